// Per-point sums over the per-pair records of the backward pass, balanced by pairs.
//
// The pairs of the listed point with rank r (its place among the listed points, in index order) occupy [offsets[r], offsets[r+1]) of the unsorted duplicate list, so the
// records to add up for one point are contiguous, but their number varies from one to thousands. Work is therefore
// cut by pairs, not by points: a wavefront owns 256 consecutive pairs (four steps of 64), finds the owning rank of
// each pair by binary search over a window of 64 range ends in LDS (64 pairs span at most 64 ranks: every visible
// point has at least one pair), and runs a segmented inclusive scan over the 64 records with DPP row shifts and row
// broadcasts (owners are sorted, so "same owner as the lane d below" is the whole segment test). A segment that
// lies inside the wavefront's 256 pairs is stored directly. Segments cut by a wavefront boundary leave a left and /
// or right piece in a small carry array, and a second kernel - one thread per boundary at which a segment starts -
// adds the pieces in order. No atomics, no zero-filled outputs, same result on every run.
#pragma once
#include "pbdr_internal.h"

namespace pbdr {

constexpr int kChunkPairs = 256;   // pairs per wavefront

// carry record per wavefront: [0..15] left piece, [16..31] right piece, then {flags, left rank, right rank, -}
constexpr int kCarryFloats = 36;
enum { kCarryHasLeft = 1, kCarryLeftThrough = 2, kCarryHasRight = 4 };

// chunk_rank[c] = rank that owns pair c * 256; written by the packing kernel (a rank writes one entry per 256 pairs it
// spans).

template <int kCtrl>
__device__ __forceinline__ float dpp_shift0(float v)    // shifted-in lanes read 0
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xf, 0xf, true));
}
template <int kCtrl>
__device__ __forceinline__ int dpp_shift_m1(int v)      // shifted-in lanes read -1
{
    return __builtin_amdgcn_update_dpp(-1, v, kCtrl, 0xf, 0xf, false);
}

// Segmented inclusive scan over the 64 lanes for non-decreasing owners: four steps inside each row of 16 lanes, then
// the last lane of row 0 / 2 into rows 1 / 3 and lane 31 into rows 2 and 3, each added where the owner matches.
template <int kVals>
__device__ __forceinline__ void seg_scan_sorted(float (&v)[kVals], int owner)
{
#define PBDR_SEG_STEP(CTRL)                                                        \
    {                                                                              \
        const bool same = dpp_shift_m1<CTRL>(owner) == owner;                      \
        _Pragma("unroll") for (int k = 0; k < kVals; ++k) {                        \
            const float t = dpp_shift0<CTRL>(v[k]);                                \
            v[k] += same ? t : 0.f;                                                \
        }                                                                          \
    }
    PBDR_SEG_STEP(0x111)   // row_shr:1
    PBDR_SEG_STEP(0x112)   // row_shr:2
    PBDR_SEG_STEP(0x114)   // row_shr:4
    PBDR_SEG_STEP(0x118)   // row_shr:8
#undef PBDR_SEG_STEP
    {   // row_bcast:15 into rows 1 and 3
        const int o = __builtin_amdgcn_update_dpp(-1, owner, 0x142, 0xa, 0xf, false);
        const bool same = o == owner;
#pragma unroll
        for (int k = 0; k < kVals; ++k) {
            const float t = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[k]), 0x142, 0xa, 0xf, false));
            v[k] += same ? t : 0.f;
        }
    }
    {   // row_bcast:31 into rows 2 and 3
        const int o = __builtin_amdgcn_update_dpp(-1, owner, 0x143, 0xc, 0xf, false);
        const bool same = o == owner;
#pragma unroll
        for (int k = 0; k < kVals; ++k) {
            const float t = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[k]), 0x143, 0xc, 0xf, false));
            v[k] += same ? t : 0.f;
        }
    }
}

// One wavefront's 256 pairs. kVec4 float4 per record, of which the first kVals floats are summed. `store(rank, v)`
// writes a finished sum for rank `rank`. sEnd: 64 words of LDS private to the wavefront.
// kTagged: the last two words of a record carry the 64-bit number of the backward call that wrote it (the workspace
// counts its backward calls from one; it starts zero-filled, so no record of an earlier call, and no record never
// written, carries the current number); a record with any other tag was not written by this call (its pair lies beyond
// the last splat its tile blended) and counts as zero. That replaces clearing all records before every backward pass.
template <int kVec4, int kVals, bool kTagged, class Store>
__device__ __forceinline__ void gather_wave(uint32_t w, int n, const uint32_t* __restrict__ status,
                                            const uint32_t* __restrict__ offsets, const uint32_t* __restrict__ chunk_rank,
                                            const float4* __restrict__ partial, uint32_t cap, float* __restrict__ carry,
                                            uint32_t* sEnd, Store store)
{
    const int lane = threadIdx.x & 63;
    const uint32_t Pc = min(status[kStNumDup], cap);
    const uint32_t m = min(status[kStNumVis], (uint32_t)n);
    const uint32_t epoch_lo = status[kStEpoch] + 1u, epoch_hi = status[kStEpoch + 1] + (epoch_lo == 0u ? 1u : 0u);
    const uint32_t wbeg = w * (uint32_t)kChunkPairs;
    if (wbeg >= Pc) return;
    const uint32_t wend = min(wbeg + (uint32_t)kChunkPairs, Pc);
    const uint32_t r0 = chunk_rank[w];
    const bool left_open = min(offsets[r0], cap) < wbeg;     // the first rank's pairs begin in an earlier wavefront
    uint32_t r_cur = r0;
    bool carry_valid = false;
    float cin[kVals];
#pragma unroll
    for (int k = 0; k < kVals; ++k) cin[k] = 0.f;
    uint32_t flags = 0, right_rank = 0;
    float* my_carry = carry + (size_t)w * kCarryFloats;
    for (uint32_t base = wbeg; base < wend; base += 64) {
        const uint32_t u = base + lane;
        const bool valid = u < wend;
        const bool last_iter = base + 64 >= wend;
        float v[kVals];
#pragma unroll
        for (int k = 0; k < kVals; ++k) v[k] = 0.f;
        if (valid) {
            float4 rec[kVec4];
#pragma unroll
            for (int q = 0; q < kVec4; ++q) rec[q] = partial[(size_t)kVec4 * u + q];
            const bool written = !kTagged || (__float_as_uint(rec[kVec4 - 1].z) == epoch_lo && __float_as_uint(rec[kVec4 - 1].w) == epoch_hi);
#pragma unroll
            for (int k = 0; k < kVals; ++k) {
                const float4 r = rec[k >> 2];
                const float x = (k & 3) == 0 ? r.x : (k & 3) == 1 ? r.y : (k & 3) == 2 ? r.z : r.w;
                v[k] = written ? x : 0.f;
            }
        }
        {   // range ends of ranks r_cur .. r_cur + 63
            const uint32_t rr = r_cur + lane;
            sEnd[lane] = (rr < m) ? min(offsets[rr + 1], cap) : 0xffffffffu;
        }
        __builtin_amdgcn_wave_barrier();
        int owner = 0;
#pragma unroll
        for (int step = 32; step >= 1; step >>= 1)
            if (sEnd[owner + step - 1] <= u) owner += step;
        const uint32_t seg_end = sEnd[min(owner, 63)];
        __builtin_amdgcn_wave_barrier();
        if (!valid) owner = 64 + lane;
        if (carry_valid && owner == 0) {      // the segment left open by the previous step continues at lane 0
            const bool head = lane == 0;
#pragma unroll
            for (int k = 0; k < kVals; ++k) v[k] += head ? cin[k] : 0.f;
        }
        seg_scan_sorted<kVals>(v, owner);
        const int onext = __shfl_down(owner, 1, 64);
        const bool end_lane = valid && (lane == 63 || onext != owner);
        const bool closed = seg_end == u + 1;               // the rank has no pair beyond this lane's
        const uint32_t rank = r_cur + (uint32_t)owner;
        const bool first_piece = left_open && rank == r0;
        if (end_lane) {
            if (closed) {
                if (first_piece) {
#pragma unroll
                    for (int k = 0; k < kVals; ++k) my_carry[k] = v[k];
                } else if (rank < m) {      // always true for consistent inputs; keeps the write in bounds regardless
                    store(rank, v);
                }
            } else if (last_iter) {
                float* dst = first_piece ? my_carry : my_carry + 16;
#pragma unroll
                for (int k = 0; k < kVals; ++k) dst[k] = v[k];
            }
        }
        // uniform bookkeeping
        const unsigned long long b_end = __ballot(end_lane);
        const unsigned long long b_left_closed = __ballot(end_lane && closed && first_piece);
        const unsigned long long b_open = __ballot(end_lane && !closed);
        if (b_left_closed) flags |= kCarryHasLeft;
        carry_valid = false;
        if (b_open) {        // at most one lane: the last valid one
            const int ol = 63 - __builtin_clzll(b_open);
            const uint32_t orank = r_cur + (uint32_t)__builtin_amdgcn_readlane(owner, ol);
            if (last_iter) {
                if (left_open && orank == r0) flags |= kCarryHasLeft | kCarryLeftThrough;
                else { flags |= kCarryHasRight; right_rank = orank; }
            } else {
                carry_valid = true;
#pragma unroll
                for (int k = 0; k < kVals; ++k)
                    cin[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v[k]), 63));
            }
            r_cur = orank;
        } else if (b_end) {
            const int ll = 63 - __builtin_clzll(b_end);
            r_cur = r_cur + (uint32_t)__builtin_amdgcn_readlane(owner, ll) + 1u;
        }
    }
    if (lane == 0) {
        uint32_t* meta = reinterpret_cast<uint32_t*>(my_carry + 32);
        meta[0] = flags; meta[1] = r0; meta[2] = right_rank; meta[3] = 0u;
    }
}

// One thread per wavefront boundary at which a cut segment starts: right piece of wavefront w, then the left pieces
// of the following wavefronts up to and including the first that is not a through piece.
template <int kVals, class Store>
__device__ __forceinline__ void gather_fixup(uint32_t w, const uint32_t* __restrict__ status, uint32_t cap,
                                             const float* __restrict__ carry, Store store)
{
    const uint32_t Pc = min(status[kStNumDup], cap);
    const uint32_t nw = (Pc + kChunkPairs - 1) / kChunkPairs;
    if (w >= nw) return;
    const float* c = carry + (size_t)w * kCarryFloats;
    const uint32_t* meta = reinterpret_cast<const uint32_t*>(c + 32);
    if (!(meta[0] & kCarryHasRight)) return;
    const uint32_t rank = meta[2];
    float v[kVals];
#pragma unroll
    for (int k = 0; k < kVals; ++k) v[k] = c[16 + k];
    for (uint32_t w2 = w + 1; w2 < nw; ++w2) {
        const float* c2 = carry + (size_t)w2 * kCarryFloats;
        const uint32_t* m2 = reinterpret_cast<const uint32_t*>(c2 + 32);
        const uint32_t f2 = m2[0];
        if (!(f2 & kCarryHasLeft) || m2[1] != rank) break;
#pragma unroll
        for (int k = 0; k < kVals; ++k) v[k] += c2[k];
        if (!(f2 & kCarryLeftThrough)) break;
    }
    store(rank, v);
}

// What k_gather_fixup does, from the side of the point: used by the kernels that read a point's record right after the
// gather, so that the fixup launch (a few microseconds for ten thousand additions) can be left out. at, count: the
// point's first pair and its number of pairs. Returns false if all of its pairs lie in one wavefront's 256 (the gather
// stored the record itself); else v = the right piece of the wavefront its first pair lies in, plus the left pieces of
// the following wavefronts up to and including the first that is not a through piece - the pieces and the order of
// gather_fixup, so the sum is bit for bit the record that kernel would store.
template <int kVals>
__device__ __forceinline__ bool record_from_carries(const CarryFold& cf, uint32_t at, uint32_t count, float (&v)[kVals])
{
    const uint32_t Pc = min(cf.status[kStNumDup], cf.cap);
    const uint32_t beg = min(at, Pc), end = min(at + count, Pc);      // (at < 2^31, count <= 2^24)
    const uint32_t w = beg / (uint32_t)kChunkPairs;
    if (end <= (w + 1u) * (uint32_t)kChunkPairs) return false;
    const uint32_t nw = (Pc + kChunkPairs - 1) / kChunkPairs;
    const float* c = cf.carry + (size_t)w * kCarryFloats;
    const uint32_t rank = reinterpret_cast<const uint32_t*>(c + 32)[2];
#pragma unroll
    for (int k = 0; k < kVals; ++k) v[k] = c[16 + k];
    for (uint32_t w2 = w + 1; w2 < nw; ++w2) {
        const float* c2 = cf.carry + (size_t)w2 * kCarryFloats;
        const uint32_t* m2 = reinterpret_cast<const uint32_t*>(c2 + 32);
        const uint32_t f2 = m2[0];
        if (!(f2 & kCarryHasLeft) || m2[1] != rank) break;
#pragma unroll
        for (int k = 0; k < kVals; ++k) v[k] += c2[k];
        if (!(f2 & kCarryLeftThrough)) break;
    }
    return true;
}

// the count of backward calls on this workspace goes up by one (k_gather_fixup does it when it runs)
__device__ __forceinline__ void close_backward_epoch(uint32_t* status)
{
    const uint32_t lo = status[kStEpoch] + 1u;
    status[kStEpoch] = lo;
    if (lo == 0u) status[kStEpoch + 1] = status[kStEpoch + 1] + 1u;
}

}  // namespace pbdr
