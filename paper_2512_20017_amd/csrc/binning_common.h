// Device code shared by the binning kernels of the 3D-Gaussian and the 2D-surfel variants: the block of 256 consecutive
// points that compacts its visible points, writes their raster records and emits their (tile, point) pairs.
#pragma once
#include "pbdr_internal.h"
#include "pair_reduce.h"

namespace pbdr {

// Pair counts are summed with saturation at 2^31 - 1: a degenerate state (many screen-filling splats) cannot wrap the
// 32-bit prefix sums; everything at or beyond the capacity (< 2^30) is dropped and reported as overflow.
constexpr uint32_t kPairSat = 0x7fffffffu;
__device__ __forceinline__ uint32_t sat_add(uint32_t a, uint32_t b)      // a, b <= kPairSat
{
    return min(a + b, kPairSat);
}

__device__ __forceinline__ uint32_t wave_inclusive_scan_sat(uint32_t v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(v, d, 64);
        if (lane >= d) v = sat_add(v, t);
    }
    return v;
}

// What the pair emission reads and writes (device pointers into the workspace).
struct BinArrays {
    const uint32_t* touched;     // [n] tiles per point, 0 = not listed
    const uint32_t* blk_vis;     // [blocks] listed points in the blocks before this one
    const uint32_t* blk_pairs;   // [blocks] pairs of the blocks before this one (saturating)
    const uint32_t* blk_order;   // [blocks] the block of points each workgroup takes: those with the most pairs first
    const uint32_t* blk_count;   // [blocks] listed points of each block
    uint32_t* order;             // [n] listed points in index order ("rank" -> point)
    uint32_t* offsets;           // [n + 1] first pair of each rank; offsets[listed] = pair total (written by the block scan)
    uint32_t* slot_base;         // [n] first pair of each listed point, by point index
    uint32_t* depth_bits;        // [n] bit pattern of the depth, by point index
    uint32_t* tkeys;             // [cap] tile id of each pair, in emission order
    uint32_t* tvals;             // [cap] point index of each pair
    uint32_t* chunk_rank;        // rank owning every 256th pair (pair_reduce.h)
    uint32_t cap;
    uint32_t* status;
};

// One block of 256 consecutive points. A listed point gets its rank among the listed points (index order), its raster
// record (pack(i), supplied by the variant), and the slots [at, at + count) of the pair list, where its pairs go in
// row-major order over its tile rectangle. Every (tile, point) pair of a wavefront's 64 consecutive points is written
// by whichever lane comes next, so the work is balanced whatever the mix of small and large splats: the pairs of those
// 64 points occupy one contiguous range (the slots are a prefix sum); lane l writes slots B + l, B + l + 64, ... and
// finds the owning point of a slot from the range starts (see the loop). Points are emitted in index
// order: the depth order of each tile's list is made afterwards, tile by tile (k_tile_depth_sort).
template <class Pack>
__device__ __forceinline__ void pack_dup_block(const BinInput& in, const CamDev& cam, const BinArrays& A,
                                               const float* __restrict__ depth, Pack pack)
{
    __shared__ uint32_t sMark[4][64];      // per wavefront: which lane's range starts at each slot of the current step
    __shared__ uint32_t sVis[4], sPairs[4];
    // the blocks with many pairs are started first: their wavefronts run longest (64 slots per step), and in index order
    // the launch ended on the few that happened to come late
    const uint32_t blk = A.blk_order[blockIdx.x];
    // a block none of whose points is listed has nothing to write (most blocks, when the view sees a tenth of a large cloud)
    if (A.blk_count[blk] == 0u) return;
    const int i = (int)(blk * 256u + threadIdx.x);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t cnt = (i < in.n) ? A.touched[i] : 0u;
    const bool vis = cnt > 0u;
    const unsigned long long vm = __ballot(vis);
    const uint32_t inc = wave_inclusive_scan_sat(cnt);
    if (lane == 63) { sVis[wave] = (uint32_t)__popcll(vm); sPairs[wave] = inc; }
    __syncthreads();
    uint32_t slot = A.blk_vis[blk] + (uint32_t)__popcll(vm & ((1ull << lane) - 1ull));
    const uint32_t below = __shfl_up(inc, 1, 64);                    // exclusive = the lane below's inclusive sum
    uint32_t at = sat_add(A.blk_pairs[blk], lane == 0 ? 0u : below);
#pragma unroll
    for (int w = 0; w < 3; ++w)
        if (w < wave) { slot += sVis[w]; at = sat_add(at, sPairs[w]); }
    int x0 = 0, y0 = 0, x1 = 0, y1 = 0;
    if (vis) {
        const float mx = in.mean2d[i], my = in.mean2d[(size_t)in.n + i];
        tile_rect(cam, mx, my, in.radius[i], x0, y0, x1, y1);
        A.order[slot] = (uint32_t)i;
        A.offsets[slot] = at;
        A.slot_base[i] = at;
        A.depth_bits[i] = __float_as_uint(depth[i]);
        pack(i);
        // which rank owns every 256th pair (for the pair-balanced gather of the backward pass)
        const uint32_t end = min(at + cnt, A.cap);
        for (uint32_t c = (at + kChunkPairs - 1) / kChunkPairs; (uint64_t)c * kChunkPairs < end; ++c) A.chunk_rank[c] = slot;
    }
    const int w = x1 - x0;
    const uint32_t first = (uint32_t)__builtin_amdgcn_readlane((int)at, 0);
    const uint32_t last_raw = (uint32_t)__builtin_amdgcn_readlane((int)(at + cnt), 63);
    const uint32_t last = min(last_raw, A.cap);        // slots at or beyond the capacity are dropped
    __builtin_amdgcn_wave_barrier();
    // Uniform trip count: every lane takes part in the cross-lane reads of each step, only lanes with a slot store.
    // The owner of slot u is the last lane whose range starts at or before u (the ranges are a prefix sum: no gaps, and
    // the ranges of listed points start at distinct slots). Per step of 64 slots: the lanes whose range starts inside
    // the step leave their number at that slot's place in LDS, and a running maximum over the lanes (DPP), carried from
    // step to step, hands every slot its owner - one LDS round trip per step where a binary search over the 64 range
    // ends took six in a row, which is what the wavefronts with thousands of pairs, the last to finish, were made of.
    int carry = -1;
    for (uint32_t base = first; base < last; base += 64) {
        const uint32_t u = base + lane;
        sMark[wave][lane] = 0xffffffffu;
        if (vis && at - base < 64u) sMark[wave][at - base] = (uint32_t)lane;      // at >= base or the difference wraps past 64
        __builtin_amdgcn_wave_barrier();
        int lo = (int)sMark[wave][lane];                  // -1 where no range starts
        __builtin_amdgcn_wave_barrier();
        lo = max(lo, __builtin_amdgcn_update_dpp(-1, lo, 0x111, 0xf, 0xf, false));      // row_shr:1
        lo = max(lo, __builtin_amdgcn_update_dpp(-1, lo, 0x112, 0xf, 0xf, false));      // row_shr:2
        lo = max(lo, __builtin_amdgcn_update_dpp(-1, lo, 0x114, 0xf, 0xf, false));      // row_shr:4
        lo = max(lo, __builtin_amdgcn_update_dpp(-1, lo, 0x118, 0xf, 0xf, false));      // row_shr:8
        lo = max(lo, __builtin_amdgcn_update_dpp(-1, lo, 0x142, 0xa, 0xf, false));      // row_bcast:15 into rows 1 and 3
        lo = max(lo, __builtin_amdgcn_update_dpp(-1, lo, 0x143, 0xc, 0xf, false));      // row_bcast:31 into rows 2 and 3
        lo = max(lo, carry);
        carry = __builtin_amdgcn_readlane(lo, 63);
        const int src = max(lo, 0);
        const int ox0 = __shfl(x0, src, 64), oy0 = __shfl(y0, src, 64), ow = __shfl(w, src, 64);
        const uint32_t oat = (uint32_t)__shfl((int)at, src, 64);
        const uint32_t oid = blk * 256u + (uint32_t)(wave * 64 + src);
        if (u < last && lo >= 0 && ow > 0) {
            const int t = (int)(u - oat);
            const int ty = oy0 + t / ow, tx = ox0 + t - (t / ow) * ow;
            A.tkeys[u] = (uint32_t)(ty * cam.TX + tx);
            A.tvals[u] = oid;
        }
    }
    if (lane == 0 && last_raw > A.cap) A.status[kStOverflow] = 1u;
}

}  // namespace pbdr
