// Stable least-significant-digit radix sort of (32-bit key, 32-bit value) pairs with a digit width chosen per pass.
//
// The order the renderer needs is the order of the 64-bit key (tile << 32 | depth bits). All duplicates of a splat
// share the low 32 bits, so the depth passes run on the n splats before duplication and only the tile passes run on
// the P pairs; the result is the same permutation a 64-bit sort of the pairs would give.
//
// Digits are at most 8 bits wide: the key bits are cut into the fewest such passes, evenly (13 tile bits = 7 + 6).
// Wider digits were measured slower although they save a pass (three 11-bit passes for the depth bits): with 2048
// bins a 2048-pair tile holds about one pair per bin, so every scattered key is a lone 4-byte write.
//
// A pass is three launches and no workgroup ever waits for another: (1) per-tile digit counts, (2) one workgroup per
// digit scans its counts over the tiles and leaves the digit's total, (3) each tile turns the totals into where
// each digit's run starts (one small scan per workgroup), ranks its pairs per wavefront with ballots and scatters.
// Per pass: 4 B (counts) + 8 B read + 8 B written per pair.
#include "pbdr_internal.h"

namespace pbdr {

constexpr int kSortPerThread = kSortItems / 256;
constexpr int kWaveItems = kSortItems / 4;        // consecutive pairs per wavefront

// Lanes of the wavefront that hold the same kBits-bit digit as this lane (among the valid ones), by kBits ballots.
template <int kBits>
__device__ __forceinline__ uint64_t digit_peers(uint32_t digit, bool valid)
{
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < kBits; ++b) {
        const bool bit = (digit >> b) & 1u;
        const uint64_t m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    return peers;
}

__device__ __forceinline__ uint32_t sort_count(const uint32_t* __restrict__ count_ptr, uint32_t count_cap)
{
    return count_ptr ? min(*count_ptr, count_cap) : count_cap;
}

// per-tile digit counts: hist[d * ntiles + tile]. One digit per valid lane goes into an LDS histogram. kPlain: every
// lane adds one (the low digits of tile ids in point order: a wavefront's 64 keys are mostly different tiles, and the
// lookup of equal digits below is then seven ballots per key for nothing; measured 10.5 -> 6.7 us at 2.9 M pairs).
// Else the lowest lane of each group of equal digits adds the group's size, so a digit shared by much of the wavefront
// (the high tile bits once the low ones are sorted) costs one add instead of a serialised atomic (8.8 us against 11.0
// with plain adds).
template <int kBits, bool kPlain>
__global__ __launch_bounds__(256) void k_radix_tile_hist(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ count_ptr,
                                                         uint32_t count_cap, int shift, uint32_t* __restrict__ hist, uint32_t ntiles)
{
    constexpr int kBins = 1 << kBits;
    constexpr uint32_t kMask = kBins - 1;
    __shared__ uint32_t h[kBins];
    const uint32_t count = sort_count(count_ptr, count_cap);
    const uint32_t base = blockIdx.x * (uint32_t)kSortItems;
    if (base >= count) return;     // uniform for the workgroup; tiles past the count are never read
    for (int d = threadIdx.x; d < kBins; d += 256) h[d] = 0;
    __syncthreads();
    const uint64_t lt_mask = (1ull << (threadIdx.x & 63)) - 1ull;
    // four consecutive keys per load (a histogram does not care which lane counts which key)
    uint32_t key[kSortPerThread];
#pragma unroll
    for (int k = 0; k < kSortPerThread / 4; ++k) {
        const uint32_t idx = base + (k * 256 + threadIdx.x) * 4u;
        if (idx + 4u <= count) {
            const uint4 v = *reinterpret_cast<const uint4*>(keys + idx);
            key[4 * k] = v.x; key[4 * k + 1] = v.y; key[4 * k + 2] = v.z; key[4 * k + 3] = v.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) key[4 * k + j] = idx + j < count ? keys[idx + j] : 0u;
        }
    }
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = base + ((k >> 2) * 256 + threadIdx.x) * 4u + (uint32_t)(k & 3);
        const bool valid = idx < count;
        const uint32_t digit = (key[k] >> shift) & kMask;
        if (kPlain) {
            if (valid) atomicAdd(&h[digit], 1u);
        } else {
            const uint64_t peers = digit_peers<kBits>(digit, valid);
            if (valid && (peers & lt_mask) == 0ull) atomicAdd(&h[digit], (uint32_t)__popcll(peers));
        }
    }
    __syncthreads();
    for (int d = threadIdx.x; d < kBins; d += 256) hist[(size_t)d * ntiles + blockIdx.x] = h[d];
}

// one workgroup per digit: exclusive scan of that digit's counts over the tiles that hold keys (in place);
// totals[digit] = their sum. 1024 threads, two consecutive counts each: 2048 tiles (4 M pairs) are one trip.
__global__ __launch_bounds__(1024) void k_radix_digit_scan(uint32_t* __restrict__ hist, uint32_t row_stride,
                                                           const uint32_t* __restrict__ count_ptr, uint32_t count_cap,
                                                           uint32_t* __restrict__ totals)
{
    __shared__ uint32_t lds[16];
    __shared__ uint32_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t ntiles = (sort_count(count_ptr, count_cap) + kSortItems - 1) / kSortItems;
    uint32_t* row = hist + (size_t)blockIdx.x * row_stride;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (uint32_t start = 0; start < ntiles; start += 2048) {
        const uint32_t idx = start + 2u * threadIdx.x;
        const uint32_t v0 = idx < ntiles ? row[idx] : 0u, v1 = idx + 1u < ntiles ? row[idx + 1u] : 0u;
        const uint32_t v = v0 + v1;
        uint32_t inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t t = __shfl_up(inc, d, 64);
            if (lane >= d) inc += t;
        }
        if (lane == 63) lds[wave] = inc;
        __syncthreads();
        uint32_t base = carry_s, chunk = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) { const uint32_t t = lds[w]; if (w < wave) base += t; chunk += t; }
        if (idx < ntiles) row[idx] = base + inc - v;
        if (idx + 1u < ntiles) row[idx + 1u] = base + inc - v1;
        __syncthreads();
        if (threadIdx.x == 0) carry_s += chunk;
        __syncthreads();
    }
    if (threadIdx.x == 0) totals[blockIdx.x] = carry_s;
}

// Scatter of one pass. The tile's pairs are first put in digit order in LDS (rank within the wavefront's round by
// ballots, then wavefront and round order: stable), then written out in that order: consecutive lanes hold
// consecutive members of a digit's run, so a run leaves as whole cache lines instead of lone 4-byte writes (measured:
// the first tile pass wrote 4x its algorithmic bytes when every lane stored its own pair straight to its place).
template <int kBits>
__global__ __launch_bounds__(256) void k_radix_scatter(const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in,
                                                       uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out,
                                                       const uint32_t* __restrict__ count_ptr, uint32_t count_cap, int shift,
                                                       const uint32_t* __restrict__ hist_scanned, uint32_t ntiles,
                                                       const uint32_t* __restrict__ totals)
{
    constexpr int kBins = 1 << kBits;
    constexpr uint32_t kMask = kBins - 1;
    constexpr int kPer = (kBins + 255) / 256;       // digits per thread in the run-start phase (consecutive digits)
    __shared__ uint32_t wave_base[4][kBins];        // per wavefront and digit: count, then next local position
    __shared__ uint32_t gdelta[kBins];              // global position minus local position, per digit
    __shared__ uint32_t sK[kSortItems], sV[kSortItems];
    __shared__ uint32_t sScan[2][4];
    const uint32_t count = sort_count(count_ptr, count_cap);
    const uint32_t block_base = blockIdx.x * (uint32_t)kSortItems;
    if (block_base >= count) return;  // uniform for the whole workgroup
    const uint32_t block_n = min((uint32_t)kSortItems, count - block_base);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t wbase = block_base + wave * kWaveItems;
    // digit totals and this tile's offset within each digit's run: loaded first, needed only after the ranking
    uint32_t tot[kPer], tile_off[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int d = threadIdx.x * kPer + j;
        tot[j] = d < kBins ? totals[d] : 0u;
        tile_off[j] = d < kBins ? hist_scanned[(size_t)d * ntiles + blockIdx.x] : 0u;
    }
    // this wavefront's consecutive pairs, in rounds of 64, kept in registers together with each pair's rank among
    // the equal digits of its round and the size of that group
    uint32_t key[kSortPerThread], val[kSortPerThread], rank[kSortPerThread], group[kSortPerThread];
    // (all sixteen loads first: written as one loop with the ranking, each round waited for its own two)
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        key[k] = 0u; val[k] = 0u;
        if (idx < count) { key[k] = keys_in[idx]; val[k] = vals_in[idx]; }
    }
    for (int d = threadIdx.x; d < kBins; d += 256) {
#pragma unroll
        for (int w = 0; w < 4; ++w) wave_base[w][d] = 0;
    }
    __syncthreads();
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        const bool valid = idx < count;
        const uint32_t digit = (key[k] >> shift) & kMask;
        const uint64_t peers = digit_peers<kBits>(digit, valid);
        rank[k] = (uint32_t)__popcll(peers & lt_mask);
        group[k] = (uint32_t)__popcll(peers);
        if (valid && rank[k] == 0u) atomicAdd(&wave_base[wave][digit], group[k]);
    }
    __syncthreads();
    {   // two exclusive scans over the digits at once: of the digit totals (where each digit's run starts globally)
        // and of this tile's digit counts (where it starts in LDS)
        uint32_t cnt[kPer], my_tot = 0, my_cnt = 0;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int d = threadIdx.x * kPer + j;
            cnt[j] = 0;
            if (d < kBins) cnt[j] = wave_base[0][d] + wave_base[1][d] + wave_base[2][d] + wave_base[3][d];
            my_tot += tot[j]; my_cnt += cnt[j];
        }
        uint32_t inc_t = my_tot, inc_c = my_cnt;
#pragma unroll
        for (int k = 1; k < 64; k <<= 1) {
            const uint32_t a = __shfl_up(inc_t, k, 64), c = __shfl_up(inc_c, k, 64);
            if (lane >= k) { inc_t += a; inc_c += c; }
        }
        if (lane == 63) { sScan[0][wave] = inc_t; sScan[1][wave] = inc_c; }
        __syncthreads();
        uint32_t below = inc_t - my_tot, lstart = inc_c - my_cnt;
#pragma unroll
        for (int w = 0; w < 3; ++w) if (w < wave) { below += sScan[0][w]; lstart += sScan[1][w]; }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int d = threadIdx.x * kPer + j;
            if (d < kBins) {
                gdelta[d] = below + tile_off[j] - lstart;
                uint32_t run = lstart;
#pragma unroll
                for (int w = 0; w < 4; ++w) { const uint32_t c = wave_base[w][d]; wave_base[w][d] = run; run += c; }
            }
            below += tot[j]; lstart += cnt[j];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        if (idx < count) {
            const uint32_t digit = (key[k] >> shift) & kMask;
            const uint32_t start = wave_base[wave][digit];          // every peer reads before the leader updates
            if (rank[k] == 0u) wave_base[wave][digit] = start + group[k];
            const uint32_t lpos = min(start + rank[k], (uint32_t)kSortItems - 1u);   // < block_n for consistent inputs
            sK[lpos] = key[k];
            sV[lpos] = val[k];
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t e = (uint32_t)k * 256u + threadIdx.x;
        if (e < block_n) {
            const uint32_t kk = sK[e];
            const uint32_t dst = e + gdelta[(kk >> shift) & kMask];
            if (dst < count_cap) {                                   // always true for consistent inputs
                keys_out[dst] = kk;
                vals_out[dst] = sV[e];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Depth order inside each tile's list. After the stable sort by tile id every tile's list holds its splats in point
// order; the list is then sorted stably by the 32 depth bits, which leaves the order of the key
// (tile << 32 | depth bits), ties by point index. One launch, every list on its own:
//   - fewer than 1023 entries (k_tile_order lists the tiles longest first and says how many have more): one WAVEFRONT
//     per list, four lists per workgroup, no workgroup barrier anywhere: up to 64 entries by counting (every lane
//     compares its key with all others through the scalar unit), else least-significant-digit radix passes with 9-bit
//     digits over the bit positions in which the list's keys differ at all (depths of one tile share sign and most
//     exponent bits: about 26 bits differ, which is three 9-bit digits where 8-bit digits took four passes; the 512
//     counters fit the space of 256 because they are 16 bits wide, two to a word). Keys and positions live in
//     registers in list order; a pass scatters them into the wavefront's 7 KB of LDS and reads them back in the new order (lists of 511 to 1022 entries took a whole workgroup
//     before: four wavefront slots for 16 us each where one wavefront now takes them, 57 -> 53 us);
//   - up to 6400 entries: the same passes by a whole workgroup, three barriers per pass. What moves is the permutation
//     (16-bit positions, two copies in LDS); the keys stay where they are, in incoming order - in LDS for lists of up
//     to 2048 entries, in the global scratch array (the spent tile ids) beyond - and are fetched through it;
//   - longer lists: keys and values move between the global scratch arrays, each wavefront sweeping its quarter of
//     the list once per pass (the first pass twice: count, then place; a placing sweep counts for the next pass).
// Under 30 KB of LDS and at most 96 registers, so that five workgroups share a compute unit: the work is a chain of
// dependent LDS and cross-lane steps per list, and what hides it is other lists in flight (measured: with 32.3 KB only
// four were resident, and the benchmark view's sort took 53.6 us instead of 50.6). That is why the per-wavefront digit
// counters double as the starting positions, at the price of the third barrier.
// A pass ranks its entries per wavefront and round of 64 by ballots (lanes with the same digit find each other), the
// first lane of each group adds the group's size to the digit's counter in LDS and gets back how many entries of that
// digit came before (earlier rounds of the wavefront: LDS executes a wavefront's operations in order), and hands that
// to its group through the LDS crossbar: equal digits keep their incoming order.
// ---------------------------------------------------------------------------------------------
constexpr int kListBits = 9;                          // digit width of the list sorts: depths of one tile differ in about 26 bits, three digits
constexpr int kListBins = 1 << kListBits;
constexpr int kListWords = kListBins / 2;             // counters in LDS are 16 bits wide, two digits to a word (the LDS adds 32-bit words)
constexpr int kPerLane = kListWords / 64;             // a wavefront's counter words, per lane
static_assert(kWaveListMax % 64 == 0, "whole rounds");
constexpr int kWgKeyMax = 2048;                       // a workgroup's list with its keys in LDS (8 rounds per wavefront)
constexpr int kWgListMax = 6400;                      // a workgroup's list with its permutation in LDS (25 rounds per wavefront)

struct WaveSortLds {      // a wavefront's share of the LDS when it sorts a list of its own
    uint32_t key[kWaveListMax];
    uint16_t idx[kWaveListMax];
    uint32_t hist[kListWords];
};
struct WgSortLds {        // the workgroup's LDS when it sorts one list together
    union {
        struct { uint32_t key[kWgKeyMax]; uint16_t idx[2][kWgKeyMax]; } a;      // keys in incoming order + the permutation, twice
        struct { uint16_t idx[2][kWgListMax]; } b;                              // the permutation alone
    } u;
    uint32_t cnt[4][kListWords];                             // per wavefront and digit: entries in the wavefront's part of the list, then where its first entry of that digit goes
    uint32_t scan[4];
    uint32_t mask;
};
union ListSortLds { WgSortLds wg; WaveSortLds wave[4]; };
static_assert(sizeof(ListSortLds) <= 30 * 1024 + 512, "five workgroups per compute unit (32.3 KB did not fit five times)");

// bit range [lo, hi] in which the keys differ -> number of kListBits-bit passes and the shift of pass p (the topmost digit
// may reach past bit hi into bits all keys share; it never reaches past bit 31)
__device__ __forceinline__ int list_passes(uint32_t diff, int& lo)
{
    lo = __builtin_ctz(diff);
    const int hi = 31 - __builtin_clz(diff);
    return (hi - lo + kListBits) / kListBits;
}
__device__ __forceinline__ int list_shift(int lo, int p) { return min(lo + kListBits * p, 32 - kListBits); }

// Entries of this wavefront with the same digit as this lane's that come before it: earlier rounds (through the
// digit's counter in `hist`, a row no other wavefront touches) plus lower lanes of this round. The lanes that share the
// digit are found bit by bit: a lane differs from this one if, for some bit, its bit (one ballot per bit) is not this
// lane's bit (sign-extended to a mask); both halves of the 64-lane sets are kept in 32-bit registers.
// kPacked: the counters are 16 bits wide, digit d in half d & 1 of word d >> 1 (for lists of fewer than 65,536 entries:
// no half ever carries into its neighbour); else one word per digit.
__device__ __forceinline__ uint32_t packed_half(uint32_t word, uint32_t digit) { return (word >> ((digit & 1u) << 4)) & 0xffffu; }

template <bool kPacked>
__device__ __forceinline__ uint32_t digit_prefix(uint32_t* hist, uint32_t digit, bool valid)
{
    const int lane = threadIdx.x & 63;
    uint32_t dlo = 0u, dhi = 0u;
#pragma unroll
    for (int bit = 0; bit < kListBits; ++bit) {
        const uint32_t ext = (uint32_t)__builtin_amdgcn_sbfe((int)digit, bit, 1);      // 0 or ~0
        const uint64_t m = __ballot(ext != 0u);
        dlo |= (uint32_t)m ^ ext;
        dhi |= (uint32_t)(m >> 32) ^ ext;
    }
    const uint64_t vm = __ballot(valid);
    const uint32_t plo = ~dlo & (uint32_t)vm, phi = ~dhi & (uint32_t)(vm >> 32);       // valid lanes with this lane's digit
    // lanes below this one among them
    const uint32_t below_lo = lane < 32 ? (1u << lane) - 1u : ~0u, below_hi = lane < 32 ? 0u : (1u << (lane - 32)) - 1u;
    const uint32_t rank = (uint32_t)__popc(plo & below_lo) + (uint32_t)__popc(phi & below_hi);
    uint32_t before = 0u;
    if (valid && rank == 0u) {
        const uint32_t group = (uint32_t)__popc(plo) + (uint32_t)__popc(phi);
        if (kPacked) before = packed_half(atomicAdd(&hist[digit >> 1], group << ((digit & 1u) << 4)), digit);
        else before = atomicAdd(&hist[digit], group);
    }
    const int leader = !valid ? lane : (plo ? __builtin_ctz(plo) : 32 + __builtin_ctz(phi));
    before = (uint32_t)__builtin_amdgcn_ds_bpermute(leader << 2, (int)before);
    return before + rank;
}

// exclusive scan over a wavefront's packed digit counters, 2 * kPerLane consecutive digits per lane, in place
__device__ __forceinline__ void wave_scan_digits(uint32_t* hist)
{
    const int lane = threadIdx.x & 63;
    uint32_t c[2 * kPerLane], tot = 0u;
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) {
        const uint32_t w = hist[kPerLane * lane + q];
        c[2 * q] = w & 0xffffu; c[2 * q + 1] = w >> 16;
        tot += c[2 * q] + c[2 * q + 1];
    }
    uint32_t inc = tot;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    uint32_t at = inc - tot;
#pragma unroll
    for (int q = 0; q < kPerLane; ++q) {
        const uint32_t a0 = at, a1 = at + c[2 * q];
        hist[kPerLane * lane + q] = a0 | (a1 << 16);
        at = a1 + c[2 * q + 1];
    }
}

__device__ __forceinline__ void wave_lds_sync()      // orders this wavefront's LDS writes before its later LDS reads
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// One wavefront sorts the list vals[0 .. L), 1 < L < kWaveListMax - 1, stably by depth_bits[val], in place.
__device__ __forceinline__ void wave_sort_list(WaveSortLds& W, uint32_t L, const uint32_t* __restrict__ depth_bits,
                                               uint32_t* __restrict__ vals)
{
    constexpr int R = kWaveListMax / 64;
    const int lane = threadIdx.x & 63;
    if (L <= 64u) {
        // rank by counting: entry j precedes entry i if its key is smaller, or equal and j < i
        uint32_t v = 0u, k = 0u;
        if ((uint32_t)lane < L) { v = vals[lane]; k = depth_bits[v]; }
        uint32_t before = 0u;
        for (uint32_t j = 0; j < L; ++j) {
            const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)k, (int)j);
            before += (kj < k || (kj == k && j < (uint32_t)lane)) ? 1u : 0u;
        }
        if ((uint32_t)lane < L) vals[min(before, L - 1u)] = v;       // every lane read its entry above
        return;
    }
    const int nr = (int)((L + 63u) / 64u);
    uint32_t key[R], id[R];      // the list in its current order: entry r * 64 + lane
#pragma unroll
    for (int r = 0; r < R; ++r) {
        id[r] = 0u;
        if (r < nr && r * 64u + lane < L) id[r] = vals[r * 64u + lane];      // (the point index, for the key fetch below)
    }
    uint32_t diff = 0u;
    const uint32_t k0 = depth_bits[(uint32_t)__builtin_amdgcn_readfirstlane((int)id[0])];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        key[r] = k0;
        if (r < nr && r * 64u + lane < L) key[r] = depth_bits[id[r]];
        diff |= key[r] ^ k0;
        id[r] = r * 64u + lane;                                              // from here on: the incoming position
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) diff |= (uint32_t)__shfl_xor((int)diff, d, 64);
    if (diff == 0u) return;                        // one depth throughout: point order is the order
    int lo;
    const int passes = list_passes(diff, lo);
    auto one_pass = [&](int shift) {
#pragma unroll
        for (int q = 0; q < kPerLane; ++q) W.hist[q * 64 + lane] = 0u;
        wave_lds_sync();
        uint32_t pre[R];
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (r < nr) pre[r] = digit_prefix<true>(W.hist, (key[r] >> shift) & (kListBins - 1u), r * 64u + lane < L);
        wave_lds_sync();
        wave_scan_digits(W.hist);
        wave_lds_sync();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r < nr && r * 64u + lane < L) {
                const uint32_t digit = (key[r] >> shift) & (kListBins - 1u);
                const uint32_t pos = min(packed_half(W.hist[digit >> 1], digit) + pre[r], L - 1u);
                W.key[pos] = key[r]; W.idx[pos] = (uint16_t)id[r];
            }
        }
        wave_lds_sync();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r < nr && r * 64u + lane < L) { key[r] = W.key[r * 64u + lane]; id[r] = W.idx[r * 64u + lane]; }
        }
        wave_lds_sync();      // (the next pass, or the next list of this wavefront, writes the buffer again)
    };
    for (int p = 0; p < passes; ++p) one_pass(list_shift(lo, p));
    // the point indices, through the sorted positions: every entry is fetched before the first is stored
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (r < nr && r * 64u + lane < L) key[r] = vals[id[r]];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (r < nr && r * 64u + lane < L) vals[r * 64u + lane] = key[r];
}

// A workgroup sorts the list vals[0 .. L). kKeysInLds: L <= kWgKeyMax and the keys are kept in LDS; else L <= kWgListMax
// and they are kept in `keys`, L words of global scratch. The permutation idx[c][i] = incoming position of the entry now
// at i goes back and forth between its two copies in LDS.
template <bool kKeysInLds>
__device__ __forceinline__ void wg_sort_list(WgSortLds& S, uint32_t L, const uint32_t* __restrict__ depth_bits,
                                             uint32_t* __restrict__ vals, uint32_t* __restrict__ keys)
{
    constexpr int R = ((kKeysInLds ? kWgKeyMax : kWgListMax) + 255) / 256;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint16_t* idx0 = kKeysInLds ? S.u.a.idx[0] : S.u.b.idx[0];
    uint16_t* idx1 = kKeysInLds ? S.u.a.idx[1] : S.u.b.idx[1];
    // keys of the list, in incoming order, and the bit positions in which they differ
    uint32_t diff = 0u;
    const uint32_t k0 = depth_bits[vals[0]];
    if (threadIdx.x == 0) S.mask = 0u;
    for (uint32_t i0 = 0; i0 < L; i0 += 8u * 256u) {      // eight independent fetches in flight, twice
        uint32_t t[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint32_t i = i0 + r * 256u + threadIdx.x;
            t[r] = i < L ? vals[i] : 0u;
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint32_t i = i0 + r * 256u + threadIdx.x;
            if (i < L) t[r] = depth_bits[t[r]];
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint32_t i = i0 + r * 256u + threadIdx.x;
            if (i < L) {
                diff |= t[r] ^ k0;
                if (kKeysInLds) S.u.a.key[i] = t[r]; else keys[i] = t[r];
                idx0[i] = (uint16_t)i;
            }
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) diff |= (uint32_t)__shfl_xor((int)diff, d, 64);
    __syncthreads();                               // S.mask is cleared; keys and permutation are in place
    if (lane == 0 && diff) atomicOr(&S.mask, diff);
    __syncthreads();
    const uint32_t mask = S.mask;
    if (mask == 0u) return;                        // one depth throughout (uniform for the workgroup)
    int lo;
    const int passes = list_passes(mask, lo);
    // each wavefront takes a contiguous quarter of the list, in rounds of 64
    const uint32_t per_wave = ((L + 255u) / 256u) * 64u;
    const int nr = (int)(per_wave / 64u);
    const uint32_t wb = wave * per_wave, we = min(L, wb + per_wave);
    uint16_t* src = idx0;
    uint16_t* dst = idx1;
    auto one_pass = [&](int shift) {
        // (this wavefront's count row was last read by the others before the barrier that ended the previous pass)
#pragma unroll
        for (int q = 0; q < kPerLane; ++q) S.cnt[wave][q * 64 + lane] = 0u;
        wave_lds_sync();
        uint32_t dp[R];      // per entry of this lane: digit | (entries of that digit before it in this wavefront's part) << kListBits
#pragma unroll
        for (int r0 = 0; r0 < R; r0 += 8) {       // eight key fetches in flight at a time
            if (r0 >= nr) break;
            uint32_t k[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t i = wb + (r0 + j) * 64u + lane;
                k[j] = 0u;
                if (r0 + j < nr && i < we) k[j] = kKeysInLds ? S.u.a.key[src[i]] : keys[src[i]];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (r0 + j < nr) {
                    const uint32_t digit = (k[j] >> shift) & (kListBins - 1u);
                    const uint32_t v = digit | (digit_prefix<true>(S.cnt[wave], digit, wb + (r0 + j) * 64u + lane < we) << kListBits);
                    if (r0 + j < R) dp[r0 + j] = v;
                }
            }
        }
        __syncthreads();      // every wavefront has counted
        {   // every wavefront works out where its own entries of each digit go: digits before, then the wavefronts before it
            uint32_t mine[2 * kPerLane], tot = 0u;
#pragma unroll
            for (int q = 0; q < kPerLane; ++q) {
                const int d = kPerLane * lane + q;
                const uint32_t w0 = S.cnt[0][d], w1 = S.cnt[1][d], w2 = S.cnt[2][d], w3 = S.cnt[3][d];
                const uint32_t before = (wave > 0 ? w0 : 0u) + (wave > 1 ? w1 : 0u) + (wave > 2 ? w2 : 0u);      // both halves at once
                const uint32_t all = w0 + w1 + w2 + w3;      // (a digit's count over the list is below 65,536)
                mine[2 * q] = tot + (before & 0xffffu);
                tot += all & 0xffffu;
                mine[2 * q + 1] = tot + (before >> 16);
                tot += all >> 16;
            }
            uint32_t inc = tot;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t t = __shfl_up(inc, d, 64);
                if (lane >= d) inc += t;
            }
            const uint32_t below = inc - tot;
            __syncthreads();      // every wavefront has read the counts: its row now takes its starting positions
#pragma unroll
            for (int q = 0; q < kPerLane; ++q) S.cnt[wave][kPerLane * lane + q] = (below + mine[2 * q]) | ((below + mine[2 * q + 1]) << 16);
        }
        wave_lds_sync();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r < nr && wb + r * 64u + lane < we) {
                const uint32_t digit = dp[r] & (kListBins - 1u);
                const uint32_t pos = min(packed_half(S.cnt[wave][digit >> 1], digit) + (dp[r] >> kListBits), L - 1u);
                dst[pos] = src[wb + r * 64u + lane];
            }
        }
        __syncthreads();      // the pass is written; the other copy of the permutation may be overwritten
        uint16_t* t = src; src = dst; dst = t;
    };
    for (int p = 0; p < passes; ++p) one_pass(list_shift(lo, p));
    // the point indices, through the sorted positions: every entry is fetched before the first is stored
    uint32_t out[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t i = r * 256u + threadIdx.x;
        out[r] = i < L ? vals[src[i]] : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t i = r * 256u + threadIdx.x;
        if (i < L) vals[i] = out[r];
    }
}

// exclusive scan of one value per thread over the workgroup's 256 threads
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* sScan)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(inc, d, 64);
        if (lane >= d) inc += t;
    }
    if (lane == 63) sScan[wave] = inc;
    __syncthreads();
    uint32_t below = inc - v;
#pragma unroll
    for (int w = 0; w < 3; ++w) if (w < wave) below += sScan[w];
    __syncthreads();
    return below;
}

// Lists too long for LDS: one stable pass by the digit at `shift` from (kin, vin) to (kout, vout), all of length L
// in global memory. Each wavefront takes a contiguous quarter of the list, in rounds of 64. `cur` holds, per wavefront
// and digit, how many of its entries have that digit: counted here in a sweep of its own if `count_first`, else by
// the previous pass, which knew where every entry went and so in whose quarter it would be (that is what `nxt` and
// `next_shift` are for: pass a negative shift when no pass follows). The counters are then turned into where the
// wavefront's first entry of each digit goes, and a sweep places the entries: digit_prefix() hands back the counter's
// value before the round's entries were added plus the lane's rank among them, which now is the entry's position.
// Nothing is kept per entry between the sweeps, so the list may be of any length.
__device__ __forceinline__ void long_list_pass(WgSortLds& S, uint32_t (*cur)[kListBins], uint32_t (*nxt)[kListBins], bool count_first, uint32_t L,
                                               int shift, int next_shift, const uint32_t* __restrict__ kin,
                                               const uint32_t* __restrict__ vin, uint32_t* __restrict__ kout, uint32_t* __restrict__ vout)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t per_wave = ((L + 255u) / 256u) * 64u;
    const uint32_t wb = min(L, wave * per_wave), we = min(L, wb + per_wave);
    if (count_first) {
#pragma unroll
        for (int q = 0; q < kListBins / 64; ++q) cur[wave][q * 64 + lane] = 0u;
        wave_lds_sync();
        for (uint32_t i0 = wb; i0 < we; i0 += 8u * 64u) {      // eight key fetches in flight at a time
            uint32_t k[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t i = i0 + j * 64u + lane;
                k[j] = i < we ? kin[i] : 0u;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (i0 + j * 64u < we) digit_prefix<false>(cur[wave], (k[j] >> shift) & (kListBins - 1u), i0 + j * 64u + lane < we);
        }
    }
    __syncthreads();      // every wavefront's counts are in
    {   // two consecutive digits per thread: a digit's run starts after all smaller digits; inside it the wavefronts follow each other
        static_assert(kListBins == 2 * 256, "two digits per thread");
        const uint32_t d0 = 2u * threadIdx.x;
        uint32_t c[2][4], tot[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int w = 0; w < 4; ++w) c[h][w] = cur[w][d0 + h];
            tot[h] = (c[h][0] + c[h][1]) + (c[h][2] + c[h][3]);
        }
        uint32_t start = block_exclusive_scan(tot[0] + tot[1], S.scan);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t at = start;
#pragma unroll
            for (int w = 0; w < 4; ++w) { cur[w][d0 + h] = at; at += c[h][w]; nxt[w][d0 + h] = 0u; }
            start += tot[h];
        }
    }
    __syncthreads();
    for (uint32_t i0 = wb; i0 < we; i0 += 8u * 64u) {
        uint32_t k[8], v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t i = i0 + j * 64u + lane;
            k[j] = 0u; v[j] = 0u;
            if (i < we) { k[j] = kin[i]; v[j] = vin[i]; }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (i0 + j * 64u < we) {
                const bool valid = i0 + j * 64u + lane < we;
                const uint32_t pos = min(digit_prefix<false>(cur[wave], (k[j] >> shift) & (kListBins - 1u), valid), L - 1u);      // < L for consistent counts
                if (valid) {
                    kout[pos] = k[j]; vout[pos] = v[j];
                    if (next_shift >= 0) {      // the next pass finds this entry in the quarter of wavefront pos / per_wave
                        const uint32_t w2 = (pos >= per_wave ? 1u : 0u) + (pos >= 2u * per_wave ? 1u : 0u) + (pos >= 3u * per_wave ? 1u : 0u);
                        atomicAdd(&nxt[w2][(k[j] >> next_shift) & (kListBins - 1u)], 1u);
                    }
                }
            }
        }
    }
    __syncthreads();      // the pass is written and the next pass's counts are complete
}

// One list too long for a wavefront, sorted by the whole workgroup (every exit is uniform for the workgroup).
__device__ __forceinline__ void wg_sort_big(WgSortLds& S, uint32_t s, uint32_t e, const uint32_t* __restrict__ depth_bits,
                                            uint32_t* __restrict__ keysA, uint32_t* __restrict__ valsA,
                                            uint32_t* __restrict__ keysB, uint32_t* __restrict__ valsB)
{
    if (e <= s + 1u) return;
    const uint32_t L = e - s;
    if (L <= (uint32_t)kWgKeyMax) { wg_sort_list<true>(S, L, depth_bits, valsA + s, keysA + s); return; }
    if (L <= (uint32_t)kWgListMax) { wg_sort_list<false>(S, L, depth_bits, valsA + s, keysA + s); return; }
    // through global memory: keys of the list and the bit positions in which they differ
    const int lane = threadIdx.x & 63;
    const uint32_t k0 = depth_bits[valsA[s]];
    uint32_t diff = 0u;
    if (threadIdx.x == 0) S.mask = 0u;
    for (uint32_t i = threadIdx.x; i < L; i += 256u) {
        const uint32_t k = depth_bits[valsA[s + i]];
        diff |= k ^ k0;
        keysA[s + i] = k;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) diff |= (uint32_t)__shfl_xor((int)diff, d, 64);
    __syncthreads();                               // S.mask is cleared, the keys are in place
    if (lane == 0 && diff) atomicOr(&S.mask, diff);
    __syncthreads();
    const uint32_t mask = S.mask;
    if (mask == 0u) return;                        // one depth throughout: point order is the order
    int lo;
    const int passes = list_passes(mask, lo);
    // two sets of full-width counters that swap roles from pass to pass, in the key / permutation area, idle here
    uint32_t (*c0)[kListBins] = reinterpret_cast<uint32_t (*)[kListBins]>(&S.u);
    uint32_t (*c1)[kListBins] = c0 + 4;
    static_assert(sizeof(S.u) >= 2 * 4 * kListBins * sizeof(uint32_t), "room for both sets of counters");
    for (int p = 0; p < passes; ++p) {
        const int next_shift = p + 1 < passes ? list_shift(lo, p + 1) : -1;
        if ((p & 1) == 0) long_list_pass(S, c0, c1, p == 0, L, list_shift(lo, p), next_shift, keysA + s, valsA + s, keysB + s, valsB + s);
        else long_list_pass(S, c1, c0, false, L, list_shift(lo, p), next_shift, keysB + s, valsB + s, keysA + s, valsA + s);
    }
    if (passes & 1)
        for (uint32_t i = threadIdx.x; i < L; i += 256u) valsA[s + i] = valsB[s + i];
}

// Work items: tile_order lists the tiles longest first and its first `nbig` tiles are too long for one wavefront, so
// workgroups 0 .. nbig - 1 take one such list each, and every later workgroup takes four shorter lists, one per
// wavefront.
__global__ __launch_bounds__(256, 5) void k_tile_depth_sort(const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
                                                            uint32_t ntiles, const uint32_t* __restrict__ status,
                                                            const uint32_t* __restrict__ depth_bits, uint32_t cap,
                                                            uint32_t* __restrict__ keysA, uint32_t* __restrict__ valsA,
                                                            uint32_t* __restrict__ keysB, uint32_t* __restrict__ valsB)
{
    __shared__ ListSortLds U;
    const uint32_t nbig = min(status[kStNumBig], ntiles);
    if (blockIdx.x < nbig) {
        const uint32_t tile = tile_order[blockIdx.x];
        wg_sort_big(U.wg, ranges[2 * tile], min(ranges[2 * tile + 1], cap), depth_bits, keysA, valsA, keysB, valsB);
        return;
    }
    const int wave = threadIdx.x >> 6;
    const uint32_t idx = nbig + (blockIdx.x - nbig) * 4u + (uint32_t)wave;
    if (idx >= ntiles) return;
    const uint32_t tile = tile_order[idx];
    const uint32_t s = ranges[2 * tile], e = min(ranges[2 * tile + 1], cap);
    if (e <= s + 1u) return;
    // (a list of kWaveListMax - 1 entries or more cannot come here: k_tile_order counted it among the first nbig)
    if (e - s < (uint32_t)kWaveListMax - 1u) wave_sort_list(U.wave[wave], e - s, depth_bits, valsA + s);
}

hipError_t launch_tile_depth_sort(const uint32_t* ranges, const uint32_t* tile_order, uint32_t ntiles, const uint32_t* status,
                                  const uint32_t* depth_bits, uint32_t cap, uint32_t* keysA, uint32_t* valsA, uint32_t* keysB,
                                  uint32_t* valsB, hipStream_t s)
{
    if (ntiles == 0) return hipSuccess;
    ProfScope prof(kKTileDepthSort, s);
    // a list of the workgroup kind has at least kWaveListMax - 1 entries, which bounds how many of them `cap` pairs can
    // hold, and so how many workgroups can have work: the rest would only start and leave, which is not free on an
    // image of 32,400 tiles
    const uint32_t big_max = min(ntiles, cap / (uint32_t)(kWaveListMax - 1) + 1u);
    const uint32_t items_max = min(ntiles, big_max + (ntiles + 3u) / 4u);
    hipLaunchKernelGGL(k_tile_depth_sort, dim3(items_max), dim3(256), 0, s, ranges, tile_order, ntiles, status, depth_bits, cap, keysA, valsA,
                       keysB, valsB);
    return hipGetLastError();
}

template <int kBits>
static void launch_pass(uint32_t* keys[2], uint32_t* vals[2], int src, const uint32_t* count_ptr, uint32_t count_cap, int shift,
                        bool low_of_several, uint32_t* totals, uint32_t* tile_hist, uint32_t nb, hipStream_t s)
{
    const int dst = src ^ 1;
    {
        ProfScope prof(kKRadixHist, s);
        if (low_of_several)
            hipLaunchKernelGGL((k_radix_tile_hist<kBits, true>), dim3(nb), dim3(256), 0, s, keys[src], count_ptr, count_cap, shift, tile_hist, nb);
        else
            hipLaunchKernelGGL((k_radix_tile_hist<kBits, false>), dim3(nb), dim3(256), 0, s, keys[src], count_ptr, count_cap, shift, tile_hist, nb);
        hipLaunchKernelGGL(k_radix_digit_scan, dim3(1u << kBits), dim3(1024), 0, s, tile_hist, nb, count_ptr, count_cap, totals);
    }
    ProfScope prof(kKRadixScatter, s);
    hipLaunchKernelGGL(k_radix_scatter<kBits>, dim3(nb), dim3(256), 0, s, keys[src], vals[src], keys[dst], vals[dst], count_ptr,
                       count_cap, shift, tile_hist, nb, totals);
}

int radix_pass_count(int key_bits)
{
    return key_bits <= 0 ? 1 : (key_bits + 7) / 8;
}

// Sorts count (device or host known) pairs on key bits [0, key_bits). Buffers ping-pong: the result is in
// (keys[p & 1], vals[p & 1]) with p = radix_pass_count(key_bits). `totals` needs kRadixMaxBins words; `tile_hist`
// kRadixMaxBins * ceil(count_cap / kSortItems).
hipError_t launch_radix_sort32(uint32_t* keys[2], uint32_t* vals[2], const uint32_t* count_ptr, uint32_t count_cap,
                               int key_bits, uint32_t* totals, uint32_t* tile_hist, hipStream_t s)
{
    if (count_cap == 0) return hipSuccess;
    const uint32_t nb = (count_cap + kSortItems - 1) / kSortItems;
    const int passes = radix_pass_count(key_bits);
    if (key_bits <= 0) key_bits = 1;
    int shift = 0;
    for (int p = 0; p < passes; ++p) {
        const int bits = (key_bits - shift + (passes - p) - 1) / (passes - p);     // remaining bits, split evenly
        const bool low = p == 0 && passes > 1;
        switch (bits) {
            case 1: launch_pass<1>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
            case 2: launch_pass<2>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
            case 3: launch_pass<3>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
            case 4: launch_pass<4>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
            case 5: launch_pass<5>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
            case 6: launch_pass<6>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
            case 7: launch_pass<7>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
            default: launch_pass<8>(keys, vals, p & 1, count_ptr, count_cap, shift, low, totals, tile_hist, nb, s); break;
        }
        shift += bits;
    }
    return hipGetLastError();
}

}  // namespace pbdr
