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

// per-tile digit counts: hist[d * ntiles + tile]. One digit per valid lane goes into an LDS histogram: the lowest
// lane of each group of equal digits adds the group's size, so a digit that is the same for the whole wavefront
// (exponent bits, high tile bits) costs one add instead of a 64-way serialised atomic.
template <int kBits>
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
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = base + k * 256 + threadIdx.x;
        const bool valid = idx < count;
        const uint32_t key = valid ? keys[idx] : 0u;
        const uint32_t digit = (key >> shift) & kMask;
        const uint64_t peers = digit_peers<kBits>(digit, valid);
        if (valid && (peers & lt_mask) == 0ull) atomicAdd(&h[digit], (uint32_t)__popcll(peers));
    }
    __syncthreads();
    for (int d = threadIdx.x; d < kBins; d += 256) hist[(size_t)d * ntiles + blockIdx.x] = h[d];
}

// one workgroup per digit: exclusive scan of that digit's counts over the tiles that hold keys (in place);
// totals[digit] = their sum
__global__ __launch_bounds__(256) void k_radix_digit_scan(uint32_t* __restrict__ hist, uint32_t row_stride,
                                                          const uint32_t* __restrict__ count_ptr, uint32_t count_cap,
                                                          uint32_t* __restrict__ totals)
{
    __shared__ uint32_t lds[4];
    __shared__ uint32_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t ntiles = (sort_count(count_ptr, count_cap) + kSortItems - 1) / kSortItems;
    uint32_t* row = hist + (size_t)blockIdx.x * row_stride;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (uint32_t start = 0; start < ntiles; start += 256) {
        const uint32_t idx = start + threadIdx.x;
        const uint32_t v = idx < ntiles ? row[idx] : 0u;
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
        for (int w = 0; w < 4; ++w) { const uint32_t t = lds[w]; if (w < wave) base += t; chunk += t; }
        if (idx < ntiles) row[idx] = base + inc - v;
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
    for (int d = threadIdx.x; d < kBins; d += 256) {
#pragma unroll
        for (int w = 0; w < 4; ++w) wave_base[w][d] = 0;
    }
    __syncthreads();
    // this wavefront's consecutive pairs, in rounds of 64, kept in registers together with each pair's rank among
    // the equal digits of its round and the size of that group
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    uint32_t key[kSortPerThread], val[kSortPerThread], rank[kSortPerThread], group[kSortPerThread];
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        const bool valid = idx < count;
        key[k] = 0u; val[k] = 0u;
        if (valid) { key[k] = keys_in[idx]; val[k] = vals_in[idx]; }
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

template <int kBits>
static void launch_pass(uint32_t* keys[2], uint32_t* vals[2], int src, const uint32_t* count_ptr, uint32_t count_cap, int shift,
                        uint32_t* totals, uint32_t* tile_hist, uint32_t nb, hipStream_t s)
{
    const int dst = src ^ 1;
    {
        ProfScope prof(kKRadixHist, s);
        hipLaunchKernelGGL(k_radix_tile_hist<kBits>, dim3(nb), dim3(256), 0, s, keys[src], count_ptr, count_cap, shift, tile_hist, nb);
        hipLaunchKernelGGL(k_radix_digit_scan, dim3(1u << kBits), dim3(256), 0, s, tile_hist, nb, count_ptr, count_cap, totals);
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
        switch (bits) {
            case 1: launch_pass<1>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
            case 2: launch_pass<2>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
            case 3: launch_pass<3>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
            case 4: launch_pass<4>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
            case 5: launch_pass<5>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
            case 6: launch_pass<6>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
            case 7: launch_pass<7>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
            default: launch_pass<8>(keys, vals, p & 1, count_ptr, count_cap, shift, totals, tile_hist, nb, s); break;
        }
        shift += bits;
    }
    return hipGetLastError();
}

}  // namespace pbdr
