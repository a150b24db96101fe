// Stable least-significant-digit radix sort of (32-bit key, 32-bit value) pairs, 8 bits per pass.
//
// The order the renderer needs is the order of the 64-bit key (tile << 32 | depth bits). All duplicates of a splat
// share the low 32 bits, so the four depth passes run on the n splats before duplication and only the tile passes
// run on the P pairs; the result is the same permutation a 64-bit sort of the pairs would give.
//
// One kernel counts every digit of every pass up front (digit totals -> where each digit's run starts). A pass is
// then three launches and no workgroup ever waits for another: (1) per-tile digit counts, (2) one workgroup per
// digit scans its counts over the tiles, (3) each 4096-pair tile ranks its pairs per wavefront with ballots and
// scatters. Per pass: 4 B (counts) + 8 B read + 8 B written per pair.
#include "pbdr_internal.h"

namespace pbdr {

constexpr int kSortPerThread = kSortItems / 256;  // 16
constexpr int kWaveItems = kSortItems / 4;        // 1024 consecutive pairs per wavefront

// Lanes of the wavefront that hold the same 8-bit digit as this lane (among the valid ones), by eight ballots.
__device__ __forceinline__ uint64_t digit_peers(uint32_t digit, bool valid)
{
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const bool bit = (digit >> b) & 1u;
        const uint64_t m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    return peers;
}

// Count one digit per valid lane into an LDS histogram: the lowest lane of each group of equal digits adds the
// group's size, so a digit that is the same for the whole wavefront (exponent bytes, high tile bits) costs one add
// instead of a 64-way serialised atomic.
__device__ __forceinline__ void hist_add(uint32_t* h, uint32_t digit, bool valid, uint64_t lt_mask)
{
    const uint64_t peers = digit_peers(digit, valid);
    if (valid && (peers & lt_mask) == 0ull) atomicAdd(&h[digit], (uint32_t)__popcll(peers));
}

__device__ __forceinline__ uint32_t sort_count(const uint32_t* __restrict__ count_ptr, uint32_t count_cap)
{
    return count_ptr ? min(*count_ptr, count_cap) : count_cap;
}

// totals[pass][256] += digit counts of this workgroup's 4096-pair tile, for `passes` digits starting at bit 0.
// The totals must be zero on entry. Integer atomics, and only for the digits that occur in the tile.
__global__ __launch_bounds__(256) void k_radix_global_hist(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ count_ptr,
                                                           uint32_t count_cap, int passes, uint32_t* __restrict__ totals)
{
    __shared__ uint32_t h[4][256];
    const uint32_t count = sort_count(count_ptr, count_cap);
    const uint32_t base = blockIdx.x * (uint32_t)kSortItems;
    if (base >= count) return;     // uniform for the workgroup
#pragma unroll
    for (int p = 0; p < 4; ++p) h[p][threadIdx.x] = 0;
    __syncthreads();
#pragma unroll 4
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = base + k * 256 + threadIdx.x;
        if (idx < count) {
            const uint32_t key = keys[idx];
            for (int p = 0; p < passes; ++p) atomicAdd(&h[p][(key >> (8 * p)) & 255u], 1u);
        }
    }
    __syncthreads();
    for (int p = 0; p < passes; ++p) {
        const uint32_t c = h[p][threadIdx.x];
        if (c) atomicAdd(&totals[p * 256 + threadIdx.x], c);
    }
}

// per-tile digit counts: hist[d * ntiles + tile]
__global__ __launch_bounds__(256) void k_radix_tile_hist(const uint32_t* __restrict__ keys, const uint32_t* __restrict__ count_ptr,
                                                         uint32_t count_cap, int shift, uint32_t* __restrict__ hist, uint32_t ntiles)
{
    __shared__ uint32_t h[256];
    const uint32_t count = sort_count(count_ptr, count_cap);
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t base = blockIdx.x * (uint32_t)kSortItems;
    const uint64_t lt_mask = (1ull << (threadIdx.x & 63)) - 1ull;
    if (base < count) {            // uniform for the workgroup
#pragma unroll 4
        for (int k = 0; k < kSortPerThread; ++k) {
            const uint32_t idx = base + k * 256 + threadIdx.x;
            const bool valid = idx < count;
            const uint32_t key = valid ? keys[idx] : 0u;
            hist_add(h, (key >> shift) & 255u, valid, lt_mask);
        }
    }
    __syncthreads();
    hist[threadIdx.x * ntiles + blockIdx.x] = h[threadIdx.x];
}

// one workgroup per digit: exclusive scan of that digit's counts over the tiles, offset by where the digit's run
// starts (= the number of keys with a smaller digit in this pass, summed here from the digit totals)
__global__ __launch_bounds__(256) void k_radix_digit_scan(uint32_t* __restrict__ hist, uint32_t ntiles,
                                                          const uint32_t* __restrict__ totals)
{
    __shared__ uint32_t lds[4];
    __shared__ uint32_t carry_s;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t* row = hist + (size_t)blockIdx.x * ntiles;
    {
        uint32_t below = (threadIdx.x < blockIdx.x) ? totals[threadIdx.x] : 0u;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) below += (uint32_t)__shfl_xor((int)below, d, 64);
        if (lane == 0) lds[wave] = below;
        __syncthreads();
        if (threadIdx.x == 0) carry_s = lds[0] + lds[1] + lds[2] + lds[3];
    }
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
}

__global__ __launch_bounds__(256) void k_radix_scatter(const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in,
                                                       uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out,
                                                       const uint32_t* __restrict__ count_ptr, uint32_t count_cap, int shift,
                                                       const uint32_t* __restrict__ hist_scanned, uint32_t ntiles)
{
    __shared__ uint32_t wave_base[4][256];
    const uint32_t count = sort_count(count_ptr, count_cap);
    const uint32_t block_base = blockIdx.x * (uint32_t)kSortItems;
    if (block_base >= count) return;  // uniform for the whole workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t wbase = block_base + wave * kWaveItems;
#pragma unroll
    for (int w = 0; w < 4; ++w) wave_base[w][threadIdx.x] = 0;
    __syncthreads();
    // this wavefront's 1024 consecutive pairs, 16 rounds of 64, kept in registers together with each pair's rank
    // among the equal digits of its round and the size of that group
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    uint32_t key[kSortPerThread], val[kSortPerThread], rank[kSortPerThread], group[kSortPerThread];
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        const bool valid = idx < count;
        key[k] = 0u; val[k] = 0u;
        if (valid) { key[k] = keys_in[idx]; val[k] = vals_in[idx]; }
        const uint32_t digit = (key[k] >> shift) & 255u;
        const uint64_t peers = digit_peers(digit, valid);
        rank[k] = (uint32_t)__popcll(peers & lt_mask);
        group[k] = (uint32_t)__popcll(peers);
        if (valid && rank[k] == 0u) atomicAdd(&wave_base[wave][digit], group[k]);
    }
    __syncthreads();
    {   // digit d: start of this tile's run, then split among the four wavefronts in order
        const int d = threadIdx.x;
        uint32_t run = hist_scanned[d * ntiles + blockIdx.x];
#pragma unroll
        for (int w = 0; w < 4; ++w) { const uint32_t c = wave_base[w][d]; wave_base[w][d] = run; run += c; }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        if (idx < count) {
            const uint32_t digit = (key[k] >> shift) & 255u;
            const uint32_t start = wave_base[wave][digit];          // every peer reads before the leader updates
            if (rank[k] == 0u) wave_base[wave][digit] = start + group[k];
            const uint32_t dst = start + rank[k];
            if (dst < count_cap) {                                   // always true for consistent inputs
                keys_out[dst] = key[k];
                vals_out[dst] = val[k];
            }
        }
    }
}

// Sorts count (device or host known) pairs on key bits [0, 8*passes). Buffers ping-pong: the result is in
// (keys[passes & 1], vals[passes & 1]). `totals` needs 4*256 words, zero on entry; `tile_hist` 256 * ceil(count_cap / 4096).
hipError_t launch_radix_sort32(uint32_t* keys[2], uint32_t* vals[2], const uint32_t* count_ptr, uint32_t count_cap,
                               int passes, uint32_t* totals, uint32_t* tile_hist, hipStream_t s)
{
    if (passes <= 0 || count_cap == 0) return hipSuccess;
    const uint32_t nb = (count_cap + kSortItems - 1) / kSortItems;
    {
        ProfScope prof(kKRadixHist, s);
        hipLaunchKernelGGL(k_radix_global_hist, dim3(nb), dim3(256), 0, s, keys[0], count_ptr, count_cap, passes, totals);
    }
    ProfScope prof(kKRadixScatter, s);
    for (int pass = 0; pass < passes; ++pass) {
        const int src = pass & 1, dst = src ^ 1, shift = 8 * pass;
        hipLaunchKernelGGL(k_radix_tile_hist, dim3(nb), dim3(256), 0, s, keys[src], count_ptr, count_cap, shift, tile_hist, nb);
        hipLaunchKernelGGL(k_radix_digit_scan, dim3(256), dim3(256), 0, s, tile_hist, nb, totals + pass * 256);
        hipLaunchKernelGGL(k_radix_scatter, dim3(nb), dim3(256), 0, s, keys[src], vals[src], keys[dst], vals[dst], count_ptr,
                           count_cap, shift, tile_hist, nb);
    }
    return hipGetLastError();
}

}  // namespace pbdr
