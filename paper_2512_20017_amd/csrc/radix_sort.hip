// Stable least-significant-digit radix sort of (uint64 key, uint32 value) pairs, 8 bits per pass, over the key
// bits that can be non-zero: 32 depth bits + ceil(log2(#tiles)) tile bits.  The pair count lives on the device
// (status word), so grids are sized for the capacity and surplus workgroups leave at once.
//
// Per pass: (1) per-block digit histogram, (2) exclusive scan of the [digit][block] count matrix, (3) scatter.
// No workgroup ever waits for another, so a pass cannot hang; the price is that keys are read twice per pass:
// 8 B (histogram) + 12 B read + 12 B write per pair per pass.
#include "pbdr_internal.h"

namespace pbdr {

constexpr int kSortPerThread = kSortItems / 256;  // 16
constexpr int kWaveItems = kSortItems / 4;        // 1024 consecutive pairs per wavefront

__global__ __launch_bounds__(256) void k_radix_hist(const uint64_t* __restrict__ keys, const uint32_t* __restrict__ status,
                                                    uint32_t cap, int shift, uint32_t* __restrict__ hist, uint32_t nblocks)
{
    __shared__ uint32_t h[256];
    const uint32_t P = min(status[kStNumDup], cap);
    h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t base = blockIdx.x * (uint32_t)kSortItems;
    if (base < P) {
#pragma unroll
        for (int k = 0; k < kSortPerThread; ++k) {
            const uint32_t idx = base + k * 256 + threadIdx.x;
            if (idx < P) atomicAdd(&h[(uint32_t)(keys[idx] >> shift) & 255u], 1u);
        }
    }
    __syncthreads();
    hist[threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(256) void k_radix_scatter(const uint64_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in,
                                                       uint64_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out,
                                                       const uint32_t* __restrict__ status, uint32_t cap, int shift,
                                                       const uint32_t* __restrict__ hist_scanned, uint32_t nblocks)
{
    __shared__ uint32_t wave_base[4][256];
    const uint32_t P = min(status[kStNumDup], cap);
    const uint32_t block_base = blockIdx.x * (uint32_t)kSortItems;
    if (block_base >= P) return;  // uniform for the whole workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t wbase = block_base + wave * kWaveItems;

#pragma unroll
    for (int w = 0; w < 4; ++w) wave_base[w][threadIdx.x] = 0;
    __syncthreads();
    // this wavefront's 1024 consecutive pairs, 16 rounds of 64, kept in registers
    uint64_t key[kSortPerThread];
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        key[k] = idx < P ? keys_in[idx] : 0ull;
        if (idx < P) atomicAdd(&wave_base[wave][(uint32_t)(key[k] >> shift) & 255u], 1u);
    }
    __syncthreads();
    {   // digit d: global start of this block's run, then split among the four wavefronts in order
        const int d = threadIdx.x;
        uint32_t run = hist_scanned[d * nblocks + blockIdx.x];
#pragma unroll
        for (int w = 0; w < 4; ++w) { const uint32_t c = wave_base[w][d]; wave_base[w][d] = run; run += c; }
    }
    __syncthreads();
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int k = 0; k < kSortPerThread; ++k) {
        const uint32_t idx = wbase + k * 64 + lane;
        const bool valid = idx < P;
        const uint32_t digit = (uint32_t)(key[k] >> shift) & 255u;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (digit >> b) & 1u;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        if (valid) {
            const uint32_t rank = (uint32_t)__popcll(peers & lt_mask);
            const uint32_t start = wave_base[wave][digit];          // every peer reads before the leader updates
            if (rank == 0) wave_base[wave][digit] = start + (uint32_t)__popcll(peers);
            keys_out[start + rank] = key[k];
            vals_out[start + rank] = vals_in[idx];
        }
    }
}

hipError_t launch_radix_sort(const Layout& L, char* ws, hipStream_t s)
{
    uint32_t* status = reinterpret_cast<uint32_t*>(ws + L.off_status);
    uint32_t* hist = reinterpret_cast<uint32_t*>(ws + L.off_hist);
    uint32_t* part = reinterpret_cast<uint32_t*>(ws + L.off_scan_part);
    uint64_t* kbuf[2] = {reinterpret_cast<uint64_t*>(ws + L.off_keys0), reinterpret_cast<uint64_t*>(ws + L.off_keys1)};
    uint32_t* vbuf[2] = {reinterpret_cast<uint32_t*>(ws + L.off_vals0), reinterpret_cast<uint32_t*>(ws + L.off_vals1)};
    const uint32_t nb = L.sort_blocks;
    for (int pass = 0; pass < L.sort_passes; ++pass) {
        const int src = pass & 1, dst = src ^ 1, shift = 8 * pass;
        {
            ProfScope prof(kKRadixHist, s);
            hipLaunchKernelGGL(k_radix_hist, dim3(nb), dim3(256), 0, s, kbuf[src], status, L.cap, shift, hist, nb);
        }
        hipError_t e = launch_exclusive_scan(hist, hist, L.hist_len, part, nullptr, s);
        if (e != hipSuccess) return e;
        ProfScope prof(kKRadixScatter, s);
        hipLaunchKernelGGL(k_radix_scatter, dim3(nb), dim3(256), 0, s, kbuf[src], vbuf[src], kbuf[dst], vbuf[dst], status,
                           L.cap, shift, hist, nb);
    }
    return hipGetLastError();
}

}  // namespace pbdr
