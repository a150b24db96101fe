// Measurement aid, not part of libpbdr: how fast gfx950 issues the kinds of vector instructions the compositing kernels
// are made of. Prints (1) the rate of independent plain v_fma_f32 (the fp32 vector peak that is reachable without packed
// math) and (2) the issue cost, in cycles per SIMD at the nominal 2.4 GHz, of a plain add, a DPP add, v_exp_f32,
// v_rcp_f32, a select and the two row-swap instructions, each measured as "two instructions per trip, one of them a
// plain op of known cost", and (3) the rate at which one compute unit's LDS returns reads of 4, 8 and 16 bytes per lane,
// all lanes reading the same address (how the compositing kernels read a staged splat) and every lane its own.
// Results are meaningless numerically (the asm strings ignore DPP wait states on purpose:
// only the issue rate is measured) and nothing is read back but one float per lane.
#include <hip/hip_runtime.h>

#include <cstdio>

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { std::printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 1; } } while (0)

__global__ __launch_bounds__(256) void k_fma(float* out, int iters)
{
    float a0 = threadIdx.x, a1 = 1, a2 = 2, a3 = 3, a4 = 4, a5 = 5, a6 = 6, a7 = 7;
    const float b = 1.0001f, c = 0.5f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            asm volatile("v_fma_f32 %0, %0, %8, %9\n\tv_fma_f32 %1, %1, %8, %9\n\tv_fma_f32 %2, %2, %8, %9\n\tv_fma_f32 %3, %3, %8, %9\n\t"
                         "v_fma_f32 %4, %4, %8, %9\n\tv_fma_f32 %5, %5, %8, %9\n\tv_fma_f32 %6, %6, %8, %9\n\tv_fma_f32 %7, %7, %8, %9"
                         : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(b), "v"(c));
        }
    }
    out[blockIdx.x * 256 + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
}

template <int kMode>
__global__ __launch_bounds__(256) void k_pair(float* out, int iters)
{
    float a = threadIdx.x * 0.5f, b = threadIdx.x * 0.25f + 1.f, c = 1.0001f, d = 0.3f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if (kMode == 0) asm volatile("v_add_f32 %0, %0, %2\n\tv_add_f32 %1, %1, %3" : "+v"(a), "+v"(b) : "v"(c), "v"(d));
            if (kMode == 1) asm volatile("v_add_f32_dpp %0, %0, %0 row_ror:8 row_mask:0xf bank_mask:0xf\n\tv_add_f32 %1, %1, %2" : "+v"(a), "+v"(b) : "v"(c));
            if (kMode == 2) asm volatile("v_exp_f32 %0, %0\n\tv_add_f32 %1, %1, %2" : "+v"(a), "+v"(b) : "v"(c));
            if (kMode == 3) asm volatile("v_rcp_f32 %0, %0\n\tv_add_f32 %1, %1, %2" : "+v"(a), "+v"(b) : "v"(c));
            if (kMode == 4) asm volatile("v_cndmask_b32 %0, %0, %2, vcc\n\tv_add_f32 %1, %1, %2" : "+v"(a), "+v"(b) : "v"(c));
            if (kMode == 5) asm volatile("v_permlane16_swap_b32 %0, %1\n\tv_add_f32 %0, %0, %2" : "+v"(a), "+v"(b) : "v"(c));
            if (kMode == 6) asm volatile("v_permlane32_swap_b32 %0, %1\n\tv_add_f32 %0, %0, %2" : "+v"(a), "+v"(b) : "v"(c));
        }
    }
    out[blockIdx.x * 256 + threadIdx.x] = a + b + c + d;
}

// kBytes per lane per read; kSame: every lane of a wavefront reads the same address
template <int kBytes, bool kSame>
__global__ __launch_bounds__(256) void k_lds_read(float* out, int iters)
{
    __shared__ float4 buf[1024];
    for (int i = threadIdx.x; i < 1024; i += 256) buf[i] = make_float4((float)i, 1.f, 2.f, 3.f);
    __syncthreads();
    float acc = 0.f;
    const unsigned addr = kSame ? (threadIdx.x >> 6) * 64u : threadIdx.x * 16u;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned a = addr + ((i * 8 + u) & 63) * 48u;      // byte address inside buf (the kernel's only LDS array)
            if (kBytes == 16) { float4 v; asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(4)" : "=v"(v) : "v"(a) : "memory"); acc += v.x; }
            if (kBytes == 8) { float2 v; asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(4)" : "=v"(v) : "v"(a) : "memory"); acc += v.x; }
            if (kBytes == 4) { float v; asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(4)" : "=v"(v) : "v"(a) : "memory"); acc += v; }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)");
    out[blockIdx.x * 256 + threadIdx.x] = acc + buf[threadIdx.x].y;
}

template <class F>
static int timed(F launch, float* ms)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    launch(8);                     // warm-up
    CHECK(hipEventRecord(e0));
    launch(0);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipEventElapsedTime(ms, e0, e1));
    CHECK(hipEventDestroy(e0)); CHECK(hipEventDestroy(e1));
    return 0;
}

int main()
{
    constexpr int kCus = 256, kSimds = 1024;
    constexpr double kClock = 2.4e9;
    float* out = nullptr;
    CHECK(hipMalloc(&out, (size_t)kCus * 16 * 256 * sizeof(float)));
    {   // 16 workgroups of 4 wavefronts per CU = 16 wavefronts per SIMD, 8 independent FMAs per lane
        const int iters = 4000, nb = kCus * 16;
        float ms = 0.f;
        if (timed([&](int warm) { hipLaunchKernelGGL(k_fma, dim3(nb), dim3(256), 0, 0, out, warm ? warm : iters); }, &ms)) return 1;
        const double flops = 2.0 * 64 * iters * 256.0 * nb, per_simd = 64.0 * iters * (nb * 4 / (double)kSimds);
        std::printf("plain v_fma_f32, 16 wavefronts per SIMD: %.1f TFLOP/s, %.2f cycles per wavefront instruction per SIMD\n",
                    flops / (ms * 1e-3) / 1e12, ms * 1e-3 * kClock / per_simd);
    }
    const char* names[7] = {"v_add_f32", "v_add_f32_dpp", "v_exp_f32", "v_rcp_f32", "v_cndmask_b32", "v_permlane16_swap_b32", "v_permlane32_swap_b32"};
    const int iters = 2000, nb = kCus * 8;                         // 8 wavefronts per SIMD
    const double per_simd = 2.0 * 16 * iters * (nb * 4 / (double)kSimds);   // instructions per SIMD
    float ms[7];
    if (timed([&](int w) { hipLaunchKernelGGL(k_pair<0>, dim3(nb), dim3(256), 0, 0, out, w ? w : iters); }, &ms[0])) return 1;
    if (timed([&](int w) { hipLaunchKernelGGL(k_pair<1>, dim3(nb), dim3(256), 0, 0, out, w ? w : iters); }, &ms[1])) return 1;
    if (timed([&](int w) { hipLaunchKernelGGL(k_pair<2>, dim3(nb), dim3(256), 0, 0, out, w ? w : iters); }, &ms[2])) return 1;
    if (timed([&](int w) { hipLaunchKernelGGL(k_pair<3>, dim3(nb), dim3(256), 0, 0, out, w ? w : iters); }, &ms[3])) return 1;
    if (timed([&](int w) { hipLaunchKernelGGL(k_pair<4>, dim3(nb), dim3(256), 0, 0, out, w ? w : iters); }, &ms[4])) return 1;
    if (timed([&](int w) { hipLaunchKernelGGL(k_pair<5>, dim3(nb), dim3(256), 0, 0, out, w ? w : iters); }, &ms[5])) return 1;
    if (timed([&](int w) { hipLaunchKernelGGL(k_pair<6>, dim3(nb), dim3(256), 0, 0, out, w ? w : iters); }, &ms[6])) return 1;
    const double plain = ms[0] * 1e-3 * kClock / per_simd;          // cycles per instruction, both plain
    for (int m = 0; m < 7; ++m) {
        const double both = ms[m] * 1e-3 * kClock / per_simd * 2.0;   // cycles per pair
        std::printf("%-24s %.2f cycles per wavefront instruction per SIMD\n", names[m], m == 0 ? plain : both - plain);
    }
    {   // LDS reads: 8 workgroups of 4 wavefronts per compute unit, up to 4 reads in flight per wavefront
        const char* lnames[4] = {"ds_read_b32, same address", "ds_read_b64, same address", "ds_read_b128, same address", "ds_read_b128, own address"};
        float lms[4];
        const int liters = 2000;
        if (timed([&](int w) { hipLaunchKernelGGL((k_lds_read<4, true>), dim3(nb), dim3(256), 0, 0, out, w ? w : liters); }, &lms[0])) return 1;
        if (timed([&](int w) { hipLaunchKernelGGL((k_lds_read<8, true>), dim3(nb), dim3(256), 0, 0, out, w ? w : liters); }, &lms[1])) return 1;
        if (timed([&](int w) { hipLaunchKernelGGL((k_lds_read<16, true>), dim3(nb), dim3(256), 0, 0, out, w ? w : liters); }, &lms[2])) return 1;
        if (timed([&](int w) { hipLaunchKernelGGL((k_lds_read<16, false>), dim3(nb), dim3(256), 0, 0, out, w ? w : liters); }, &lms[3])) return 1;
        const double per_cu = (double)nb * 4 / kCus * liters * 8;      // wavefront reads per compute unit
        for (int m = 0; m < 4; ++m)
            std::printf("%-28s %.2f cycles per wavefront read per compute unit\n", lnames[m], lms[m] * 1e-3 * kClock / per_cu);
    }
    CHECK(hipFree(out));
    return 0;
}
