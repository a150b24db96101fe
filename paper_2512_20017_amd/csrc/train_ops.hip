// The two steps of a training iteration that sit around the rasterizer on the GPU that renders a view (paper Alg. 1):
// the loss with its gradient (lines 13 and 16: loss_fn, loss_fn.backward) and the parameter update (line 27:
// AdamUpdate; App. E.1: the "selective" Adam, which touches only points that were visible in the batch).
// Both are single passes over memory: HBM-bound, no reuse, 16-byte accesses per lane.
#include "pbdr_internal.h"

#include <cmath>

namespace pbdr {

// loss += mean |image - target| ; dL = sign(image - target) / count. One float4 per lane and trip; block sums are
// formed in registers and LDS and leave the workgroup as one float atomic.
__global__ __launch_bounds__(256) void k_l1_loss(const float* __restrict__ image, const float* __restrict__ target,
                                                 size_t count, float inv_count, float* __restrict__ loss,
                                                 float* __restrict__ dL)
{
    __shared__ float sWave[4];
    const size_t nvec = count / 4;
    const size_t stride = (size_t)gridDim.x * 256;
    float acc = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += stride) {
        const float4 a = reinterpret_cast<const float4*>(image)[i];
        const float4 b = reinterpret_cast<const float4*>(target)[i];
        const float d0 = a.x - b.x, d1 = a.y - b.y, d2 = a.z - b.z, d3 = a.w - b.w;
        acc += (fabsf(d0) + fabsf(d1)) + (fabsf(d2) + fabsf(d3));
        float4 g;
        g.x = d0 > 0.f ? inv_count : (d0 < 0.f ? -inv_count : 0.f);
        g.y = d1 > 0.f ? inv_count : (d1 < 0.f ? -inv_count : 0.f);
        g.z = d2 > 0.f ? inv_count : (d2 < 0.f ? -inv_count : 0.f);
        g.w = d3 > 0.f ? inv_count : (d3 < 0.f ? -inv_count : 0.f);
        reinterpret_cast<float4*>(dL)[i] = g;
    }
    if (blockIdx.x == 0 && threadIdx.x < (count & 3)) {      // up to three trailing elements
        const size_t i = nvec * 4 + threadIdx.x;
        const float d = image[i] - target[i];
        acc += fabsf(d);
        dL[i] = d > 0.f ? inv_count : (d < 0.f ? -inv_count : 0.f);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if ((threadIdx.x & 63) == 0) sWave[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(loss, ((sWave[0] + sWave[1]) + (sWave[2] + sWave[3])) * inv_count);
}

// visible[i] |= radius[i] > 0 : the union over the views of a batch of the points each view uses
__global__ __launch_bounds__(256) void k_mark_visible(int n, const int32_t* __restrict__ radius, uint8_t* __restrict__ visible)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n && radius[i] > 0) visible[i] = 1;
}

// blockIdx.y = plane of the [planes][n] tensors; a lane owns four consecutive points (n % 4 == 0 here).
// A lane none of whose points is visible reads four mask bytes and nothing else.
__global__ __launch_bounds__(256) void k_adam_selective_vec(int n, float* __restrict__ param, float* __restrict__ grad,
                                                            float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
                                                            const uint8_t* __restrict__ visible, AdamDev c)
{
    const int q = blockIdx.x * 256 + threadIdx.x;          // group of four points
    if (q >= n / 4) return;
    const uint32_t vis = reinterpret_cast<const uint32_t*>(visible)[q];
    if (vis == 0u) return;
    const size_t at = (size_t)blockIdx.y * n / 4 + q;
    float4 p = reinterpret_cast<float4*>(param)[at];
    const float4 g = reinterpret_cast<const float4*>(grad)[at];
    float4 m = reinterpret_cast<float4*>(exp_avg)[at];
    float4 v = reinterpret_cast<float4*>(exp_avg_sq)[at];
    if (vis & 0x000000ffu) adam_one(c, p.x, g.x, m.x, v.x);
    if (vis & 0x0000ff00u) adam_one(c, p.y, g.y, m.y, v.y);
    if (vis & 0x00ff0000u) adam_one(c, p.z, g.z, m.z, v.z);
    if (vis & 0xff000000u) adam_one(c, p.w, g.w, m.w, v.w);
    reinterpret_cast<float4*>(param)[at] = p;
    reinterpret_cast<float4*>(exp_avg)[at] = m;
    reinterpret_cast<float4*>(exp_avg_sq)[at] = v;
    if (c.zero_grad) {
        float4 z = g;
        if (vis & 0x000000ffu) z.x = 0.f;
        if (vis & 0x0000ff00u) z.y = 0.f;
        if (vis & 0x00ff0000u) z.z = 0.f;
        if (vis & 0xff000000u) z.w = 0.f;
        reinterpret_cast<float4*>(grad)[at] = z;
    }
}

// any n: one point per lane
__global__ __launch_bounds__(256) void k_adam_selective(int n, float* __restrict__ param, float* __restrict__ grad,
                                                        float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
                                                        const uint8_t* __restrict__ visible, AdamDev c)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n || visible[i] == 0) return;
    const size_t at = (size_t)blockIdx.y * n + i;
    float p = param[at], m = exp_avg[at], v = exp_avg_sq[at];
    adam_one(c, p, grad[at], m, v);
    param[at] = p; exp_avg[at] = m; exp_avg_sq[at] = v;
    if (c.zero_grad) grad[at] = 0.f;
}

AdamDev make_adam(float lr, float beta1, float beta2, float eps, int step, int zero_grad)
{
    AdamDev c;
    c.beta1 = beta1; c.beta2 = beta2;
    c.one_m_beta1 = (float)(1.0 - (double)beta1); c.one_m_beta2 = (float)(1.0 - (double)beta2);
    const double bc1 = 1.0 - std::pow((double)beta1, (double)step), bc2 = 1.0 - std::pow((double)beta2, (double)step);
    c.step_size = (float)((double)lr / bc1);
    c.inv_sqrt_bc2 = (float)(1.0 / std::sqrt(bc2));
    c.eps = eps; c.zero_grad = zero_grad;
    return c;
}

hipError_t launch_l1_loss(int W, int H, const float* image, const float* target, float* loss, float* dL, hipStream_t s)
{
    const size_t count = (size_t)3 * W * H;
    const size_t nvec = count / 4;
    unsigned blocks = (unsigned)((nvec + 256 * 4 - 1) / (256 * 4));     // four float4 per lane
    if (blocks < 1) blocks = 1;
    // every workgroup ends in one float atomic on the same word, and those serialise: at 1080p 1,519 workgroups (four
    // float4 per lane) took 31 us, 512 (grid-stride) take 20; 256 are too few wavefronts to stream at full rate (26 us)
    if (blocks > 512) blocks = 512;
    ProfScope prof(kKLoss, s);
    hipLaunchKernelGGL(k_l1_loss, dim3(blocks), dim3(256), 0, s, image, target, count, (float)(1.0 / (double)count), loss, dL);
    return hipGetLastError();
}

hipError_t launch_mark_visible(int n, const int32_t* radius, uint8_t* visible, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_mark_visible, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, n, radius, visible);
    return hipGetLastError();
}

hipError_t launch_adam_selective(int n, int planes, float* param, float* grad, float* exp_avg, float* exp_avg_sq,
                                 const uint8_t* visible, float lr, float beta1, float beta2, float eps, int step,
                                 int zero_grad, hipStream_t s)
{
    if (n == 0 || planes == 0) return hipSuccess;
    const AdamDev c = make_adam(lr, beta1, beta2, eps, step, zero_grad);
    ProfScope prof(kKAdam, s);
    if ((n & 3) == 0)
        hipLaunchKernelGGL(k_adam_selective_vec, dim3((unsigned)((n / 4 + 255) / 256), (unsigned)planes), dim3(256), 0, s, n, param,
                           grad, exp_avg, exp_avg_sq, visible, c);
    else
        hipLaunchKernelGGL(k_adam_selective, dim3((unsigned)((n + 255) / 256), (unsigned)planes), dim3(256), 0, s, n, param, grad,
                           exp_avg, exp_avg_sq, visible, c);
    return hipGetLastError();
}

}  // namespace pbdr
