// Point-group frustum culling (paper App. D.1 "frustum culling of point groups"; Sec. 4.2.1 for the groups: runs of
// consecutive points of a cloud stored in Z-order).
//
// Once per cloud: one axis-aligned box around the centres of each group, and the group's largest scale. Once per
// view: one thread per group decides from the box alone whether every point of the group would be culled by the
// per-point tests anyway; the per-point kernel then skips such groups without reading a single parameter.
//
// The paper tests the eight box corners against the frustum. A box can meet the frustum with no corner inside it and
// splats have an extent, so here the test is the conservative one: the corners against the near and far planes and
// against the four side planes of the image, each pushed out by an upper bound of any member's extent.
// "Conservative" refers to the fp32 per-point kernel: every threshold carries a margin for the rounding of both
// sides, so the splat state is identical with and without groups.
#include "pbdr_internal.h"

namespace pbdr {

// bounds planes: [0..2] min xyz, [3..5] max xyz, [6] largest scale (exp of the largest log-scale); [7][n_groups]
__global__ __launch_bounds__(256) void k_group_bounds(SceneDev sc, int group_size, int n_groups, float* __restrict__ bounds)
{
    __shared__ float red[7][4];
    const int g = blockIdx.x;
    const int lo = g * group_size, hi = min(lo + group_size, sc.n);
    const size_t N = (size_t)sc.n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float inf = __builtin_huge_valf();
    float v[7] = {inf, inf, inf, -inf, -inf, -inf, -inf};
    for (int i = lo + (int)threadIdx.x; i < hi; i += 256) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const float m = sc.mean[(size_t)k * N + i];
            v[k] = fminf(v[k], m); v[3 + k] = fmaxf(v[3 + k], m);
            v[6] = fmaxf(v[6], sc.log_scale[(size_t)k * N + i]);
        }
    }
#pragma unroll
    for (int k = 0; k < 7; ++k) {
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const float o = __shfl_xor(v[k], d, 64);
            v[k] = (k < 3) ? fminf(v[k], o) : fmaxf(v[k], o);
        }
        if (lane == 0) red[k][wave] = v[k];
    }
    __syncthreads();
    if (threadIdx.x < 7) {
        const int k = threadIdx.x;
        const float a = red[k][0], b = red[k][1], c = red[k][2], d = red[k][3];
        float r = (k < 3) ? fminf(fminf(a, b), fminf(c, d)) : fmaxf(fmaxf(a, b), fmaxf(c, d));
        if (k == 6) r = expf(r);
        bounds[(size_t)k * n_groups + g] = r;
    }
}

// keep[g] = 0 if every point of group g is certain to be culled for this view: all eight corners of its box behind
// the near plane, or beyond the far plane, or beyond one image side's plane pushed out by the largest extent a member
// can have. A member at depth z has extent <= k1 s_max / z + k0 (k1 = 3 |clamped Jacobian|_F z, k0 = blur, eigenvalue
// floor and ceil), and its tile rectangle is empty on the right if mean2d_x - extent >= 16 TX + 1, on the left if
// mean2d_x + extent < 0; times z > 0 these are linear in the camera-space position, so corners decide for the box.
// Each comparison carries 4e-6 of the sum of the magnitudes of its terms as margin towards keeping.
__device__ __forceinline__ uint8_t group_keep(const CamDev& cam, int g, int n_groups, const float* __restrict__ bounds)
{
    float b[7];
#pragma unroll
    for (int k = 0; k < 7; ++k) b[k] = bounds[(size_t)k * n_groups + g];
    const float kRel = 4e-6f;
    const float F2 = cam.fx * cam.fx * (1.f + cam.lim_x * cam.lim_x) + cam.fy * cam.fy * (1.f + cam.lim_y * cam.lim_y);
    const float k1s = 3.0f * sqrtf(F2) * b[6] * 1.00001f;
    const float k0 = (3.0f * sqrtf(kBlur + sqrtf(kEigFloor)) + 1.0f) * 1.00001f;
    // (coefficient of p_x or p_y, coefficient of p_z) of the four side planes: right, left, bottom, top
    const float cxy[4] = {cam.fx, -cam.fx, cam.fy, -cam.fy};
    const float cz[4] = {-(16.0f * (float)(cam.otx + cam.TX) + 1.0f + k0 - cam.cx), -(cam.cx - 16.0f * (float)cam.otx + k0),
                         -(16.0f * (float)(cam.oty + cam.TY) + 1.0f + k0 - cam.cy), -(cam.cy - 16.0f * (float)cam.oty + k0)};
    bool behind = true, beyond = true;
    bool outside[4] = {true, true, true, true};
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float c0 = b[(k & 1) ? 3 : 0], c1 = b[(k & 2) ? 4 : 1], c2 = b[(k & 4) ? 5 : 2];
        float p[3], m[3];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const float t0 = cam.R[3 * i] * c0, t1 = cam.R[3 * i + 1] * c1, t2 = cam.R[3 * i + 2] * c2;
            p[i] = t0 + t1 + t2 + cam.t[i];
            m[i] = fabsf(t0) + fabsf(t1) + fabsf(t2) + fabsf(cam.t[i]);
        }
        behind = behind && (p[2] + kRel * m[2] < cam.near_p);
        beyond = beyond && (p[2] - kRel * m[2] > cam.far_p);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float q = (i < 2) ? p[0] : p[1], mq = (i < 2) ? m[0] : m[1];
            const float f = cxy[i] * q + cz[i] * p[2] - k1s;
            const float mag = fabsf(cxy[i]) * mq + fabsf(cz[i]) * m[2] + k1s;
            outside[i] = outside[i] && (f - kRel * mag > 0.f);
        }
    }
    const bool drop = behind || beyond || outside[0] || outside[1] || outside[2] || outside[3];
    return drop ? 0 : 1;
}

__global__ __launch_bounds__(256) void k_group_cull(CamDev cam, int n_groups, const float* __restrict__ bounds,
                                                    uint8_t* __restrict__ keep)
{
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= n_groups) return;
    keep[g] = group_keep(cam, g, n_groups, bounds);
}

// the same test for every view of a batch: blockIdx.y = view, keep is [views][groups]
__global__ __launch_bounds__(256) void k_group_cull_batch(BatchCams cams, int n_groups, const float* __restrict__ bounds,
                                                          uint8_t* __restrict__ keep)
{
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= n_groups) return;
    const int v = blockIdx.y;
    keep[(size_t)v * n_groups + g] = group_keep(cams.cam[v], g, n_groups, bounds);
}

hipError_t launch_group_bounds(const SceneDev& sc, int group_size, float* bounds, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const int ng = (sc.n + group_size - 1) / group_size;
    hipLaunchKernelGGL(k_group_bounds, dim3((unsigned)ng), dim3(256), 0, s, sc, group_size, ng, bounds);
    return hipGetLastError();
}

hipError_t launch_group_cull(const CamDev& cam, int n_groups, const float* bounds, uint8_t* keep, hipStream_t s)
{
    if (n_groups == 0) return hipSuccess;
    ProfScope prof(kKGroupCull, s);
    hipLaunchKernelGGL(k_group_cull, dim3((unsigned)((n_groups + 255) / 256)), dim3(256), 0, s, cam, n_groups, bounds, keep);
    return hipGetLastError();
}

hipError_t launch_group_cull_batch(const BatchCams& cams, int n_groups, const float* bounds, uint8_t* keep, hipStream_t s)
{
    if (n_groups == 0 || cams.count == 0) return hipSuccess;
    ProfScope prof(kKGroupCull, s);
    hipLaunchKernelGGL(k_group_cull_batch, dim3((unsigned)((n_groups + 255) / 256), (unsigned)cams.count), dim3(256), 0, s, cams,
                       n_groups, bounds, keep);
    return hipGetLastError();
}

}  // namespace pbdr
