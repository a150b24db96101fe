// Per-tile compositing, forward and backward (image_render and image_render.backward: paper Sec. 2.1 "computes the
// color of each pixel front to back, blending the overlapping splats until full opacity is reached"; Alg. 1
// lines 12 and 18).
//
// One workgroup (4 wavefronts of 64) per 16x16 tile; each wavefront owns an 8x8 pixel block so that a splat that
// misses the block costs the wavefront nothing past the test. The tile's depth-sorted list is staged through LDS
// 256 splats at a time (one 48-byte record per thread, three 16-byte loads), then every lane walks the batch with
// LDS broadcast reads. Plain VALU work: there is no dense contraction here, so no MFMA.
#include "pbdr_internal.h"

namespace pbdr {

constexpr int kBatch = 256;

struct TileCtx {
    int px, py;
    bool inside;
    uint32_t pix;
    uint32_t start, end;
};

__device__ __forceinline__ TileCtx tile_ctx(const CamDev& cam, const uint32_t* __restrict__ ranges)
{
    TileCtx c;
    const int tile = blockIdx.x;
    const int ty = tile / cam.TX, tx = tile - ty * cam.TX;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    c.px = tx * kTile + (wave & 1) * 8 + (lane & 7);
    c.py = ty * kTile + (wave >> 1) * 8 + (lane >> 3);
    c.inside = c.px < cam.W && c.py < cam.H;
    c.pix = (uint32_t)c.py * (uint32_t)cam.W + (uint32_t)c.px;
    c.start = ranges[2 * tile];
    c.end = ranges[2 * tile + 1];
    return c;
}

__global__ __launch_bounds__(256) void k_composite_fwd(CamDev cam, const uint32_t* __restrict__ ranges,
                                                       const uint32_t* __restrict__ vals, const Packed* __restrict__ packed,
                                                       float bg0, float bg1, float bg2, float* __restrict__ image,
                                                       float* __restrict__ final_T, uint32_t* __restrict__ last_idx)
{
    __shared__ float4 sA[kBatch];  // mx, my, qa, qb
    __shared__ float4 sB[kBatch];  // qc, o, r, g
    __shared__ float sC[kBatch];   // b
    const TileCtx c = tile_ctx(cam, ranges);
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    float T = 1.f, C0 = 0.f, C1 = 0.f, C2 = 0.f;
    uint32_t last = 0;
    bool done = !c.inside;
    for (uint32_t base = c.start; base < c.end; base += kBatch) {
        if (__syncthreads_count(!done) == 0) break;   // also fences the previous batch's LDS reads
        const uint32_t idx = base + threadIdx.x;
        if (idx < c.end) {
            const float4* rec = reinterpret_cast<const float4*>(packed + vals[idx]);
            const float4 a = rec[0], b = rec[1], d = rec[2];
            sA[threadIdx.x] = a; sB[threadIdx.x] = b; sC[threadIdx.x] = d.x;
        }
        __syncthreads();
        const int cnt = (int)min((uint32_t)kBatch, c.end - base);
        if (!done) {
            for (int j = 0; j < cnt; ++j) {
                const float4 a = sA[j];
                const float4 b = sB[j];
                const float dx = fx - a.x, dy = fy - a.y;
                const float sigma = 0.5f * (a.z * dx * dx + b.x * dy * dy) + a.w * dx * dy;
                if (sigma < 0.f) continue;
                const float alpha = fminf(kAlphaMax, b.y * __expf(-sigma));
                if (alpha < kAlphaMin) continue;
                const float Tn = T * (1.f - alpha);
                if (Tn < kTStop) { done = true; break; }
                const float w = alpha * T;
                C0 += b.z * w; C1 += b.w * w; C2 += sC[j] * w;
                T = Tn;
                last = (base - c.start) + (uint32_t)j + 1u;
            }
        }
    }
    if (c.inside) {
        const size_t HW = (size_t)cam.W * cam.H;
        image[c.pix] = C0 + T * bg0;
        image[HW + c.pix] = C1 + T * bg1;
        image[2 * HW + c.pix] = C2 + T * bg2;
        final_T[c.pix] = T;
        last_idx[c.pix] = last;
    }
}

// Sum over the 64 lanes of a wavefront with DPP row shifts and row broadcasts (no LDS traffic); the total ends
// up in lane 63 and is returned in every lane through a readlane.
__device__ __forceinline__ float wave_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x111, 0xf, 0xf, true));  // row_shr:1
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x112, 0xf, 0xf, true));  // row_shr:2
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xf, 0xf, true));  // row_shr:4
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xf, 0xf, true));  // row_shr:8
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xa, 0xf, false)); // row_bcast:15
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xc, 0xf, false)); // row_bcast:31
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__global__ __launch_bounds__(256) void k_composite_bwd(CamDev cam, const uint32_t* __restrict__ ranges,
                                                       const uint32_t* __restrict__ vals, const Packed* __restrict__ packed,
                                                       float bg0, float bg1, float bg2, const float* __restrict__ final_T,
                                                       const uint32_t* __restrict__ last_idx, const float* __restrict__ dL_dimage,
                                                       int n, SplatGradDev g2)
{
    __shared__ float4 sA[kBatch];
    __shared__ float4 sB[kBatch];
    __shared__ float sC[kBatch];
    __shared__ uint32_t sId[kBatch];
    __shared__ uint32_t sMax[4];
    const TileCtx c = tile_ctx(cam, ranges);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    const size_t HW = (size_t)cam.W * cam.H;
    const size_t N = (size_t)n;
    float T = 1.f, g0 = 0.f, g1 = 0.f, g2c = 0.f;
    uint32_t last = 0;
    if (c.inside) {
        T = final_T[c.pix];
        last = min(last_idx[c.pix], c.end - c.start);   // never walk past the tile's list, whatever the caller passed
        g0 = dL_dimage[c.pix]; g1 = dL_dimage[HW + c.pix]; g2c = dL_dimage[2 * HW + c.pix];
    }
    // S = sum over splats behind the current one of w_i (c_i . g), plus the background term
    float S = T * (bg0 * g0 + bg1 * g1 + bg2 * g2c);
    // the deepest list position any pixel of the tile blended
    uint32_t wmax = last;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) wmax = max(wmax, (uint32_t)__shfl_xor((int)wmax, d, 64));
    if (lane == 0) sMax[wave] = wmax;
    __syncthreads();
    const uint32_t tile_last = max(max(sMax[0], sMax[1]), max(sMax[2], sMax[3]));
    if (tile_last == 0) return;
    const int nbatch = (int)((tile_last + kBatch - 1) / kBatch);
    for (int bi = nbatch - 1; bi >= 0; --bi) {
        const uint32_t boff = (uint32_t)bi * kBatch;               // 0-based list position of the batch's first splat
        const int cnt = (int)min((uint32_t)kBatch, tile_last - boff);
        __syncthreads();
        if ((int)threadIdx.x < cnt) {
            const uint32_t id = vals[c.start + boff + threadIdx.x];
            const float4* rec = reinterpret_cast<const float4*>(packed + id);
            const float4 a = rec[0], b = rec[1], d = rec[2];
            sA[threadIdx.x] = a; sB[threadIdx.x] = b; sC[threadIdx.x] = d.x; sId[threadIdx.x] = id;
        }
        __syncthreads();
        if (wmax <= boff) continue;   // nothing of this batch was blended by this wavefront (uniform per wave)
        for (int j = cnt - 1; j >= 0; --j) {
            const uint32_t pos = boff + (uint32_t)j + 1u;           // 1-based list position
            const float4 a = sA[j];
            const float4 b = sB[j];
            const float cb = sC[j];
            const float dx = fx - a.x, dy = fy - a.y;
            const float sigma = 0.5f * (a.z * dx * dx + b.x * dy * dy) + a.w * dx * dy;
            const float gauss = __expf(-sigma);
            const float araw = b.y * gauss;
            const float alpha = fminf(kAlphaMax, araw);
            const bool hit = (pos <= last) && (sigma >= 0.f) && (alpha >= kAlphaMin);
            if (__ballot(hit) == 0ull) continue;                   // uniform per wave
            float d_r = 0.f, d_g = 0.f, d_b = 0.f, d_o = 0.f, d_qa = 0.f, d_qb = 0.f, d_qc = 0.f, d_mx = 0.f, d_my = 0.f;
            if (hit) {
                const float oma = 1.f - alpha;
                const float ioma = 1.f / oma;
                T *= ioma;                                          // transmittance in front of this splat
                const float w = alpha * T;
                const float cg = b.z * g0 + b.w * g1 + cb * g2c;
                const float dL_dalpha = T * cg - S * ioma;
                S += w * cg;
                d_r = w * g0; d_g = w * g1; d_b = w * g2c;
                if (araw < kAlphaMax) {
                    const float ds = -alpha * dL_dalpha;
                    d_o = gauss * dL_dalpha;
                    d_qa = 0.5f * dx * dx * ds; d_qb = dx * dy * ds; d_qc = 0.5f * dy * dy * ds;
                    d_mx = -(a.z * dx + a.w * dy) * ds;
                    d_my = -(b.x * dy + a.w * dx) * ds;
                }
            }
            d_r = wave_sum(d_r); d_g = wave_sum(d_g); d_b = wave_sum(d_b); d_o = wave_sum(d_o);
            d_qa = wave_sum(d_qa); d_qb = wave_sum(d_qb); d_qc = wave_sum(d_qc);
            d_mx = wave_sum(d_mx); d_my = wave_sum(d_my);
            if (lane == 0) {
                const uint32_t id = sId[j];
                atomicAdd(g2.color + id, d_r); atomicAdd(g2.color + N + id, d_g); atomicAdd(g2.color + 2 * N + id, d_b);
                atomicAdd(g2.opacity + id, d_o);
                atomicAdd(g2.conic + id, d_qa); atomicAdd(g2.conic + N + id, d_qb); atomicAdd(g2.conic + 2 * N + id, d_qc);
                atomicAdd(g2.mean2d + id, d_mx); atomicAdd(g2.mean2d + N + id, d_my);
            }
        }
    }
}


// Measurement aid: the forward walk with counters instead of colours. counters[0] += list entries examined per pixel
// (up to and including the one that ends the pixel), counters[1] += pairs blended.
__global__ __launch_bounds__(256) void k_render_stats(CamDev cam, const uint32_t* __restrict__ ranges,
                                                      const uint32_t* __restrict__ vals, const Packed* __restrict__ packed,
                                                      unsigned long long* __restrict__ counters)
{
    __shared__ float4 sA[kBatch];
    __shared__ float4 sB[kBatch];
    __shared__ unsigned long long sCnt[2];
    const TileCtx c = tile_ctx(cam, ranges);
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    float T = 1.f;
    uint32_t examined = 0, blended = 0;
    bool done = !c.inside;
    if (threadIdx.x < 2) sCnt[threadIdx.x] = 0ull;
    for (uint32_t base = c.start; base < c.end; base += kBatch) {
        if (__syncthreads_count(!done) == 0) break;
        const uint32_t idx = base + threadIdx.x;
        if (idx < c.end) {
            const float4* rec = reinterpret_cast<const float4*>(packed + vals[idx]);
            sA[threadIdx.x] = rec[0]; sB[threadIdx.x] = rec[1];
        }
        __syncthreads();
        const int cnt = (int)min((uint32_t)kBatch, c.end - base);
        if (!done) {
            for (int j = 0; j < cnt; ++j) {
                const float4 a = sA[j];
                const float4 b = sB[j];
                const float dx = fx - a.x, dy = fy - a.y;
                const float sigma = 0.5f * (a.z * dx * dx + b.x * dy * dy) + a.w * dx * dy;
                ++examined;
                if (sigma < 0.f) continue;
                const float alpha = fminf(kAlphaMax, b.y * __expf(-sigma));
                if (alpha < kAlphaMin) continue;
                const float Tn = T * (1.f - alpha);
                if (Tn < kTStop) { done = true; break; }
                T = Tn;
                ++blended;
            }
        }
    }
    __syncthreads();
    atomicAdd(&sCnt[0], (unsigned long long)examined);
    atomicAdd(&sCnt[1], (unsigned long long)blended);
    __syncthreads();
    if (threadIdx.x < 2 && sCnt[threadIdx.x]) atomicAdd(&counters[threadIdx.x], sCnt[threadIdx.x]);
}

__global__ __launch_bounds__(256) void k_fill_f32(float* __restrict__ p, float v, size_t count)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = v;
}

hipError_t launch_composite_fwd(const CamDev& cam, const Layout& L, char* ws, const float bg[3], float* image,
                                float* final_T, uint32_t* last_idx, hipStream_t s)
{
    const uint32_t* ranges = reinterpret_cast<const uint32_t*>(ws + L.off_ranges);
    const uint32_t* vals = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    const Packed* packed = reinterpret_cast<const Packed*>(ws + L.off_packed);
    ProfScope prof(kKCompositeFwd, s);
    hipLaunchKernelGGL(k_composite_fwd, dim3((unsigned)L.tiles), dim3(256), 0, s, cam, ranges, vals, packed, bg[0], bg[1],
                       bg[2], image, final_T, last_idx);
    return hipGetLastError();
}

hipError_t launch_composite_bwd(const CamDev& cam, const Layout& L, char* ws, int n, const float bg[3],
                                const float* final_T, const uint32_t* last_idx, const float* dL_dimage,
                                const SplatGradDev& g2, hipStream_t s)
{
    const uint32_t* ranges = reinterpret_cast<const uint32_t*>(ws + L.off_ranges);
    const uint32_t* vals = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    const Packed* packed = reinterpret_cast<const Packed*>(ws + L.off_packed);
    if (n > 0) {
        ProfScope prof(kKFill, s);
        const size_t N = (size_t)n;
        const auto zero = [&](float* p, size_t count) {
            hipLaunchKernelGGL(k_fill_f32, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s, p, 0.f, count);
        };
        zero(g2.mean2d, 2 * N); zero(g2.conic, 3 * N); zero(g2.opacity, N); zero(g2.color, 3 * N);
    }
    ProfScope prof(kKCompositeBwd, s);
    hipLaunchKernelGGL(k_composite_bwd, dim3((unsigned)L.tiles), dim3(256), 0, s, cam, ranges, vals, packed, bg[0], bg[1],
                       bg[2], final_T, last_idx, dL_dimage, n, g2);
    return hipGetLastError();
}

hipError_t launch_render_stats(const CamDev& cam, const Layout& L, char* ws, uint64_t* counters, hipStream_t s)
{
    const uint32_t* ranges = reinterpret_cast<const uint32_t*>(ws + L.off_ranges);
    const uint32_t* vals = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    const Packed* packed = reinterpret_cast<const Packed*>(ws + L.off_packed);
    ProfScope prof(kKStats, s);
    hipLaunchKernelGGL(k_fill_f32, dim3(1), dim3(256), 0, s, reinterpret_cast<float*>(counters), 0.f, (size_t)4);
    hipLaunchKernelGGL(k_render_stats, dim3((unsigned)L.tiles), dim3(256), 0, s, cam, ranges, vals, packed,
                       reinterpret_cast<unsigned long long*>(counters));
    return hipGetLastError();
}

}  // namespace pbdr
