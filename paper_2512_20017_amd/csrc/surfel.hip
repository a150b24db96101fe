// 2D Gaussian surfels (the paper's 2DGS configuration: Sec. 5 "Applications"; Table 3b state of 20 floats; App. B
// "2DGS models [the projection] more accurately"): per-point projection and its derivative, raster record, and the
// per-tile compositing kernels with a ray-disk intersection per (pixel, splat) pair instead of a projected conic.
//
// A point is an oriented disk: centre, two raw tangent vectors made orthonormal by Gram-Schmidt, two scales, opacity,
// SH colour. ray_transform T = K [R s_u t_u | R s_v t_v | R mean + t] maps disk coordinates (u, v, 1) to homogeneous
// pixels. A pixel's ray meets the disk plane at (u, v) = (p_0, p_1) / p_2 with p = h_u x h_v, h_u = x T_2 - T_0,
// h_v = y T_2 - T_1 (rows of T); G = exp(-(u^2+v^2)/2), low-pass G^ = max(G, exp(-|pixel - mean2d|^2)),
// alpha = min(0.99, o G^); skip / stop / order rules as for 3D Gaussians.
//
// fp32 care: x T_2 - T_0 subtracts numbers of size (pixel x depth) to leave one of size (offset x depth). The raster
// record therefore stores rows centred on the projected centre, T_0' = T_0 - mx T_2 and T_1' = T_1 - my T_2 (one fused
// multiply-add each, so exactly rounded), and the kernels use h_u = dx T_2 - T_0' with dx = x - mx. The same value of
// mx is used on both sides, so this is the same number as x T_2 - T_0, without the cancellation.
#include "composite_common.h"
#include "pair_reduce.h"
#include "binning_common.h"
#include "sh_basis.h"

namespace pbdr {

// 64-byte raster record
struct __attribute__((aligned(16))) Packed2D {
    float t0x, t0y, t1x, t1y;      // centred rows T_0', T_1' (first two components)
    float t2x, t2y, t2z, o;        // T_2, opacity
    float mx, my, r, g;            // mean2d, red, green
    float b, radius_bits, t0z, t1z;  // blue, integer extent (bit-cast), third components of the centred rows (rounding residue)
};
static_assert(sizeof(Packed2D) == 64, "surfel raster record is 64 bytes");

struct Frame2D {
    float tu[3], tv[3], w[3], ainv, winv, btu, su, sv;
    float H[9];   // row-major; columns R s_u t_u, R s_v t_v, R mean + t
};

__device__ __forceinline__ void surfel_frame(const CamDev& cam, const float m[3], const float a[3], const float b[3],
                                             float ls0, float ls1, Frame2D& F)
{
    F.su = expf(ls0); F.sv = expf(ls1);
    F.ainv = 1.0f / sqrtf(a[0] * a[0] + a[1] * a[1] + a[2] * a[2]);
#pragma unroll
    for (int i = 0; i < 3; ++i) F.tu[i] = a[i] * F.ainv;
    F.btu = b[0] * F.tu[0] + b[1] * F.tu[1] + b[2] * F.tu[2];
#pragma unroll
    for (int i = 0; i < 3; ++i) F.w[i] = b[i] - F.btu * F.tu[i];
    F.winv = 1.0f / sqrtf(F.w[0] * F.w[0] + F.w[1] * F.w[1] + F.w[2] * F.w[2]);
#pragma unroll
    for (int i = 0; i < 3; ++i) F.tv[i] = F.w[i] * F.winv;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        F.H[3 * i] = F.su * (cam.R[3 * i] * F.tu[0] + cam.R[3 * i + 1] * F.tu[1] + cam.R[3 * i + 2] * F.tu[2]);
        F.H[3 * i + 1] = F.sv * (cam.R[3 * i] * F.tv[0] + cam.R[3 * i + 1] * F.tv[1] + cam.R[3 * i + 2] * F.tv[2]);
        F.H[3 * i + 2] = cam.R[3 * i] * m[0] + cam.R[3 * i + 1] * m[1] + cam.R[3 * i + 2] * m[2] + cam.t[i];
    }
}

template <int kDeg>
__global__ __launch_bounds__(256) void k_preprocess2d(Scene2DDev sc, CamDev cam, Splats2DDev out)
{
    const int n = sc.n;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const size_t N = (size_t)n;
    const float m[3] = {sc.mean[i], sc.mean[N + i], sc.mean[2 * N + i]};
    const float pz = cam.R[6] * m[0] + cam.R[7] * m[1] + cam.R[8] * m[2] + cam.t[2];
    if (!(pz >= cam.near_p && pz <= cam.far_p)) { out.radius[i] = 0; return; }
    const float a[3] = {sc.tan_u[i], sc.tan_u[N + i], sc.tan_u[2 * N + i]};
    const float b[3] = {sc.tan_v[i], sc.tan_v[N + i], sc.tan_v[2 * N + i]};
    Frame2D F;
    surfel_frame(cam, m, a, b, sc.log_scale[i], sc.log_scale[N + i], F);
    float T[9];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        T[k] = cam.fx * F.H[k] + cam.cx * F.H[6 + k];
        T[3 + k] = cam.fy * F.H[3 + k] + cam.cy * F.H[6 + k];
        T[6 + k] = F.H[6 + k];
    }
    const float aa = 9.f * (T[6] * T[6] + T[7] * T[7]) - T[8] * T[8];
    if (!(aa < 0.f)) { out.radius[i] = 0; return; }
    const float iz = 1.0f / T[8];
    // projected centre, formed from the camera-space columns so that cx, cy do not cancel
    const float mx = cam.fx * F.H[2] * iz + cam.cx, my = cam.fy * F.H[5] * iz + cam.cy;
    float reach = 0.f;
    {
        // Bounding box of the perspective image of the 3-sigma rim, in coordinates centred on the projected centre:
        // rows U_i = f_i (H_i - (H_i2 / H_22) H_2), whose third components vanish, so neither the principal point nor
        // the centre's own pixel coordinate enters (no cancellation of large numbers).
        const float ia = 1.0f / (9.f * (F.H[6] * F.H[6] + F.H[7] * F.H[7]) - F.H[8] * F.H[8]);
        const float f2[2] = {cam.fx, cam.fy};
#pragma unroll
        for (int ax = 0; ax < 2; ++ax) {
            const float* Hi = F.H + 3 * ax;
            const float sl = Hi[2] * iz;
            const float u0 = f2[ax] * (Hi[0] - sl * F.H[6]), u1 = f2[ax] * (Hi[1] - sl * F.H[7]);
            const float bb = 9.f * (u0 * F.H[6] + u1 * F.H[7]);
            const float cc = 9.f * (u0 * u0 + u1 * u1);
            const float c0 = bb * ia;
            const float half = sqrtf(fmaxf(1e-4f, c0 * c0 - cc * ia));
            reach = fmaxf(reach, fabsf(c0) + half);
        }
    }
    float ext = fmaxf(3.f, ceilf(reach));
    const int r = (ext < (float)kRadiusMax) ? (int)ext : kRadiusMax;
    if ((float)r <= cam.radius_clip) { out.radius[i] = 0; return; }
    {
        int x0, y0, x1, y1;
        tile_rect(cam, mx, my, r, x0, y0, x1, y1);
        if ((x1 - x0) * (y1 - y0) <= 0) { out.radius[i] = 0; return; }
    }
    const float vx = m[0] - cam.campos[0], vy = m[1] - cam.campos[1], vz = m[2] - cam.campos[2];
    const float vinv = 1.0f / sqrtf(vx * vx + vy * vy + vz * vz);
    float Y[16];
    sh_basis(kDeg, vx * vinv, vy * vinv, vz * vinv, Y);
    constexpr int K = (kDeg + 1) * (kDeg + 1);
    // all coefficients asked for before the first is used (written as one loop with the sums, every load was waited for
    // on its own: 48 round trips in a row per point)
    float coef[3 * K];
#pragma unroll
    for (int j = 0; j < 3 * K; ++j) coef[j] = __builtin_nontemporal_load(&sc.sh[(size_t)j * N + i]);
    const float lg = __builtin_nontemporal_load(&sc.logit[i]);
    float rgb[3] = {0.5f, 0.5f, 0.5f};
#pragma unroll
    for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int c = 0; c < 3; ++c) rgb[c] += Y[k] * coef[3 * k + c];
    }
    // normal = R (t_u x t_v), turned towards the camera
    float nw[3] = {F.tu[1] * F.tv[2] - F.tu[2] * F.tv[1], F.tu[2] * F.tv[0] - F.tu[0] * F.tv[2], F.tu[0] * F.tv[1] - F.tu[1] * F.tv[0]};
    float nc[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) nc[k] = cam.R[3 * k] * nw[0] + cam.R[3 * k + 1] * nw[1] + cam.R[3 * k + 2] * nw[2];
    const float facing = nc[0] * F.H[2] + nc[1] * F.H[5] + nc[2] * F.H[8];
    const float sgn = facing > 0.f ? -1.f : 1.f;
    out.mean2d[i] = mx; out.mean2d[N + i] = my;
#pragma unroll
    for (int k = 0; k < 9; ++k) out.T[(size_t)k * N + i] = T[k];
    out.opacity[i] = 1.0f / (1.0f + expf(-lg));
#pragma unroll
    for (int c = 0; c < 3; ++c) { out.color[(size_t)c * N + i] = fmaxf(rgb[c], 0.f); out.normal[(size_t)c * N + i] = sgn * nc[c]; }
    out.radius[i] = r;
    out.depth[i] = T[8];
}

// kFirst, kFromRecords: see the 3D variant. With kFromRecords the splat-state gradient of a point is the 64-byte record
// the gather of the compositing backward left in the workspace (`rec`), and `radius` is the tiles-touched count.
template <int kDeg, bool kFirst, bool kFromRecords>
__global__ __launch_bounds__(256) void k_preprocess2d_bwd(Scene2DDev sc, CamDev cam, const int32_t* __restrict__ radius,
                                                          const float* __restrict__ Tst, Splat2DGradDev g2,
                                                          const float4* __restrict__ rec, CarryFold cf, Scene2DGradDev g)
{
    const int n = sc.n;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const size_t N = (size_t)n;
    if (radius[i] <= 0) {
        if (kFirst) {
            constexpr int K0 = (kDeg + 1) * (kDeg + 1);
            // zeros and SH / opacity reads: non-temporal, as in the 3D kernels (see preprocess.hip)
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                __builtin_nontemporal_store(0.f, &g.mean[(size_t)k * N + i]);
                __builtin_nontemporal_store(0.f, &g.tan_u[(size_t)k * N + i]);
                __builtin_nontemporal_store(0.f, &g.tan_v[(size_t)k * N + i]);
            }
            __builtin_nontemporal_store(0.f, &g.log_scale[i]); __builtin_nontemporal_store(0.f, &g.log_scale[N + i]);
            __builtin_nontemporal_store(0.f, &g.logit[i]);
#pragma unroll
            for (int k = 0; k < 3 * K0; ++k) __builtin_nontemporal_store(0.f, &g.sh[(size_t)k * N + i]);
        }
        return;
    }
    // dL/d(splat state): T (nine), mean2d (two), opacity, colour (three), in the record's order
    float gs[15];
    if (kFromRecords) {
        const float4 ra = rec[(size_t)4 * i], rb = rec[(size_t)4 * i + 1], rc = rec[(size_t)4 * i + 2], rd = rec[(size_t)4 * i + 3];
        const float v[15] = {ra.x, ra.y, ra.z, ra.w, rb.x, rb.y, rb.z, rb.w, rc.x, rc.y, rc.z, rc.w, rd.x, rd.y, rd.z};
#pragma unroll
        for (int k = 0; k < 15; ++k) gs[k] = v[k];
        // a point whose pairs are cut by a wavefront boundary of the gather: its record is still in pieces (this launch
        // stands in for k_gather2d_fixup, see pair_reduce.h)
        if (cf.carry != nullptr) (void)record_from_carries<15>(cf, cf.slot_base[i], (uint32_t)radius[i], gs);
    } else {
#pragma unroll
        for (int k = 0; k < 9; ++k) gs[k] = g2.T[(size_t)k * N + i];
        gs[9] = g2.mean2d[i]; gs[10] = g2.mean2d[N + i];
        gs[11] = g2.opacity[i];
        gs[12] = g2.color[i]; gs[13] = g2.color[N + i]; gs[14] = g2.color[2 * N + i];
    }
    const float m[3] = {sc.mean[i], sc.mean[N + i], sc.mean[2 * N + i]};
    const float a[3] = {sc.tan_u[i], sc.tan_u[N + i], sc.tan_u[2 * N + i]};
    const float b[3] = {sc.tan_v[i], sc.tan_v[N + i], sc.tan_v[2 * N + i]};
    Frame2D F;
    surfel_frame(cam, m, a, b, sc.log_scale[i], sc.log_scale[N + i], F);
    {
        const float o = 1.0f / (1.0f + expf(-__builtin_nontemporal_load(&sc.logit[i])));
        grad_out<kFirst>(&g.logit[i], gs[11] * o * (1.f - o));
    }
    float dmu[3] = {0.f, 0.f, 0.f};
    {
        const float vx = m[0] - cam.campos[0], vy = m[1] - cam.campos[1], vz = m[2] - cam.campos[2];
        const float vinv = 1.0f / sqrtf(vx * vx + vy * vy + vz * vz);
        const float dx = vx * vinv, dy = vy * vinv, dz = vz * vinv;
        float Y[16];
        float dY[16][3];
        sh_basis(kDeg, dx, dy, dz, Y);
        sh_basis_grad(kDeg, dx, dy, dz, dY);
        constexpr int K = (kDeg + 1) * (kDeg + 1);
        float gd0 = 0.f, gd1 = 0.f, gd2 = 0.f;
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            float raw = 0.5f, t0 = 0.f, t1 = 0.f, t2 = 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const float co = __builtin_nontemporal_load(&sc.sh[(size_t)(3 * k + c) * N + i]);
                raw += Y[k] * co;
                t0 += dY[k][0] * co; t1 += dY[k][1] * co; t2 += dY[k][2] * co;
            }
            const float gc = raw > 0.f ? gs[12 + c] : 0.f;
            if (kFirst || gc != 0.f) {
#pragma unroll
                for (int k = 0; k < K; ++k) grad_out<kFirst>(&g.sh[(size_t)(3 * k + c) * N + i], Y[k] * gc);
            }
            gd0 += gc * t0; gd1 += gc * t1; gd2 += gc * t2;
        }
        const float dot = gd0 * dx + gd1 * dy + gd2 * dz;
        dmu[0] += (gd0 - dx * dot) * vinv; dmu[1] += (gd1 - dy * dot) * vinv; dmu[2] += (gd2 - dz * dot) * vinv;
    }
    // gradient w.r.t. the stored transform, plus mean2d_i = T_i2 / T_22
    float GT[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) GT[k] = gs[k];
    {
        const float T02 = Tst[2 * N + i], T12 = Tst[5 * N + i], T22 = Tst[8 * N + i];
        const float iz = 1.0f / T22, gmx = gs[9], gmy = gs[10];
        GT[2] += gmx * iz; GT[5] += gmy * iz;
        GT[8] -= (gmx * T02 + gmy * T12) * iz * iz;
    }
    float GH[9];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        GH[k] = cam.fx * GT[k];
        GH[3 + k] = cam.fy * GT[3 + k];
        GH[6 + k] = cam.cx * GT[k] + cam.cy * GT[3 + k] + GT[6 + k];
    }
    float gcol[3][3];   // world-space gradients of the three column vectors
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int r = 0; r < 3; ++r) gcol[k][r] = cam.R[r] * GH[k] + cam.R[3 + r] * GH[3 + k] + cam.R[6 + r] * GH[6 + k];
#pragma unroll
    for (int r = 0; r < 3; ++r) grad_out<kFirst>(&g.mean[(size_t)r * N + i], dmu[r] + gcol[2][r]);
    grad_out<kFirst>(&g.log_scale[i], F.su * (gcol[0][0] * F.tu[0] + gcol[0][1] * F.tu[1] + gcol[0][2] * F.tu[2]));
    grad_out<kFirst>(&g.log_scale[N + i], F.sv * (gcol[1][0] * F.tv[0] + gcol[1][1] * F.tv[1] + gcol[1][2] * F.tv[2]));
    {
        float gtu[3], gtv[3], gw[3];
#pragma unroll
        for (int r = 0; r < 3; ++r) { gtu[r] = F.su * gcol[0][r]; gtv[r] = F.sv * gcol[1][r]; }
        float dot = gtv[0] * F.tv[0] + gtv[1] * F.tv[1] + gtv[2] * F.tv[2];
#pragma unroll
        for (int r = 0; r < 3; ++r) gw[r] = (gtv[r] - F.tv[r] * dot) * F.winv;
        const float gbtu = -(gw[0] * F.tu[0] + gw[1] * F.tu[1] + gw[2] * F.tu[2]);
        float gx[3];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            grad_out<kFirst>(&g.tan_v[(size_t)r * N + i], gw[r] + gbtu * F.tu[r]);
            gx[r] = gtu[r] - F.btu * gw[r] + gbtu * b[r];
        }
        dot = gx[0] * F.tu[0] + gx[1] * F.tu[1] + gx[2] * F.tu[2];
#pragma unroll
        for (int r = 0; r < 3; ++r) grad_out<kFirst>(&g.tan_u[(size_t)r * N + i], (gx[r] - F.tu[r] * dot) * F.ainv);
    }
}

// Surfels: the 64-byte raster record of a listed point, with centred rows (see binning_common.h for the rest of the
// block's work: compaction and pair emission as for 3D Gaussians).
__global__ __launch_bounds__(256) void k_pack_dup2d(Splats2DDev sp, CamDev cam, BinArrays A, Packed2D* __restrict__ packed)
{
    const size_t N = (size_t)sp.n;
    pack_dup_block(BinInput{sp.n, sp.mean2d, sp.radius}, cam, A, sp.depth, [&](int i) {
        const float mx = sp.mean2d[i], my = sp.mean2d[N + i];
        const float t2x = sp.T[6 * N + i], t2y = sp.T[7 * N + i], t2z = sp.T[8 * N + i];
        float4* dst = reinterpret_cast<float4*>(packed + i);
        dst[0] = make_float4(fmaf(-mx, t2x, sp.T[i]), fmaf(-mx, t2y, sp.T[N + i]), fmaf(-my, t2x, sp.T[3 * N + i]),
                             fmaf(-my, t2y, sp.T[4 * N + i]));
        dst[1] = make_float4(t2x, t2y, t2z, sp.opacity[i]);
        dst[2] = make_float4(mx, my, sp.color[i], sp.color[N + i]);
        dst[3] = make_float4(sp.color[2 * N + i], __int_as_float(sp.radius[i]), fmaf(-mx, t2z, sp.T[2 * N + i]),
                             fmaf(-my, t2z, sp.T[5 * N + i]));
    });
}

constexpr int kAccStride2D = 17;   // floats between the LDS accumulators of consecutive surfels of a batch (odd)

// LDS image of one staged batch of kB surfels (kB a multiple of 64, at most the workgroup size)
template <int kB>
struct Stage2D {
    float4 a[kB];   // t0x, t0y, t1x, t1y
    float4 b[kB];   // t2x, t2y, t2z, log2(opacity)
    float4 c[kB];   // mx, my, red, green
    float4 d[kB];   // blue, t0z, t1z, -
    unsigned long long mask[4][kB / 64];
};

// Stage list entries [first, first+count): one per thread. A quadrant is kept for a splat if the bounding box of the
// image of the disk rim where alpha falls to 1/255 (rho^2 = 2 ln(255 o)), or the low-pass support around the centre,
// meets the quadrant's pixel centres; taken conservatively. count <= kB. All 256 threads must call it.
template <int kB>
__device__ __forceinline__ void stage_batch2d(Stage2D<kB>& S, const TileCtx& t, const uint32_t* __restrict__ vals,
                                              const Packed2D* __restrict__ packed, uint32_t first, int count, uint32_t& id,
                                              float4& r0, float4& r1, float4& r2, float4& r3)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool have = (int)threadIdx.x < count;
    bool reach[4] = {false, false, false, false};
    id = 0;
    r0 = r1 = r2 = r3 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (have) {
        id = vals[first + threadIdx.x];
        const float4* rec = reinterpret_cast<const float4*>(packed + id);
        r0 = rec[0]; r1 = rec[1]; r2 = rec[2]; r3 = rec[3];
        const float L = __log2f(r1.w);
        S.a[threadIdx.x] = r0;
        S.b[threadIdx.x] = make_float4(r1.x, r1.y, r1.z, L);
        S.c[threadIdx.x] = r2;
        S.d[threadIdx.x] = make_float4(r3.x, r3.z, r3.w, 0.f);
        const float tau = (L + kLog2_255) * 0.6931471805599453f;      // ln(255 o): alpha >= 1/255 <=> -ln G^ <= tau
        if (!(tau < -0.02f)) {
            const float rho2 = 2.f * fmaxf(tau, 0.f) + 0.05f;          // rim of the disk part, with margin
            const float lp = sqrtf(fmaxf(tau, 0.f)) + 0.05f;           // radius of the low-pass part, with margin
            // image of the rim u^2 + v^2 = rho2, relative to the projected centre: rows T_0', T_1', T_2
            const float aa = rho2 * (r1.x * r1.x + r1.y * r1.y) - r1.z * r1.z;
            float lo[2] = {-lp, -lp}, hi[2] = {lp, lp};
            const bool bounded = aa < -0.02f * r1.z * r1.z;   // else the rim at this level comes (almost) to the camera plane: keep all
            if (bounded) {
                const float ia = 1.0f / aa;
                const float bx = rho2 * (r0.x * r1.x + r0.y * r1.y) - r3.z * r1.z, by = rho2 * (r0.z * r1.x + r0.w * r1.y) - r3.w * r1.z;
                const float cx = rho2 * (r0.x * r0.x + r0.y * r0.y) - r3.z * r3.z, cy = rho2 * (r0.z * r0.z + r0.w * r0.w) - r3.w * r3.w;
                const float c0x = bx * ia, c0y = by * ia;
                const float hx = sqrtf(fmaxf(0.f, c0x * c0x - cx * ia)) * 1.001f + 0.01f;
                const float hy = sqrtf(fmaxf(0.f, c0y * c0y - cy * ia)) * 1.001f + 0.01f;
                lo[0] = fminf(lo[0], c0x - hx); hi[0] = fmaxf(hi[0], c0x + hx);
                lo[1] = fminf(lo[1], c0y - hy); hi[1] = fmaxf(hi[1], c0y + hy);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float qx0 = (float)(t.tx0 + (q & 1) * 8) + 0.5f - r2.x, qy0 = (float)(t.ty0 + (q >> 1) * 8) + 0.5f - r2.y;
                // keep unless the box lies wholly outside the quadrant's span of pixel centres (NaN keeps)
                const bool out = (hi[0] < qx0) || (lo[0] > qx0 + 7.f) || (hi[1] < qy0) || (lo[1] > qy0 + 7.f);
                reach[q] = !bounded || !out;
            }
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const unsigned long long m = __ballot(reach[q]);
        if (lane == 0 && wave < kB / 64) S.mask[q][wave] = m;
    }
}

// per-pair evaluation shared by forward and backward: exponent of G^ in log2 units and the pieces the backward needs
struct Pair2D {
    float dx, dy, hu0, hu1, hu2, hv0, hv1, hv2, p2, ip2, u, v, e1, e2;
};

__device__ __forceinline__ void eval_pair2d(const float4& a, const float4& b, const float4& c, const float4& d, float fx, float fy,
                                            Pair2D& E)
{
    E.dx = fx - c.x; E.dy = fy - c.y;
    E.hu0 = E.dx * b.x - a.x; E.hu1 = E.dx * b.y - a.y; E.hu2 = E.dx * b.z - d.y;
    E.hv0 = E.dy * b.x - a.z; E.hv1 = E.dy * b.y - a.w; E.hv2 = E.dy * b.z - d.z;
    const float p0 = E.hu1 * E.hv2 - E.hu2 * E.hv1;
    const float p1 = E.hu2 * E.hv0 - E.hu0 * E.hv2;
    E.p2 = E.hu0 * E.hv1 - E.hu1 * E.hv0;
    E.ip2 = __builtin_amdgcn_rcpf(E.p2);
    E.u = p0 * E.ip2; E.v = p1 * E.ip2;
    E.e1 = (-0.5f * kLog2e) * (E.u * E.u + E.v * E.v);
    E.e2 = -kLog2e * (E.dx * E.dx + E.dy * E.dy);
}

__global__ __launch_bounds__(256) void k_composite2d_fwd(CamDev cam, const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
                                                         const uint32_t* __restrict__ vals, const Packed2D* __restrict__ packed,
                                                         float bg0, float bg1, float bg2, float* __restrict__ image,
                                                         float* __restrict__ final_T, uint32_t* __restrict__ last_idx)
{
    __shared__ Stage2D<kBatch> S;
    const TileCtx c = tile_ctx(cam, ranges, tile_order);
    const int wave = threadIdx.x >> 6;
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    float T = 1.f, C0 = 0.f, C1 = 0.f, C2 = 0.f;
    uint32_t last = 0;
    bool live = c.inside;
    for (uint32_t base = c.start; base < c.end; base += kBatch) {
        if (__syncthreads_count(live) == 0) break;
        const int cnt = (int)min((uint32_t)kBatch, c.end - base);
        uint32_t id; float4 r0, r1, r2, r3;
        stage_batch2d(S, c, vals, packed, base, cnt, id, r0, r1, r2, r3);
        __syncthreads();
        if (__ballot(live) == 0ull) continue;
        const uint32_t pos0 = base - c.start + 1u;
        // alpha of one visit: everything that does not depend on the pixel's running state
        auto eval = [&](int j, float& alpha, bool& ok, float& r, float& g, float& bl) {
            const float4 a = S.a[j], b = S.b[j], cc = S.c[j], dd = S.d[j];
            bl = dd.x; r = cc.z; g = cc.w;
            Pair2D E;
            eval_pair2d(a, b, cc, dd, fx, fy, E);
            const float ex = (E.p2 != 0.f) ? fmaxf(E.e1, E.e2) : -1e30f;
            alpha = fminf(kAlphaMax, __builtin_amdgcn_exp2f(b.w + ex));
            ok = (E.p2 != 0.f) && (alpha >= kAlphaMin);
        };
        auto blend_one = [&](int j, float alpha, bool ok, float r, float g, float bl) {
            const bool valid = live && ok;
            const float aT = alpha * T;
            const float Tn = T - aT;            // T (1 - alpha), with the product the weight needs anyway
            const bool stop = valid && (Tn < kTStop);
            const bool blend = valid && !stop;
            live = live && !stop;
            const float w = blend ? aT : 0.f;
            C0 += r * w; C1 += g * w; C2 += bl * w;
            T = blend ? Tn : T;
            last = blend ? pos0 + (uint32_t)j : last;
        };
        for (int k = 0; k < 4; ++k) {
            unsigned long long m = uniform_u64(S.mask[wave][k]);
            // two visits per trip while there are two (independent alphas, blends in list order), as in the 3D kernel
            while (m & (m - 1ull)) {
                const int j0 = k * 64 + __builtin_ctzll(m);
                m &= m - 1ull;
                const int j1 = k * 64 + __builtin_ctzll(m);
                m &= m - 1ull;
                float al0, red0, grn0, blu0, al1, red1, grn1, blu1;
                bool ok0, ok1;
                eval(j0, al0, ok0, red0, grn0, blu0);
                eval(j1, al1, ok1, red1, grn1, blu1);
                blend_one(j0, al0, ok0, red0, grn0, blu0);
                blend_one(j1, al1, ok1, red1, grn1, blu1);
            }
            if (m) {
                const int j0 = k * 64 + __builtin_ctzll(m);
                float al0, red0, grn0, blu0;
                bool ok0;
                eval(j0, al0, ok0, red0, grn0, blu0);
                blend_one(j0, al0, ok0, red0, grn0, blu0);
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

// Backward. With dp = dL/dp for p = h_u x h_v (three numbers per pair), the gradient of the transform is a lane sum of
// the moments S0 = sum dp, Sx = sum dx dp, Sy = sum dy dp (dx, dy from the projected centre):
//   sum dL/dh_u = T_2 x Sy - T_1' x S0,   sum dL/dh_v = Sx x T_2 - S0 x T_0',
//   dT_0 = -sum dL/dh_u, dT_1 = -sum dL/dh_v, dT_2 = mx sum dL/dh_u + my sum dL/dh_v - T_1' x Sx - Sy x T_0'.
// Together with 3 colour sums, d opacity and the 2 low-pass sums for mean2d: 15 sums per splat, through two row
// butterflies, an LDS accumulator for the tile and one 64-byte record per (tile, splat) pair.
constexpr int kBwdBatch2D = 64;    // surfels staged at a time by the backward kernel: what the per-quadrant accumulators leave room for

__global__ __launch_bounds__(256, 6) void k_composite2d_bwd(CamDev cam, const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
                                                         const uint32_t* __restrict__ vals, const Packed2D* __restrict__ packed,
                                                         const uint32_t* __restrict__ slot_base, float bg0, float bg1, float bg2,
                                                         const float* __restrict__ final_T, const uint32_t* __restrict__ last_idx,
                                                         const float* __restrict__ dL_dimage, uint32_t cap,
                                                         float4* __restrict__ partial)
{
    __shared__ Stage2D<kBwdBatch2D> S;
    // [quadrant][splat of the batch][value], 17 floats apart (odd: the stores of one visit and the per-thread reads at
    // the end of a batch spread over the LDS banks). A wavefront visits a splat at most once per batch, so it writes its
    // quadrant's sums with plain stores and the thread that staged the splat adds the four up: no LDS float atomics,
    // which cost the LDS about 2.5 cycles per active lane.
    __shared__ float sAcc[4][kAccStride2D * kBwdBatch2D];
    __shared__ uint32_t sMax[4];
    const TileCtx c = tile_ctx(cam, ranges, tile_order);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float fx = (float)c.px + 0.5f, fy = (float)c.py + 0.5f;
    const size_t HW = (size_t)cam.W * cam.H;
    float T = 1.f, g0 = 0.f, g1 = 0.f, g2c = 0.f;
    uint32_t last = 0;
    if (c.inside) {
        T = final_T[c.pix];
        last = min(last_idx[c.pix], c.end - c.start);
        g0 = dL_dimage[c.pix]; g1 = dL_dimage[HW + c.pix]; g2c = dL_dimage[2 * HW + c.pix];
    }
    float Sfx = T * (bg0 * g0 + bg1 * g1 + bg2 * g2c);
    uint32_t wmax = last;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) wmax = max(wmax, (uint32_t)__shfl_xor((int)wmax, d, 64));
    if (lane == 0) sMax[wave] = wmax;
    __syncthreads();
    const uint32_t tile_last = max(max(sMax[0], sMax[1]), max(sMax[2], sMax[3]));
    const int tile_x = c.tix, tile_y = c.tiy;
    // The pairs behind the last splat any pixel of the tile blended are never staged; the gather adds up the records of
    // all pairs, so theirs are written as zeros here (every pair is in exactly one tile's list: each record is written
    // exactly once per call, here or at the end of its batch, and no fill of the whole array is needed beforehand).
    for (uint32_t p = tile_last + threadIdx.x; p < c.end - c.start; p += 256u) {
        const uint32_t idz = vals[c.start + p];
        const float4* rz = reinterpret_cast<const float4*>(packed + idz);
        const float4 z2 = rz[2], z3 = rz[3];
        int x0, y0, x1, y1;
        tile_rect(cam, z2.x, z2.y, __float_as_int(z3.y), x0, y0, x1, y1);
        const uint32_t u = slot_base[idz] + (uint32_t)((tile_y - y0) * (x1 - x0) + (tile_x - x0));
        if (u < cap && tile_x >= x0 && tile_x < x1 && tile_y >= y0 && tile_y < y1) {
            float4* dst = partial + (size_t)4 * u;
            const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
            dst[0] = zero; dst[1] = zero; dst[2] = zero; dst[3] = zero;
        }
    }
    if (tile_last == 0) return;
    const bool bit1 = (lane & 2) != 0;
    const int acc_slot = ((lane & 1) ? 8 : 0) + ((lane >> 1) & 7);     // see row_sum8: odd lanes take the second eight sums
    float* const sAccW = sAcc[wave];
    const int nbatch = (int)((tile_last + kBwdBatch2D - 1) / kBwdBatch2D);
    for (int bi = nbatch - 1; bi >= 0; --bi) {
        const uint32_t boff = (uint32_t)bi * kBwdBatch2D;
        const int cnt = (int)min((uint32_t)kBwdBatch2D, tile_last - boff);
        uint32_t id; float4 q0, q1, q2, q3;
        stage_batch2d(S, c, vals, packed, c.start + boff, cnt, id, q0, q1, q2, q3);
#pragma unroll
        for (int k = 0; k < 4 * kAccStride2D * kBwdBatch2D / 256; ++k) (&sAcc[0][0])[k * 256 + threadIdx.x] = 0.f;
        __syncthreads();
        if (wmax > boff) {
            for (int k = kBwdBatch2D / 64 - 1; k >= 0; --k) {
                unsigned long long m = uniform_u64(S.mask[wave][k]);
                while (m) {
                    const int bit = 63 - __builtin_clzll(m);
                    m &= ~(1ull << bit);
                    const int j = k * 64 + bit;
                    const uint32_t pos = boff + (uint32_t)j + 1u;
                    const float4 a = S.a[j], b = S.b[j], cc = S.c[j], dd = S.d[j];
                    const float blue = dd.x;
                    Pair2D E;
                    eval_pair2d(a, b, cc, dd, fx, fy, E);
                    const bool disk = E.e1 > E.e2;                         // which part of the max is active (false for NaN)
                    const float ex = disk ? E.e1 : E.e2;
                    const float gh = __builtin_amdgcn_exp2f(ex);           // G^
                    const float araw = __builtin_amdgcn_exp2f(b.w + ex);   // o G^
                    const float alpha = fminf(kAlphaMax, araw);
                    const bool hit = (pos <= last) && (E.p2 != 0.f) && (alpha >= kAlphaMin);
                    if (__ballot(hit) == 0ull) continue;
                    const float ioma = __builtin_amdgcn_rcpf(1.f - alpha);
                    const float Tk = T * ioma;
                    const float w = hit ? alpha * Tk : 0.f;
                    const float cg = cc.z * g0 + cc.w * g1 + blue * g2c;
                    const float dL_dalpha = Tk * cg - Sfx * ioma;
                    const float da = (hit && araw < kAlphaMax) ? dL_dalpha : 0.f;     // zero where alpha was clamped
                    T = hit ? Tk : T;
                    Sfx += w * cg;
                    const float d_o = gh * da;
                    const float dgh = araw * da;                             // o G^ dL/dalpha (zero unless hit)
                    // disk part: dL/du = -u G o dL/dalpha; low-pass part: dL/dmx = 2 dx G2 o dL/dalpha.
                    // u, v, 1/p2 are finite wherever the disk part is the active one; elsewhere they are replaced by 0
                    // so that no 0 * inf reaches the sums.
                    const float us = disk ? E.u : 0.f, vs = disk ? E.v : 0.f, ips = disk ? E.ip2 : 0.f;
                    const float du = -us * dgh, dv = -vs * dgh;
                    const float dmx = disk ? 0.f : 2.f * E.dx * dgh, dmy = disk ? 0.f : 2.f * E.dy * dgh;
                    const float dp0 = du * ips, dp1 = dv * ips, dp2 = -(du * us + dv * vs) * ips;
                    const float va[8] = {dp0, dp1, dp2, E.dx * dp0, E.dx * dp1, E.dx * dp2, E.dy * dp0, E.dy * dp1};
                    const float vb[8] = {E.dy * dp2, w * g0, w * g1, w * g2c, d_o, dmx, dmy, 0.f};
                    const float pa = row_sum8(va, bit1);
                    const float pb = row_sum8(vb, bit1);
                    // even lanes of a row keep the first eight sums, odd lanes (their copies) take the second eight;
                    // the four rows are added lane by lane, and the 16 lanes of the last row store the sums
                    const float tot = sum_rows((lane & 1) ? pb : pa);
                    int acc_base = kAccStride2D * j;
                    asm volatile("" : "+s"(acc_base));      // keep the product on the scalar unit (as in the 3D kernel)
                    if (lane >= 48) sAccW[acc_base + acc_slot] = tot;
                }
            }
        }
        __syncthreads();
        if ((int)threadIdx.x < cnt) {
            int x0, y0, x1, y1;
            tile_rect(cam, q2.x, q2.y, __float_as_int(q3.y), x0, y0, x1, y1);
            const uint32_t u = slot_base[id] + (uint32_t)((tile_y - y0) * (x1 - x0) + (tile_x - x0));
            if (u < cap && tile_x >= x0 && tile_x < x1 && tile_y >= y0 && tile_y < y1) {
                float acc[15];
#pragma unroll
                for (int k = 0; k < 15; ++k) {
                    const int e = kAccStride2D * (int)threadIdx.x + k;
                    acc[k] = (sAcc[0][e] + sAcc[1][e]) + (sAcc[2][e] + sAcc[3][e]);
                }
                const float s0[3] = {acc[0], acc[1], acc[2]};
                const float sx[3] = {acc[3], acc[4], acc[5]};
                const float sy[3] = {acc[6], acc[7], acc[8]};
                const float t0[3] = {q0.x, q0.y, q3.z}, t1[3] = {q0.z, q0.w, q3.w}, t2[3] = {q1.x, q1.y, q1.z};
                const float mx = q2.x, my = q2.y;
                float dhu[3], dhv[3], ex[3];
                // sum dL/dh_u = T2 x Sy - T1' x S0
                dhu[0] = (t2[1] * sy[2] - t2[2] * sy[1]) - (t1[1] * s0[2] - t1[2] * s0[1]);
                dhu[1] = (t2[2] * sy[0] - t2[0] * sy[2]) - (t1[2] * s0[0] - t1[0] * s0[2]);
                dhu[2] = (t2[0] * sy[1] - t2[1] * sy[0]) - (t1[0] * s0[1] - t1[1] * s0[0]);
                // sum dL/dh_v = Sx x T2 - S0 x T0'
                dhv[0] = (sx[1] * t2[2] - sx[2] * t2[1]) - (s0[1] * t0[2] - s0[2] * t0[1]);
                dhv[1] = (sx[2] * t2[0] - sx[0] * t2[2]) - (s0[2] * t0[0] - s0[0] * t0[2]);
                dhv[2] = (sx[0] * t2[1] - sx[1] * t2[0]) - (s0[0] * t0[1] - s0[1] * t0[0]);
                // - T1' x Sx - Sy x T0'
                ex[0] = -(t1[1] * sx[2] - t1[2] * sx[1]) - (sy[1] * t0[2] - sy[2] * t0[1]);
                ex[1] = -(t1[2] * sx[0] - t1[0] * sx[2]) - (sy[2] * t0[0] - sy[0] * t0[2]);
                ex[2] = -(t1[0] * sx[1] - t1[1] * sx[0]) - (sy[0] * t0[1] - sy[1] * t0[0]);
                float4* dst = partial + (size_t)4 * u;
                dst[0] = make_float4(-dhu[0], -dhu[1], -dhu[2], -dhv[0]);                                     // dT0, dT1.x
                dst[1] = make_float4(-dhv[1], -dhv[2], mx * dhu[0] + my * dhv[0] + ex[0], mx * dhu[1] + my * dhv[1] + ex[1]);
                dst[2] = make_float4(mx * dhu[2] + my * dhv[2] + ex[2], acc[13], acc[14],   // dT2.z, d mean2d
                                     acc[12]);                                                          // d opacity
                dst[3] = make_float4(acc[9], acc[10], acc[11], 0.f);        // d colour
            }
        }
        __syncthreads();
    }
}

// Per point: add up the 64-byte partial records of its pairs (balanced by pairs, see pair_reduce.h).
struct StoreSplat2DGrad {      // one 64-byte record per point, by point index (see the 3D variant)
    float4* rec;
    const uint32_t* order;
    __device__ __forceinline__ void operator()(uint32_t rank, const float (&v)[15]) const
    {
        float4* dst = rec + (size_t)4 * order[rank];
        dst[0] = make_float4(v[0], v[1], v[2], v[3]);
        dst[1] = make_float4(v[4], v[5], v[6], v[7]);
        dst[2] = make_float4(v[8], v[9], v[10], v[11]);
        dst[3] = make_float4(v[12], v[13], v[14], 0.f);
    }
};

__global__ __launch_bounds__(256) void k_gather2d(int n, const uint32_t* __restrict__ status, const uint32_t* __restrict__ order,
                                                  const uint32_t* __restrict__ offsets, const uint32_t* __restrict__ chunk_rank,
                                                  const float4* __restrict__ partial, uint32_t cap, float* __restrict__ carry,
                                                  float4* __restrict__ rec)
{
    __shared__ uint32_t sEnd[4][64];
    const uint32_t w = blockIdx.x * 4u + (threadIdx.x >> 6);
    gather_wave<4, 15, false>(w, n, status, offsets, chunk_rank, partial, cap, carry, sEnd[threadIdx.x >> 6], StoreSplat2DGrad{rec, order});
}

__global__ __launch_bounds__(256) void k_gather2d_fixup(int n, const uint32_t* __restrict__ status, const uint32_t* __restrict__ order,
                                                        uint32_t cap, const float* __restrict__ carry, float4* __restrict__ rec)
{
    gather_fixup<15>(blockIdx.x * 256u + threadIdx.x, status, cap, carry, StoreSplat2DGrad{rec, order});
}

__global__ __launch_bounds__(256) void k_grad_records_to_planes2d(int n, const uint32_t* __restrict__ tiles_touched,
                                                                  const float4* __restrict__ rec, Splat2DGradDev g2)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n || tiles_touched[i] == 0) return;
    const size_t N = (size_t)n;
    const float4 a = rec[(size_t)4 * i], b = rec[(size_t)4 * i + 1], c = rec[(size_t)4 * i + 2], d = rec[(size_t)4 * i + 3];
    const float v[15] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w, c.x, c.y, c.z, c.w, d.x, d.y, d.z};
#pragma unroll
    for (int k = 0; k < 9; ++k) g2.T[(size_t)k * N + i] = v[k];
    g2.mean2d[i] = v[9]; g2.mean2d[N + i] = v[10];
    g2.opacity[i] = v[11];
    g2.color[i] = v[12]; g2.color[N + i] = v[13]; g2.color[2 * N + i] = v[14];
}

// Measurement aid: the forward walk with counters instead of colours (see the 3D variant).
__global__ __launch_bounds__(256) void k_render_stats2d(CamDev cam, const uint32_t* __restrict__ ranges, const uint32_t* __restrict__ tile_order,
                                                        const uint32_t* __restrict__ vals, const Packed2D* __restrict__ packed,
                                                        unsigned long long* __restrict__ counters)
{
    __shared__ float4 sR[4][kBatch];
    __shared__ unsigned long long sCnt[2];
    const TileCtx c = tile_ctx(cam, ranges, tile_order);
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
#pragma unroll
            for (int k = 0; k < 4; ++k) sR[k][threadIdx.x] = rec[k];
        }
        __syncthreads();
        const int cnt = (int)min((uint32_t)kBatch, c.end - base);
        if (!done) {
            for (int j = 0; j < cnt; ++j) {
                const float4 a = sR[0][j], b = sR[1][j], cc = sR[2][j], r3 = sR[3][j];
                Pair2D E;
                eval_pair2d(a, b, cc, make_float4(r3.x, r3.z, r3.w, 0.f), fx, fy, E);
                ++examined;
                if (E.p2 == 0.f) continue;
                const float alpha = fminf(kAlphaMax, b.w * __builtin_amdgcn_exp2f(fmaxf(E.e1, E.e2)));
                if (!(alpha >= kAlphaMin)) continue;
                const float Tn = T - alpha * T;     // as the forward kernel forms it
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

__global__ __launch_bounds__(64) void k_zero_counters2d(unsigned long long* __restrict__ counters)
{
    if (threadIdx.x < 2) counters[threadIdx.x] = 0ull;
}

// ---------------------------------------------------------------------------------------------------- launchers
hipError_t launch_preprocess2d(const Scene2DDev& sc, const CamDev& cam, const Splats2DDev& out, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    ProfScope prof(kKPreprocess, s);
    switch (sc.sh_degree) {
        case 0: hipLaunchKernelGGL(k_preprocess2d<0>, dim3(blocks), dim3(256), 0, s, sc, cam, out); break;
        case 1: hipLaunchKernelGGL(k_preprocess2d<1>, dim3(blocks), dim3(256), 0, s, sc, cam, out); break;
        case 2: hipLaunchKernelGGL(k_preprocess2d<2>, dim3(blocks), dim3(256), 0, s, sc, cam, out); break;
        default: hipLaunchKernelGGL(k_preprocess2d<3>, dim3(blocks), dim3(256), 0, s, sc, cam, out); break;
    }
    return hipGetLastError();
}

template <bool kFirst, bool kFromRecords>
static void launch_preprocess2d_bwd_t(const Scene2DDev& sc, const CamDev& cam, const int32_t* used, const float* Tst,
                                      const Splat2DGradDev& g2, const float4* rec, const CarryFold& cf, const Scene2DGradDev& g, unsigned blocks,
                                      hipStream_t s)
{
    switch (sc.sh_degree) {
        case 0: hipLaunchKernelGGL((k_preprocess2d_bwd<0, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, Tst, g2, rec, cf, g); break;
        case 1: hipLaunchKernelGGL((k_preprocess2d_bwd<1, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, Tst, g2, rec, cf, g); break;
        case 2: hipLaunchKernelGGL((k_preprocess2d_bwd<2, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, Tst, g2, rec, cf, g); break;
        default: hipLaunchKernelGGL((k_preprocess2d_bwd<3, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, Tst, g2, rec, cf, g); break;
    }
}

hipError_t launch_preprocess2d_bwd(const Scene2DDev& sc, const CamDev& cam, const Splats2DDev& sp, const Splat2DGradDev& g2,
                                   const Scene2DGradDev& g, bool first_view, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    ProfScope prof(kKPreprocessBwd, s);
    const CarryFold no_fold{nullptr, nullptr, nullptr, 0u};
    if (first_view) launch_preprocess2d_bwd_t<true, false>(sc, cam, sp.radius, sp.T, g2, nullptr, no_fold, g, blocks, s);
    else launch_preprocess2d_bwd_t<false, false>(sc, cam, sp.radius, sp.T, g2, nullptr, no_fold, g, blocks, s);
    return hipGetLastError();
}

// the same from the per-point gradient records in the workspace (see k_preprocess2d_bwd)
hipError_t launch_preprocess2d_bwd_records(const Scene2DDev& sc, const CamDev& cam, const Splats2DDev& sp, const uint32_t* tiles_touched,
                                           const float4* rec, const CarryFold& cf, const Scene2DGradDev& g, bool first_view, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    const int32_t* used = reinterpret_cast<const int32_t*>(tiles_touched);     // counts are far below 2^31
    const Splat2DGradDev none{nullptr, nullptr, nullptr, nullptr};
    ProfScope prof(kKPreprocessBwd, s);
    if (first_view) launch_preprocess2d_bwd_t<true, true>(sc, cam, used, sp.T, none, rec, cf, g, blocks, s);
    else launch_preprocess2d_bwd_t<false, true>(sc, cam, used, sp.T, none, rec, cf, g, blocks, s);
    return hipGetLastError();
}

hipError_t launch_bin_sort2d(const Splats2DDev& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s)
{
    if (sp.n == 0) return launch_bin_begin(L, ws, s);      // nothing to count: only the cleared status words and ranges
    hipError_t e = launch_count_visible(BinInput{sp.n, sp.mean2d, sp.radius}, cam, L, ws, s);
    if (e != hipSuccess) return e;
    {
        ProfScope prof(kKDuplicate, s);
        hipLaunchKernelGGL(k_pack_dup2d, dim3((unsigned)((sp.n + 255) / 256)), dim3(256), 0, s, sp, cam, bin_arrays(L, ws),
                           reinterpret_cast<Packed2D*>(ws + L.off_packed));
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return launch_bin_finish(BinInput{sp.n, sp.mean2d, sp.radius}, cam, L, ws, s);
}

hipError_t launch_composite2d_fwd(const CamDev& cam, const Layout& L, char* ws, const float bg[3], float* image,
                                  float* final_T, uint32_t* last_idx, hipStream_t s)
{
    ProfScope prof(kKCompositeFwd, s);
    hipLaunchKernelGGL(k_composite2d_fwd, dim3((unsigned)(cam.TX * cam.TY)), dim3(256), 0, s, cam,
                       reinterpret_cast<const uint32_t*>(ws + L.off_ranges), reinterpret_cast<const uint32_t*>(ws + L.off_tile_order),
                       reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L)),
                       reinterpret_cast<const Packed2D*>(ws + L.off_packed), bg[0], bg[1], bg[2], image, final_T, last_idx);
    return hipGetLastError();
}

hipError_t launch_composite2d_bwd(const CamDev& cam, const Layout& L, char* ws, int n, const float bg[3], const float* final_T,
                                  const uint32_t* last_idx, const float* dL_dimage, const Splat2DGradDev& g2, hipStream_t s)
{
    const uint32_t* status = reinterpret_cast<const uint32_t*>(ws + L.off_status);
    float4* partial = reinterpret_cast<float4*>(ws + L.off_partial);
    {
        ProfScope prof(kKCompositeBwd, s);
        hipLaunchKernelGGL(k_composite2d_bwd, dim3((unsigned)(cam.TX * cam.TY)), dim3(256), 0, s, cam,
                           reinterpret_cast<const uint32_t*>(ws + L.off_ranges), reinterpret_cast<const uint32_t*>(ws + L.off_tile_order),
                       reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L)),
                           reinterpret_cast<const Packed2D*>(ws + L.off_packed), reinterpret_cast<const uint32_t*>(ws + L.off_slot_base),
                           bg[0], bg[1], bg[2], final_T, last_idx, dL_dimage, L.cap, partial);
    }
    if (n > 0) {
        ProfScope prof(kKGather, s);
        const uint32_t* order = reinterpret_cast<const uint32_t*>(ws + L.off_order);
        const uint32_t* offsets = reinterpret_cast<const uint32_t*>(ws + L.off_offsets);
        const uint32_t* chunk_rank = reinterpret_cast<const uint32_t*>(ws + L.off_chunk_rank);
        float* carry = reinterpret_cast<float*>(ws + L.off_carry);
        const unsigned nwave = (unsigned)((L.cap + kChunkPairs - 1) / kChunkPairs);
        float4* rec = reinterpret_cast<float4*>(ws + L.off_grad_rec);
        hipLaunchKernelGGL(k_gather2d, dim3((nwave + 3) / 4), dim3(256), 0, s, n, status, order, offsets, chunk_rank, partial,
                           L.cap, carry, rec);
        if (g2.mean2d != nullptr) {      // else the caller goes on from the records, pieces included (launch_preprocess2d_bwd_records)
            hipLaunchKernelGGL(k_gather2d_fixup, dim3((nwave + 255) / 256), dim3(256), 0, s, n, status, order, L.cap, carry, rec);
            hipLaunchKernelGGL(k_grad_records_to_planes2d, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, n,
                               reinterpret_cast<const uint32_t*>(ws + L.off_touched), rec, g2);
        }
    }
    return hipGetLastError();
}

hipError_t launch_render_stats2d(const CamDev& cam, const Layout& L, char* ws, uint64_t* counters, hipStream_t s)
{
    ProfScope prof(kKStats, s);
    hipLaunchKernelGGL(k_zero_counters2d, dim3(1), dim3(64), 0, s, reinterpret_cast<unsigned long long*>(counters));
    hipLaunchKernelGGL(k_render_stats2d, dim3((unsigned)(cam.TX * cam.TY)), dim3(256), 0, s, cam,
                       reinterpret_cast<const uint32_t*>(ws + L.off_ranges), reinterpret_cast<const uint32_t*>(ws + L.off_tile_order),
                       reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L)),
                       reinterpret_cast<const Packed2D*>(ws + L.off_packed), reinterpret_cast<unsigned long long*>(counters));
    return hipGetLastError();
}

}  // namespace pbdr
