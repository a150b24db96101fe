// Per-point kernels: cull + project + SH colour (pts_culling + pts_splatting, paper Sec. 3.1 / 3.2, Alg. 1
// lines 2-4) and its derivative (pts_splatting.backward, Alg. 1 lines 22-24).
//
// One thread per point, structure-of-arrays planes: a wavefront reads 64 consecutive floats of every
// attribute (256-byte coalesced segments); the 48 SH planes are only touched by points that survive culling.
// HBM-bound: 236 B read + 44 B written per surviving point, 12 B + 4 B per point culled by depth.
#include "pbdr_internal.h"
#include "pair_reduce.h"

// No fused multiply-adds formed by the compiler in this file. Which products get fused into which sums depends on how
// the surrounding code is laid out (what shares a basic block after inlining, hoisting and unrolling), so the one-view
// and the batched kernels, which run the same per-point functions inside different loops, would otherwise differ in
// the last bit here and there, and with them, rarely, an extent or a cull decision. With contraction off every
// operation rounds as written and the variants agree bit for bit. These kernels wait on memory, not on the ALU.
#pragma clang fp contract(off)

#include "sh_basis.h"      // (after the pragma: the basis functions round as written here too)

namespace pbdr {

struct Proj {
    float s[3], q[4], qinv, Rq[9], A[9], T[6];
    float px, py, pz, iz, tx, ty;
    bool tx_free, ty_free;
    float J00, J02, J11, J12;
    float a, b, c, det;
};

__device__ __forceinline__ void quat_rot(const float q[4], float R[9])
{
    const float w = q[0], x = q[1], y = q[2], z = q[3];
    R[0] = 1.f - 2.f * (y * y + z * z); R[1] = 2.f * (x * y - w * z);       R[2] = 2.f * (x * z + w * y);
    R[3] = 2.f * (x * y + w * z);       R[4] = 1.f - 2.f * (x * x + z * z); R[5] = 2.f * (y * z - w * x);
    R[6] = 2.f * (x * z - w * y);       R[7] = 2.f * (y * z + w * x);       R[8] = 1.f - 2.f * (x * x + y * y);
}

// Covariance projection of a point already known to pass the depth test.
// cov2d = T T^T + blur I with T = J R_cam R_q diag(s): never forms the 3D covariance.
__device__ __forceinline__ void project_cov(const CamDev& cam, const float ls[3], const float qraw[4], Proj& P)
{
#pragma unroll
    for (int k = 0; k < 3; ++k) P.s[k] = expf(ls[k]);
    P.qinv = 1.0f / sqrtf(qraw[0] * qraw[0] + qraw[1] * qraw[1] + qraw[2] * qraw[2] + qraw[3] * qraw[3]);
#pragma unroll
    for (int k = 0; k < 4; ++k) P.q[k] = qraw[k] * P.qinv;
    quat_rot(P.q, P.Rq);
    // A = R_cam * Rq * diag(s)
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j)
            P.A[3 * i + j] = (cam.R[3 * i] * P.Rq[j] + cam.R[3 * i + 1] * P.Rq[3 + j] + cam.R[3 * i + 2] * P.Rq[6 + j]) * P.s[j];
    P.iz = 1.0f / P.pz;
    float tx = P.px * P.iz, ty = P.py * P.iz;
    P.tx_free = (tx <= cam.lim_x) && (tx >= -cam.lim_x);
    P.ty_free = (ty <= cam.lim_y) && (ty >= -cam.lim_y);
    tx = fminf(cam.lim_x, fmaxf(-cam.lim_x, tx));
    ty = fminf(cam.lim_y, fmaxf(-cam.lim_y, ty));
    P.tx = tx; P.ty = ty;
    P.J00 = cam.fx * P.iz; P.J02 = -cam.fx * tx * P.iz;
    P.J11 = cam.fy * P.iz; P.J12 = -cam.fy * ty * P.iz;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        P.T[j] = P.J00 * P.A[j] + P.J02 * P.A[6 + j];
        P.T[3 + j] = P.J11 * P.A[3 + j] + P.J12 * P.A[6 + j];
    }
    const float a0 = P.T[0] * P.T[0] + P.T[1] * P.T[1] + P.T[2] * P.T[2];
    const float c0 = P.T[3] * P.T[3] + P.T[4] * P.T[4] + P.T[5] * P.T[5];
    P.b = P.T[0] * P.T[3] + P.T[1] * P.T[4] + P.T[2] * P.T[5];
    // |T0|^2 |T1|^2 - (T0.T1)^2 = |T0 x T1|^2 : the determinant without the cancellation of a*c - b*b
    const float xx = P.T[1] * P.T[5] - P.T[2] * P.T[4];
    const float xy = P.T[2] * P.T[3] - P.T[0] * P.T[5];
    const float xz = P.T[0] * P.T[4] - P.T[1] * P.T[3];
    P.a = a0 + kBlur; P.c = c0 + kBlur;
    P.det = (xx * xx + xy * xy + xz * xz) + kBlur * (a0 + c0) + kBlur * kBlur;
}

// Where a point's raw parameters come from. The per-view work asks for them in the order it needs them - centre,
// then shape (scales, rotation) once the depth test is passed, then appearance (SH coefficients, opacity) once the
// point is known to be visible - so that culled points cost 12 bytes.
// DirectSrc reads every value from memory where it is used (one view per launch). CachedSrc keeps what it has read
// in registers, for launches that take a point through several views.
template <int kDeg>
struct DirectSrc {
    const SceneDev& sc;
    int i;
    size_t N;
    float m[3], ls[3], qr[4];
    __device__ __forceinline__ DirectSrc(const SceneDev& sc_, int i_) : sc(sc_), i(i_), N((size_t)sc_.n)
    {
        m[0] = sc.mean[i]; m[1] = sc.mean[N + i]; m[2] = sc.mean[2 * N + i];
    }
    __device__ __forceinline__ void need_shape()
    {
#pragma unroll
        for (int k = 0; k < 3; ++k) ls[k] = sc.log_scale[(size_t)k * N + i];
#pragma unroll
        for (int k = 0; k < 4; ++k) qr[k] = sc.quat[(size_t)k * N + i];
    }
    __device__ __forceinline__ void need_appearance() {}
    // read once by the forward kernel and once, after everything else of the view, by the backward kernel: non-temporal,
    // so that these 49 planes do not push what the next kernels re-read (splat state, sort buffers) out of the caches
    // (forward kernel 48 -> 41 us at 1M points). The same on the other parameters, on the gradient stores or on the
    // per-pair records of the gather was measured slower for the step as a whole.
    __device__ __forceinline__ float sh(int j) const { return __builtin_nontemporal_load(&sc.sh[(size_t)j * N + i]); }
    __device__ __forceinline__ float logit() const { return __builtin_nontemporal_load(&sc.logit[i]); }
};

template <int kDeg>
struct CachedSrc {
    static constexpr int K3 = 3 * (kDeg + 1) * (kDeg + 1);
    const SceneDev& sc;
    int i;
    size_t N;
    float m[3], ls[3], qr[4];
    float shv[K3], lg;
    bool has_shape, has_app;
    __device__ __forceinline__ CachedSrc(const SceneDev& sc_, int i_) : sc(sc_), i(i_), N((size_t)sc_.n), has_shape(false), has_app(false)
    {
        m[0] = sc.mean[i]; m[1] = sc.mean[N + i]; m[2] = sc.mean[2 * N + i];
    }
    __device__ __forceinline__ void need_shape()
    {
        if (has_shape) return;
#pragma unroll
        for (int k = 0; k < 3; ++k) ls[k] = sc.log_scale[(size_t)k * N + i];
#pragma unroll
        for (int k = 0; k < 4; ++k) qr[k] = sc.quat[(size_t)k * N + i];
        has_shape = true;
    }
    __device__ __forceinline__ void need_appearance()
    {
        if (has_app) return;
#pragma unroll
        for (int j = 0; j < K3; ++j) shv[j] = sc.sh[(size_t)j * N + i];
        lg = sc.logit[i];
        has_app = true;
    }
    __device__ __forceinline__ float sh(int j) const { return shv[j]; }
    __device__ __forceinline__ float logit() const { return lg; }
};

// One point through one view: cull, project, colour; writes the view's splat state (radius 0 for a culled point).
template <int kDeg, class Src>
__device__ __forceinline__ void preprocess_point(const CamDev& cam, Src& src, const SplatsDev& out)
{
    const int i = src.i;
    const size_t N = src.N;
    const float m0 = src.m[0], m1 = src.m[1], m2 = src.m[2];
    Proj P;
    P.px = cam.R[0] * m0 + cam.R[1] * m1 + cam.R[2] * m2 + cam.t[0];
    P.py = cam.R[3] * m0 + cam.R[4] * m1 + cam.R[5] * m2 + cam.t[1];
    P.pz = cam.R[6] * m0 + cam.R[7] * m1 + cam.R[8] * m2 + cam.t[2];
    if (!(P.pz >= cam.near_p && P.pz <= cam.far_p)) { out.radius[i] = 0; return; }
    src.need_shape();
    project_cov(cam, src.ls, src.qr, P);
    if (!(P.det > 0.f)) { out.radius[i] = 0; return; }
    const float idet = 1.0f / P.det;
    const float mx = cam.fx * P.px * P.iz + cam.cx;
    const float my = cam.fy * P.py * P.iz + cam.cy;
    const float mid = 0.5f * (P.a + P.c);
    // (a-c)^2/4 + b^2 is mid^2 - (a c - b^2) written without cancellation
    const float hd = 0.5f * (P.a - P.c);
    const float disc = fmaxf(kEigFloor, hd * hd + P.b * P.b);
    const float ext = ceilf(3.0f * sqrtf(mid + sqrtf(disc)));
    const int r = (ext < (float)kRadiusMax) ? (int)ext : kRadiusMax;
    if ((float)r <= cam.radius_clip) { out.radius[i] = 0; return; }
    int x0, y0, x1, y1;
    tile_rect(cam, mx, my, r, x0, y0, x1, y1);
    if ((x1 - x0) * (y1 - y0) <= 0) { out.radius[i] = 0; return; }
    // colour
    src.need_appearance();
    const float vx = m0 - cam.campos[0], vy = m1 - cam.campos[1], vz = m2 - cam.campos[2];
    const float vinv = 1.0f / sqrtf(vx * vx + vy * vy + vz * vz);
    float Y[16];
    sh_basis(kDeg, vx * vinv, vy * vinv, vz * vinv, Y);
    constexpr int K = (kDeg + 1) * (kDeg + 1);
    float rgb[3] = {0.5f, 0.5f, 0.5f};
#pragma unroll
    for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int c = 0; c < 3; ++c) rgb[c] += Y[k] * src.sh(3 * k + c);
    }
    const float o = 1.0f / (1.0f + expf(-src.logit()));
    out.mean2d[i] = mx; out.mean2d[N + i] = my;
    out.conic[i] = P.c * idet; out.conic[N + i] = -P.b * idet; out.conic[2 * N + i] = P.a * idet;
    out.opacity[i] = o;
    out.color[i] = fmaxf(rgb[0], 0.f); out.color[N + i] = fmaxf(rgb[1], 0.f); out.color[2 * N + i] = fmaxf(rgb[2], 0.f);
    out.radius[i] = r;
    out.depth[i] = P.pz;
}

// keep / blocks_per_group: optional point-group culling (App. D.1). keep[g] == 0 means every point of group g is
// known to be culled for this view; the workgroup then only marks its 256 points culled and reads no parameter.
template <int kDeg>
__global__ __launch_bounds__(256) void k_preprocess(SceneDev sc, CamDev cam, SplatsDev out, const uint8_t* __restrict__ keep,
                                                    int blocks_per_group)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= sc.n) return;
    if (keep != nullptr && keep[blockIdx.x / blocks_per_group] == 0) { out.radius[i] = 0; return; }
    DirectSrc<kDeg> src(sc, i);
    preprocess_point<kDeg>(cam, src, out);
}

// All views of a batch in one pass over the points (App. D.1: view-by-view preprocessing reads the cloud once per
// view, O(batch x points)). A thread takes its point through every view and reads each parameter at most once; the
// per-view arithmetic is preprocess_point, so each view's splat state is what k_preprocess writes for it.
// keep: [views][groups] flags of the group test, or null.
template <int kDeg>
__global__ __launch_bounds__(256) void k_preprocess_batch(SceneDev sc, BatchCams cams, BatchSplats outs,
                                                          const uint8_t* __restrict__ keep, int blocks_per_group, int n_groups)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= sc.n) return;
    const int g = blockIdx.x / blocks_per_group;
    CachedSrc<kDeg> src(sc, i);
    for (int v = 0; v < cams.count; ++v) {
        if (keep != nullptr && keep[(size_t)v * n_groups + g] == 0) { outs.view[v].radius[i] = 0; continue; }
        preprocess_point<kDeg>(cams.cam[v], src, outs.view[v]);
    }
}

// dL/d(splat state) of one point in one view
struct SplatGradIn {
    float mean2d[2], conic[3], opacity, color[3];
    __device__ __forceinline__ void load(const SplatGradDev& g2, int i, size_t N)
    {
        mean2d[0] = g2.mean2d[i]; mean2d[1] = g2.mean2d[N + i];
        conic[0] = g2.conic[i]; conic[1] = g2.conic[N + i]; conic[2] = g2.conic[2 * N + i];
        opacity = g2.opacity[i];
        color[0] = g2.color[i]; color[1] = g2.color[N + i]; color[2] = g2.color[2 * N + i];
    }
    // from the nine sums in the record's order
    __device__ __forceinline__ void from_values(const float (&v)[9])
    {
        mean2d[0] = v[0]; mean2d[1] = v[1];
        conic[0] = v[2]; conic[1] = v[3]; conic[2] = v[4];
        opacity = v[5];
        color[0] = v[6]; color[1] = v[7]; color[2] = v[8];
    }
    // from the 48-byte per-point record the gather of the compositing backward leaves in the workspace
    __device__ __forceinline__ void load_record(const float4* __restrict__ rec, int i)
    {
        const float4 a = rec[(size_t)3 * i], b = rec[(size_t)3 * i + 1], c = rec[(size_t)3 * i + 2];
        mean2d[0] = a.x; mean2d[1] = a.y;
        conic[0] = a.z; conic[1] = a.w; conic[2] = b.x;
        opacity = b.y;
        color[0] = b.z; color[1] = b.w; color[2] = c.x;
    }
};

// Where the parameter gradients of a point go. MemSink puts each value into the caller's buffer as it is produced
// (one view per launch): "+=" (Alg. 1 lines 22-24), or a plain store for the first view of a batch, which folds the
// zero-initialisation of line 21 into it. RegSink adds the views of a batch up in registers first.
template <int kDeg, bool kFirst>
struct MemSink {
    const SceneGradDev& g;
    int i;
    size_t N;
    static constexpr bool kSkipZeroChannel = !kFirst;     // adding zeros to sixteen planes is sixteen wasted updates
    __device__ __forceinline__ void logit(float v) { grad_out<kFirst>(&g.logit[i], v); }
    __device__ __forceinline__ void sh(int j, float v) { grad_out<kFirst>(&g.sh[(size_t)j * N + i], v); }
    __device__ __forceinline__ void mean(int k, float v) { grad_out<kFirst>(&g.mean[(size_t)k * N + i], v); }
    __device__ __forceinline__ void log_scale(int k, float v) { grad_out<kFirst>(&g.log_scale[(size_t)k * N + i], v); }
    __device__ __forceinline__ void quat(int k, float v) { grad_out<kFirst>(&g.quat[(size_t)k * N + i], v); }
};

template <int kDeg>
struct RegSink {
    static constexpr int K3 = 3 * (kDeg + 1) * (kDeg + 1);
    static constexpr bool kSkipZeroChannel = true;
    float a_logit, a_sh[K3], a_mean[3], a_ls[3], a_quat[4];
    __device__ __forceinline__ RegSink()
    {
        a_logit = 0.f;
#pragma unroll
        for (int j = 0; j < K3; ++j) a_sh[j] = 0.f;
#pragma unroll
        for (int k = 0; k < 3; ++k) { a_mean[k] = 0.f; a_ls[k] = 0.f; }
#pragma unroll
        for (int k = 0; k < 4; ++k) a_quat[k] = 0.f;
    }
    __device__ __forceinline__ void logit(float v) { a_logit += v; }
    __device__ __forceinline__ void sh(int j, float v) { a_sh[j] += v; }
    __device__ __forceinline__ void mean(int k, float v) { a_mean[k] += v; }
    __device__ __forceinline__ void log_scale(int k, float v) { a_ls[k] += v; }
    __device__ __forceinline__ void quat(int k, float v) { a_quat[k] += v; }
};

// Derivative of preprocess_point for a point that the view uses (radius > 0): dL/d(splat state) -> dL/d(parameters).
// src must hold shape and appearance.
template <int kDeg, class Src, class Sink>
__device__ __forceinline__ void preprocess_point_bwd(const CamDev& cam, const Src& src, const SplatGradIn& in, Sink& sink)
{
    const float m0 = src.m[0], m1 = src.m[1], m2 = src.m[2];
    Proj P;
    P.px = cam.R[0] * m0 + cam.R[1] * m1 + cam.R[2] * m2 + cam.t[0];
    P.py = cam.R[3] * m0 + cam.R[4] * m1 + cam.R[5] * m2 + cam.t[1];
    P.pz = cam.R[6] * m0 + cam.R[7] * m1 + cam.R[8] * m2 + cam.t[2];
    project_cov(cam, src.ls, src.qr, P);
    const float idet = 1.0f / P.det;
    const float qa = P.c * idet, qb = -P.b * idet, qc = P.a * idet;

    // ---- opacity
    {
        const float o = 1.0f / (1.0f + expf(-src.logit()));
        sink.logit(in.opacity * o * (1.f - o));
    }
    float dmu0 = 0.f, dmu1 = 0.f, dmu2 = 0.f;
    // ---- colour: SH coefficients and the view direction
    {
        const float vx = m0 - cam.campos[0], vy = m1 - cam.campos[1], vz = m2 - cam.campos[2];
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
            float raw = 0.5f;
            float t0 = 0.f, t1 = 0.f, t2 = 0.f;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const float co = src.sh(3 * k + c);
                raw += Y[k] * co;
                t0 += dY[k][0] * co; t1 += dY[k][1] * co; t2 += dY[k][2] * co;
            }
            const float gc = raw > 0.f ? in.color[c] : 0.f;
            if (!Sink::kSkipZeroChannel || gc != 0.f) {
#pragma unroll
                for (int k = 0; k < K; ++k) sink.sh(3 * k + c, Y[k] * gc);
            }
            gd0 += gc * t0; gd1 += gc * t1; gd2 += gc * t2;
        }
        const float dot = gd0 * dx + gd1 * dy + gd2 * dz;
        dmu0 += (gd0 - dx * dot) * vinv; dmu1 += (gd1 - dy * dot) * vinv; dmu2 += (gd2 - dz * dot) * vinv;
    }
    // ---- conic -> cov2d:  G = -Q G_Q Q with G_Q = [[ga, gb/2],[gb/2, gc]]
    float G00, G01, G11;
    {
        const float ga = in.conic[0], gb = 0.5f * in.conic[1], gc = in.conic[2];
        const float u00 = qa * ga + qb * gb, u01 = qa * gb + qb * gc;
        const float u10 = qb * ga + qc * gb, u11 = qb * gb + qc * gc;
        G00 = -(u00 * qa + u01 * qb);
        G01 = -(u00 * qb + u01 * qc);
        G11 = -(u10 * qb + u11 * qc);
    }
    // ---- cov2d = T T^T:  G_T = 2 G T
    float GT[6];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        GT[j] = 2.f * (G00 * P.T[j] + G01 * P.T[3 + j]);
        GT[3 + j] = 2.f * (G01 * P.T[j] + G11 * P.T[3 + j]);
    }
    // ---- T = J A
    const float GJ00 = GT[0] * P.A[0] + GT[1] * P.A[1] + GT[2] * P.A[2];
    const float GJ02 = GT[0] * P.A[6] + GT[1] * P.A[7] + GT[2] * P.A[8];
    const float GJ11 = GT[3] * P.A[3] + GT[4] * P.A[4] + GT[5] * P.A[5];
    const float GJ12 = GT[3] * P.A[6] + GT[4] * P.A[7] + GT[5] * P.A[8];
    float GA[9];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        GA[j] = P.J00 * GT[j];
        GA[3 + j] = P.J11 * GT[3 + j];
        GA[6 + j] = P.J02 * GT[j] + P.J12 * GT[3 + j];
    }
    // ---- J and mean2d as functions of the camera-space position
    float dp0, dp1, dp2;
    {
        const float iz = P.iz, iz2 = iz * iz;
        const float gmx = in.mean2d[0], gmy = in.mean2d[1];
        const float gtx = -cam.fx * iz * GJ02, gty = -cam.fy * iz * GJ12;
        dp2 = (-cam.fx * GJ00 + cam.fx * P.tx * GJ02 - cam.fy * GJ11 + cam.fy * P.ty * GJ12) * iz2;
        dp0 = gmx * cam.fx * iz; dp1 = gmy * cam.fy * iz;
        dp2 -= (gmx * cam.fx * P.px + gmy * cam.fy * P.py) * iz2;
        if (P.tx_free) { dp0 += gtx * iz; dp2 -= gtx * P.px * iz2; }
        if (P.ty_free) { dp1 += gty * iz; dp2 -= gty * P.py * iz2; }
    }
    dmu0 += cam.R[0] * dp0 + cam.R[3] * dp1 + cam.R[6] * dp2;
    dmu1 += cam.R[1] * dp0 + cam.R[4] * dp1 + cam.R[7] * dp2;
    dmu2 += cam.R[2] * dp0 + cam.R[5] * dp1 + cam.R[8] * dp2;
    sink.mean(0, dmu0); sink.mean(1, dmu1); sink.mean(2, dmu2);
    // ---- A = R_cam W, W = Rq diag(s)
    float GRq[9];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        float gs = 0.f;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const float gw = cam.R[r] * GA[j] + cam.R[3 + r] * GA[3 + j] + cam.R[6 + r] * GA[6 + j];
            gs += gw * P.Rq[3 * r + j];
            GRq[3 * r + j] = gw * P.s[j];
        }
        sink.log_scale(j, gs * P.s[j]);
    }
    // ---- Rq as a function of the unit quaternion, then the normalisation
    {
        const float w = P.q[0], x = P.q[1], y = P.q[2], z = P.q[3];
        const float* G = GRq;
        float gq[4];
        gq[0] = 2.f * (-z * G[1] + y * G[2] + z * G[3] - x * G[5] - y * G[6] + x * G[7]);
        gq[1] = 2.f * (y * G[1] + z * G[2] + y * G[3] - 2.f * x * G[4] - w * G[5] + z * G[6] + w * G[7] - 2.f * x * G[8]);
        gq[2] = 2.f * (-2.f * y * G[0] + x * G[1] + w * G[2] + x * G[3] + z * G[5] - w * G[6] + z * G[7] - 2.f * y * G[8]);
        gq[3] = 2.f * (-2.f * z * G[0] - w * G[1] + x * G[2] + w * G[3] - 2.f * z * G[4] + y * G[5] + x * G[6] + y * G[7]);
        const float dot = gq[0] * w + gq[1] * x + gq[2] * y + gq[3] * z;
#pragma unroll
        for (int k = 0; k < 4; ++k) sink.quat(k, (gq[k] - P.q[k] * dot) * P.qinv);
    }
}

// zeros for a point no view of the batch uses, when the buffer is written rather than added to. Non-temporal: nobody
// reads these zeros back within the step, and kept out of the caches they leave the scene parameters there for the
// next view's forward kernel (measured: 8 us per step at 1M points; the same on the non-zero entries was slower).
template <int kDeg>
__device__ __forceinline__ void zero_point_grads(const SceneGradDev& g, int i, size_t N)
{
    constexpr int K0 = (kDeg + 1) * (kDeg + 1);
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        __builtin_nontemporal_store(0.f, &g.mean[(size_t)k * N + i]);
        __builtin_nontemporal_store(0.f, &g.log_scale[(size_t)k * N + i]);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) __builtin_nontemporal_store(0.f, &g.quat[(size_t)k * N + i]);
    __builtin_nontemporal_store(0.f, &g.logit[i]);
#pragma unroll
    for (int k = 0; k < 3 * K0; ++k) __builtin_nontemporal_store(0.f, &g.sh[(size_t)k * N + i]);
}

// kFirst: the first view of a batch. The gradient buffer is then written, not added to, and points this view does not
// use get zeros, so the caller need not clear the buffer beforehand.
// kFromRecords: the splat-state gradient comes straight from the per-point records of the compositing backward
// (`rec`), and the points to work on are those binning listed (`used` = tiles touched); otherwise from the planes of
// g2, for the points with radius > 0 (`used` = radius).
template <int kDeg, bool kFirst, bool kFromRecords>
__global__ __launch_bounds__(256) void k_preprocess_bwd(SceneDev sc, CamDev cam, const int32_t* __restrict__ used,
                                                        SplatGradDev g2, const float4* __restrict__ rec, CarryFold cf, SceneGradDev g)
{
    const int n = sc.n;
    const int i = blockIdx.x * 256 + threadIdx.x;
    // (with cf.carry this launch stands in for k_gather_fixup: it also closes the backward call's epoch)
    if (kFromRecords && cf.carry != nullptr && i == 0) close_backward_epoch(cf.status);
    if (i >= n) return;
    const size_t N = (size_t)n;
    if (used[i] <= 0) {
        if (kFirst) zero_point_grads<kDeg>(g, i, N);
        return;
    }
    DirectSrc<kDeg> src(sc, i);
    src.need_shape();
    SplatGradIn in;
    if (kFromRecords) {
        in.load_record(rec, i);
        if (cf.carry != nullptr) {      // a point whose pairs are cut by a wavefront boundary of the gather: its record is still in pieces
            float v[9];
            if (record_from_carries<9>(cf, cf.slot_base[i], (uint32_t)used[i], v)) in.from_values(v);
        }
    } else {
        in.load(g2, i, N);
    }
    MemSink<kDeg, kFirst> sink{g, i, N};
    preprocess_point_bwd<kDeg>(cam, src, in, sink);
}

// The views of a batch in one pass over the points (Alg. 1 lines 21-24: the gradients of the batch's views are summed
// into one buffer). A thread reads its point's parameters once, runs the per-view derivative for every view that uses
// the point, adds the results up in registers in view order and touches the gradient buffer once: a store (kFirst) or
// one "+=". View by view the same work reads the parameters and reads and writes the 236-byte gradient row once per
// view.
template <int kDeg, bool kFirst>
__global__ __launch_bounds__(256) void k_preprocess_bwd_batch(SceneDev sc, BatchCams cams, BatchSplatGrads in_all, SceneGradDev g)
{
    const int n = sc.n;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const size_t N = (size_t)n;
    uint32_t used = 0u;
    for (int v = 0; v < cams.count; ++v) used |= (in_all.radius[v][i] > 0 ? 1u : 0u) << v;
    if (used == 0u) {
        if (kFirst) zero_point_grads<kDeg>(g, i, N);
        return;
    }
    CachedSrc<kDeg> src(sc, i);
    src.need_shape();
    src.need_appearance();
    RegSink<kDeg> acc;
    for (int v = 0; v < cams.count; ++v) {
        if (!((used >> v) & 1u)) continue;
        SplatGradIn in;
        in.load(in_all.grad[v], i, N);
        preprocess_point_bwd<kDeg>(cams.cam[v], src, in, acc);
    }
    constexpr int K3 = 3 * (kDeg + 1) * (kDeg + 1);
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        grad_out<kFirst>(&g.mean[(size_t)k * N + i], acc.a_mean[k]);
        grad_out<kFirst>(&g.log_scale[(size_t)k * N + i], acc.a_ls[k]);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) grad_out<kFirst>(&g.quat[(size_t)k * N + i], acc.a_quat[k]);
    grad_out<kFirst>(&g.logit[i], acc.a_logit);
#pragma unroll
    for (int j = 0; j < K3; ++j) grad_out<kFirst>(&g.sh[(size_t)j * N + i], acc.a_sh[j]);
}

// The same, with the optimizer step in the same pass (Alg. 1 lines 21-27 for one batch): the summed gradient of a point
// never leaves the registers; the thread updates the point's 11 + 3K parameters and both Adam moments in place. Points no
// view of the batch uses are left alone (the "selective" Adam of App. E.1: the union of the views' visible points).
template <int kDeg>
__global__ __launch_bounds__(256) void k_preprocess_bwd_batch_adam(SceneDev sc, BatchCams cams, BatchSplatGrads in_all, BatchAdam opt)
{
    const int n = sc.n;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const size_t N = (size_t)n;
    uint32_t used = 0u;
    for (int v = 0; v < cams.count; ++v) used |= (in_all.radius[v][i] > 0 ? 1u : 0u) << v;
    if (used == 0u) return;
    CachedSrc<kDeg> src(sc, i);
    src.need_shape();
    src.need_appearance();
    RegSink<kDeg> acc;
    for (int v = 0; v < cams.count; ++v) {
        if (!((used >> v) & 1u)) continue;
        SplatGradIn in;
        in.load(in_all.grad[v], i, N);
        preprocess_point_bwd<kDeg>(cams.cam[v], src, in, acc);
    }
    constexpr int K3 = 3 * (kDeg + 1) * (kDeg + 1);
    // parameter planes are written through the scene's own pointers
    float* p_mean = const_cast<float*>(sc.mean);
    float* p_ls = const_cast<float*>(sc.log_scale);
    float* p_quat = const_cast<float*>(sc.quat);
    float* p_logit = const_cast<float*>(sc.logit);
    float* p_sh = const_cast<float*>(sc.sh);
    // Entries are taken in runs of up to 16: all moments of a run are asked for before the first is used, so the run
    // costs one memory round trip and not one per entry.
    auto run = [&](int attr, float* param, float* mom1, float* mom2, const float* value, const float* grad, int first, int count) {
        float m[16], v2[16];
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (k < count) { const size_t at = (size_t)(first + k) * N + i; m[k] = mom1[at]; v2[k] = mom2[at]; }
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if (k < count) {
                const size_t at = (size_t)(first + k) * N + i;
                float p = value[first + k];
                adam_one(opt.attr[attr], p, grad[first + k], m[k], v2[k]);
                param[at] = p; mom1[at] = m[k]; mom2[at] = v2[k];
            }
    };
    run(0, p_mean, opt.m_mean, opt.v_mean, src.m, acc.a_mean, 0, 3);
    run(1, p_ls, opt.m_log_scale, opt.v_log_scale, src.ls, acc.a_ls, 0, 3);
    run(2, p_quat, opt.m_quat, opt.v_quat, src.qr, acc.a_quat, 0, 4);
    run(3, p_logit, opt.m_logit, opt.v_logit, &src.lg, &acc.a_logit, 0, 1);
#pragma unroll
    for (int j0 = 0; j0 < K3; j0 += 16) run(4, p_sh, opt.m_sh, opt.v_sh, src.shv, acc.a_sh, j0, (K3 - j0 < 16) ? K3 - j0 : 16);
}


hipError_t launch_preprocess(const SceneDev& sc, const CamDev& cam, const SplatsDev& out, const uint8_t* keep,
                             int group_size, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    const int bpg = keep ? group_size / 256 : 1;
    ProfScope prof(kKPreprocess, s);
    switch (sc.sh_degree) {
        case 0: hipLaunchKernelGGL(k_preprocess<0>, dim3(blocks), dim3(256), 0, s, sc, cam, out, keep, bpg); break;
        case 1: hipLaunchKernelGGL(k_preprocess<1>, dim3(blocks), dim3(256), 0, s, sc, cam, out, keep, bpg); break;
        case 2: hipLaunchKernelGGL(k_preprocess<2>, dim3(blocks), dim3(256), 0, s, sc, cam, out, keep, bpg); break;
        default: hipLaunchKernelGGL(k_preprocess<3>, dim3(blocks), dim3(256), 0, s, sc, cam, out, keep, bpg); break;
    }
    return hipGetLastError();
}

template <bool kFirst, bool kFromRecords>
static void launch_preprocess_bwd_t(const SceneDev& sc, const CamDev& cam, const int32_t* used, const SplatGradDev& g2,
                                    const float4* rec, const CarryFold& cf, const SceneGradDev& g, unsigned blocks, hipStream_t s)
{
    switch (sc.sh_degree) {
        case 0: hipLaunchKernelGGL((k_preprocess_bwd<0, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, g2, rec, cf, g); break;
        case 1: hipLaunchKernelGGL((k_preprocess_bwd<1, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, g2, rec, cf, g); break;
        case 2: hipLaunchKernelGGL((k_preprocess_bwd<2, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, g2, rec, cf, g); break;
        default: hipLaunchKernelGGL((k_preprocess_bwd<3, kFirst, kFromRecords>), dim3(blocks), dim3(256), 0, s, sc, cam, used, g2, rec, cf, g); break;
    }
}

hipError_t launch_preprocess_bwd(const SceneDev& sc, const CamDev& cam, const int32_t* radius, const SplatGradDev& g2,
                                 const SceneGradDev& g, bool first_view, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    ProfScope prof(kKPreprocessBwd, s);
    const CarryFold none{nullptr, nullptr, nullptr, 0u};
    if (first_view) launch_preprocess_bwd_t<true, false>(sc, cam, radius, g2, nullptr, none, g, blocks, s);
    else launch_preprocess_bwd_t<false, false>(sc, cam, radius, g2, nullptr, none, g, blocks, s);
    return hipGetLastError();
}

// the same from the per-point gradient records in the workspace (see k_preprocess_bwd)
hipError_t launch_preprocess_bwd_records(const SceneDev& sc, const CamDev& cam, const uint32_t* tiles_touched, const float4* rec,
                                         const CarryFold& cf, const SceneGradDev& g, bool first_view, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    const int32_t* used = reinterpret_cast<const int32_t*>(tiles_touched);     // counts are far below 2^31
    const SplatGradDev none{nullptr, nullptr, nullptr, nullptr};
    ProfScope prof(kKPreprocessBwd, s);
    if (first_view) launch_preprocess_bwd_t<true, true>(sc, cam, used, none, rec, cf, g, blocks, s);
    else launch_preprocess_bwd_t<false, true>(sc, cam, used, none, rec, cf, g, blocks, s);
    return hipGetLastError();
}

hipError_t launch_preprocess_batch(const SceneDev& sc, const BatchCams& cams, const BatchSplats& outs, const uint8_t* keep,
                                   int group_size, hipStream_t s)
{
    if (sc.n == 0 || cams.count == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    const int bpg = keep ? group_size / 256 : 1;
    const int ng = keep ? (sc.n + group_size - 1) / group_size : 0;
    ProfScope prof(kKPreprocess, s);
    switch (sc.sh_degree) {
        case 0: hipLaunchKernelGGL(k_preprocess_batch<0>, dim3(blocks), dim3(256), 0, s, sc, cams, outs, keep, bpg, ng); break;
        case 1: hipLaunchKernelGGL(k_preprocess_batch<1>, dim3(blocks), dim3(256), 0, s, sc, cams, outs, keep, bpg, ng); break;
        case 2: hipLaunchKernelGGL(k_preprocess_batch<2>, dim3(blocks), dim3(256), 0, s, sc, cams, outs, keep, bpg, ng); break;
        default: hipLaunchKernelGGL(k_preprocess_batch<3>, dim3(blocks), dim3(256), 0, s, sc, cams, outs, keep, bpg, ng); break;
    }
    return hipGetLastError();
}

template <bool kFirst>
static void launch_preprocess_bwd_batch_t(const SceneDev& sc, const BatchCams& cams, const BatchSplatGrads& in, const SceneGradDev& g,
                                          unsigned blocks, hipStream_t s)
{
    switch (sc.sh_degree) {
        case 0: hipLaunchKernelGGL((k_preprocess_bwd_batch<0, kFirst>), dim3(blocks), dim3(256), 0, s, sc, cams, in, g); break;
        case 1: hipLaunchKernelGGL((k_preprocess_bwd_batch<1, kFirst>), dim3(blocks), dim3(256), 0, s, sc, cams, in, g); break;
        case 2: hipLaunchKernelGGL((k_preprocess_bwd_batch<2, kFirst>), dim3(blocks), dim3(256), 0, s, sc, cams, in, g); break;
        default: hipLaunchKernelGGL((k_preprocess_bwd_batch<3, kFirst>), dim3(blocks), dim3(256), 0, s, sc, cams, in, g); break;
    }
}

hipError_t launch_preprocess_bwd_batch(const SceneDev& sc, const BatchCams& cams, const BatchSplatGrads& in, const SceneGradDev& g,
                                       bool first_view, hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    ProfScope prof(kKPreprocessBwd, s);
    if (first_view) launch_preprocess_bwd_batch_t<true>(sc, cams, in, g, blocks, s);
    else launch_preprocess_bwd_batch_t<false>(sc, cams, in, g, blocks, s);
    return hipGetLastError();
}

hipError_t launch_preprocess_bwd_batch_adam(const SceneDev& sc, const BatchCams& cams, const BatchSplatGrads& in, const BatchAdam& opt,
                                            hipStream_t s)
{
    if (sc.n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((sc.n + 255) / 256);
    ProfScope prof(kKPreprocessBwd, s);
    switch (sc.sh_degree) {
        case 0: hipLaunchKernelGGL(k_preprocess_bwd_batch_adam<0>, dim3(blocks), dim3(256), 0, s, sc, cams, in, opt); break;
        case 1: hipLaunchKernelGGL(k_preprocess_bwd_batch_adam<1>, dim3(blocks), dim3(256), 0, s, sc, cams, in, opt); break;
        case 2: hipLaunchKernelGGL(k_preprocess_bwd_batch_adam<2>, dim3(blocks), dim3(256), 0, s, sc, cams, in, opt); break;
        default: hipLaunchKernelGGL(k_preprocess_bwd_batch_adam<3>, dim3(blocks), dim3(256), 0, s, sc, cams, in, opt); break;
    }
    return hipGetLastError();
}

}  // namespace pbdr
