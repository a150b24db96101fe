/*
 * pbdr_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, double-precision CPU implementation of the per-view hot path
 * of point-based differentiable rendering with 3D Gaussians: cull, project to a
 * 2D splat, sort splats by distance to the camera plane, blend front to back per
 * pixel until (near) full opacity, and the derivative of all that (paper Sec. 2.1,
 * "PBDR models and their rendering"; Sec. 3.1 pts_culling / pts_splatting /
 * image_render; Sec. 3.2 "3DGS"; Alg. 1 compute lines; Table 3a splat state).
 *
 * It shares no code, header, table or constant generator with the HIP library.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * The paper delegates the rasterizer's numerics to its rendering kernels and
 * states only the pipeline. The numeric rules used here (the readings) are:
 *   - learnable parameters are raw: scale = exp(log_scale), rotation =
 *     normalised quaternion (w,x,y,z), opacity = sigmoid(logit);
 *   - depth is the camera-space z ("distance to the camera plane", Sec. 2.1);
 *   - "affine approximation of perspective projection" (App. B): first-order
 *     (Jacobian) push-forward of the 3D covariance, with the ray slope clamped
 *     to 1.3x the half field of view, plus a 0.3 px^2 screen-space blur;
 *   - extent = ceil(3 sigma_max); a splat touches the 16x16 tiles of the
 *     bounding square of that extent; the splat is *restricted* to those tiles;
 *   - colour = max(0, 0.5 + sum_k Y_k(dir) sh_k), real spherical harmonics up
 *     to degree 3;
 *   - blending: alpha = min(0.99, o exp(-sigma)); alpha < 1/255 is skipped; the
 *     splat that would take transmittance below 1e-4 is not blended and ends
 *     the pixel; image = C + T bg;
 *   - ties in depth are broken by ascending point index;
 *   - the backward pass is the exact derivative with every discrete decision
 *     (cull, extent, skip, stop, order, clamps) frozen.
 *
 * Layouts follow the paper's "S x l" tensors: mean[n][3], log_scale[n][3],
 * quat[n][4], logit[n], sh[n][K][3] with K=(deg+1)^2; splat state per Table 3a:
 * mean2d[n][2], conic[n][3], opacity[n], color[n][3], radius[n], depth[n].
 * Images are [H][W][3].
 *
 * parity pins: see tests/test_oracle_*.py (closed forms, rule scenes, white
 * furnace, finite differences, brute-force binning, SH quadrature, rigid-motion
 * invariance, projection-Jacobian push-forward, permutation invariance).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_TILE 16
#define ORC_BLUR 0.3
#define ORC_ALPHA_MAX 0.99
#define ORC_ALPHA_MIN (1.0 / 255.0)
#define ORC_T_STOP 1e-4
#define ORC_GUARD 1.3
#define ORC_EIG_FLOOR 0.1
#define ORC_RADIUS_MAX (1 << 20)    /* overflow guard only */
#define ORC_PIX_MAX 1073741824.0    /* overflow guard only: |floor(mean2d)| <= 2^30 */

/* fragile-pixel flags (a knife-edge decision lies within rounding of fp32) */
#define ORC_FRAG_ALPHA_MIN 1
#define ORC_FRAG_T_STOP 2
#define ORC_FRAG_SIGMA 4
#define ORC_FRAG_ALPHA_MAX 8

typedef struct {
    int32_t width, height;
    double fx, fy, cx, cy;
    double R[9]; /* world -> camera, row-major; +x right, +y down, +z forward */
    double t[3];
    double near_plane, far_plane, radius_clip;
} orc_camera;

/* ------------------------------------------------------------------ */
/* Real spherical harmonics, degree <= 3, index k = l*l + l + m.       */
/* Y[k] as polynomials in the unit direction (x,y,z); dY[k][a] are the */
/* partial derivatives of those polynomials w.r.t. (x,y,z).            */
/* ------------------------------------------------------------------ */
static void sh_eval(int deg, const double d[3], double Y[16], double dY[16][3])
{
    const double pi = 3.14159265358979323846;
    const double x = d[0], y = d[1], z = d[2];
    const double c0 = sqrt(1.0 / (4.0 * pi));
    const double c1 = sqrt(3.0 / (4.0 * pi));
    const double c2a = sqrt(15.0 / (4.0 * pi));
    const double c2b = sqrt(5.0 / (16.0 * pi));
    const double c2c = sqrt(15.0 / (16.0 * pi));
    const double c3a = sqrt(35.0 / (32.0 * pi));
    const double c3b = sqrt(105.0 / (4.0 * pi));
    const double c3c = sqrt(21.0 / (32.0 * pi));
    const double c3d = sqrt(7.0 / (16.0 * pi));
    const double c3e = sqrt(105.0 / (16.0 * pi));
    int k;
    for (k = 0; k < 16; ++k) { Y[k] = 0.0; dY[k][0] = dY[k][1] = dY[k][2] = 0.0; }
    Y[0] = c0;
    if (deg < 1) return;
    Y[1] = -c1 * y;  dY[1][1] = -c1;
    Y[2] =  c1 * z;  dY[2][2] =  c1;
    Y[3] = -c1 * x;  dY[3][0] = -c1;
    if (deg < 2) return;
    Y[4] =  c2a * x * y;  dY[4][0] =  c2a * y;  dY[4][1] =  c2a * x;
    Y[5] = -c2a * y * z;  dY[5][1] = -c2a * z;  dY[5][2] = -c2a * y;
    Y[6] =  c2b * (2.0 * z * z - x * x - y * y);
    dY[6][0] = -2.0 * c2b * x;  dY[6][1] = -2.0 * c2b * y;  dY[6][2] = 4.0 * c2b * z;
    Y[7] = -c2a * x * z;  dY[7][0] = -c2a * z;  dY[7][2] = -c2a * x;
    Y[8] =  c2c * (x * x - y * y);  dY[8][0] = 2.0 * c2c * x;  dY[8][1] = -2.0 * c2c * y;
    if (deg < 3) return;
    Y[9]  = -c3a * y * (3.0 * x * x - y * y);
    dY[9][0] = -c3a * 6.0 * x * y;  dY[9][1] = -c3a * (3.0 * x * x - 3.0 * y * y);
    Y[10] =  c3b * x * y * z;
    dY[10][0] = c3b * y * z;  dY[10][1] = c3b * x * z;  dY[10][2] = c3b * x * y;
    Y[11] = -c3c * y * (4.0 * z * z - x * x - y * y);
    dY[11][0] = c3c * 2.0 * x * y;
    dY[11][1] = -c3c * (4.0 * z * z - x * x - 3.0 * y * y);
    dY[11][2] = -c3c * 8.0 * y * z;
    Y[12] =  c3d * z * (2.0 * z * z - 3.0 * x * x - 3.0 * y * y);
    dY[12][0] = -c3d * 6.0 * x * z;  dY[12][1] = -c3d * 6.0 * y * z;
    dY[12][2] = c3d * (6.0 * z * z - 3.0 * x * x - 3.0 * y * y);
    Y[13] = -c3c * x * (4.0 * z * z - x * x - y * y);
    dY[13][0] = -c3c * (4.0 * z * z - 3.0 * x * x - y * y);
    dY[13][1] = c3c * 2.0 * x * y;
    dY[13][2] = -c3c * 8.0 * x * z;
    Y[14] =  c3e * z * (x * x - y * y);
    dY[14][0] = c3e * 2.0 * x * z;  dY[14][1] = -c3e * 2.0 * y * z;  dY[14][2] = c3e * (x * x - y * y);
    Y[15] = -c3a * x * (x * x - 3.0 * y * y);
    dY[15][0] = -c3a * (3.0 * x * x - 3.0 * y * y);  dY[15][1] = c3a * 6.0 * x * y;
}

/* exported for the quadrature / library pin */
void orc_sh_basis(int deg, const double dir[3], double Y[16])
{
    double dY[16][3];
    sh_eval(deg, dir, Y, dY);
}

/* ------------------------------------------------------------------ */
/* Tile rectangle of a splat: the 16x16 tiles met by the square of     */
/* half-side `radius` around mean2d, clamped to the tile grid.         */
/* floor((m - r)/16) is evaluated as floordiv(floor(m) - r, 16), which */
/* is the same number because r and 16 are integers.                   */
/* rect = {x0, y0, x1, y1}, upper bounds exclusive.                    */
/* ------------------------------------------------------------------ */
static int64_t floordiv16(int64_t v) { return (v >= 0) ? v / 16 : -((-v + 15) / 16); }
static int64_t clampi(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

void orc_tile_rect(double mx, double my, int radius, int width, int height, int32_t rect[4])
{
    const int64_t TX = (width + ORC_TILE - 1) / ORC_TILE, TY = (height + ORC_TILE - 1) / ORC_TILE;
    double fmx = floor(mx), fmy = floor(my);
    if (fmx > ORC_PIX_MAX) fmx = ORC_PIX_MAX;
    if (fmx < -ORC_PIX_MAX) fmx = -ORC_PIX_MAX;
    if (fmy > ORC_PIX_MAX) fmy = ORC_PIX_MAX;
    if (fmy < -ORC_PIX_MAX) fmy = -ORC_PIX_MAX;
    {
        const int64_t ix = (int64_t)fmx, iy = (int64_t)fmy, r = radius;
        rect[0] = (int32_t)clampi(floordiv16(ix - r), 0, TX);
        rect[1] = (int32_t)clampi(floordiv16(iy - r), 0, TY);
        rect[2] = (int32_t)clampi(floordiv16(ix + r + 15), 0, TX);
        rect[3] = (int32_t)clampi(floordiv16(iy + r + 15), 0, TY);
    }
}

/* ------------------------------------------------------------------ */
/* Projection of one point, keeping every intermediate (used by the    */
/* forward and by its derivative).                                     */
/* ------------------------------------------------------------------ */
typedef struct {
    int visible;
    double s[3], qn[4], qlen, o;
    double Rq[9];
    double p[3];
    double Sigma[9];
    double lim_x, lim_y, tx, ty;
    int tx_clamped, ty_clamped;
    double J[6], M[6];
    double a, b, c, det; /* 2D covariance incl. blur */
    double conic[3];
    double mean2d[2];
    double extent; /* 3 sqrt(lambda_max) before ceil */
    int radius;
    int32_t rect[4];
    double v[3], vlen, dir[3];
    double Y[16], dY[16][3];
    double rgb_raw[3], rgb[3];
} orc_proj;

static void quat_to_rot(const double q[4], double R[9])
{
    const double w = q[0], x = q[1], y = q[2], z = q[3];
    R[0] = 1.0 - 2.0 * (y * y + z * z); R[1] = 2.0 * (x * y - w * z);       R[2] = 2.0 * (x * z + w * y);
    R[3] = 2.0 * (x * y + w * z);       R[4] = 1.0 - 2.0 * (x * x + z * z); R[5] = 2.0 * (y * z - w * x);
    R[6] = 2.0 * (x * z - w * y);       R[7] = 2.0 * (y * z + w * x);       R[8] = 1.0 - 2.0 * (x * x + y * y);
}

static void project_one(int sh_degree, const double mean[3], const double log_scale[3], const double quat[4],
                        double logit, const double* sh /* [K][3] */, const orc_camera* cam, orc_proj* P)
{
    int i, j, k, c;
    const int K = (sh_degree + 1) * (sh_degree + 1);
    memset(P, 0, sizeof(*P));
    /* activations */
    for (i = 0; i < 3; ++i) P->s[i] = exp(log_scale[i]);
    P->qlen = sqrt(quat[0] * quat[0] + quat[1] * quat[1] + quat[2] * quat[2] + quat[3] * quat[3]);
    for (i = 0; i < 4; ++i) P->qn[i] = quat[i] / P->qlen;
    P->o = 1.0 / (1.0 + exp(-logit));
    quat_to_rot(P->qn, P->Rq);
    /* camera space */
    for (i = 0; i < 3; ++i)
        P->p[i] = cam->R[3 * i] * mean[0] + cam->R[3 * i + 1] * mean[1] + cam->R[3 * i + 2] * mean[2] + cam->t[i];
    if (P->p[2] < cam->near_plane || P->p[2] > cam->far_plane) return;
    /* 3D covariance  Rq diag(s^2) Rq^T */
    for (i = 0; i < 3; ++i)
        for (j = 0; j < 3; ++j) {
            double acc = 0.0;
            for (k = 0; k < 3; ++k) acc += P->Rq[3 * i + k] * P->s[k] * P->s[k] * P->Rq[3 * j + k];
            P->Sigma[3 * i + j] = acc;
        }
    /* Jacobian of the pinhole projection at p, ray slopes clamped to the guard band */
    {
        const double z = P->p[2];
        double tx = P->p[0] / z, ty = P->p[1] / z;
        P->lim_x = ORC_GUARD * (0.5 * cam->width) / cam->fx;
        P->lim_y = ORC_GUARD * (0.5 * cam->height) / cam->fy;
        if (tx > P->lim_x) { tx = P->lim_x; P->tx_clamped = 1; }
        if (tx < -P->lim_x) { tx = -P->lim_x; P->tx_clamped = 1; }
        if (ty > P->lim_y) { ty = P->lim_y; P->ty_clamped = 1; }
        if (ty < -P->lim_y) { ty = -P->lim_y; P->ty_clamped = 1; }
        P->tx = tx; P->ty = ty;
        P->J[0] = cam->fx / z; P->J[1] = 0.0;         P->J[2] = -cam->fx * tx / z;
        P->J[3] = 0.0;         P->J[4] = cam->fy / z; P->J[5] = -cam->fy * ty / z;
    }
    for (i = 0; i < 2; ++i)
        for (j = 0; j < 3; ++j) {
            double acc = 0.0;
            for (k = 0; k < 3; ++k) acc += P->J[3 * i + k] * cam->R[3 * k + j];
            P->M[3 * i + j] = acc;
        }
    {
        double S2[4];
        for (i = 0; i < 2; ++i)
            for (j = 0; j < 2; ++j) {
                double acc = 0.0;
                int l;
                for (k = 0; k < 3; ++k)
                    for (l = 0; l < 3; ++l) acc += P->M[3 * i + k] * P->Sigma[3 * k + l] * P->M[3 * j + l];
                S2[2 * i + j] = acc;
            }
        P->a = S2[0] + ORC_BLUR; P->b = 0.5 * (S2[1] + S2[2]); P->c = S2[3] + ORC_BLUR;
    }
    P->det = P->a * P->c - P->b * P->b;
    if (!(P->det > 0.0)) return;
    P->conic[0] = P->c / P->det; P->conic[1] = -P->b / P->det; P->conic[2] = P->a / P->det;
    P->mean2d[0] = cam->fx * P->p[0] / P->p[2] + cam->cx;
    P->mean2d[1] = cam->fy * P->p[1] / P->p[2] + cam->cy;
    {
        const double m = 0.5 * (P->a + P->c);
        double disc = m * m - P->det, r;
        if (disc < ORC_EIG_FLOOR) disc = ORC_EIG_FLOOR;
        P->extent = 3.0 * sqrt(m + sqrt(disc));
        r = ceil(P->extent);
        if (!(r < (double)ORC_RADIUS_MAX)) r = (double)ORC_RADIUS_MAX;
        P->radius = (int)r;
    }
    if ((double)P->radius <= cam->radius_clip) { P->radius = 0; return; }
    orc_tile_rect(P->mean2d[0], P->mean2d[1], P->radius, cam->width, cam->height, P->rect);
    if ((P->rect[2] - P->rect[0]) * (P->rect[3] - P->rect[1]) <= 0) { P->radius = 0; return; }
    /* view-dependent colour */
    {
        double campos[3];
        for (i = 0; i < 3; ++i)
            campos[i] = -(cam->R[i] * cam->t[0] + cam->R[3 + i] * cam->t[1] + cam->R[6 + i] * cam->t[2]);
        for (i = 0; i < 3; ++i) P->v[i] = mean[i] - campos[i];
        P->vlen = sqrt(P->v[0] * P->v[0] + P->v[1] * P->v[1] + P->v[2] * P->v[2]);
        for (i = 0; i < 3; ++i) P->dir[i] = P->v[i] / P->vlen;
        sh_eval(sh_degree, P->dir, P->Y, P->dY);
        for (c = 0; c < 3; ++c) {
            double acc = 0.5;
            for (k = 0; k < K; ++k) acc += P->Y[k] * sh[3 * k + c];
            P->rgb_raw[c] = acc;
            P->rgb[c] = acc > 0.0 ? acc : 0.0;
        }
    }
    P->visible = 1;
}

/*
 * pts_culling + pts_splatting for one view (Sec. 3.1; Alg. 1's culling and splatting steps): fills the
 * Table 3a state. A culled point gets radius 0 and zeros elsewhere.
 * Optional outputs (may be NULL): rect[n][4]; cov2d[n][3] = (a,b,c) incl. blur;
 * near_tie[n] = 1 where an integer decision (extent ceil, tile rectangle, a cull
 * test) is within `tau` of flipping, so an fp32 evaluation may legitimately differ.
 */
void orc_preprocess(int n, int sh_degree, const double* mean, const double* log_scale, const double* quat,
                    const double* logit, const double* sh, const orc_camera* cam, double* mean2d, double* conic,
                    double* opacity, double* color, int32_t* radius, double* depth, int32_t* rect, double* cov2d,
                    uint8_t* near_tie, double tau)
{
    const int K = (sh_degree + 1) * (sh_degree + 1);
    int i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; ++i) {
        orc_proj P;
        int k;
        project_one(sh_degree, mean + 3 * i, log_scale + 3 * i, quat + 4 * i, logit[i], sh + (size_t)3 * K * i, cam, &P);
        mean2d[2 * i] = mean2d[2 * i + 1] = 0.0;
        conic[3 * i] = conic[3 * i + 1] = conic[3 * i + 2] = 0.0;
        opacity[i] = 0.0; depth[i] = 0.0; radius[i] = 0;
        color[3 * i] = color[3 * i + 1] = color[3 * i + 2] = 0.0;
        if (rect) for (k = 0; k < 4; ++k) rect[4 * i + k] = 0;
        if (cov2d) for (k = 0; k < 3; ++k) cov2d[3 * i + k] = 0.0;
        if (near_tie) {
            /* decisions that an fp32 evaluation could take the other way */
            int flag = 0;
            const double z = P.p[2];
            if (fabs(z - cam->near_plane) < tau * fabs(z) || fabs(z - cam->far_plane) < tau * fabs(z)) flag = 1;
            if (z >= cam->near_plane && z <= cam->far_plane && P.det > 0.0) {
                int32_t ra[4], rb[4];
                int rlo, rhi;
                if (fabs(P.extent - floor(P.extent + 0.5)) < tau * (1.0 + P.extent)) flag = 1;
                rlo = (int)ceil(P.extent * (1.0 - tau) - tau); rhi = (int)ceil(P.extent * (1.0 + tau) + tau);
                if (rlo < 0) rlo = 0;
                if (((double)rlo <= cam->radius_clip) != ((double)rhi <= cam->radius_clip)) flag = 1;
                orc_tile_rect(P.mean2d[0] - tau * (1.0 + fabs(P.mean2d[0])), P.mean2d[1] - tau * (1.0 + fabs(P.mean2d[1])),
                              P.radius > 0 ? P.radius : rhi, cam->width, cam->height, ra);
                orc_tile_rect(P.mean2d[0] + tau * (1.0 + fabs(P.mean2d[0])), P.mean2d[1] + tau * (1.0 + fabs(P.mean2d[1])),
                              P.radius > 0 ? P.radius : rhi, cam->width, cam->height, rb);
                for (k = 0; k < 4; ++k) if (ra[k] != rb[k]) flag = 1;
            }
            near_tie[i] = (uint8_t)flag;
        }
        if (!P.visible) continue;
        mean2d[2 * i] = P.mean2d[0]; mean2d[2 * i + 1] = P.mean2d[1];
        for (k = 0; k < 3; ++k) { conic[3 * i + k] = P.conic[k]; color[3 * i + k] = P.rgb[k]; }
        opacity[i] = P.o; depth[i] = P.p[2]; radius[i] = P.radius;
        if (rect) for (k = 0; k < 4; ++k) rect[4 * i + k] = P.rect[k];
        if (cov2d) { cov2d[3 * i] = P.a; cov2d[3 * i + 1] = P.b; cov2d[3 * i + 2] = P.c; }
    }
}

/* ------------------------------------------------------------------ */
/* Tile lists: duplicate each visible splat into every tile of its     */
/* rectangle, order by (tile, depth as fp32 bit pattern, point index). */
/* ------------------------------------------------------------------ */
typedef struct { uint64_t key; uint32_t id; } orc_pair;

static int pair_cmp(const void* pa, const void* pb)
{
    const orc_pair* a = (const orc_pair*)pa;
    const orc_pair* b = (const orc_pair*)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->id != b->id) return a->id < b->id ? -1 : 1;
    return 0;
}

/* number of (tile, splat) pairs */
uint64_t orc_count_pairs(int n, const double* mean2d, const int32_t* radius, int width, int height)
{
    uint64_t total = 0;
    int i;
    for (i = 0; i < n; ++i) {
        int32_t r[4];
        if (radius[i] <= 0) continue;
        orc_tile_rect(mean2d[2 * i], mean2d[2 * i + 1], radius[i], width, height, r);
        total += (uint64_t)(r[2] - r[0]) * (uint64_t)(r[3] - r[1]);
    }
    return total;
}

/*
 * keys[P], vals[P]: sorted pairs, key = tile_id << 32 | bits(depth_f32), tile_id = ty*TX + tx.
 * ranges[tiles][2]: [start, end) of each tile's run in the sorted list; empty tile = {0,0}.
 * Returns P.
 */
uint64_t orc_bin_sort(int n, const double* mean2d, const int32_t* radius, const float* depth32, int width, int height,
                      uint64_t* keys, uint32_t* vals, uint32_t* ranges)
{
    const int TX = (width + ORC_TILE - 1) / ORC_TILE, TY = (height + ORC_TILE - 1) / ORC_TILE;
    const uint64_t P = orc_count_pairs(n, mean2d, radius, width, height);
    orc_pair* list = (orc_pair*)malloc((P ? P : 1) * sizeof(orc_pair));
    uint64_t w = 0, j;
    int i, tx, ty;
    for (i = 0; i < n; ++i) {
        int32_t r[4];
        uint32_t bits;
        if (radius[i] <= 0) continue;
        orc_tile_rect(mean2d[2 * i], mean2d[2 * i + 1], radius[i], width, height, r);
        memcpy(&bits, &depth32[i], 4);
        for (ty = r[1]; ty < r[3]; ++ty)
            for (tx = r[0]; tx < r[2]; ++tx) {
                list[w].key = ((uint64_t)(uint32_t)(ty * TX + tx) << 32) | bits;
                list[w].id = (uint32_t)i;
                ++w;
            }
    }
    qsort(list, (size_t)P, sizeof(orc_pair), pair_cmp);
    memset(ranges, 0, (size_t)TX * TY * 2 * sizeof(uint32_t));
    for (j = 0; j < P; ++j) {
        const uint32_t tile = (uint32_t)(list[j].key >> 32);
        keys[j] = list[j].key; vals[j] = list[j].id;
        if (j == 0 || (uint32_t)(list[j - 1].key >> 32) != tile) ranges[2 * tile] = (uint32_t)j;
        if (j + 1 == P || (uint32_t)(list[j + 1].key >> 32) != tile) ranges[2 * tile + 1] = (uint32_t)(j + 1);
    }
    free(list);
    return P;
}

/* ------------------------------------------------------------------ */
/* Blending of one pixel over a list of splat indices.                 */
/* Writes the blended splats (position in list, alpha, T before it).   */
/* ------------------------------------------------------------------ */
typedef struct { uint32_t pos; double alpha, T, gauss; int clamped; } orc_hit;

static void blend_pixel(double px, double py, const uint32_t* list, uint32_t len, const double* mean2d,
                        const double* conic, const double* opacity, const double* color, const double bg[3],
                        double rgb_out[3], double* T_out, uint32_t* last_out, uint8_t* fragile_out,
                        uint64_t* n_eval, uint64_t* n_blend, orc_hit* hits, uint32_t* n_hits)
{
    double T = 1.0, C[3] = {0.0, 0.0, 0.0};
    uint32_t last = 0, k, nh = 0;
    uint8_t frag = 0;
    uint64_t ev = 0;
    for (k = 0; k < len; ++k) {
        const uint32_t g = list[k];
        const double dx = px - mean2d[2 * g], dy = py - mean2d[2 * g + 1];
        const double sigma = 0.5 * (conic[3 * g] * dx * dx + conic[3 * g + 2] * dy * dy) + conic[3 * g + 1] * dx * dy;
        double gauss, araw, alpha, Tn;
        ++ev;
        /* the sign decision below is within fp32 rounding of flipping: the error of sigma evaluated in fp32 grows
         * with the size of its three terms, which matters for conics close to degenerate (terms that cancel) */
        if (fabs(sigma) < 1e-6 + 4e-7 * (0.5 * (fabs(conic[3 * g]) * dx * dx + fabs(conic[3 * g + 2]) * dy * dy) +
                                         fabs(conic[3 * g + 1] * dx * dy)))
            frag |= ORC_FRAG_SIGMA;
        if (sigma < 0.0) continue;
        gauss = exp(-sigma);
        araw = opacity[g] * gauss;
        alpha = araw < ORC_ALPHA_MAX ? araw : ORC_ALPHA_MAX;
        if (fabs(araw - ORC_ALPHA_MAX) < 1e-5) frag |= ORC_FRAG_ALPHA_MAX;
        /* the skip decision is within fp32 rounding of flipping. An fp32 evaluation of alpha = o exp(-sigma) carries a
         * relative error of at most about 1e-6 (logarithm of o, exponential, the final product) + 2.5e-7 x the size of
         * sigma's three terms (a few roundings of each); the flag is raised within twice that of the threshold */
        if (fabs(alpha - ORC_ALPHA_MIN) <
            ORC_ALPHA_MIN * (2e-6 + 5e-7 * (0.5 * (fabs(conic[3 * g]) * dx * dx + fabs(conic[3 * g + 2]) * dy * dy) +
                                            fabs(conic[3 * g + 1] * dx * dy))))
            frag |= ORC_FRAG_ALPHA_MIN;
        if (alpha < ORC_ALPHA_MIN) continue;
        Tn = T * (1.0 - alpha);
        if (fabs(Tn - ORC_T_STOP) < 1e-8) frag |= ORC_FRAG_T_STOP;
        if (Tn < ORC_T_STOP) break;
        C[0] += color[3 * g] * alpha * T; C[1] += color[3 * g + 1] * alpha * T; C[2] += color[3 * g + 2] * alpha * T;
        if (hits) { hits[nh].pos = k; hits[nh].alpha = alpha; hits[nh].T = T; hits[nh].gauss = gauss; hits[nh].clamped = !(araw < ORC_ALPHA_MAX); }
        ++nh;
        T = Tn;
        last = k + 1;
    }
    rgb_out[0] = C[0] + T * bg[0]; rgb_out[1] = C[1] + T * bg[1]; rgb_out[2] = C[2] + T * bg[2];
    *T_out = T; *last_out = last;
    if (fragile_out) *fragile_out = frag;
    if (n_eval) *n_eval = ev;
    if (n_blend) *n_blend = nh;
    if (n_hits) *n_hits = nh;
}

/*
 * image_render forward (Sec. 2.1 blending; Sec. 3.1 image_render): per pixel over its
 * tile's sorted list. image[H][W][3], final_T[H][W], last_idx[H][W] = 1-based position
 * in the tile's list of the last blended splat (0 = none). fragile[H][W] optional.
 * counters[0] = list entries examined (summed over pixels), counters[1] = blended pairs.
 */
void orc_render_fwd(int width, int height, const double* mean2d, const double* conic, const double* opacity,
                    const double* color, const uint32_t* vals, const uint32_t* ranges, const double bg[3],
                    double* image, double* final_T, uint32_t* last_idx, uint8_t* fragile, uint64_t* counters)
{
    const int TX = (width + ORC_TILE - 1) / ORC_TILE;
    uint64_t tot_eval = 0, tot_blend = 0;
    int y;
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : tot_eval, tot_blend)
    for (y = 0; y < height; ++y) {
        int x;
        for (x = 0; x < width; ++x) {
            const int tile = (y / ORC_TILE) * TX + (x / ORC_TILE);
            const uint32_t s = ranges[2 * tile], e = ranges[2 * tile + 1];
            const size_t pix = (size_t)y * width + x;
            uint64_t ev, nb;
            blend_pixel(x + 0.5, y + 0.5, vals + s, e - s, mean2d, conic, opacity, color, bg, image + 3 * pix,
                        final_T + pix, last_idx + pix, fragile ? fragile + pix : NULL, &ev, &nb, NULL, NULL);
            tot_eval += ev; tot_blend += nb;
        }
    }
    if (counters) { counters[0] = tot_eval; counters[1] = tot_blend; }
}

/*
 * The definition the tile lists implement, written without tile lists: every pixel walks
 * the single global list `order` (all visible splats by (depth bits, index)) and keeps the
 * splats whose tile rectangle contains the pixel's tile. Slow; for small scenes.
 */
void orc_render_fwd_global(int width, int height, int n_order, const uint32_t* order, const int32_t* rect,
                           const double* mean2d, const double* conic, const double* opacity, const double* color,
                           const double bg[3], double* image, double* final_T)
{
    uint32_t* mine = (uint32_t*)malloc((size_t)(n_order ? n_order : 1) * sizeof(uint32_t));
    int x, y, k;
    for (y = 0; y < height; ++y)
        for (x = 0; x < width; ++x) {
            const int tx = x / ORC_TILE, ty = y / ORC_TILE;
            const size_t pix = (size_t)y * width + x;
            uint32_t len = 0, last;
            for (k = 0; k < n_order; ++k) {
                const int32_t* r = rect + 4 * order[k];
                if (tx >= r[0] && tx < r[2] && ty >= r[1] && ty < r[3]) mine[len++] = order[k];
            }
            blend_pixel(x + 0.5, y + 0.5, mine, len, mean2d, conic, opacity, color, bg, image + 3 * pix, final_T + pix,
                        &last, NULL, NULL, NULL, NULL, NULL);
        }
    free(mine);
}

/*
 * image_render.backward (Alg. 1): gradient of L w.r.t. the splat state given
 * dL/dimage [H][W][3]. Outputs are ACCUMULATED (+=): d_mean2d[n][2], d_conic[n][3],
 * d_opacity[n], d_color[n][3]. The forward blend is recomputed per pixel and the suffix
 * sums are formed directly (no divide-back recurrence).
 */
void orc_render_bwd(int width, int height, const double* mean2d, const double* conic, const double* opacity,
                    const double* color, const uint32_t* vals, const uint32_t* ranges, const double bg[3],
                    const double* dL_dimage, double* d_mean2d, double* d_conic, double* d_opacity, double* d_color)
{
    const int TX = (width + ORC_TILE - 1) / ORC_TILE;
    int y;
#pragma omp parallel for schedule(dynamic, 4)
    for (y = 0; y < height; ++y) {
        int x;
        uint32_t cap = 0;
        orc_hit* hits = NULL;
        for (x = 0; x < width; ++x) {
            const int tile = (y / ORC_TILE) * TX + (x / ORC_TILE);
            const uint32_t s = ranges[2 * tile], e = ranges[2 * tile + 1];
            const size_t pix = (size_t)y * width + x;
            const double* g = dL_dimage + 3 * pix;
            const double px = x + 0.5, py = y + 0.5;
            double rgb[3], T_final, suffix;
            uint32_t last, nh;
            int k;
            if (e - s > cap) { cap = e - s; free(hits); hits = (orc_hit*)malloc((size_t)cap * sizeof(orc_hit)); }
            if (e == s) continue;
            blend_pixel(px, py, vals + s, e - s, mean2d, conic, opacity, color, bg, rgb, &T_final, &last, NULL, NULL,
                        NULL, hits, &nh);
            /* suffix = sum_{i>k} w_i (rgb_i . g) + T_final (bg . g) */
            suffix = T_final * (bg[0] * g[0] + bg[1] * g[1] + bg[2] * g[2]);
            for (k = (int)nh - 1; k >= 0; --k) {
                const uint32_t gi = vals[s + hits[k].pos];
                const double alpha = hits[k].alpha, T = hits[k].T, w = alpha * T;
                const double cg = color[3 * gi] * g[0] + color[3 * gi + 1] * g[1] + color[3 * gi + 2] * g[2];
                const double dL_dalpha = T * cg - suffix / (1.0 - alpha);
                int c;
                for (c = 0; c < 3; ++c) {
#pragma omp atomic
                    d_color[3 * gi + c] += w * g[c];
                }
                if (!hits[k].clamped) {
                    const double dx = px - mean2d[2 * gi], dy = py - mean2d[2 * gi + 1];
                    const double dL_dsigma = -alpha * dL_dalpha;
                    const double qa = conic[3 * gi], qb = conic[3 * gi + 1], qc = conic[3 * gi + 2];
#pragma omp atomic
                    d_opacity[gi] += hits[k].gauss * dL_dalpha;
#pragma omp atomic
                    d_conic[3 * gi] += 0.5 * dx * dx * dL_dsigma;
#pragma omp atomic
                    d_conic[3 * gi + 1] += dx * dy * dL_dsigma;
#pragma omp atomic
                    d_conic[3 * gi + 2] += 0.5 * dy * dy * dL_dsigma;
#pragma omp atomic
                    d_mean2d[2 * gi] += -(qa * dx + qb * dy) * dL_dsigma;
#pragma omp atomic
                    d_mean2d[2 * gi + 1] += -(qc * dy + qb * dx) * dL_dsigma;
                }
                suffix += w * cg;
            }
        }
        free(hits);
    }
}

/*
 * pts_splatting.backward (Alg. 1, the step that sums the views' gradients): chain rule from the splat-state gradient to
 * the raw point parameters, ACCUMULATED (+=) into g_mean[n][3], g_log_scale[n][3],
 * g_quat[n][4], g_logit[n], g_sh[n][K][3]. Depth and radius carry no gradient.
 */
void orc_preprocess_bwd(int n, int sh_degree, const double* mean, const double* log_scale, const double* quat,
                        const double* logit, const double* sh, const orc_camera* cam, const double* d_mean2d,
                        const double* d_conic, const double* d_opacity, const double* d_color, double* g_mean,
                        double* g_log_scale, double* g_quat, double* g_logit, double* g_sh)
{
    const int K = (sh_degree + 1) * (sh_degree + 1);
    int idx;
#pragma omp parallel for schedule(static)
    for (idx = 0; idx < n; ++idx) {
        orc_proj P;
        double dp[3] = {0, 0, 0}, dmu[3] = {0, 0, 0};
        double GS2[4], GM[6], GSigma[9], GJ[6], GW[9], GRq[9], gs[3], gqn[4];
        int i, j, k, c;
        project_one(sh_degree, mean + 3 * idx, log_scale + 3 * idx, quat + 4 * idx, logit[idx],
                    sh + (size_t)3 * K * idx, cam, &P);
        if (!P.visible) continue;
        /* opacity = sigmoid(logit) */
        g_logit[idx] += d_opacity[idx] * P.o * (1.0 - P.o);
        /* colour = max(0, 0.5 + sum_k Y_k(dir) sh_k), dir = v/|v|, v = mean - campos */
        {
            double ddir[3] = {0, 0, 0}, dot;
            for (c = 0; c < 3; ++c) {
                const double gc = P.rgb_raw[c] > 0.0 ? d_color[3 * idx + c] : 0.0;
                for (k = 0; k < K; ++k) {
                    g_sh[(size_t)3 * K * idx + 3 * k + c] += P.Y[k] * gc;
                    for (i = 0; i < 3; ++i) ddir[i] += gc * P.dY[k][i] * sh[(size_t)3 * K * idx + 3 * k + c];
                }
            }
            dot = ddir[0] * P.dir[0] + ddir[1] * P.dir[1] + ddir[2] * P.dir[2];
            for (i = 0; i < 3; ++i) dmu[i] += (ddir[i] - P.dir[i] * dot) / P.vlen;
        }
        /* conic = inverse of the 2D covariance: G_cov = -Q G_Q Q, with G_Q symmetric */
        {
            const double Q[4] = {P.conic[0], P.conic[1], P.conic[1], P.conic[2]};
            const double GQ[4] = {d_conic[3 * idx], 0.5 * d_conic[3 * idx + 1], 0.5 * d_conic[3 * idx + 1],
                                  d_conic[3 * idx + 2]};
            double tmp[4];
            for (i = 0; i < 2; ++i)
                for (j = 0; j < 2; ++j) tmp[2 * i + j] = Q[2 * i] * GQ[j] + Q[2 * i + 1] * GQ[2 + j];
            for (i = 0; i < 2; ++i)
                for (j = 0; j < 2; ++j) GS2[2 * i + j] = -(tmp[2 * i] * Q[j] + tmp[2 * i + 1] * Q[2 + j]);
        }
        /* cov2d = M Sigma M^T (+ const):  G_Sigma = M^T G M,  G_M = 2 G M Sigma */
        for (i = 0; i < 3; ++i)
            for (j = 0; j < 3; ++j) {
                double acc = 0.0;
                int a, b;
                for (a = 0; a < 2; ++a)
                    for (b = 0; b < 2; ++b) acc += P.M[3 * a + i] * GS2[2 * a + b] * P.M[3 * b + j];
                GSigma[3 * i + j] = acc;
            }
        for (i = 0; i < 2; ++i)
            for (j = 0; j < 3; ++j) {
                double acc = 0.0;
                int a;
                for (a = 0; a < 2; ++a)
                    for (k = 0; k < 3; ++k) acc += 2.0 * GS2[2 * i + a] * P.M[3 * a + k] * P.Sigma[3 * k + j];
                GM[3 * i + j] = acc;
            }
        /* M = J R_cam:  G_J = G_M R_cam^T */
        for (i = 0; i < 2; ++i)
            for (j = 0; j < 3; ++j) {
                double acc = 0.0;
                for (k = 0; k < 3; ++k) acc += GM[3 * i + k] * cam->R[3 * j + k];
                GJ[3 * i + j] = acc;
            }
        /* J entries as functions of p (slopes tx, ty frozen when clamped) */
        {
            const double x = P.p[0], y = P.p[1], z = P.p[2], fx = cam->fx, fy = cam->fy;
            const double gtx = GJ[2] * (-fx / z), gty = GJ[5] * (-fy / z);
            dp[2] += GJ[0] * (-fx / (z * z)) + GJ[2] * (fx * P.tx / (z * z)) + GJ[4] * (-fy / (z * z)) +
                     GJ[5] * (fy * P.ty / (z * z));
            if (!P.tx_clamped) { dp[0] += gtx / z; dp[2] += -gtx * x / (z * z); }
            if (!P.ty_clamped) { dp[1] += gty / z; dp[2] += -gty * y / (z * z); }
            /* mean2d = (fx x/z + cx, fy y/z + cy) */
            dp[0] += d_mean2d[2 * idx] * fx / z;
            dp[2] += -d_mean2d[2 * idx] * fx * x / (z * z);
            dp[1] += d_mean2d[2 * idx + 1] * fy / z;
            dp[2] += -d_mean2d[2 * idx + 1] * fy * y / (z * z);
        }
        /* p = R_cam mean + t */
        for (i = 0; i < 3; ++i) dmu[i] += cam->R[i] * dp[0] + cam->R[3 + i] * dp[1] + cam->R[6 + i] * dp[2];
        for (i = 0; i < 3; ++i) g_mean[3 * idx + i] += dmu[i];
        /* Sigma = W W^T, W = Rq diag(s):  G_W = 2 G_Sigma W */
        for (i = 0; i < 3; ++i)
            for (j = 0; j < 3; ++j) {
                double acc = 0.0;
                for (k = 0; k < 3; ++k) acc += 2.0 * GSigma[3 * i + k] * P.Rq[3 * k + j] * P.s[j];
                GW[3 * i + j] = acc;
            }
        for (j = 0; j < 3; ++j) {
            gs[j] = 0.0;
            for (i = 0; i < 3; ++i) { gs[j] += GW[3 * i + j] * P.Rq[3 * i + j]; GRq[3 * i + j] = GW[3 * i + j] * P.s[j]; }
            g_log_scale[3 * idx + j] += gs[j] * P.s[j];
        }
        /* Rq entries as functions of the unit quaternion (w,x,y,z) */
        {
            const double w = P.qn[0], x = P.qn[1], y = P.qn[2], z = P.qn[3], *G = GRq;
            double dot;
            gqn[0] = 2.0 * (-z * G[1] + y * G[2] + z * G[3] - x * G[5] - y * G[6] + x * G[7]);
            gqn[1] = 2.0 * (y * G[1] + z * G[2] + y * G[3] - 2.0 * x * G[4] - w * G[5] + z * G[6] + w * G[7] - 2.0 * x * G[8]);
            gqn[2] = 2.0 * (-2.0 * y * G[0] + x * G[1] + w * G[2] + x * G[3] + z * G[5] - w * G[6] + z * G[7] - 2.0 * y * G[8]);
            gqn[3] = 2.0 * (-2.0 * z * G[0] - w * G[1] + x * G[2] + w * G[3] - 2.0 * z * G[4] + y * G[5] + x * G[6] + y * G[7]);
            /* normalisation q/|q| */
            dot = gqn[0] * P.qn[0] + gqn[1] * P.qn[1] + gqn[2] * P.qn[2] + gqn[3] * P.qn[3];
            for (i = 0; i < 4; ++i) g_quat[4 * idx + i] += (gqn[i] - P.qn[i] * dot) / P.qlen;
        }
    }
}

int orc_num_threads(void)
{
    int nthreads = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        nthreads = omp_get_num_threads();
    }
#endif
    return nthreads;
}

/* ====================================================================================== */
/* Point-group frustum culling (App. D.1; Sec. 4.2.1 for the Z-order and the group size).   */
/*                                                                                        */
/* Points stored in Z-order are cut into groups of G consecutive points; each group keeps   */
/* an axis-aligned box around its centres and its largest scale. Per view, a whole group   */
/* is dropped when its box shows that every point in it would be culled anyway, so the      */
/* per-point work is spent on in-frustum groups only.                                      */
/* Reading: the paper tests the 8 box corners against the frustum; a box can meet the       */
/* frustum with no corner inside, and splats have an extent, so that test can drop          */
/* visible points. Here the test is made conservative with respect to THIS file's           */
/* per-point culls, so that grouped and ungrouped preprocessing give identical results.     */
/* With p = R c + t a corner in camera space, a group is dropped if                         */
/*   every corner has p_z < near, or every corner has p_z > far, or                         */
/*   for one of the four image sides every corner lies beyond that side's plane pushed      */
/*   out by the largest extent a member can have. A member at depth z has extent            */
/*     ceil(3 sqrt(lambda)) <= k1 s_max / z + k0,                                           */
/*     k1 = 3 sqrt(F2),  F2 = fx^2 (1 + lim_x^2) + fy^2 (1 + lim_y^2)  (Frobenius norm of    */
/*     the clamped Jacobian times z),  k0 = 3 sqrt(0.3 + sqrt(0.1)) + 1  (blur, the floor    */
/*     under the root of the eigenvalue formula, the ceil),                                 */
/*   and its tile rectangle is empty on the right if mean2d_x - extent >= 16 TX + 1, on      */
/*   the left if mean2d_x + extent < 0 (same in y). Multiplied by z > 0 these are linear     */
/*   in p, e.g. right:  fx p_x - (16 TX + 1 + k0 - cx) p_z - k1 s_max >= 0,                  */
/*   so they hold throughout the box if they hold at its corners; members behind the        */
/*   camera are culled by the near test whatever the planes say.                            */
/* bounds[g] = (min x, min y, min z, max x, max y, max z, s_max).                          */
/* ====================================================================================== */
void orc_group_bounds(int n, int group_size, const double* mean, const double* log_scale, double* bounds)
{
    const int ng = (n + group_size - 1) / group_size;
    int g;
#pragma omp parallel for schedule(static)
    for (g = 0; g < ng; ++g) {
        const int lo = g * group_size, hi = (lo + group_size < n) ? lo + group_size : n;
        double* b = bounds + 7 * g;
        int i, k;
        for (k = 0; k < 3; ++k) { b[k] = mean[3 * lo + k]; b[3 + k] = mean[3 * lo + k]; }
        b[6] = 0.0;
        for (i = lo; i < hi; ++i) {
            for (k = 0; k < 3; ++k) {
                const double v = mean[3 * i + k], sc = exp(log_scale[3 * i + k]);
                if (v < b[k]) b[k] = v;
                if (v > b[3 + k]) b[3 + k] = v;
                if (sc > b[6]) b[6] = sc;
            }
        }
    }
}

/* The rule. Every comparison is moved by eps times the sum of the magnitudes of its terms: towards keeping for
 * eps > 0, towards dropping for eps < 0 (used to flag decisions that rounding could flip). */
static int group_keep(const double* b, const orc_camera* cam, double eps)
{
    const int TX = (cam->width + ORC_TILE - 1) / ORC_TILE, TY = (cam->height + ORC_TILE - 1) / ORC_TILE;
    const double lim_x = ORC_GUARD * (0.5 * cam->width) / cam->fx, lim_y = ORC_GUARD * (0.5 * cam->height) / cam->fy;
    const double F2 = cam->fx * cam->fx * (1.0 + lim_x * lim_x) + cam->fy * cam->fy * (1.0 + lim_y * lim_y);
    const double k1 = 3.0 * sqrt(F2), k0 = 3.0 * sqrt(ORC_BLUR + sqrt(ORC_EIG_FLOOR)) + 1.0;
    /* side planes as (coefficient of p_x, of p_y, of p_z): right, left, bottom, top */
    const double side[4][3] = {{cam->fx, 0.0, -(16.0 * TX + 1.0 + k0 - cam->cx)}, {-cam->fx, 0.0, -(cam->cx + k0)},
                               {0.0, cam->fy, -(16.0 * TY + 1.0 + k0 - cam->cy)}, {0.0, -cam->fy, -(cam->cy + k0)}};
    double p[8][3], mag[8][3];
    int k, i, j, behind = 1, beyond = 1;
    for (k = 0; k < 8; ++k) {
        const double c[3] = {b[(k & 1) ? 3 : 0], b[(k & 2) ? 4 : 1], b[(k & 4) ? 5 : 2]};
        for (i = 0; i < 3; ++i) {
            p[k][i] = cam->t[i]; mag[k][i] = fabs(cam->t[i]);
            for (j = 0; j < 3; ++j) { p[k][i] += cam->R[3 * i + j] * c[j]; mag[k][i] += fabs(cam->R[3 * i + j] * c[j]); }
        }
        if (!(p[k][2] + eps * mag[k][2] < cam->near_plane)) behind = 0;
        if (!(p[k][2] - eps * mag[k][2] > cam->far_plane)) beyond = 0;
    }
    if (behind || beyond) return 0;
    for (i = 0; i < 4; ++i) {
        int outside = 1;
        for (k = 0; k < 8 && outside; ++k) {
            const double f = side[i][0] * p[k][0] + side[i][1] * p[k][1] + side[i][2] * p[k][2] - k1 * b[6];
            const double m = fabs(side[i][0]) * mag[k][0] + fabs(side[i][1]) * mag[k][1] + fabs(side[i][2]) * mag[k][2] + k1 * b[6];
            if (!(f - eps * m > 0.0)) outside = 0;
        }
        if (outside) return 0;
    }
    return 1;
}

/* keep[g] = 0 if group g is dropped for this view. near_tie[g] (optional) = 1 if moving the thresholds by +-tau flips it. */
void orc_group_cull(int n_groups, const double* bounds, const orc_camera* cam, uint8_t* keep, uint8_t* near_tie, double tau)
{
    int g;
#pragma omp parallel for schedule(static)
    for (g = 0; g < n_groups; ++g) {
        keep[g] = (uint8_t)group_keep(bounds + 7 * g, cam, 0.0);
        if (near_tie) near_tie[g] = (uint8_t)(group_keep(bounds + 7 * g, cam, tau) != group_keep(bounds + 7 * g, cam, -tau));
    }
}

/* orc_preprocess restricted to the groups that survive orc_group_cull: the state of Table 3a, culled groups zeroed */
void orc_preprocess_grouped(int n, int sh_degree, int group_size, const double* mean, const double* log_scale,
                            const double* quat, const double* logit, const double* sh, const orc_camera* cam,
                            double* mean2d, double* conic, double* opacity, double* color, int32_t* radius, double* depth,
                            uint8_t* keep_out)
{
    const int K = (sh_degree + 1) * (sh_degree + 1);
    const int ng = (n + group_size - 1) / group_size;
    double* bounds = (double*)malloc((size_t)(ng > 0 ? ng : 1) * 7 * sizeof(double));
    uint8_t* keep = (uint8_t*)malloc((size_t)(ng > 0 ? ng : 1));
    int i;
    orc_group_bounds(n, group_size, mean, log_scale, bounds);
    orc_group_cull(ng, bounds, cam, keep, NULL, 0.0);
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; ++i) {
        orc_proj P;
        int k;
        mean2d[2 * i] = mean2d[2 * i + 1] = 0.0;
        conic[3 * i] = conic[3 * i + 1] = conic[3 * i + 2] = 0.0;
        opacity[i] = 0.0; depth[i] = 0.0; radius[i] = 0;
        color[3 * i] = color[3 * i + 1] = color[3 * i + 2] = 0.0;
        if (!keep[i / group_size]) continue;
        project_one(sh_degree, mean + 3 * i, log_scale + 3 * i, quat + 4 * i, logit[i], sh + (size_t)3 * K * i, cam, &P);
        if (!P.visible) continue;
        mean2d[2 * i] = P.mean2d[0]; mean2d[2 * i + 1] = P.mean2d[1];
        for (k = 0; k < 3; ++k) { conic[3 * i + k] = P.conic[k]; color[3 * i + k] = P.rgb[k]; }
        opacity[i] = P.o; depth[i] = P.p[2]; radius[i] = P.radius;
    }
    if (keep_out) memcpy(keep_out, keep, (size_t)ng);
    free(bounds); free(keep);
}

/* ====================================================================================== */
/* 2D Gaussian surfels (the paper's 2DGS configuration: Sec. 5 "Applications", Table 3b,   */
/* App. B: "2DGS models [the projection] more accurately").                                */
/*                                                                                        */
/* A point is an oriented disk: centre mean, two raw tangent vectors (a, b) made           */
/* orthonormal by Gram-Schmidt (t_u = a/|a|, t_v = (b - (b.t_u) t_u)/|.|, n = t_u x t_v),   */
/* two scales exp(log_scale), opacity = sigmoid(logit), SH colour as for 3D Gaussians.     */
/* Readings (the paper gives only the state layout of Table 3b):                           */
/*   - ray_transforms T = K [R (s_u t_u) | R (s_v t_v) | R mean + t]: maps disk            */
/*     coordinates (u, v, 1) to homogeneous pixel coordinates;                             */
/*   - a pixel (x, y) meets the disk plane where the two planes x and y of its ray,        */
/*     pulled back through T, intersect: h_u = x T_2 - T_0, h_v = y T_2 - T_1 (rows of T), */
/*     p = h_u x h_v, (u, v) = (p_0, p_1)/p_2; G = exp(-(u^2+v^2)/2);                       */
/*   - screen-space low-pass: G^ = max(G, exp(-|pixel - mean2d|^2)) (sigma = sqrt(2)/2);    */
/*   - alpha = min(0.99, o G^), then the same skip / stop / order rules as above;           */
/*   - extent: exact bounding box of the perspective image of the 3-sigma disk, radius =   */
/*     ceil of its largest reach from mean2d, at least 3 (the low-pass support); a disk     */
/*     whose 3-sigma rim reaches the camera plane is culled; depth = z of the centre;       */
/*   - normal = R n, turned to face the camera (output only).                               */
/* Layouts: tan_u[n][3], tan_v[n][3], log_scale2[n][2]; T[n][9] row-major; normal[n][3].    */
/* ====================================================================================== */
#define ORC_FRAG_LOWPASS 16
#define ORC_FRAG_GRAZING 32

typedef struct {
    int visible;
    double tu[3], tv[3], nrm[3], alen, w[3], wlen, btu;
    double su, sv, o;
    double Hm[9], T[9];
    double mean2d[2], bc[2], half[2];
    double arim, reach; /* rim-vs-camera-plane discriminant and largest reach of the bounding box (set when in depth range) */
    int radius;
    int32_t rect[4];
    double ncam[3];
    double v[3], vlen, dir[3];
    double Y[16], dY[16][3];
    double rgb_raw[3], rgb[3];
} orc2d_proj;

static void cross3(const double a[3], const double b[3], double c[3])
{
    c[0] = a[1] * b[2] - a[2] * b[1]; c[1] = a[2] * b[0] - a[0] * b[2]; c[2] = a[0] * b[1] - a[1] * b[0];
}

static void project2d_one(int sh_degree, const double mean[3], const double ta[3], const double tb[3], const double ls[2],
                          double logit, const double* sh, const orc_camera* cam, orc2d_proj* P)
{
    int i, k, c;
    const int K = (sh_degree + 1) * (sh_degree + 1);
    double col[3][3]; /* camera-space columns of H */
    memset(P, 0, sizeof(*P));
    P->su = exp(ls[0]); P->sv = exp(ls[1]); P->o = 1.0 / (1.0 + exp(-logit));
    P->alen = sqrt(ta[0] * ta[0] + ta[1] * ta[1] + ta[2] * ta[2]);
    for (i = 0; i < 3; ++i) P->tu[i] = ta[i] / P->alen;
    P->btu = tb[0] * P->tu[0] + tb[1] * P->tu[1] + tb[2] * P->tu[2];
    for (i = 0; i < 3; ++i) P->w[i] = tb[i] - P->btu * P->tu[i];
    P->wlen = sqrt(P->w[0] * P->w[0] + P->w[1] * P->w[1] + P->w[2] * P->w[2]);
    for (i = 0; i < 3; ++i) P->tv[i] = P->w[i] / P->wlen;
    cross3(P->tu, P->tv, P->nrm);
    for (i = 0; i < 3; ++i) {
        col[0][i] = P->su * (cam->R[3 * i] * P->tu[0] + cam->R[3 * i + 1] * P->tu[1] + cam->R[3 * i + 2] * P->tu[2]);
        col[1][i] = P->sv * (cam->R[3 * i] * P->tv[0] + cam->R[3 * i + 1] * P->tv[1] + cam->R[3 * i + 2] * P->tv[2]);
        col[2][i] = cam->R[3 * i] * mean[0] + cam->R[3 * i + 1] * mean[1] + cam->R[3 * i + 2] * mean[2] + cam->t[i];
    }
    for (i = 0; i < 3; ++i) for (k = 0; k < 3; ++k) P->Hm[3 * i + k] = col[k][i];
    for (k = 0; k < 3; ++k) {
        P->T[k] = cam->fx * P->Hm[k] + cam->cx * P->Hm[6 + k];
        P->T[3 + k] = cam->fy * P->Hm[3 + k] + cam->cy * P->Hm[6 + k];
        P->T[6 + k] = P->Hm[6 + k];
    }
    if (P->T[8] < cam->near_plane || P->T[8] > cam->far_plane) return;
    {
        const double a = 9.0 * (P->T[6] * P->T[6] + P->T[7] * P->T[7]) - P->T[8] * P->T[8];
        double reach = 0.0, r;
        P->arim = a;
        if (!(a < 0.0)) return; /* the 3-sigma rim reaches the camera plane */
        for (i = 0; i < 2; ++i) {
            const double* Ti = P->T + 3 * i;
            const double b = 9.0 * (Ti[0] * P->T[6] + Ti[1] * P->T[7]) - Ti[2] * P->T[8];
            const double cc = 9.0 * (Ti[0] * Ti[0] + Ti[1] * Ti[1]) - Ti[2] * Ti[2];
            double disc;
            P->bc[i] = b / a;
            disc = P->bc[i] * P->bc[i] - cc / a;
            if (disc < 1e-4) disc = 1e-4;
            P->half[i] = sqrt(disc);
            P->mean2d[i] = Ti[2] / P->T[8];
            r = fabs(P->bc[i] - P->mean2d[i]) + P->half[i];
            if (r > reach) reach = r;
        }
        P->reach = reach;
        r = ceil(reach);
        if (r < 3.0) r = 3.0;
        if (!(r < (double)ORC_RADIUS_MAX)) r = (double)ORC_RADIUS_MAX;
        P->radius = (int)r;
    }
    if ((double)P->radius <= cam->radius_clip) { P->radius = 0; return; }
    orc_tile_rect(P->mean2d[0], P->mean2d[1], P->radius, cam->width, cam->height, P->rect);
    if ((P->rect[2] - P->rect[0]) * (P->rect[3] - P->rect[1]) <= 0) { P->radius = 0; return; }
    {
        double dotp = 0.0;
        for (i = 0; i < 3; ++i) {
            P->ncam[i] = cam->R[3 * i] * P->nrm[0] + cam->R[3 * i + 1] * P->nrm[1] + cam->R[3 * i + 2] * P->nrm[2];
            dotp += P->ncam[i] * col[2][i];
        }
        if (dotp > 0.0) for (i = 0; i < 3; ++i) P->ncam[i] = -P->ncam[i];
    }
    {
        double campos[3];
        for (i = 0; i < 3; ++i)
            campos[i] = -(cam->R[i] * cam->t[0] + cam->R[3 + i] * cam->t[1] + cam->R[6 + i] * cam->t[2]);
        for (i = 0; i < 3; ++i) P->v[i] = mean[i] - campos[i];
        P->vlen = sqrt(P->v[0] * P->v[0] + P->v[1] * P->v[1] + P->v[2] * P->v[2]);
        for (i = 0; i < 3; ++i) P->dir[i] = P->v[i] / P->vlen;
        sh_eval(sh_degree, P->dir, P->Y, P->dY);
        for (c = 0; c < 3; ++c) {
            double acc = 0.5;
            for (k = 0; k < K; ++k) acc += P->Y[k] * sh[3 * k + c];
            P->rgb_raw[c] = acc;
            P->rgb[c] = acc > 0.0 ? acc : 0.0;
        }
    }
    P->visible = 1;
}

/* Table 3b state: mean2d[n][2], T[n][9] (ray_transforms), opacity[n], color[n][3], radius[n], depth[n], normal[n][3].
 * Optional: bbox[n][4] = (centre_x, centre_y, half_x, half_y) of the 3-sigma disk's image; near_tie[n] = 1 where an
 * integer decision (a cull test, the extent's ceil, the tile rectangle) is within `tau` of flipping, or where the rim
 * comes so close to the camera plane that the extent is ill-conditioned, so an fp32 evaluation may differ. */
void orc2d_preprocess(int n, int sh_degree, const double* mean, const double* tan_u, const double* tan_v,
                      const double* log_scale2, const double* logit, const double* sh, const orc_camera* cam,
                      double* mean2d, double* T, double* opacity, double* color, int32_t* radius, double* depth,
                      double* normal, double* bbox, uint8_t* near_tie, double tau)
{
    const int K = (sh_degree + 1) * (sh_degree + 1);
    int i;
#pragma omp parallel for schedule(static)
    for (i = 0; i < n; ++i) {
        orc2d_proj P;
        int k;
        project2d_one(sh_degree, mean + 3 * i, tan_u + 3 * i, tan_v + 3 * i, log_scale2 + 2 * i, logit[i],
                      sh + (size_t)3 * K * i, cam, &P);
        mean2d[2 * i] = mean2d[2 * i + 1] = 0.0; opacity[i] = 0.0; depth[i] = 0.0; radius[i] = 0;
        for (k = 0; k < 9; ++k) T[9 * i + k] = 0.0;
        for (k = 0; k < 3; ++k) { color[3 * i + k] = 0.0; normal[3 * i + k] = 0.0; }
        if (bbox) for (k = 0; k < 4; ++k) bbox[4 * i + k] = 0.0;
        if (near_tie) {
            int flag = 0;
            const double z = P.T[8];
            if (fabs(z - cam->near_plane) < tau * fabs(z) || fabs(z - cam->far_plane) < tau * fabs(z)) flag = 1;
            if (z >= cam->near_plane && z <= cam->far_plane) {
                if (fabs(P.arim) < 0.02 * z * z) flag = 1;
                if (P.arim < 0.0) {
                    int32_t ra[4], rb[4];
                    double elo = P.reach * (1.0 - tau) - tau, ehi = P.reach * (1.0 + tau) + tau;
                    int rlo, rhi;
                    if (fabs(P.reach - floor(P.reach + 0.5)) < tau * (1.0 + P.reach)) flag = 1;
                    if (elo < 3.0) elo = 3.0;
                    if (ehi < 3.0) ehi = 3.0;
                    rlo = (int)ceil(elo); rhi = (int)ceil(ehi);
                    if (((double)rlo <= cam->radius_clip) != ((double)rhi <= cam->radius_clip)) flag = 1;
                    orc_tile_rect(P.mean2d[0] - tau * (1.0 + fabs(P.mean2d[0])), P.mean2d[1] - tau * (1.0 + fabs(P.mean2d[1])),
                                  P.radius > 0 ? P.radius : rhi, cam->width, cam->height, ra);
                    orc_tile_rect(P.mean2d[0] + tau * (1.0 + fabs(P.mean2d[0])), P.mean2d[1] + tau * (1.0 + fabs(P.mean2d[1])),
                                  P.radius > 0 ? P.radius : rhi, cam->width, cam->height, rb);
                    for (k = 0; k < 4; ++k) if (ra[k] != rb[k]) flag = 1;
                }
            }
            near_tie[i] = (uint8_t)flag;
        }
        if (!P.visible) continue;
        mean2d[2 * i] = P.mean2d[0]; mean2d[2 * i + 1] = P.mean2d[1];
        for (k = 0; k < 9; ++k) T[9 * i + k] = P.T[k];
        for (k = 0; k < 3; ++k) { color[3 * i + k] = P.rgb[k]; normal[3 * i + k] = P.ncam[k]; }
        opacity[i] = P.o; depth[i] = P.T[8]; radius[i] = P.radius;
        if (bbox) { bbox[4 * i] = P.bc[0]; bbox[4 * i + 1] = P.bc[1]; bbox[4 * i + 2] = P.half[0]; bbox[4 * i + 3] = P.half[1]; }
    }
}

/* How ill-conditioned the ray-disk intersection of pixel position (x, y) is: |h_u| |h_v| / |h_u x h_v| (>= 1). The
 * cross product p = h_u x h_v cancels when the disk is seen nearly edge-on from this pixel (h_u and h_v nearly
 * parallel); (u, v) = (p_0, p_1) / p_2 evaluated in fp32 then carries about 2.5e-7 x this number of relative error. */
static double ray_uv_condition(const double T[9], double x, double y)
{
    double hu[3], hv[3], p[3], nu, nv, np_;
    int k;
    for (k = 0; k < 3; ++k) { hu[k] = x * T[6 + k] - T[k]; hv[k] = y * T[6 + k] - T[3 + k]; }
    cross3(hu, hv, p);
    nu = sqrt(hu[0] * hu[0] + hu[1] * hu[1] + hu[2] * hu[2]);
    nv = sqrt(hv[0] * hv[0] + hv[1] * hv[1] + hv[2] * hv[2]);
    np_ = sqrt(p[0] * p[0] + p[1] * p[1] + p[2] * p[2]);
    return np_ > 0.0 ? nu * nv / np_ : 1e300;
}

/* disk coordinates (u, v) where the ray of pixel position (x, y) meets the surfel's plane; returns 0 if parallel */
int orc2d_ray_uv(const double T[9], double x, double y, double uv[2])
{
    double hu[3], hv[3], p[3];
    int k;
    for (k = 0; k < 3; ++k) { hu[k] = x * T[6 + k] - T[k]; hv[k] = y * T[6 + k] - T[3 + k]; }
    cross3(hu, hv, p);
    if (p[2] == 0.0) return 0;
    uv[0] = p[0] / p[2]; uv[1] = p[1] / p[2];
    return 1;
}

typedef struct { uint32_t pos; double alpha, Tr, ghat, u, v, g, g2; int clamped, lowpass; } orc2d_hit;

static void blend_pixel2d(double px, double py, const uint32_t* list, uint32_t len, const double* mean2d, const double* Tm,
                          const double* opacity, const double* color, const double bg[3], double rgb_out[3],
                          double* T_out, uint32_t* last_out, uint8_t* fragile_out, uint64_t* n_eval, uint64_t* n_blend,
                          orc2d_hit* hits, uint32_t* n_hits)
{
    double Tr = 1.0, C[3] = {0.0, 0.0, 0.0};
    uint32_t last = 0, k, nh = 0;
    uint8_t frag = 0;
    uint64_t ev = 0;
    for (k = 0; k < len; ++k) {
        const uint32_t g = list[k];
        double uv[2], G, G2, ghat, araw, alpha, Tn, dx, dy;
        ++ev;
        if (!orc2d_ray_uv(Tm + 9 * g, px, py, uv)) continue;
        G = exp(-0.5 * (uv[0] * uv[0] + uv[1] * uv[1]));
        dx = px - mean2d[2 * g]; dy = py - mean2d[2 * g + 1];
        G2 = exp(-(dx * dx + dy * dy));
        ghat = G > G2 ? G : G2;
        araw = opacity[g] * ghat;
        alpha = araw < ORC_ALPHA_MAX ? araw : ORC_ALPHA_MAX;
        if (fabs(araw - ORC_ALPHA_MAX) < 1e-5) frag |= ORC_FRAG_ALPHA_MAX;
        if (fabs(alpha - ORC_ALPHA_MIN) < 2e-7) frag |= ORC_FRAG_ALPHA_MIN;
        /* a disk seen nearly edge-on from this pixel: an fp32 evaluation of (u, v) is off by `rel`, relatively, so G by
         * the factor exp(+- rel (u^2 + v^2)). If that exceeds 1.25e-4 (the gradient tolerance is 1e-3) and the pair is
         * blended, or would be with G at the upper end of that range, the pixel's result is not pinned by fp32 */
        {
            const double rel = 2.5e-7 * ray_uv_condition(Tm + 9 * g, px, py);
            if (rel > 1.25e-4) {
                const double r2 = uv[0] * uv[0] + uv[1] * uv[1];
                const double Gup = exp(-0.5 * r2 * (1.0 - (rel < 0.5 ? 2.0 * rel : 1.0)));
                if (opacity[g] * (Gup > G2 ? Gup : G2) >= ORC_ALPHA_MIN) frag |= ORC_FRAG_GRAZING;
            }
        }
        if (alpha < ORC_ALPHA_MIN) continue;
        if (fabs(G - G2) < 1e-6) frag |= ORC_FRAG_LOWPASS;
        Tn = Tr * (1.0 - alpha);
        if (fabs(Tn - ORC_T_STOP) < 1e-8) frag |= ORC_FRAG_T_STOP;
        if (Tn < ORC_T_STOP) break;
        C[0] += color[3 * g] * alpha * Tr; C[1] += color[3 * g + 1] * alpha * Tr; C[2] += color[3 * g + 2] * alpha * Tr;
        if (hits) {
            hits[nh].pos = k; hits[nh].alpha = alpha; hits[nh].Tr = Tr; hits[nh].ghat = ghat; hits[nh].u = uv[0];
            hits[nh].v = uv[1]; hits[nh].g = G; hits[nh].g2 = G2; hits[nh].clamped = !(araw < ORC_ALPHA_MAX);
            hits[nh].lowpass = !(G > G2);
        }
        ++nh;
        Tr = Tn;
        last = k + 1;
    }
    rgb_out[0] = C[0] + Tr * bg[0]; rgb_out[1] = C[1] + Tr * bg[1]; rgb_out[2] = C[2] + Tr * bg[2];
    *T_out = Tr; *last_out = last;
    if (fragile_out) *fragile_out = frag;
    if (n_eval) *n_eval = ev;
    if (n_blend) *n_blend = nh;
    if (n_hits) *n_hits = nh;
}

void orc2d_render_fwd(int width, int height, const double* mean2d, const double* Tm, const double* opacity,
                      const double* color, const uint32_t* vals, const uint32_t* ranges, const double bg[3],
                      double* image, double* final_T, uint32_t* last_idx, uint8_t* fragile, uint64_t* counters)
{
    const int TX = (width + ORC_TILE - 1) / ORC_TILE;
    uint64_t tot_eval = 0, tot_blend = 0;
    int y;
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : tot_eval, tot_blend)
    for (y = 0; y < height; ++y) {
        int x;
        for (x = 0; x < width; ++x) {
            const int tile = (y / ORC_TILE) * TX + (x / ORC_TILE);
            const uint32_t s = ranges[2 * tile], e = ranges[2 * tile + 1];
            const size_t pix = (size_t)y * width + x;
            uint64_t ev, nb;
            blend_pixel2d(x + 0.5, y + 0.5, vals + s, e - s, mean2d, Tm, opacity, color, bg, image + 3 * pix, final_T + pix,
                          last_idx + pix, fragile ? fragile + pix : NULL, &ev, &nb, NULL, NULL);
            tot_eval += ev; tot_blend += nb;
        }
    }
    if (counters) { counters[0] = tot_eval; counters[1] = tot_blend; }
}

/* gradient w.r.t. the splat state: d_T[n][9], d_mean2d[n][2] (through the low-pass branch only), d_opacity, d_color; += */
void orc2d_render_bwd(int width, int height, const double* mean2d, const double* Tm, const double* opacity,
                      const double* color, const uint32_t* vals, const uint32_t* ranges, const double bg[3],
                      const double* dL_dimage, double* d_T, double* d_mean2d, double* d_opacity, double* d_color)
{
    const int TX = (width + ORC_TILE - 1) / ORC_TILE;
    int y;
#pragma omp parallel for schedule(dynamic, 4)
    for (y = 0; y < height; ++y) {
        int x;
        uint32_t cap = 0;
        orc2d_hit* hits = NULL;
        for (x = 0; x < width; ++x) {
            const int tile = (y / ORC_TILE) * TX + (x / ORC_TILE);
            const uint32_t s = ranges[2 * tile], e = ranges[2 * tile + 1];
            const size_t pix = (size_t)y * width + x;
            const double* g = dL_dimage + 3 * pix;
            const double px = x + 0.5, py = y + 0.5;
            double rgb[3], T_final, suffix;
            uint32_t last, nh;
            int k;
            if (e - s > cap) { cap = e - s; free(hits); hits = (orc2d_hit*)malloc((size_t)cap * sizeof(orc2d_hit)); }
            if (e == s) continue;
            blend_pixel2d(px, py, vals + s, e - s, mean2d, Tm, opacity, color, bg, rgb, &T_final, &last, NULL, NULL, NULL,
                          hits, &nh);
            suffix = T_final * (bg[0] * g[0] + bg[1] * g[1] + bg[2] * g[2]);
            for (k = (int)nh - 1; k >= 0; --k) {
                const uint32_t gi = vals[s + hits[k].pos];
                const double alpha = hits[k].alpha, Tr = hits[k].Tr, w = alpha * Tr;
                const double cg = color[3 * gi] * g[0] + color[3 * gi + 1] * g[1] + color[3 * gi + 2] * g[2];
                const double dL_dalpha = Tr * cg - suffix / (1.0 - alpha);
                int c;
                for (c = 0; c < 3; ++c) {
#pragma omp atomic
                    d_color[3 * gi + c] += w * g[c];
                }
                if (!hits[k].clamped) {
                    const double dL_dghat = opacity[gi] * dL_dalpha;
#pragma omp atomic
                    d_opacity[gi] += hits[k].ghat * dL_dalpha;
                    if (hits[k].lowpass) {
                        const double dx = px - mean2d[2 * gi], dy = py - mean2d[2 * gi + 1];
                        /* G2 = exp(-(dx^2+dy^2)), dx = px - mx */
#pragma omp atomic
                        d_mean2d[2 * gi] += dL_dghat * hits[k].g2 * 2.0 * dx;
#pragma omp atomic
                        d_mean2d[2 * gi + 1] += dL_dghat * hits[k].g2 * 2.0 * dy;
                    } else {
                        const double* Tg = Tm + 9 * gi;
                        const double du = -hits[k].u * hits[k].g * dL_dghat, dv = -hits[k].v * hits[k].g * dL_dghat;
                        double hu[3], hv[3], p[3], dp[3], dhu[3], dhv[3];
                        int q;
                        for (q = 0; q < 3; ++q) { hu[q] = px * Tg[6 + q] - Tg[q]; hv[q] = py * Tg[6 + q] - Tg[3 + q]; }
                        cross3(hu, hv, p);
                        dp[0] = du / p[2]; dp[1] = dv / p[2]; dp[2] = -(du * p[0] + dv * p[1]) / (p[2] * p[2]);
                        cross3(hv, dp, dhu);   /* p = hu x hv  =>  dL/dhu = hv x dL/dp */
                        cross3(dp, hu, dhv);   /*                  dL/dhv = dL/dp x hu */
                        for (q = 0; q < 3; ++q) {
#pragma omp atomic
                            d_T[9 * gi + q] += -dhu[q];
#pragma omp atomic
                            d_T[9 * gi + 3 + q] += -dhv[q];
#pragma omp atomic
                            d_T[9 * gi + 6 + q] += px * dhu[q] + py * dhv[q];
                        }
                    }
                }
                suffix += w * cg;
            }
        }
        free(hits);
    }
}

/* chain rule from (d_T, d_mean2d, d_opacity, d_color) to the raw surfel parameters; accumulated (+=) */
void orc2d_preprocess_bwd(int n, int sh_degree, const double* mean, const double* tan_u, const double* tan_v,
                          const double* log_scale2, const double* logit, const double* sh, const orc_camera* cam,
                          const double* d_T, const double* d_mean2d, const double* d_opacity, const double* d_color,
                          double* g_mean, double* g_tan_u, double* g_tan_v, double* g_log_scale2, double* g_logit,
                          double* g_sh)
{
    const int K = (sh_degree + 1) * (sh_degree + 1);
    int idx;
#pragma omp parallel for schedule(static)
    for (idx = 0; idx < n; ++idx) {
        orc2d_proj P;
        double GT[9], GH[9], gcol[3][3], dmu[3] = {0, 0, 0}, gtu[3], gtv[3], gx[3], gw[3], gb[3], ga[3];
        int i, k, c;
        project2d_one(sh_degree, mean + 3 * idx, tan_u + 3 * idx, tan_v + 3 * idx, log_scale2 + 2 * idx, logit[idx],
                      sh + (size_t)3 * K * idx, cam, &P);
        if (!P.visible) continue;
        g_logit[idx] += d_opacity[idx] * P.o * (1.0 - P.o);
        {
            double ddir[3] = {0, 0, 0}, dot;
            for (c = 0; c < 3; ++c) {
                const double gc = P.rgb_raw[c] > 0.0 ? d_color[3 * idx + c] : 0.0;
                for (k = 0; k < K; ++k) {
                    g_sh[(size_t)3 * K * idx + 3 * k + c] += P.Y[k] * gc;
                    for (i = 0; i < 3; ++i) ddir[i] += gc * P.dY[k][i] * sh[(size_t)3 * K * idx + 3 * k + c];
                }
            }
            dot = ddir[0] * P.dir[0] + ddir[1] * P.dir[1] + ddir[2] * P.dir[2];
            for (i = 0; i < 3; ++i) dmu[i] += (ddir[i] - P.dir[i] * dot) / P.vlen;
        }
        for (k = 0; k < 9; ++k) GT[k] = d_T[9 * idx + k];
        /* mean2d_i = T_i2 / T_22 */
        GT[2] += d_mean2d[2 * idx] / P.T[8];
        GT[5] += d_mean2d[2 * idx + 1] / P.T[8];
        GT[8] += -(d_mean2d[2 * idx] * P.T[2] + d_mean2d[2 * idx + 1] * P.T[5]) / (P.T[8] * P.T[8]);
        /* T0 = fx H0 + cx H2, T1 = fy H1 + cy H2, T2 = H2 (rows) */
        for (k = 0; k < 3; ++k) {
            GH[k] = cam->fx * GT[k];
            GH[3 + k] = cam->fy * GT[3 + k];
            GH[6 + k] = cam->cx * GT[k] + cam->cy * GT[3 + k] + GT[6 + k];
        }
        /* columns of H: R (su tu), R (sv tv), R mean + t  ->  world-space gradients of the three column vectors */
        for (k = 0; k < 3; ++k)
            for (i = 0; i < 3; ++i)
                gcol[k][i] = cam->R[i] * GH[k] + cam->R[3 + i] * GH[3 + k] + cam->R[6 + i] * GH[6 + k];
        for (i = 0; i < 3; ++i) dmu[i] += gcol[2][i];
        for (i = 0; i < 3; ++i) g_mean[3 * idx + i] += dmu[i];
        g_log_scale2[2 * idx] += P.su * (gcol[0][0] * P.tu[0] + gcol[0][1] * P.tu[1] + gcol[0][2] * P.tu[2]);
        g_log_scale2[2 * idx + 1] += P.sv * (gcol[1][0] * P.tv[0] + gcol[1][1] * P.tv[1] + gcol[1][2] * P.tv[2]);
        for (i = 0; i < 3; ++i) { gtu[i] = P.su * gcol[0][i]; gtv[i] = P.sv * gcol[1][i]; }
        /* Gram-Schmidt: tv = w/|w|, w = b - (b.tu) tu, tu = a/|a| */
        {
            double dot = gtv[0] * P.tv[0] + gtv[1] * P.tv[1] + gtv[2] * P.tv[2], wtu, gbtu;
            for (i = 0; i < 3; ++i) gw[i] = (gtv[i] - P.tv[i] * dot) / P.wlen;
            wtu = gw[0] * P.tu[0] + gw[1] * P.tu[1] + gw[2] * P.tu[2];
            gbtu = -wtu;                                  /* d/d(b.tu) */
            for (i = 0; i < 3; ++i) {
                gb[i] = gw[i] + gbtu * P.tu[i];
                gx[i] = gtu[i] - P.btu * gw[i] + gbtu * tan_v[3 * idx + i];   /* total gradient w.r.t. tu */
            }
            dot = gx[0] * P.tu[0] + gx[1] * P.tu[1] + gx[2] * P.tu[2];
            for (i = 0; i < 3; ++i) ga[i] = (gx[i] - P.tu[i] * dot) / P.alen;
        }
        for (i = 0; i < 3; ++i) { g_tan_u[3 * idx + i] += ga[i]; g_tan_v[3 * idx + i] += gb[i]; }
    }
}
