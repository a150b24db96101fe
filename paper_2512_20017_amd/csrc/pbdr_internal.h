// Internal declarations shared by the HIP translation units of libpbdr (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "profile.h"

namespace pbdr {

constexpr int kTile = 16;
constexpr float kBlur = 0.3f;
constexpr float kAlphaMax = 0.99f;
constexpr float kAlphaMin = 1.0f / 255.0f;
constexpr float kTStop = 1e-4f;
constexpr float kGuard = 1.3f;
constexpr float kEigFloor = 0.1f;
constexpr int kRadiusMax = 1 << 20;
constexpr float kPixMax = 1073741824.0f;

// Camera as the kernels see it (passed by value as a kernel argument -> lives in SGPRs).
// A call may render one rectangular patch of the image (App. D.2 of the paper): W, H are then the patch's size (the
// size of the output buffers), [rx0, rx1) x [ry0, ry1) its pixels in image coordinates, and TX x TY the part of the
// image's tile grid that meets it, starting at tile (otx, oty). Tiles stay aligned to the image's own 16 x 16 grid, so
// a patch holds exactly the pixels the whole-image render would give. Whole image: otx = oty = 0, patch = image.
struct CamDev {
    int W, H, TX, TY;
    int otx, oty, rx0, ry0, rx1, ry1;
    float fx, fy, cx, cy;
    float R[9];
    float t[3];
    float campos[3];
    float near_p, far_p, radius_clip;
    float lim_x, lim_y;
};

// Tile rectangle [x0, x1) x [y0, y1) of a splat, in tiles of the call's grid: floor((m -+ r) / 16) evaluated as integer
// floor-division of floor(m) -+ r (the same number, exact), clamped to the grid.
__device__ __forceinline__ void tile_rect(const CamDev& cam, float mx, float my, int r, int& x0, int& y0, int& x1, int& y1)
{
    const int ix = (int)fminf(kPixMax, fmaxf(-kPixMax, floorf(mx)));
    const int iy = (int)fminf(kPixMax, fmaxf(-kPixMax, floorf(my)));
    x0 = min(max(((ix - r) >> 4) - cam.otx, 0), cam.TX);
    y0 = min(max(((iy - r) >> 4) - cam.oty, 0), cam.TY);
    x1 = min(max(((ix + r + 15) >> 4) - cam.otx, 0), cam.TX);
    y1 = min(max(((iy + r + 15) >> 4) - cam.oty, 0), cam.TY);
}

// Gradient write-out of the splatting backward: "+=" into the caller's buffer (Alg. 1 lines 22-24), or a plain store
// for the first view of a batch, which folds the zero-initialisation of line 21 into it.
// The "+=" is an add performed by the memory side with no value returned (one thread per address and launch, so the
// sum is what load, add, store would give, and the same on every run): as load, add, store the compiler keeps the 59
// entries of a point in program order, each load waiting behind the store before it - a chain of 59 round trips.
template <bool kFirst>
__device__ __forceinline__ void grad_out(float* __restrict__ p, float v)
{
    if (kFirst) *p = v;
    else (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Raster record: everything the compositing kernels need about one splat, gathered with three 16-byte loads.
struct __attribute__((aligned(16))) Packed {
    float mx, my, qa, qb;   // mean2d, conic a, b
    float qc, o, r, g;      // conic c, opacity, red, green
    float b, radius_bits, depth, pad2;  // radius_bits: the integer extent, bit-cast
};
static_assert(sizeof(Packed) == 48, "raster record is 48 bytes");

struct SceneDev {
    int n, sh_degree;
    const float *mean, *log_scale, *quat, *logit, *sh;
};
struct SceneGradDev {
    float *mean, *log_scale, *quat, *logit, *sh;
};
struct SplatsDev {
    int n;
    float *mean2d, *conic, *opacity, *color;
    int32_t* radius;
    float* depth;
};
struct SplatGradDev {
    float *mean2d, *conic, *opacity, *color;
};

// Up to kMaxBatchViews views handed to one launch by value (kernel arguments): cameras, the splat states to write,
// the radii and splat-state gradients to read.
constexpr int kMaxBatchViews = 16;
struct BatchCams {
    int count;
    CamDev cam[kMaxBatchViews];
};
struct BatchSplats {
    SplatsDev view[kMaxBatchViews];
};
struct BatchSplatGrads {
    const int32_t* radius[kMaxBatchViews];
    SplatGradDev grad[kMaxBatchViews];
};

// 2D Gaussian surfels: raw parameters, per-view state (Table 3b of the paper) and their gradients
struct Scene2DDev {
    int n, sh_degree;
    const float *mean, *tan_u, *tan_v, *log_scale, *logit, *sh;
};
struct Scene2DGradDev {
    float *mean, *tan_u, *tan_v, *log_scale, *logit, *sh;
};
struct Splats2DDev {
    int n;
    float *mean2d, *T, *opacity, *color;
    int32_t* radius;
    float *depth, *normal;
};
struct Splat2DGradDev {
    float *mean2d, *T, *opacity, *color;
};

// Status words at the head of the workspace.
// pair count, overflow flag, visible-point count, number of tiles whose list is too long for one wavefront to sort
// (written by k_tile_order): cleared by every binning. kStEpoch (two words) is never cleared by a call: the 64-bit
// number of backward passes this workspace has seen plus one, stamped into the per-pair records a pass writes (see
// k_composite_bwd); it relies on the workspace having been zero-filled once before its first use.
enum { kStNumDup = 0, kStOverflow = 1, kStNumVis = 2, kStNumBig = 3, kStCleared = 32, kStEpoch = 32, kStWords = 64 };

// Workspace layout for (n, W, H, capacity). All offsets are multiples of 256 bytes.
enum Variant { kVariant3D = 0, kVariant2D = 1 };   // 3D Gaussians / 2D Gaussian surfels

struct Layout {
    int n, W, H, TX, TY, tiles;
    int variant;
    size_t record_bytes;      // raster record per point: 48 (3D) or 64 (2D)
    int partial_vec4;         // float4s of partial gradient sums per pair: 3 (3D) or 4 (2D)
    uint32_t cap;
    int tile_bits, tile_passes;   // key bits / radix passes spent on the tile id
    size_t off_status, off_packed, off_depth_bits, off_blk_vis, off_blk_pairs, off_blk_vis_at, off_blk_pairs_at, off_blk_order, off_touched, off_offsets, off_slot_base, off_order,
        off_tkey0, off_tval0, off_tkey1, off_tval1, off_totals, off_tile_hist, off_ranges,
        off_partial, off_keys64, off_chunk_rank, off_carry, off_grad_rec, off_reach, off_tile_order, total;
};
constexpr int kSortItems = 2048;   // pairs per radix-sort block
// A tile's list of fewer than kWaveListMax - 1 entries is put in depth order by one wavefront, a longer one by a whole
// workgroup (radix_sort.hip); k_tile_order (binning.hip) counts the longer ones, so the value must be where two of its
// length classes meet: a power of two or 1.5 times one.
constexpr int kWaveListMax = 1024;
constexpr int kRadixMaxBins = 256;   // widest digit: 8 bits
int radix_pass_count(int key_bits);  // passes launch_radix_sort32 takes for this many key bits
bool make_layout(int n, int W, int H, uint64_t cap, int variant, Layout* L);

// ---- launchers (each enqueues on `s` and returns the launch status) ----
// keep == nullptr: every point is tested; else keep[point / group_size] == 0 skips the point (group_size % 256 == 0)
hipError_t launch_preprocess(const SceneDev& sc, const CamDev& cam, const SplatsDev& out, const uint8_t* keep,
                             int group_size, hipStream_t s);
hipError_t launch_group_bounds(const SceneDev& sc, int group_size, float* bounds, hipStream_t s);
hipError_t launch_group_cull(const CamDev& cam, int n_groups, const float* bounds, uint8_t* keep, hipStream_t s);
// For the kernels that read a point's gradient record straight after the gather and finish the records cut by
// wavefront boundaries themselves (pair_reduce.h: record_from_carries), in place of the k_gather_fixup launch.
struct CarryFold {
    const float* carry;             // null: the records are complete (k_gather_fixup has run)
    const uint32_t* slot_base;      // [n] first pair of each listed point
    uint32_t* status;
    uint32_t cap;
};
CarryFold carry_fold(const Layout& L, char* ws);

hipError_t launch_preprocess_bwd_records(const SceneDev& sc, const CamDev& cam, const uint32_t* tiles_touched, const float4* rec, const CarryFold& cf,
                                         const SceneGradDev& g, bool first_view, hipStream_t s);
hipError_t launch_group_cull_batch(const BatchCams& cams, int n_groups, const float* bounds, uint8_t* keep, hipStream_t s);
hipError_t launch_preprocess_batch(const SceneDev& sc, const BatchCams& cams, const BatchSplats& outs, const uint8_t* keep,
                                   int group_size, hipStream_t s);
hipError_t launch_preprocess_bwd_batch(const SceneDev& sc, const BatchCams& cams, const BatchSplatGrads& in, const SceneGradDev& g,
                                       bool first_view, hipStream_t s);
hipError_t launch_preprocess_bwd(const SceneDev& sc, const CamDev& cam, const int32_t* radius, const SplatGradDev& g2,
                                 const SceneGradDev& g, bool first_view, hipStream_t s);
// what binning needs of a splat state, whatever the variant
struct BinInput {
    int n;
    const float* mean2d;      // [2][n]
    const int32_t* radius;    // [n]
};
struct BinArrays;
BinArrays bin_arrays(const Layout& L, char* ws);                                             // see binning_common.h
hipError_t launch_bin_begin(const Layout& L, char* ws, hipStream_t s);                       // zero status / totals / ranges
hipError_t launch_count_visible(const BinInput& in, const CamDev& cam, const Layout& L, char* ws, hipStream_t s);
hipError_t launch_bin_finish(const BinInput& in, const CamDev& cam, const Layout& L, char* ws, hipStream_t s);
hipError_t launch_bin_sort(const SplatsDev& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s);
hipError_t launch_composite_fwd(const CamDev& cam, const Layout& L, char* ws, const float bg[3], float* image,
                                float* final_T, uint32_t* last_idx, hipStream_t s);
hipError_t launch_composite_bwd(const CamDev& cam, const Layout& L, char* ws, int n, const float bg[3],
                                const float* final_T, const uint32_t* last_idx, const float* dL_dimage,
                                const SplatGradDev& g2, hipStream_t s);

hipError_t launch_render_stats(const CamDev& cam, const Layout& L, char* ws, uint64_t* counters, hipStream_t s);

// stable sort of every tile's list [ranges[2t], ranges[2t+1]) of (keysA, valsA) by depth_bits[val]; keysA's contents are
// overwritten, (keysB, valsB) are scratch; the result is in valsA
hipError_t launch_tile_depth_sort(const uint32_t* ranges, const uint32_t* tile_order, uint32_t ntiles, const uint32_t* status,
                                  const uint32_t* depth_bits, uint32_t cap, uint32_t* keysA, uint32_t* valsA, uint32_t* keysB, uint32_t* valsB, hipStream_t s);
hipError_t launch_radix_sort32(uint32_t* keys[2], uint32_t* vals[2], const uint32_t* count_ptr, uint32_t count_cap,
                               int key_bits, uint32_t* totals, uint32_t* tile_hist, hipStream_t s);
hipError_t launch_make_keys64(const Layout& L, char* ws, hipStream_t s);

// 2D Gaussian surfel variant (workspace laid out with kVariant2D)
hipError_t launch_preprocess2d(const Scene2DDev& sc, const CamDev& cam, const Splats2DDev& out, hipStream_t s);
hipError_t launch_preprocess2d_bwd(const Scene2DDev& sc, const CamDev& cam, const Splats2DDev& sp, const Splat2DGradDev& g2,
                                   const Scene2DGradDev& g, bool first_view, hipStream_t s);
hipError_t launch_preprocess2d_bwd_records(const Scene2DDev& sc, const CamDev& cam, const Splats2DDev& sp, const uint32_t* tiles_touched,
                                           const float4* rec, const CarryFold& cf, const Scene2DGradDev& g, bool first_view, hipStream_t s);
hipError_t launch_bin_sort2d(const Splats2DDev& sp, const CamDev& cam, const Layout& L, char* ws, hipStream_t s);
hipError_t launch_composite2d_fwd(const CamDev& cam, const Layout& L, char* ws, const float bg[3], float* image,
                                  float* final_T, uint32_t* last_idx, hipStream_t s);
hipError_t launch_composite2d_bwd(const CamDev& cam, const Layout& L, char* ws, int n, const float bg[3], const float* final_T,
                                  const uint32_t* last_idx, const float* dL_dimage, const Splat2DGradDev& g2, hipStream_t s);

hipError_t launch_render_stats2d(const CamDev& cam, const Layout& L, char* ws, uint64_t* counters, hipStream_t s);

// loss and optimizer step (Alg. 1 lines 13, 16, 27)
// Adam with bias correction for one value (Alg. 1 line 27). The constants are formed on the host in double.
struct AdamDev {
    float beta1, beta2, one_m_beta1, one_m_beta2;
    float step_size;      // lr / (1 - beta1^t)
    float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^t)
    float eps;
    int zero_grad;
};
AdamDev make_adam(float lr, float beta1, float beta2, float eps, int step, int zero_grad);

__device__ __forceinline__ void adam_one(const AdamDev& c, float& p, float g, float& m, float& v)
{
#pragma clang fp contract(off)      // the same roundings wherever this is inlined (see preprocess.hip)
    m = c.beta1 * m + c.one_m_beta1 * g;
    v = c.beta2 * v + c.one_m_beta2 * g * g;
    p -= c.step_size * m / (sqrtf(v) * c.inv_sqrt_bc2 + c.eps);
}

struct BatchAdam {          // one AdamDev per attribute: mean, log_scale, quat, opacity logit, SH
    AdamDev attr[5];
    float *m_mean, *m_log_scale, *m_quat, *m_logit, *m_sh;
    float *v_mean, *v_log_scale, *v_quat, *v_logit, *v_sh;
};
hipError_t launch_preprocess_bwd_batch_adam(const SceneDev& sc, const BatchCams& cams, const BatchSplatGrads& in, const BatchAdam& opt,
                                            hipStream_t s);
hipError_t launch_l1_loss(int W, int H, const float* image, const float* target, float* loss, float* dL, hipStream_t s);
hipError_t launch_mark_visible(int n, const int32_t* radius, uint8_t* visible, hipStream_t s);
hipError_t launch_adam_selective(int n, int planes, float* param, float* grad, float* exp_avg, float* exp_avg_sq,
                                 const uint8_t* visible, float lr, float beta1, float beta2, float eps, int step,
                                 int zero_grad, hipStream_t s);

// final location of the sorted pair lists (depends on the parity of the tile pass count)
inline size_t sorted_tkeys_off(const Layout& L) { return (L.tile_passes & 1) ? L.off_tkey1 : L.off_tkey0; }
inline size_t sorted_vals_off(const Layout& L) { return (L.tile_passes & 1) ? L.off_tval1 : L.off_tval0; }

}  // namespace pbdr
