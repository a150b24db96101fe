/*
 * pbdr.h -- C ABI of the MI355X (gfx950) splatting rasterizer: the per-view compute of point-based
 * differentiable rendering with 3D Gaussians, forward and backward.
 *
 * The three main calls follow the paper's three-function view of a PBDR algorithm (Sec. 3.1):
 *   pbdr_preprocess   = pts_culling + pts_splatting : point parameters + camera -> per-view splat state
 *   pbdr_render_fwd   = image_render                : splat state -> image (+ what the backward needs)
 *   pbdr_render_bwd   = image_render.backward + pts_splatting.backward (Alg. 1 lines 17-18, 22-24)
 *
 * Conventions for every call
 *   - Pointers inside the structs and the image / workspace pointers are DEVICE pointers owned by the caller
 *     (e.g. PyTorch allocations). The structs themselves, `bg` and the camera live in HOST memory.
 *   - The library allocates, frees and retains nothing. Work is enqueued on `hip_stream` (a hipStream_t, NULL =
 *     default stream) and the call returns without synchronising, except pbdr_query_lists which synchronises.
 *   - All arrays are fp32 / int32 / uint32 planes ("structure of arrays"): an attribute with l components of n
 *     points is stored as [l][n], i.e. component-major, so that one wavefront reads 64 consecutive floats.
 *     This is the paper's S x l tensor (Sec. 3.1) transposed. Every pointer must be 16-byte aligned.
 *   - Return value: PBDR_OK or a negative pbdr_status. Invalid arguments are detected on the host before
 *     anything is enqueued. No exceptions or C++ types cross this boundary.
 *   - Calls that share a workspace, a gradient buffer or an output must be ordered on one stream by the caller.
 *
 * Numerical rules (the paper leaves them to its rendering kernels; these are this library's readings, and the
 * CPU oracle states the same): scale = exp(log_scale), rotation = normalised quaternion (w,x,y,z), opacity =
 * sigmoid(logit); depth = camera-space z; first-order ("affine", App. B) projection of the covariance with the
 * ray slope clamped to 1.3 x the half field of view and 0.3 px^2 blur; extent = ceil(3 sigma_max); 16x16 tiles;
 * colour = max(0, 0.5 + SH(dir)); alpha = min(0.99, o exp(-sigma)); alpha < 1/255 skipped; a splat that would
 * take the transmittance below 1e-4 is not blended and ends the pixel; depth ties ordered by point index.
 */
#ifndef PBDR_H
#define PBDR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PBDR_TILE 16
#define PBDR_VERSION 100

typedef enum pbdr_status {
    PBDR_OK = 0,
    PBDR_ERR_INVALID_ARG = -1,         /* null / misaligned pointer, n < 0, sh_degree outside 0..3, bad image size */
    PBDR_ERR_WORKSPACE_TOO_SMALL = -2, /* workspace smaller than pbdr_workspace_bytes() for these sizes */
    PBDR_ERR_CAPACITY = -3,            /* more (tile, splat) pairs than dup_capacity (reported by pbdr_query_lists) */
    PBDR_ERR_HIP = -4,                 /* a HIP call failed; see pbdr_last_hip_error() */
    PBDR_ERR_STATIC_LIMIT = -5         /* pbdr_render_fwd_static: more points or a larger image than its fixed scratch serves */
} pbdr_status;

/* Point cloud shard ("model state", Sec. 3.1; 3DGS attributes Sec. 2.1 / 3.2): 59 floats per point at degree 3. */
typedef struct pbdr_scene {
    int32_t n;                  /* number of points, >= 0 */
    int32_t sh_degree;          /* 0..3; K = (sh_degree+1)^2 coefficients per colour channel */
    const float* mean;          /* [3][n] world-space position */
    const float* log_scale;     /* [3][n] */
    const float* quat;          /* [4][n] (w,x,y,z), need not be normalised */
    const float* opacity_logit; /* [n] */
    const float* sh;            /* [K][3][n] coefficient-major, then channel */
} pbdr_scene;

/* Gradient w.r.t. pbdr_scene, same layout. pbdr_render_bwd / pbdr_preprocess_bwd ACCUMULATE (+=) into it,
 * which is how Alg. 1 lines 22-24 sum the views of a batch; the caller zeroes it once per batch (line 21).
 * first_view != 0 folds that zeroing into the call for the first view of a batch: the buffer's previous contents
 * are ignored and every entry of every point is written - the view's gradient, or zero for points it does not use -
 * which leaves what zeroing and then accumulating leaves (up to the rounding of the last multiply-add), without the
 * extra pass over 236 bytes per point. */
typedef struct pbdr_scene_grads {
    int32_t n;
    int32_t sh_degree;
    float* mean;
    float* log_scale;
    float* quat;
    float* opacity_logit;
    float* sh;
    int32_t first_view;
} pbdr_scene_grads;

/* Pinhole view. World -> camera: p = R x + t, R row-major; camera axes +x right, +y down, +z forward.
 * Pixel (i,j) has its centre at (i+0.5, j+0.5). far_plane and radius_clip are the two per-view filters the paper
 * uses for street scenes (App. E.1); radius_clip = 0 and far_plane = 1e10 disable them. near_plane must be > 0. */
typedef struct pbdr_camera {
    int32_t width, height;
    float fx, fy, cx, cy;
    float R[9];
    float t[3];
    float near_plane, far_plane, radius_clip;
} pbdr_camera;

/* Per-view splat state, exactly the 11 elements / 44 bytes per point of Table 3a.
 * radius == 0 marks a culled point; its other fields are then unspecified. */
typedef struct pbdr_splats {
    int32_t n;
    float* mean2d;   /* [2][n] pixel coordinates */
    float* conic;    /* [3][n] inverse 2D covariance (a, b, c) */
    float* opacity;  /* [n] */
    float* color;    /* [3][n] */
    int32_t* radius; /* [n] extent in pixels */
    float* depth;    /* [n] camera-space z */
} pbdr_splats;

/* Gradient w.r.t. the differentiable part of pbdr_splats (what Alg. 1 line 19-20 sends back). Overwritten for every
 * point that binning lists: radius > 0 and a tile rectangle that meets the rendered image or patch (every point with
 * radius > 0 of a state written by the matching preprocessing call). Entries of other points are left untouched, and
 * the second half of pbdr_render_bwd does not read them: such points receive no parameter gradient (zeros with
 * first_view). pbdr_preprocess_bwd on its own selects by splats->radius > 0 and reads g_splats of all those points. */
typedef struct pbdr_splat_grads {
    int32_t n;
    float* mean2d;  /* [2][n] */
    float* conic;   /* [3][n] */
    float* opacity; /* [n] */
    float* color;   /* [3][n] */
} pbdr_splat_grads;

/* Bytes of workspace that pbdr_render_fwd / pbdr_render_bwd / pbdr_bin_sort need for n points, a width x height
 * image and at most dup_capacity (tile, splat) pairs. The workspace must be 256-byte aligned and ZERO-FILLED ONCE
 * before its first use (pbdr_workspace_init, or any device memset of the caller's): the backward pass tells the
 * per-pair records it wrote from older ones by the number of the call, which the workspace counts from zero. Calls
 * never need it cleared again, and a workspace may be reused for other sizes after being zero-filled again. */
int pbdr_workspace_bytes(int32_t n, int32_t width, int32_t height, uint64_t dup_capacity, size_t* out_bytes);

/* Zero-fills `bytes` bytes of workspace (a fill kernel on hip_stream; bytes a multiple of 16). Once per allocation. */
int pbdr_workspace_init(void* workspace, size_t bytes, void* hip_stream);

/* pts_culling + pts_splatting (Sec. 3.1, Sec. 3.2 "3DGS"; Alg. 1 lines 2-4). One pass over the shard: near/far
 * cull, covariance projection, conic, extent, off-screen and radius_clip cull, SH colour. Writes all of `out`. */
int pbdr_preprocess(const pbdr_scene* scene, const pbdr_camera* cam, pbdr_splats* out, void* hip_stream);

/* Point-group frustum culling (App. D.1; the groups are those of Sec. 4.2.1: runs of group_size consecutive points of
 * a cloud stored in Z-order, so that a group is spatially compact). group_size: a multiple of 256 in [256, 2^20].
 * pbdr_group_count returns ceil(n / group_size), or a negative status.
 * pbdr_group_bounds: once per cloud (again whenever means or scales have changed): bounds [7][n_groups] (device) =
 * planes min x, min y, min z, max x, max y, max z of the group's centres and the group's largest scale.
 * pbdr_preprocess_grouped = pbdr_preprocess preceded by one test per group: keep [n_groups] (device, uint8, written)
 * is 0 for a group whose box shows that each of its points would be culled for this view (behind the near plane,
 * beyond the far plane, or off screen by more than any member's extent); such groups cost 4 bytes written per point
 * and no parameter read. The paper tests the eight box corners against the frustum; here the test is conservative
 * with respect to the per-point culls, so `out` is identical to what pbdr_preprocess writes (radius == 0 for every
 * point of a dropped group). */
int pbdr_group_count(int32_t n, int32_t group_size);
int pbdr_group_bounds(const pbdr_scene* scene, int32_t group_size, float* bounds, void* hip_stream);
int pbdr_preprocess_grouped(const pbdr_scene* scene, const pbdr_camera* cam, int32_t group_size, const float* bounds,
                            uint8_t* keep, pbdr_splats* out, void* hip_stream);

/* The views of a batch in one pass over the points (App. D.1: view-by-view preprocessing reads the cloud once per
 * view, O(batch x points); Alg. 1 lines 2-4 for every view of the batch, lines 21-24 for their gradients).
 * num_views in [1, PBDR_MAX_BATCH_VIEWS]; `cams`, `outs`, `splats`, `g_splats` are host arrays of num_views structs
 * (the pointers inside them are device pointers, every n equal to scene->n).
 * pbdr_preprocess_batch: outs[v] receives exactly what pbdr_preprocess(scene, &cams[v], &outs[v]) writes; every
 * parameter of a point is read at most once for the whole batch. group_size == 0: no group test (bounds and keep are
 * ignored). Otherwise bounds is what pbdr_group_bounds wrote and keep [num_views][n_groups] (device, uint8) receives
 * the per-view flags of pbdr_preprocess_grouped; a group that no view keeps costs no parameter read.
 * pbdr_preprocess_bwd_batch: grads (+)= sum over v of what pbdr_preprocess_bwd(scene, &cams[v], &splats[v],
 * &g_splats[v], grads) adds, the views added in index order before the buffer is touched once (a store when
 * grads->first_view != 0, else one "+="). Of splats[v] only radius is read. Equal to the view-by-view sequence up to
 * the rounding of fused multiply-adds. */
#define PBDR_MAX_BATCH_VIEWS 16
int pbdr_preprocess_batch(const pbdr_scene* scene, int32_t num_views, const pbdr_camera* cams, const pbdr_splats* outs,
                          int32_t group_size, const float* bounds, uint8_t* keep, void* hip_stream);
int pbdr_preprocess_bwd_batch(const pbdr_scene* scene, int32_t num_views, const pbdr_camera* cams, const pbdr_splats* splats,
                              const pbdr_splat_grads* g_splats, pbdr_scene_grads* grads, void* hip_stream);

/* Image patches (Sec. 4.2.2: the unit of rendering work is an H/p x W/p patch of an image, p = 2..8; App. D.2: the
 * rendering kernels are restricted to the patch). A patch is the pixel rectangle [x0, x1) x [y0, y1) of the camera's
 * image, any size and position inside it. The *_patch calls do what their whole-image namesakes do for those pixels
 * only: tiles stay aligned to the image's own 16 x 16 grid and only tiles that meet the patch are listed, sorted and
 * composited, so image / final_T / last_idx - here [3][h][w], [h][w], [h][w] with w = x1 - x0, h = y1 - y0 - hold
 * exactly the values the whole-image render has at those pixels, and dL_dimage is [3][h][w]. pbdr_preprocess_patch
 * additionally culls points whose tile rectangle misses the patch (radius = 0), which is what makes a patch cheaper
 * than the image; the other fields of a visible point do not depend on the patch. The workspace is sized for the
 * whole image (pbdr_workspace_bytes with the camera's width and height); pbdr_lists_view then shows tile ids
 * relative to the patch's tile grid (its first tile is 0, row length = tiles across the patch). The three calls of
 * one patch must be given the same patch. pbdr_preprocess_bwd serves patches unchanged. */
typedef struct pbdr_patch {
    int32_t x0, y0, x1, y1;
} pbdr_patch;

int pbdr_preprocess_patch(const pbdr_scene* scene, const pbdr_camera* cam, const pbdr_patch* patch, pbdr_splats* out,
                          void* hip_stream);
int pbdr_render_fwd_patch(const pbdr_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                          uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                          size_t workspace_bytes, void* hip_stream);
int pbdr_render_bwd_patch(const pbdr_scene* scene, const pbdr_splats* splats, const pbdr_camera* cam,
                          const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                          const uint32_t* last_idx, const float* dL_dimage, pbdr_splat_grads* g_splats,
                          pbdr_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The sorting half of image_render (Sec. 2.1: "sorts these view-dependent splats by their distance to the camera
 * plane"): per-splat tile count, device prefix sum, duplication in point order, and a sort into the order of the key
 * (tile << 32 | depth bits), ties by point index - a stable radix sort of the pairs by tile id, then every tile's
 * list by depth bits - and per-tile ranges.
 * Results stay in the workspace; pbdr_lists_view gives their addresses. If more than dup_capacity pairs exist the
 * excess is dropped, nothing is written out of bounds, and pbdr_query_lists reports PBDR_ERR_CAPACITY. */
int pbdr_bin_sort(const pbdr_splats* splats, const pbdr_camera* cam, uint64_t dup_capacity, void* workspace,
                  size_t workspace_bytes, void* hip_stream);

/* image_render forward (Sec. 2.1 blending; Alg. 1 line 12) = pbdr_bin_sort followed by per-tile front-to-back
 * compositing. image [3][H][W], final_T [H][W], last_idx [H][W] = 1-based position, within the pixel's tile list,
 * of the last splat blended into the pixel (0 = none). The workspace keeps the lists for pbdr_render_bwd. */
int pbdr_render_fwd(const pbdr_splats* splats, const pbdr_camera* cam, const float bg[3], uint64_t dup_capacity,
                    float* image, float* final_T, uint32_t* last_idx, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/* pbdr_render_fwd for callers that cannot allocate device memory at all (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels in the same order, with the workspace taken from a fixed
 * array of PBDR_STATIC_SCRATCH_BYTES that lives in the library's device image (each GPU the library runs on holds its
 * own copy until the process ends) instead of from the caller. The call allocates and frees nothing; its first use on
 * a device only looks up that device's address of the array. Limits: splats->n <= PBDR_STATIC_MAX_POINTS, width and
 * height <= PBDR_STATIC_MAX_SIDE, at most PBDR_STATIC_MAX_PAIRS (tile, splat) pairs (the dup_capacity of the call; the
 * excess is dropped as pbdr_render_fwd drops it). Larger n or image: PBDR_ERR_STATIC_LIMIT, nothing enqueued.
 * image, final_T, last_idx as pbdr_render_fwd, bit for bit what it writes for dup_capacity = PBDR_STATIC_MAX_PAIRS.
 * pair_count: device pointer to one uint32 that receives the number of pairs found (before clamping; a value above
 * PBDR_STATIC_MAX_PAIRS means the lists were truncated), or NULL. Rendering only: the lists stay in the library's
 * array, there is no matching backward call. Every call on one GPU uses that GPU's one array, whatever its stream:
 * calls that may overlap in time on one GPU race with each other - order them on one stream or with events. */
#define PBDR_STATIC_MAX_POINTS 16384
#define PBDR_STATIC_MAX_SIDE 512
#define PBDR_STATIC_MAX_PAIRS 262144
#define PBDR_STATIC_SCRATCH_BYTES (24u << 20)
int pbdr_render_fwd_static(const pbdr_splats* splats, const pbdr_camera* cam, const float bg[3], float* image,
                           float* final_T, uint32_t* last_idx, uint32_t* pair_count, void* hip_stream);

/* image_render.backward then pts_splatting.backward (Alg. 1 lines 17-18 and 22-24). Needs the workspace exactly
 * as pbdr_render_fwd left it for the same splats, camera and dup_capacity. dL_dimage [3][H][W]. g_splats is overwritten with
 * dL/d(splat state). If scene and grads are both non-NULL the parameter gradient is then ACCUMULATED into grads;
 * if both are NULL the call stops after g_splats (the point where the paper's system exchanges gradients).
 * g_splats may be NULL when scene and grads are given: the splat-state gradient then stays in the workspace (one
 * 48-byte record per point) and the second half reads it there, which saves writing and re-reading its nine planes. */
int pbdr_render_bwd(const pbdr_scene* scene, const pbdr_splats* splats, const pbdr_camera* cam, const float bg[3],
                    uint64_t dup_capacity, const float* final_T, const uint32_t* last_idx, const float* dL_dimage,
                    pbdr_splat_grads* g_splats, pbdr_scene_grads* grads, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/* pts_splatting.backward alone (Alg. 1 lines 22-24): chain rule from g_splats to the raw parameters, ACCUMULATED
 * into grads. Points with splats->radius == 0 receive nothing. Depth and radius carry no gradient. */
int pbdr_preprocess_bwd(const pbdr_scene* scene, const pbdr_camera* cam, const pbdr_splats* splats,
                        const pbdr_splat_grads* g_splats, pbdr_scene_grads* grads, void* hip_stream);

/* Device addresses, inside a workspace laid out for these sizes, of the results of pbdr_bin_sort / pbdr_render_fwd:
 * sorted keys [P] (tile << 32 | bits(depth)), vals [P] (point index), ranges [tiles][2] ([start,end) per tile,
 * {0,0} for an empty tile), num_dup [1] (P before clamping to dup_capacity). Any out pointer may be NULL.
 * The 64-bit keys are not kept by the sort; asking for them enqueues one small kernel on hip_stream that rebuilds
 * them into a scratch part of the workspace (valid until the next call that uses this workspace). */
int pbdr_lists_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                    uint64_t dup_capacity, void* hip_stream, const uint64_t** keys, const uint32_t** vals,
                    const uint32_t** ranges, const uint32_t** num_dup);

/* Device address, inside a workspace laid out for these sizes, of the order in which the compositing kernels of the
 * last pbdr_bin_sort / pbdr_render_fwd (surfel_workspace == 0) or pbdr2d_render_fwd (!= 0) take the tiles:
 * tile_order [tiles of the call's grid], a permutation of the tile ids as pbdr_lists_view shows them. An
 * implementation detail with no effect on any result (Sec. 2.1 composites every tile independently of the others):
 * tiles with longer lists come first, in classes of list length L, two per octave of L + 1 (class = 2 floor(log2(L + 1))
 * + the next lower bit of L + 1, classes of 2^19.5 and more merged), and within a class in ascending id. */
int pbdr_tile_order_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                         uint64_t dup_capacity, int32_t surfel_workspace, const uint32_t** tile_order);

/* Device address, inside a workspace of either kind laid out for these sizes, of three words that the last
 * pbdr_bin_sort / pbdr_render_fwd / pbdr2d_render_fwd on it left: {pairs found (before clamping to dup_capacity;
 * saturates at 2^31 - 1), overflow flag (1 = pairs beyond dup_capacity were dropped), listed points}. The caller can
 * poll them with a copy of its own, ordered after the call on its stream: nothing here synchronises. */
int pbdr_status_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                     uint64_t dup_capacity, const uint32_t** status_words);

/* Synchronises hip_stream and reads back the number of (tile, splat) pairs found by the last pbdr_bin_sort /
 * pbdr_render_fwd on this workspace. Returns PBDR_ERR_CAPACITY if it exceeded dup_capacity (the lists were then
 * truncated), else PBDR_OK. Optional: callers that know a safe capacity never need to call it. */
int pbdr_query_lists(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                     uint64_t dup_capacity, void* hip_stream, uint64_t* num_dup);

/* Measurement aid, not part of the hot path: counts, for the lists now in the workspace, the (pixel, splat) pairs a
 * forward pass examines (every list entry up to and including the one that ends the pixel) and the pairs it blends.
 * counters: device pointer to 2 uint64 {examined, blended}, overwritten. */
int pbdr_render_stats(const pbdr_camera* cam, int32_t n, uint64_t dup_capacity, uint64_t* counters, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------------------
 * 2D Gaussian surfels: the same three calls for the paper's 2DGS configuration (Sec. 5 "Applications"; per-view
 * state of Table 3b, 20 floats; App. B notes that 2DGS projects more accurately than the affine approximation).
 * The paper gives only the state layout; this library's readings, which the CPU oracle states too:
 *   - a point is a disk: centre, two raw tangent vectors made orthonormal by Gram-Schmidt (t_u = a/|a|, t_v = the
 *     normalised part of b orthogonal to t_u), scales exp(log_scale) along them, opacity, SH colour;
 *   - ray_transform T = K [R s_u t_u | R s_v t_v | R mean + t] (row-major 3x3) maps disk coordinates (u, v, 1) to
 *     homogeneous pixels; a pixel (x, y) meets the disk plane at (u, v) = (p_0, p_1) / p_2, p = h_u x h_v,
 *     h_u = x T_2 - T_0, h_v = y T_2 - T_1 (rows of T); G = exp(-(u^2 + v^2) / 2);
 *   - screen-space low-pass G^ = max(G, exp(-|pixel - mean2d|^2)); alpha = min(0.99, o G^); a pair with p_2 = 0 is
 *     skipped; skip / stop / order rules as for 3D Gaussians;
 *   - extent = max(3, ceil(largest reach, from mean2d, of the exact bounding box of the 3-sigma rim's perspective
 *     image)); a disk whose 3-sigma rim reaches the camera plane is culled; depth = camera-space z of the centre;
 *   - normal = R (t_u x t_v), turned to face the camera (an output; carries no gradient).
 * Workspaces are laid out differently from the 3D calls: size them with pbdr2d_workspace_bytes and inspect them with
 * pbdr2d_lists_view. pbdr_query_lists serves both kinds of workspace (the pair count sits at the same place). */
typedef struct pbdr2d_scene {
    int32_t n;
    int32_t sh_degree;
    const float* mean;          /* [3][n] */
    const float* tan_u;         /* [3][n] raw first tangent, any non-zero length */
    const float* tan_v;         /* [3][n] raw second tangent, not parallel to tan_u */
    const float* log_scale;     /* [2][n] */
    const float* opacity_logit; /* [n] */
    const float* sh;            /* [K][3][n] */
} pbdr2d_scene;

typedef struct pbdr2d_scene_grads { /* accumulated (+=); first_view as in pbdr_scene_grads */
    int32_t n;
    int32_t sh_degree;
    float* mean;
    float* tan_u;
    float* tan_v;
    float* log_scale;
    float* opacity_logit;
    float* sh;
    int32_t first_view;
} pbdr2d_scene_grads;

/* Per-view surfel state: the 20 floats per point of Table 3b (radius counted as one). radius == 0 = culled. */
typedef struct pbdr2d_splats {
    int32_t n;
    float* mean2d;        /* [2][n] */
    float* ray_transform; /* [9][n] T row-major: plane k holds T[k/3][k%3] */
    float* opacity;       /* [n] */
    float* color;         /* [3][n] */
    int32_t* radius;      /* [n] */
    float* depth;         /* [n] */
    float* normal;        /* [3][n] camera-space unit normal facing the camera */
} pbdr2d_splats;

typedef struct pbdr2d_splat_grads { /* overwritten for points with radius > 0, untouched for culled points */
    int32_t n;
    float* mean2d;        /* [2][n] through the low-pass term only */
    float* ray_transform; /* [9][n] */
    float* opacity;       /* [n] */
    float* color;         /* [3][n] */
} pbdr2d_splat_grads;

int pbdr2d_workspace_bytes(int32_t n, int32_t width, int32_t height, uint64_t dup_capacity, size_t* out_bytes);

/* pts_culling + pts_splatting for surfels (Sec. 3.1; state of Table 3b). Writes all of `out`. */
int pbdr2d_preprocess(const pbdr2d_scene* scene, const pbdr_camera* cam, pbdr2d_splats* out, void* hip_stream);

/* image_render forward for surfels: binning and sorting exactly as pbdr_bin_sort (Sec. 2.1), then per-tile
 * front-to-back compositing with one ray-disk intersection per (pixel, splat) pair. Outputs as pbdr_render_fwd. */
int pbdr2d_render_fwd(const pbdr2d_splats* splats, const pbdr_camera* cam, const float bg[3], uint64_t dup_capacity,
                      float* image, float* final_T, uint32_t* last_idx, void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/* image_render.backward then pts_splatting.backward for surfels (Alg. 1 lines 17-18, 22-24); arguments and the
 * scene/grads NULL rule and the g_splats NULL rule (64-byte records here) as pbdr_render_bwd. */
int pbdr2d_render_bwd(const pbdr2d_scene* scene, const pbdr2d_splats* splats, const pbdr_camera* cam, const float bg[3],
                      uint64_t dup_capacity, const float* final_T, const uint32_t* last_idx, const float* dL_dimage,
                      pbdr2d_splat_grads* g_splats, pbdr2d_scene_grads* grads, void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/* pts_splatting.backward alone for surfels; accumulates into grads. */
int pbdr2d_preprocess_bwd(const pbdr2d_scene* scene, const pbdr_camera* cam, const pbdr2d_splats* splats,
                          const pbdr2d_splat_grads* g_splats, pbdr2d_scene_grads* grads, void* hip_stream);

/* Image patches for surfels: as pbdr_preprocess_patch / pbdr_render_fwd_patch / pbdr_render_bwd_patch (App. D.2 restricts
 * the kernels of every evaluated algorithm to a patch); workspace sized by pbdr2d_workspace_bytes for the whole image. */
int pbdr2d_preprocess_patch(const pbdr2d_scene* scene, const pbdr_camera* cam, const pbdr_patch* patch, pbdr2d_splats* out,
                            void* hip_stream);
int pbdr2d_render_fwd_patch(const pbdr2d_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                            uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                            size_t workspace_bytes, void* hip_stream);
int pbdr2d_render_bwd_patch(const pbdr2d_scene* scene, const pbdr2d_splats* splats, const pbdr_camera* cam,
                            const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                            const uint32_t* last_idx, const float* dL_dimage, pbdr2d_splat_grads* g_splats,
                            pbdr2d_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream);

/* As pbdr_lists_view, for a workspace used by pbdr2d_render_fwd. */
int pbdr2d_lists_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                      uint64_t dup_capacity, void* hip_stream, const uint64_t** keys, const uint32_t** vals,
                      const uint32_t** ranges, const uint32_t** num_dup);

/* As pbdr_render_stats, for a workspace used by pbdr2d_render_fwd. */
int pbdr2d_render_stats(const pbdr_camera* cam, int32_t n, uint64_t dup_capacity, uint64_t* counters, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------------------------------
 * The two steps of a training iteration around the rasterizer (Alg. 1): loss and parameter update. The paper names
 * them only (loss_fn, loss_fn.backward, AdamUpdate; App. E.1: the "selective" Adam); the readings here, stated by the
 * CPU oracle too: mean-L1 loss against the target image (what the benchmark configurations use), and the textbook
 * Adam update with bias correction applied to the points that were visible in the batch, every other point's
 * parameter and moments left untouched.
 *
 * pbdr_l1_loss (Alg. 1 lines 13 and 16, one pass): *loss += mean |image - target| over the 3 x H x W values (device
 * float, accumulated like line 14's loss_total; the caller zeroes it), dL_dimage = sign(image - target) / (3 H W),
 * zero where they are equal. image, target, dL_dimage: [3][H][W]. For a patch pass the patch's width and height.
 *
 * pbdr_mark_visible: visible[i] = 1 where radius[i] > 0, other entries kept: called once per view of a batch on a
 * zeroed uint8 [n], it leaves the union of the points the batch's views use.
 *
 * pbdr_adam_selective (Alg. 1 line 27) on one attribute tensor of `planes` planes, [planes][n]: for each point i with
 * visible[i] != 0 and each plane,  m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
 * param -= lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps);  step counts from 1. If zero_grad != 0 the
 * gradient entries that were consumed are set to zero (Alg. 1 line 21 for the next iteration: entries of invisible
 * points are zero already, nothing accumulated into them). A point that is not visible costs one byte read. */
typedef struct pbdr_adam_config {
    float lr, beta1, beta2, eps;
    int32_t step;
    int32_t zero_grad;
} pbdr_adam_config;

int pbdr_l1_loss(int32_t width, int32_t height, const float* image, const float* target, float* loss, float* dL_dimage,
                 void* hip_stream);
int pbdr_mark_visible(int32_t n, const int32_t* radius, uint8_t* visible, void* hip_stream);
int pbdr_adam_selective(int32_t n, int32_t planes, float* param, float* grad, float* exp_avg, float* exp_avg_sq,
                        const uint8_t* visible, const pbdr_adam_config* cfg, void* hip_stream);

/* pts_splatting.backward for the views of a batch and the optimizer step in one pass over the points (Alg. 1 lines
 * 21-27): exactly what pbdr_preprocess_bwd_batch with first_view = 1, pbdr_mark_visible once per view and
 * pbdr_adam_selective once per attribute do, bit for bit, without the parameter gradient going through memory.
 * The arrays `scene` points to are UPDATED IN PLACE for the points at least one view uses (radius > 0); exp_avg and
 * exp_avg_sq are the two Adam moments, laid out like the scene (their first_view field is ignored). lr[5]: learning
 * rates of mean, log_scale, quat, opacity_logit, sh. Of cfg, beta1, beta2, eps and step are used. */
int pbdr_preprocess_bwd_batch_adam(const pbdr_scene* scene, int32_t num_views, const pbdr_camera* cams, const pbdr_splats* splats,
                                   const pbdr_splat_grads* g_splats, pbdr_scene_grads* exp_avg, pbdr_scene_grads* exp_avg_sq,
                                   const float lr[5], const pbdr_adam_config* cfg, void* hip_stream);

/* Optional per-kernel timing for benchmarks, with HIP events recorded on the stream each kernel is launched on.
 * kernel_mask: bit i enables kernel id i (ids 0 .. pbdr_profile_kernel_count()-1, names from
 * pbdr_profile_kernel_name). At most max_records launches are timed between begin/reset and collect.
 * collect synchronises the recorded events and returns the summed duration and number of records of one kernel id.
 * Process-global and not thread-safe; creates HIP events (host objects), no device memory. */
int pbdr_profile_begin(uint32_t kernel_mask, int32_t max_records);
int pbdr_profile_collect(int32_t kernel_id, double* total_ms, int32_t* records);
int pbdr_profile_reset(void);
int pbdr_profile_end(void);
const char* pbdr_profile_kernel_name(int32_t kernel_id);
int pbdr_profile_kernel_count(void);

const char* pbdr_status_string(int status);
int pbdr_last_hip_error(void); /* hipError_t of the most recent PBDR_ERR_HIP on this thread */
int pbdr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PBDR_H */
