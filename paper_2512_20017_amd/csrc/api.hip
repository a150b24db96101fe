// C ABI of libpbdr: argument checks, workspace layout, camera conversion, kernel sequencing. No allocation here.
#include "../../include/pbdr.h"
#include "pbdr_internal.h"

#include <cmath>
#include <mutex>

namespace pbdr {

// Workspace of pbdr_render_fwd_static: part of the library's device image, one copy per GPU. Host code never uses this
// name as an address; static_scratch() asks the runtime where the current device keeps its copy.
static __device__ __align__(256) unsigned char scratch[PBDR_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];      // per device, filled on first use
static std::mutex g_scratch_mutex;

static hipError_t static_scratch(void** out)
{
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr || (reinterpret_cast<uintptr_t>(p) & 255u) != 0) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

__global__ __launch_bounds__(256) void k_zero_fill(uint4* __restrict__ p, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (size_t)gridDim.x * 256) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ void k_copy_word(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = *src;
}

static thread_local int g_last_hip_error = 0;

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

bool make_layout(int n, int W, int H, uint64_t cap, int variant, Layout* L)
{
    if (n < 0 || W <= 0 || H <= 0 || W > 65536 || H > 65536) return false;
    if (cap == 0) cap = 1;
    if (cap > 0x3fffffffull) return false;
    L->n = n; L->W = W; L->H = H;
    L->variant = variant;
    L->record_bytes = variant == kVariant2D ? 64 : sizeof(Packed);
    L->partial_vec4 = variant == kVariant2D ? 4 : 3;
    L->TX = (W + kTile - 1) / kTile; L->TY = (H + kTile - 1) / kTile;
    L->tiles = L->TX * L->TY;
    L->cap = (uint32_t)cap;
    L->tile_bits = 0;
    while ((1 << L->tile_bits) < L->tiles) ++L->tile_bits;
    L->tile_passes = radix_pass_count(L->tile_bits);
    const size_t nblk_t = ((size_t)cap + kSortItems - 1) / kSortItems;
    size_t off = 0;
    const auto take = [&](size_t bytes) { const size_t at = off; off = align256(off + bytes); return at; };
    L->off_status = take(kStWords * sizeof(uint32_t));
    L->off_packed = take((size_t)n * L->record_bytes);
    L->off_depth_bits = take((size_t)n * sizeof(uint32_t));
    L->off_blk_vis = take(((size_t)n / 256 + 8) * sizeof(uint32_t));
    L->off_blk_pairs = take(((size_t)n / 256 + 8) * sizeof(uint32_t));
    L->off_blk_vis_at = take(((size_t)n / 256 + 8) * sizeof(uint32_t));  // exclusive sums of the two above
    L->off_blk_pairs_at = take(((size_t)n / 256 + 8) * sizeof(uint32_t));
    L->off_blk_order = take(((size_t)n / 256 + 8) * sizeof(uint32_t));   // blocks of points in the order the packing kernel takes them
    L->off_touched = take((size_t)n * sizeof(uint32_t));
    L->off_offsets = take(((size_t)n + 1) * sizeof(uint32_t));
    L->off_slot_base = take((size_t)n * sizeof(uint32_t));
    L->off_order = take((size_t)n * sizeof(uint32_t));       // listed points in index order ("rank" -> point)
    L->off_tkey0 = take((size_t)cap * sizeof(uint32_t));
    L->off_tval0 = take((size_t)cap * sizeof(uint32_t));
    L->off_tkey1 = take((size_t)cap * sizeof(uint32_t));
    L->off_tval1 = take((size_t)cap * sizeof(uint32_t));
    L->off_totals = take((size_t)kRadixMaxBins * sizeof(uint32_t));      // digit totals of a pass of the tile sort
    L->off_tile_hist = take(nblk_t * kRadixMaxBins * sizeof(uint32_t));
    L->off_ranges = take((size_t)L->tiles * 2 * sizeof(uint32_t));
    L->off_partial = take((size_t)cap * L->partial_vec4 * 4 * sizeof(float));
    L->off_keys64 = take((size_t)cap * sizeof(uint64_t));
    L->off_chunk_rank = take(((size_t)cap / 256 + 2) * sizeof(uint32_t));         // see pair_reduce.h
    L->off_carry = take(((size_t)cap / 256 + 2) * 36 * sizeof(float));
    L->off_grad_rec = take((size_t)n * L->partial_vec4 * 4 * sizeof(float));      // per-point gradient records, by point index
    L->off_reach = take((size_t)4 * cap);  // per sorted pair and quadrant of its tile: can the splat reach it (forward -> backward)
    L->off_tile_order = take((size_t)L->tiles * sizeof(uint32_t));   // tiles in the order the compositing kernels take them
    L->total = off;
    return true;
}

static inline bool aligned16(const void* p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static bool check_camera(const pbdr_camera* cam)
{
    if (!cam) return false;
    if (cam->width <= 0 || cam->height <= 0 || cam->width > 65536 || cam->height > 65536) return false;
    if (!(cam->fx > 0.f) || !(cam->fy > 0.f) || !(cam->near_plane > 0.f) || !(cam->far_plane > cam->near_plane)) return false;
    if (!(cam->radius_clip >= 0.f)) return false;
    for (int i = 0; i < 9; ++i) if (!std::isfinite(cam->R[i])) return false;
    for (int i = 0; i < 3; ++i) if (!std::isfinite(cam->t[i])) return false;
    return std::isfinite(cam->cx) && std::isfinite(cam->cy);
}

static bool check_patch(const pbdr_camera* cam, const pbdr_patch* p)
{
    return p && p->x0 >= 0 && p->y0 >= 0 && p->x0 < p->x1 && p->y0 < p->y1 && p->x1 <= cam->width && p->y1 <= cam->height;
}

// patch == nullptr: the whole image
static CamDev to_dev(const pbdr_camera* cam, const pbdr_patch* patch = nullptr)
{
    CamDev c;
    const pbdr_patch whole = {0, 0, cam->width, cam->height};
    const pbdr_patch& r = patch ? *patch : whole;
    c.W = r.x1 - r.x0; c.H = r.y1 - r.y0;
    c.rx0 = r.x0; c.ry0 = r.y0; c.rx1 = r.x1; c.ry1 = r.y1;
    c.otx = r.x0 / kTile; c.oty = r.y0 / kTile;
    c.TX = (r.x1 + kTile - 1) / kTile - c.otx; c.TY = (r.y1 + kTile - 1) / kTile - c.oty;
    c.fx = cam->fx; c.fy = cam->fy; c.cx = cam->cx; c.cy = cam->cy;
    for (int i = 0; i < 9; ++i) c.R[i] = cam->R[i];
    for (int i = 0; i < 3; ++i) c.t[i] = cam->t[i];
    for (int i = 0; i < 3; ++i)   // camera centre = -R^T t, formed in double on the host
        c.campos[i] = (float)(-((double)cam->R[i] * cam->t[0] + (double)cam->R[3 + i] * cam->t[1] + (double)cam->R[6 + i] * cam->t[2]));
    c.near_p = cam->near_plane; c.far_p = cam->far_plane; c.radius_clip = cam->radius_clip;
    c.lim_x = (float)((double)kGuard * 0.5 * cam->width / cam->fx);
    c.lim_y = (float)((double)kGuard * 0.5 * cam->height / cam->fy);
    return c;
}

static bool check_scene(const pbdr_scene* sc)
{
    if (!sc || sc->n < 0 || sc->sh_degree < 0 || sc->sh_degree > 3) return false;
    if (sc->n == 0) return true;
    return aligned16(sc->mean) && aligned16(sc->log_scale) && aligned16(sc->quat) && aligned16(sc->opacity_logit) && aligned16(sc->sh);
}
static bool check_scene_grads(const pbdr_scene_grads* g, const pbdr_scene* sc)
{
    if (!g || g->n != sc->n || g->sh_degree != sc->sh_degree) return false;
    if (g->n == 0) return true;
    return aligned16(g->mean) && aligned16(g->log_scale) && aligned16(g->quat) && aligned16(g->opacity_logit) && aligned16(g->sh);
}
static bool check_splats(const pbdr_splats* sp)
{
    if (!sp || sp->n < 0) return false;
    if (sp->n == 0) return true;
    return aligned16(sp->mean2d) && aligned16(sp->conic) && aligned16(sp->opacity) && aligned16(sp->color) &&
           aligned16(sp->radius) && aligned16(sp->depth);
}
static bool check_splat_grads(const pbdr_splat_grads* g, int n)
{
    if (!g || g->n != n) return false;
    if (n == 0) return true;
    return aligned16(g->mean2d) && aligned16(g->conic) && aligned16(g->opacity) && aligned16(g->color);
}

static SceneDev dev(const pbdr_scene* s) { return SceneDev{s->n, s->sh_degree, s->mean, s->log_scale, s->quat, s->opacity_logit, s->sh}; }
static SceneGradDev dev(const pbdr_scene_grads* g) { return SceneGradDev{g->mean, g->log_scale, g->quat, g->opacity_logit, g->sh}; }
static SplatsDev dev(const pbdr_splats* s) { return SplatsDev{s->n, s->mean2d, s->conic, s->opacity, s->color, s->radius, s->depth}; }
static SplatGradDev dev(const pbdr_splat_grads* g) { return SplatGradDev{g->mean2d, g->conic, g->opacity, g->color}; }

static bool check_scene2d(const pbdr2d_scene* sc)
{
    if (!sc || sc->n < 0 || sc->sh_degree < 0 || sc->sh_degree > 3) return false;
    if (sc->n == 0) return true;
    return aligned16(sc->mean) && aligned16(sc->tan_u) && aligned16(sc->tan_v) && aligned16(sc->log_scale) &&
           aligned16(sc->opacity_logit) && aligned16(sc->sh);
}
static bool check_scene2d_grads(const pbdr2d_scene_grads* g, const pbdr2d_scene* sc)
{
    if (!g || g->n != sc->n || g->sh_degree != sc->sh_degree) return false;
    if (g->n == 0) return true;
    return aligned16(g->mean) && aligned16(g->tan_u) && aligned16(g->tan_v) && aligned16(g->log_scale) &&
           aligned16(g->opacity_logit) && aligned16(g->sh);
}
static bool check_splats2d(const pbdr2d_splats* sp)
{
    if (!sp || sp->n < 0) return false;
    if (sp->n == 0) return true;
    return aligned16(sp->mean2d) && aligned16(sp->ray_transform) && aligned16(sp->opacity) && aligned16(sp->color) &&
           aligned16(sp->radius) && aligned16(sp->depth) && aligned16(sp->normal);
}
static bool check_splat2d_grads(const pbdr2d_splat_grads* g, int n)
{
    if (!g || g->n != n) return false;
    if (n == 0) return true;
    return aligned16(g->mean2d) && aligned16(g->ray_transform) && aligned16(g->opacity) && aligned16(g->color);
}
static Scene2DDev dev(const pbdr2d_scene* s)
{
    return Scene2DDev{s->n, s->sh_degree, s->mean, s->tan_u, s->tan_v, s->log_scale, s->opacity_logit, s->sh};
}
static Scene2DGradDev dev(const pbdr2d_scene_grads* g) { return Scene2DGradDev{g->mean, g->tan_u, g->tan_v, g->log_scale, g->opacity_logit, g->sh}; }
static Splats2DDev dev(const pbdr2d_splats* s)
{
    return Splats2DDev{s->n, s->mean2d, s->ray_transform, s->opacity, s->color, s->radius, s->depth, s->normal};
}
static Splat2DGradDev dev(const pbdr2d_splat_grads* g) { return Splat2DGradDev{g->mean2d, g->ray_transform, g->opacity, g->color}; }

static int hip_result(hipError_t e)
{
    if (e == hipSuccess) return PBDR_OK;
    g_last_hip_error = (int)e;
    return PBDR_ERR_HIP;
}

static int workspace_ok(void* ws, size_t bytes, int n, int W, int H, uint64_t cap, Layout* L, int variant = kVariant3D)
{
    if (!make_layout(n, W, H, cap, variant, L)) return PBDR_ERR_INVALID_ARG;
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return PBDR_ERR_INVALID_ARG;
    if (bytes < L->total) return PBDR_ERR_WORKSPACE_TOO_SMALL;
    return PBDR_OK;
}

}  // namespace pbdr

using namespace pbdr;

extern "C" {

int pbdr_version(void) { return PBDR_VERSION; }

int pbdr_last_hip_error(void) { return g_last_hip_error; }

const char* pbdr_status_string(int status)
{
    switch (status) {
        case PBDR_OK: return "ok";
        case PBDR_ERR_INVALID_ARG: return "invalid argument";
        case PBDR_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case PBDR_ERR_CAPACITY: return "more (tile, splat) pairs than dup_capacity";
        case PBDR_ERR_HIP: return "HIP error";
        case PBDR_ERR_STATIC_LIMIT: return "more points or a larger image than the static scratch buffer serves";
        default: return "unknown status";
    }
}

int pbdr_workspace_init(void* workspace, size_t bytes, void* hip_stream)
{
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 15u) != 0 || (bytes & 15u) != 0) return PBDR_ERR_INVALID_ARG;
    if (bytes == 0) return PBDR_OK;
    const size_t count = bytes / 16;
    const unsigned blocks = (unsigned)((count + 255) / 256 < 16384 ? (count + 255) / 256 : 16384);
    hipLaunchKernelGGL(k_zero_fill, dim3(blocks), dim3(256), 0, (hipStream_t)hip_stream, reinterpret_cast<uint4*>(workspace), count);
    return hip_result(hipGetLastError());
}

int pbdr_status_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                     uint64_t dup_capacity, const uint32_t** status_words)
{
    Layout L;
    if (!status_words) return PBDR_ERR_INVALID_ARG;
    // the status block heads both kinds of workspace; the 3D layout is the smaller one, so its size check serves both
    const int st = workspace_ok(workspace, workspace_bytes, n, width, height, dup_capacity, &L);
    if (st != PBDR_OK) return st;
    *status_words = reinterpret_cast<const uint32_t*>((char*)workspace + L.off_status);
    return PBDR_OK;
}

int pbdr_workspace_bytes(int32_t n, int32_t width, int32_t height, uint64_t dup_capacity, size_t* out_bytes)
{
    Layout L;
    if (!out_bytes || !make_layout(n, width, height, dup_capacity, kVariant3D, &L)) return PBDR_ERR_INVALID_ARG;
    *out_bytes = L.total;
    return PBDR_OK;
}

static int preprocess_impl(const pbdr_scene* scene, const pbdr_camera* cam, const pbdr_patch* patch, pbdr_splats* out,
                           void* hip_stream)
{
    if (!check_scene(scene) || !check_camera(cam) || !check_splats(out) || out->n != scene->n) return PBDR_ERR_INVALID_ARG;
    if (patch && !check_patch(cam, patch)) return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_preprocess(dev(scene), to_dev(cam, patch), dev(out), nullptr, 0, (hipStream_t)hip_stream));
}

int pbdr_preprocess(const pbdr_scene* scene, const pbdr_camera* cam, pbdr_splats* out, void* hip_stream)
{
    return preprocess_impl(scene, cam, nullptr, out, hip_stream);
}

int pbdr_preprocess_patch(const pbdr_scene* scene, const pbdr_camera* cam, const pbdr_patch* patch, pbdr_splats* out,
                          void* hip_stream)
{
    if (!patch) return PBDR_ERR_INVALID_ARG;
    return preprocess_impl(scene, cam, patch, out, hip_stream);
}

static bool check_group_size(int32_t group_size)
{
    return group_size >= 256 && group_size <= (1 << 20) && (group_size % 256) == 0;
}

int pbdr_group_count(int32_t n, int32_t group_size)
{
    if (n < 0 || !check_group_size(group_size)) return PBDR_ERR_INVALID_ARG;
    return (int)(((int64_t)n + group_size - 1) / group_size);
}

int pbdr_group_bounds(const pbdr_scene* scene, int32_t group_size, float* bounds, void* hip_stream)
{
    if (!check_scene(scene) || !check_group_size(group_size)) return PBDR_ERR_INVALID_ARG;
    if (scene->n > 0 && !aligned16(bounds)) return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_group_bounds(dev(scene), group_size, bounds, (hipStream_t)hip_stream));
}

int pbdr_preprocess_grouped(const pbdr_scene* scene, const pbdr_camera* cam, int32_t group_size, const float* bounds,
                            uint8_t* keep, pbdr_splats* out, void* hip_stream)
{
    if (!check_scene(scene) || !check_camera(cam) || !check_splats(out) || out->n != scene->n || !check_group_size(group_size))
        return PBDR_ERR_INVALID_ARG;
    if (scene->n == 0) return PBDR_OK;
    if (!aligned16(bounds) || !aligned16(keep)) return PBDR_ERR_INVALID_ARG;
    const CamDev c = to_dev(cam);
    const int ng = (int)(((int64_t)scene->n + group_size - 1) / group_size);
    const hipError_t e = launch_group_cull(c, ng, bounds, keep, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_result(e);
    return hip_result(launch_preprocess(dev(scene), c, dev(out), keep, group_size, (hipStream_t)hip_stream));
}

int pbdr_preprocess_batch(const pbdr_scene* scene, int32_t num_views, const pbdr_camera* cams, const pbdr_splats* outs,
                          int32_t group_size, const float* bounds, uint8_t* keep, void* hip_stream)
{
    if (!check_scene(scene) || num_views < 1 || num_views > PBDR_MAX_BATCH_VIEWS || !cams || !outs) return PBDR_ERR_INVALID_ARG;
    if (group_size != 0 && !check_group_size(group_size)) return PBDR_ERR_INVALID_ARG;
    BatchCams bc;
    BatchSplats bs;
    bc.count = num_views;
    for (int v = 0; v < num_views; ++v) {
        if (!check_camera(&cams[v]) || !check_splats(&outs[v]) || outs[v].n != scene->n) return PBDR_ERR_INVALID_ARG;
        bc.cam[v] = to_dev(&cams[v]);
        bs.view[v] = dev(&outs[v]);
    }
    for (int v = num_views; v < kMaxBatchViews; ++v) { bc.cam[v] = bc.cam[0]; bs.view[v] = bs.view[0]; }
    if (scene->n == 0) return PBDR_OK;
    const uint8_t* use_keep = nullptr;
    if (group_size != 0) {
        if (!aligned16(bounds) || !aligned16(keep)) return PBDR_ERR_INVALID_ARG;
        const int ng = (int)(((int64_t)scene->n + group_size - 1) / group_size);
        const hipError_t e = launch_group_cull_batch(bc, ng, bounds, keep, (hipStream_t)hip_stream);
        if (e != hipSuccess) return hip_result(e);
        use_keep = keep;
    }
    return hip_result(launch_preprocess_batch(dev(scene), bc, bs, use_keep, group_size, (hipStream_t)hip_stream));
}

int pbdr_preprocess_bwd_batch(const pbdr_scene* scene, int32_t num_views, const pbdr_camera* cams, const pbdr_splats* splats,
                              const pbdr_splat_grads* g_splats, pbdr_scene_grads* grads, void* hip_stream)
{
    if (!check_scene(scene) || num_views < 1 || num_views > PBDR_MAX_BATCH_VIEWS || !cams || !splats || !g_splats ||
        !check_scene_grads(grads, scene))
        return PBDR_ERR_INVALID_ARG;
    BatchCams bc;
    BatchSplatGrads bg;
    bc.count = num_views;
    for (int v = 0; v < num_views; ++v) {
        if (!check_camera(&cams[v]) || !check_splats(&splats[v]) || splats[v].n != scene->n ||
            !check_splat_grads(&g_splats[v], scene->n))
            return PBDR_ERR_INVALID_ARG;
        bc.cam[v] = to_dev(&cams[v]);
        bg.radius[v] = splats[v].radius;
        bg.grad[v] = dev(&g_splats[v]);
    }
    for (int v = num_views; v < kMaxBatchViews; ++v) { bc.cam[v] = bc.cam[0]; bg.radius[v] = bg.radius[0]; bg.grad[v] = bg.grad[0]; }
    return hip_result(launch_preprocess_bwd_batch(dev(scene), bc, bg, dev(grads), grads->first_view != 0, (hipStream_t)hip_stream));
}

int pbdr_bin_sort(const pbdr_splats* splats, const pbdr_camera* cam, uint64_t dup_capacity, void* workspace,
                  size_t workspace_bytes, void* hip_stream)
{
    if (!check_splats(splats) || !check_camera(cam)) return PBDR_ERR_INVALID_ARG;
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, splats->n, cam->width, cam->height, dup_capacity, &L);
    if (st != PBDR_OK) return st;
    return hip_result(launch_bin_sort(dev(splats), to_dev(cam), L, (char*)workspace, (hipStream_t)hip_stream));
}

static int render_fwd_impl(const pbdr_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                           uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

int pbdr_render_fwd(const pbdr_splats* splats, const pbdr_camera* cam, const float bg[3], uint64_t dup_capacity,
                    float* image, float* final_T, uint32_t* last_idx, void* workspace, size_t workspace_bytes,
                    void* hip_stream)
{
    return render_fwd_impl(splats, cam, nullptr, bg, dup_capacity, image, final_T, last_idx, workspace, workspace_bytes, hip_stream);
}

int pbdr_render_fwd_patch(const pbdr_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                          uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                          size_t workspace_bytes, void* hip_stream)
{
    if (!patch) return PBDR_ERR_INVALID_ARG;
    return render_fwd_impl(splats, cam, patch, bg, dup_capacity, image, final_T, last_idx, workspace, workspace_bytes, hip_stream);
}

static int render_fwd_impl(const pbdr_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                           uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                           size_t workspace_bytes, void* hip_stream)
{
    if (!check_splats(splats) || !check_camera(cam) || !bg || !aligned16(image) || !aligned16(final_T) || !aligned16(last_idx))
        return PBDR_ERR_INVALID_ARG;
    if (patch && !check_patch(cam, patch)) return PBDR_ERR_INVALID_ARG;
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, splats->n, cam->width, cam->height, dup_capacity, &L);
    if (st != PBDR_OK) return st;
    const CamDev c = to_dev(cam, patch);
    hipError_t e = launch_bin_sort(dev(splats), c, L, (char*)workspace, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_result(e);
    return hip_result(launch_composite_fwd(c, L, (char*)workspace, bg, image, final_T, last_idx, (hipStream_t)hip_stream));
}

int pbdr_render_fwd_static(const pbdr_splats* splats, const pbdr_camera* cam, const float bg[3], float* image,
                           float* final_T, uint32_t* last_idx, uint32_t* pair_count, void* hip_stream)
{
    if (!check_splats(splats) || !check_camera(cam) || !bg || !aligned16(image) || !aligned16(final_T) || !aligned16(last_idx))
        return PBDR_ERR_INVALID_ARG;
    if (pair_count && (reinterpret_cast<uintptr_t>(pair_count) & 3u)) return PBDR_ERR_INVALID_ARG;
    if (splats->n > PBDR_STATIC_MAX_POINTS || cam->width > PBDR_STATIC_MAX_SIDE || cam->height > PBDR_STATIC_MAX_SIDE)
        return PBDR_ERR_STATIC_LIMIT;
    Layout L;
    if (!make_layout(splats->n, cam->width, cam->height, PBDR_STATIC_MAX_PAIRS, kVariant3D, &L)) return PBDR_ERR_INVALID_ARG;
    if (L.total > (size_t)PBDR_STATIC_SCRATCH_BYTES) return PBDR_ERR_STATIC_LIMIT;
    void* ws = nullptr;
    hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return hip_result(e);
    // nothing of the array needs clearing here: binning's first kernel zeroes the status words and the tile ranges,
    // and every other part is written by this call before this call reads it
    const CamDev c = to_dev(cam);
    e = launch_bin_sort(dev(splats), c, L, (char*)ws, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_result(e);
    e = launch_composite_fwd(c, L, (char*)ws, bg, image, final_T, last_idx, (hipStream_t)hip_stream);
    if (e != hipSuccess || !pair_count) return hip_result(e);
    hipLaunchKernelGGL(k_copy_word, dim3(1), dim3(64), 0, (hipStream_t)hip_stream,
                       reinterpret_cast<const uint32_t*>((char*)ws + L.off_status) + kStNumDup, pair_count);
    return hip_result(hipGetLastError());
}

int pbdr_preprocess_bwd(const pbdr_scene* scene, const pbdr_camera* cam, const pbdr_splats* splats,
                        const pbdr_splat_grads* g_splats, pbdr_scene_grads* grads, void* hip_stream)
{
    if (!check_scene(scene) || !check_camera(cam) || !check_splats(splats) || splats->n != scene->n ||
        !check_splat_grads(g_splats, scene->n) || !check_scene_grads(grads, scene))
        return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_preprocess_bwd(dev(scene), to_dev(cam), splats->radius, dev(g_splats), dev(grads),
                                            grads->first_view != 0, (hipStream_t)hip_stream));
}

static int render_bwd_impl(const pbdr_scene* scene, const pbdr_splats* splats, const pbdr_camera* cam,
                           const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                           const uint32_t* last_idx, const float* dL_dimage, pbdr_splat_grads* g_splats,
                           pbdr_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream);

int pbdr_render_bwd(const pbdr_scene* scene, const pbdr_splats* splats, const pbdr_camera* cam, const float bg[3],
                    uint64_t dup_capacity, const float* final_T, const uint32_t* last_idx, const float* dL_dimage,
                    pbdr_splat_grads* g_splats, pbdr_scene_grads* grads, void* workspace, size_t workspace_bytes,
                    void* hip_stream)
{
    return render_bwd_impl(scene, splats, cam, nullptr, bg, dup_capacity, final_T, last_idx, dL_dimage, g_splats, grads,
                           workspace, workspace_bytes, hip_stream);
}

int pbdr_render_bwd_patch(const pbdr_scene* scene, const pbdr_splats* splats, const pbdr_camera* cam,
                          const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                          const uint32_t* last_idx, const float* dL_dimage, pbdr_splat_grads* g_splats,
                          pbdr_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!patch) return PBDR_ERR_INVALID_ARG;
    return render_bwd_impl(scene, splats, cam, patch, bg, dup_capacity, final_T, last_idx, dL_dimage, g_splats, grads,
                           workspace, workspace_bytes, hip_stream);
}

static int render_bwd_impl(const pbdr_scene* scene, const pbdr_splats* splats, const pbdr_camera* cam,
                           const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                           const uint32_t* last_idx, const float* dL_dimage, pbdr_splat_grads* g_splats,
                           pbdr_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!check_splats(splats) || !check_camera(cam) || !bg || !aligned16(final_T) || !aligned16(last_idx) || !aligned16(dL_dimage))
        return PBDR_ERR_INVALID_ARG;
    if (g_splats ? !check_splat_grads(g_splats, splats->n) : scene == nullptr) return PBDR_ERR_INVALID_ARG;
    if (patch && !check_patch(cam, patch)) return PBDR_ERR_INVALID_ARG;
    if ((scene == nullptr) != (grads == nullptr)) return PBDR_ERR_INVALID_ARG;
    if (scene && (!check_scene(scene) || scene->n != splats->n || !check_scene_grads(grads, scene))) return PBDR_ERR_INVALID_ARG;
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, splats->n, cam->width, cam->height, dup_capacity, &L);
    if (st != PBDR_OK) return st;
    const CamDev c = to_dev(cam, patch);
    const SplatGradDev g2 = g_splats ? dev(g_splats) : SplatGradDev{nullptr, nullptr, nullptr, nullptr};
    hipError_t e = launch_composite_bwd(c, L, (char*)workspace, splats->n, bg, final_T, last_idx, dL_dimage, g2, (hipStream_t)hip_stream);
    if (e != hipSuccess || !scene) return hip_result(e);
    if (!g_splats)      // no splat-state gradient asked for: the splatting backward reads the workspace's per-point records
        return hip_result(launch_preprocess_bwd_records(dev(scene), c, reinterpret_cast<const uint32_t*>((char*)workspace + L.off_touched),
                                                        reinterpret_cast<const float4*>((char*)workspace + L.off_grad_rec),
                                                        carry_fold(L, (char*)workspace), dev(grads), grads->first_view != 0,
                                                        (hipStream_t)hip_stream));
    // g_splats holds this call's values for exactly the points binning listed (tile count > 0), so those, not
    // radius > 0, are the points the second half may read: a whole-image state rendered through a patch, or a
    // caller-made state with an empty tile rectangle, has radius > 0 points that were never listed
    return hip_result(launch_preprocess_bwd(dev(scene), c, reinterpret_cast<const int32_t*>((char*)workspace + L.off_touched), g2,
                                            dev(grads), grads->first_view != 0, (hipStream_t)hip_stream));
}

int pbdr_render_stats(const pbdr_camera* cam, int32_t n, uint64_t dup_capacity, uint64_t* counters, void* workspace,
                      size_t workspace_bytes, void* hip_stream)
{
    if (!check_camera(cam) || !aligned16(counters)) return PBDR_ERR_INVALID_ARG;
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, n, cam->width, cam->height, dup_capacity, &L);
    if (st != PBDR_OK) return st;
    return hip_result(launch_render_stats(to_dev(cam), L, (char*)workspace, counters, (hipStream_t)hip_stream));
}

static int lists_view(int variant, void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                      uint64_t dup_capacity, void* hip_stream, const uint64_t** keys, const uint32_t** vals,
                      const uint32_t** ranges, const uint32_t** num_dup)
{
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, n, width, height, dup_capacity, &L, variant);
    if (st != PBDR_OK) return st;
    char* ws = (char*)workspace;
    if (keys) {
        if (n > 0) {
            const hipError_t e = launch_make_keys64(L, ws, (hipStream_t)hip_stream);
            if (e != hipSuccess) return hip_result(e);
        }
        *keys = reinterpret_cast<const uint64_t*>(ws + L.off_keys64);
    }
    if (vals) *vals = reinterpret_cast<const uint32_t*>(ws + sorted_vals_off(L));
    if (ranges) *ranges = reinterpret_cast<const uint32_t*>(ws + L.off_ranges);
    if (num_dup) *num_dup = reinterpret_cast<const uint32_t*>(ws + L.off_status) + kStNumDup;
    return PBDR_OK;
}

int pbdr_tile_order_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                         uint64_t dup_capacity, int32_t surfel_workspace, const uint32_t** tile_order)
{
    Layout L;
    if (!tile_order) return PBDR_ERR_INVALID_ARG;
    const int st = workspace_ok(workspace, workspace_bytes, n, width, height, dup_capacity, &L, surfel_workspace ? kVariant2D : kVariant3D);
    if (st != PBDR_OK) return st;
    *tile_order = reinterpret_cast<const uint32_t*>((char*)workspace + L.off_tile_order);
    return PBDR_OK;
}

int pbdr_lists_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                    uint64_t dup_capacity, void* hip_stream, const uint64_t** keys, const uint32_t** vals,
                    const uint32_t** ranges, const uint32_t** num_dup)
{
    return lists_view(kVariant3D, workspace, workspace_bytes, n, width, height, dup_capacity, hip_stream, keys, vals, ranges, num_dup);
}

int pbdr2d_lists_view(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                      uint64_t dup_capacity, void* hip_stream, const uint64_t** keys, const uint32_t** vals,
                      const uint32_t** ranges, const uint32_t** num_dup)
{
    return lists_view(kVariant2D, workspace, workspace_bytes, n, width, height, dup_capacity, hip_stream, keys, vals, ranges, num_dup);
}

int pbdr2d_workspace_bytes(int32_t n, int32_t width, int32_t height, uint64_t dup_capacity, size_t* out_bytes)
{
    Layout L;
    if (!out_bytes || !make_layout(n, width, height, dup_capacity, kVariant2D, &L)) return PBDR_ERR_INVALID_ARG;
    *out_bytes = L.total;
    return PBDR_OK;
}

static int preprocess2d_impl(const pbdr2d_scene* scene, const pbdr_camera* cam, const pbdr_patch* patch, pbdr2d_splats* out,
                             void* hip_stream)
{
    if (!check_scene2d(scene) || !check_camera(cam) || !check_splats2d(out) || out->n != scene->n) return PBDR_ERR_INVALID_ARG;
    if (patch && !check_patch(cam, patch)) return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_preprocess2d(dev(scene), to_dev(cam, patch), dev(out), (hipStream_t)hip_stream));
}

int pbdr2d_preprocess(const pbdr2d_scene* scene, const pbdr_camera* cam, pbdr2d_splats* out, void* hip_stream)
{
    return preprocess2d_impl(scene, cam, nullptr, out, hip_stream);
}

int pbdr2d_preprocess_patch(const pbdr2d_scene* scene, const pbdr_camera* cam, const pbdr_patch* patch, pbdr2d_splats* out,
                            void* hip_stream)
{
    if (!patch) return PBDR_ERR_INVALID_ARG;
    return preprocess2d_impl(scene, cam, patch, out, hip_stream);
}

static int render2d_fwd_impl(const pbdr2d_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                             uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                             size_t workspace_bytes, void* hip_stream);

int pbdr2d_render_fwd(const pbdr2d_splats* splats, const pbdr_camera* cam, const float bg[3], uint64_t dup_capacity,
                      float* image, float* final_T, uint32_t* last_idx, void* workspace, size_t workspace_bytes,
                      void* hip_stream)
{
    return render2d_fwd_impl(splats, cam, nullptr, bg, dup_capacity, image, final_T, last_idx, workspace, workspace_bytes, hip_stream);
}

int pbdr2d_render_fwd_patch(const pbdr2d_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                            uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                            size_t workspace_bytes, void* hip_stream)
{
    if (!patch) return PBDR_ERR_INVALID_ARG;
    return render2d_fwd_impl(splats, cam, patch, bg, dup_capacity, image, final_T, last_idx, workspace, workspace_bytes, hip_stream);
}

static int render2d_fwd_impl(const pbdr2d_splats* splats, const pbdr_camera* cam, const pbdr_patch* patch, const float bg[3],
                             uint64_t dup_capacity, float* image, float* final_T, uint32_t* last_idx, void* workspace,
                             size_t workspace_bytes, void* hip_stream)
{
    if (!check_splats2d(splats) || !check_camera(cam) || !bg || !aligned16(image) || !aligned16(final_T) || !aligned16(last_idx))
        return PBDR_ERR_INVALID_ARG;
    if (patch && !check_patch(cam, patch)) return PBDR_ERR_INVALID_ARG;
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, splats->n, cam->width, cam->height, dup_capacity, &L, kVariant2D);
    if (st != PBDR_OK) return st;
    const CamDev c = to_dev(cam, patch);
    hipError_t e = launch_bin_sort2d(dev(splats), c, L, (char*)workspace, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_result(e);
    return hip_result(launch_composite2d_fwd(c, L, (char*)workspace, bg, image, final_T, last_idx, (hipStream_t)hip_stream));
}

int pbdr2d_render_stats(const pbdr_camera* cam, int32_t n, uint64_t dup_capacity, uint64_t* counters, void* workspace,
                        size_t workspace_bytes, void* hip_stream)
{
    if (!check_camera(cam) || !aligned16(counters)) return PBDR_ERR_INVALID_ARG;
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, n, cam->width, cam->height, dup_capacity, &L, kVariant2D);
    if (st != PBDR_OK) return st;
    return hip_result(launch_render_stats2d(to_dev(cam), L, (char*)workspace, counters, (hipStream_t)hip_stream));
}

int pbdr2d_preprocess_bwd(const pbdr2d_scene* scene, const pbdr_camera* cam, const pbdr2d_splats* splats,
                          const pbdr2d_splat_grads* g_splats, pbdr2d_scene_grads* grads, void* hip_stream)
{
    if (!check_scene2d(scene) || !check_camera(cam) || !check_splats2d(splats) || splats->n != scene->n ||
        !check_splat2d_grads(g_splats, scene->n) || !check_scene2d_grads(grads, scene))
        return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_preprocess2d_bwd(dev(scene), to_dev(cam), dev(splats), dev(g_splats), dev(grads), grads->first_view != 0,
                                              (hipStream_t)hip_stream));
}

static int render2d_bwd_impl(const pbdr2d_scene* scene, const pbdr2d_splats* splats, const pbdr_camera* cam,
                             const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                             const uint32_t* last_idx, const float* dL_dimage, pbdr2d_splat_grads* g_splats,
                             pbdr2d_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream);

int pbdr2d_render_bwd(const pbdr2d_scene* scene, const pbdr2d_splats* splats, const pbdr_camera* cam, const float bg[3],
                      uint64_t dup_capacity, const float* final_T, const uint32_t* last_idx, const float* dL_dimage,
                      pbdr2d_splat_grads* g_splats, pbdr2d_scene_grads* grads, void* workspace, size_t workspace_bytes,
                      void* hip_stream)
{
    return render2d_bwd_impl(scene, splats, cam, nullptr, bg, dup_capacity, final_T, last_idx, dL_dimage, g_splats, grads,
                             workspace, workspace_bytes, hip_stream);
}

int pbdr2d_render_bwd_patch(const pbdr2d_scene* scene, const pbdr2d_splats* splats, const pbdr_camera* cam,
                            const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                            const uint32_t* last_idx, const float* dL_dimage, pbdr2d_splat_grads* g_splats,
                            pbdr2d_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!patch) return PBDR_ERR_INVALID_ARG;
    return render2d_bwd_impl(scene, splats, cam, patch, bg, dup_capacity, final_T, last_idx, dL_dimage, g_splats, grads,
                             workspace, workspace_bytes, hip_stream);
}

static int render2d_bwd_impl(const pbdr2d_scene* scene, const pbdr2d_splats* splats, const pbdr_camera* cam,
                             const pbdr_patch* patch, const float bg[3], uint64_t dup_capacity, const float* final_T,
                             const uint32_t* last_idx, const float* dL_dimage, pbdr2d_splat_grads* g_splats,
                             pbdr2d_scene_grads* grads, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!check_splats2d(splats) || !check_camera(cam) || !bg || !aligned16(final_T) || !aligned16(last_idx) || !aligned16(dL_dimage))
        return PBDR_ERR_INVALID_ARG;
    if (g_splats ? !check_splat2d_grads(g_splats, splats->n) : scene == nullptr) return PBDR_ERR_INVALID_ARG;
    if (patch && !check_patch(cam, patch)) return PBDR_ERR_INVALID_ARG;
    if ((scene == nullptr) != (grads == nullptr)) return PBDR_ERR_INVALID_ARG;
    if (scene && (!check_scene2d(scene) || scene->n != splats->n || !check_scene2d_grads(grads, scene))) return PBDR_ERR_INVALID_ARG;
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, splats->n, cam->width, cam->height, dup_capacity, &L, kVariant2D);
    if (st != PBDR_OK) return st;
    const CamDev c = to_dev(cam, patch);
    const Splat2DGradDev g2 = g_splats ? dev(g_splats) : Splat2DGradDev{nullptr, nullptr, nullptr, nullptr};
    hipError_t e = launch_composite2d_bwd(c, L, (char*)workspace, splats->n, bg, final_T, last_idx, dL_dimage, g2,
                                          (hipStream_t)hip_stream);
    if (e != hipSuccess || !scene) return hip_result(e);
    if (!g_splats)      // no splat-state gradient asked for: the splatting backward reads the workspace's per-point records
        return hip_result(launch_preprocess2d_bwd_records(dev(scene), c, dev(splats),
                                                          reinterpret_cast<const uint32_t*>((char*)workspace + L.off_touched),
                                                          reinterpret_cast<const float4*>((char*)workspace + L.off_grad_rec),
                                                          carry_fold(L, (char*)workspace), dev(grads), grads->first_view != 0,
                                                          (hipStream_t)hip_stream));
    Splats2DDev listed = dev(splats);      // as in the 3D call: the points binning listed are the ones g_splats was written for
    listed.radius = reinterpret_cast<int32_t*>((char*)workspace + L.off_touched);
    return hip_result(launch_preprocess2d_bwd(dev(scene), c, listed, dev(g_splats), dev(grads), grads->first_view != 0,
                                              (hipStream_t)hip_stream));
}

int pbdr_l1_loss(int32_t width, int32_t height, const float* image, const float* target, float* loss, float* dL_dimage,
                 void* hip_stream)
{
    if (width <= 0 || height <= 0 || width > 65536 || height > 65536) return PBDR_ERR_INVALID_ARG;
    if (!aligned16(image) || !aligned16(target) || !aligned16(dL_dimage) || loss == nullptr || (reinterpret_cast<uintptr_t>(loss) & 3u))
        return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_l1_loss(width, height, image, target, loss, dL_dimage, (hipStream_t)hip_stream));
}

int pbdr_mark_visible(int32_t n, const int32_t* radius, uint8_t* visible, void* hip_stream)
{
    if (n < 0) return PBDR_ERR_INVALID_ARG;
    if (n > 0 && (!aligned16(radius) || !aligned16(visible))) return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_mark_visible(n, radius, visible, (hipStream_t)hip_stream));
}

int pbdr_adam_selective(int32_t n, int32_t planes, float* param, float* grad, float* exp_avg, float* exp_avg_sq,
                        const uint8_t* visible, const pbdr_adam_config* cfg, void* hip_stream)
{
    if (n < 0 || planes < 0 || planes > 65535 || !cfg) return PBDR_ERR_INVALID_ARG;
    if (!(cfg->lr >= 0.f) || !(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f) ||
        !(cfg->eps > 0.f) || cfg->step < 1)
        return PBDR_ERR_INVALID_ARG;
    if (n > 0 && planes > 0 &&
        (!aligned16(param) || !aligned16(grad) || !aligned16(exp_avg) || !aligned16(exp_avg_sq) || !aligned16(visible)))
        return PBDR_ERR_INVALID_ARG;
    return hip_result(launch_adam_selective(n, planes, param, grad, exp_avg, exp_avg_sq, visible, cfg->lr, cfg->beta1,
                                            cfg->beta2, cfg->eps, cfg->step, cfg->zero_grad, (hipStream_t)hip_stream));
}

int pbdr_preprocess_bwd_batch_adam(const pbdr_scene* scene, int32_t num_views, const pbdr_camera* cams, const pbdr_splats* splats,
                                   const pbdr_splat_grads* g_splats, pbdr_scene_grads* exp_avg, pbdr_scene_grads* exp_avg_sq,
                                   const float lr[5], const pbdr_adam_config* cfg, void* hip_stream)
{
    if (!check_scene(scene) || num_views < 1 || num_views > PBDR_MAX_BATCH_VIEWS || !cams || !splats || !g_splats || !lr || !cfg ||
        !check_scene_grads(exp_avg, scene) || !check_scene_grads(exp_avg_sq, scene))
        return PBDR_ERR_INVALID_ARG;
    if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f) || !(cfg->beta2 >= 0.f && cfg->beta2 < 1.f) || !(cfg->eps > 0.f) || cfg->step < 1)
        return PBDR_ERR_INVALID_ARG;
    BatchCams bc;
    BatchSplatGrads bg;
    BatchAdam opt;
    bc.count = num_views;
    for (int v = 0; v < num_views; ++v) {
        if (!check_camera(&cams[v]) || !check_splats(&splats[v]) || splats[v].n != scene->n ||
            !check_splat_grads(&g_splats[v], scene->n))
            return PBDR_ERR_INVALID_ARG;
        bc.cam[v] = to_dev(&cams[v]);
        bg.radius[v] = splats[v].radius;
        bg.grad[v] = dev(&g_splats[v]);
    }
    for (int v = num_views; v < kMaxBatchViews; ++v) { bc.cam[v] = bc.cam[0]; bg.radius[v] = bg.radius[0]; bg.grad[v] = bg.grad[0]; }
    for (int a = 0; a < 5; ++a) {
        if (!(lr[a] >= 0.f)) return PBDR_ERR_INVALID_ARG;
        opt.attr[a] = make_adam(lr[a], cfg->beta1, cfg->beta2, cfg->eps, cfg->step, 0);
    }
    const SceneGradDev m = dev(exp_avg), v2 = dev(exp_avg_sq);
    opt.m_mean = m.mean; opt.m_log_scale = m.log_scale; opt.m_quat = m.quat; opt.m_logit = m.logit; opt.m_sh = m.sh;
    opt.v_mean = v2.mean; opt.v_log_scale = v2.log_scale; opt.v_quat = v2.quat; opt.v_logit = v2.logit; opt.v_sh = v2.sh;
    return hip_result(launch_preprocess_bwd_batch_adam(dev(scene), bc, bg, opt, (hipStream_t)hip_stream));
}

int pbdr_query_lists(void* workspace, size_t workspace_bytes, int32_t n, int32_t width, int32_t height,
                     uint64_t dup_capacity, void* hip_stream, uint64_t* num_dup)
{
    Layout L;
    const int st = workspace_ok(workspace, workspace_bytes, n, width, height, dup_capacity, &L);
    if (st != PBDR_OK) return st;
    uint32_t host[4] = {0, 0, 0, 0};
    hipError_t e = hipMemcpyAsync(host, (char*)workspace + L.off_status, sizeof(host), hipMemcpyDeviceToHost,
                                  (hipStream_t)hip_stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_result(e);
    if (num_dup) *num_dup = host[kStNumDup];
    return (host[kStNumDup] > L.cap) ? PBDR_ERR_CAPACITY : PBDR_OK;
}

}  // extern "C"
