// Event-based kernel timing for benchmarks: pbdr_profile_begin/collect/end. Host-side bookkeeping only.
#include "../../include/pbdr.h"
#include "profile.h"

#include <cstdlib>

namespace pbdr {
ProfState g_prof;

static const char* const kKernelNames[kKernelCount] = {
    "k_preprocess", "k_count_visible", "(unused)", "k_pack_dup", "k_radix_hist", "k_radix_scatter", "k_tile_ranges",
    "fill", "k_composite_fwd", "k_composite_bwd", "k_preprocess_bwd", "k_render_stats", "k_gather_splat_grads", "k_group_cull", "k_l1_loss", "k_adam_selective",
    "k_tile_depth_sort"};

static void release()
{
    for (int i = 0; i < g_prof.capacity; ++i) {
        (void)hipEventDestroy(g_prof.start[i]);
        (void)hipEventDestroy(g_prof.stop[i]);
    }
    std::free(g_prof.start); std::free(g_prof.stop); std::free(g_prof.kernel);
    g_prof = ProfState();
}
}  // namespace pbdr

using namespace pbdr;

extern "C" {

int pbdr_profile_begin(uint32_t kernel_mask, int32_t max_records)
{
    if (max_records <= 0 || max_records > (1 << 20)) return PBDR_ERR_INVALID_ARG;
    if (g_prof.capacity) release();
    g_prof.start = (hipEvent_t*)std::calloc((size_t)max_records, sizeof(hipEvent_t));
    g_prof.stop = (hipEvent_t*)std::calloc((size_t)max_records, sizeof(hipEvent_t));
    g_prof.kernel = (int*)std::calloc((size_t)max_records, sizeof(int));
    if (!g_prof.start || !g_prof.stop || !g_prof.kernel) { release(); return PBDR_ERR_INVALID_ARG; }
    for (int i = 0; i < max_records; ++i) {
        // timing only: nobody reads device data on the strength of these events, so they need not make the kernels'
        // writes visible to the host when they complete (measured: 3 us less per step of a run that times one kernel)
        if (hipEventCreateWithFlags(&g_prof.start[i], hipEventDisableSystemFence) != hipSuccess ||
            hipEventCreateWithFlags(&g_prof.stop[i], hipEventDisableSystemFence) != hipSuccess) {
            g_prof.capacity = i; release(); return PBDR_ERR_HIP;
        }
        g_prof.capacity = i + 1;
    }
    g_prof.mask = kernel_mask;
    return PBDR_OK;
}

int pbdr_profile_collect(int32_t kernel_id, double* total_ms, int32_t* records)
{
    if (kernel_id < 0 || kernel_id >= kKernelCount || !total_ms || !records) return PBDR_ERR_INVALID_ARG;
    double tot = 0.0; int cnt = 0;
    for (int i = 0; i < g_prof.used; ++i) {
        if (g_prof.kernel[i] != kernel_id) continue;
        if (hipEventSynchronize(g_prof.stop[i]) != hipSuccess) return PBDR_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.start[i], g_prof.stop[i]) != hipSuccess) return PBDR_ERR_HIP;
        tot += ms; ++cnt;
    }
    *total_ms = tot; *records = cnt;
    return PBDR_OK;
}

int pbdr_profile_reset(void) { g_prof.used = 0; return PBDR_OK; }

int pbdr_profile_end(void) { release(); return PBDR_OK; }

const char* pbdr_profile_kernel_name(int32_t kernel_id)
{
    return (kernel_id >= 0 && kernel_id < kKernelCount) ? kKernelNames[kernel_id] : "";
}

int pbdr_profile_kernel_count(void) { return kKernelCount; }

}  // extern "C"
