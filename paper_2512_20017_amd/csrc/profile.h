// Optional per-kernel timing with HIP events on the stream the kernels run on (off by default; no cost when off).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbdr {

enum KernelId {
    kKPreprocess = 0, kKCountPack, kKScan, kKDuplicate, kKRadixHist, kKRadixScatter, kKTileRanges, kKFill,
    kKCompositeFwd, kKCompositeBwd, kKPreprocessBwd, kKStats, kKGather, kKGroupCull, kKLoss, kKAdam, kKTileDepthSort, kKernelCount
};

struct ProfState {
    uint32_t mask = 0;
    int capacity = 0;   // event pairs available
    int used = 0;
    hipEvent_t* start = nullptr;
    hipEvent_t* stop = nullptr;
    int* kernel = nullptr;
};
extern ProfState g_prof;

// Records a start event at construction and a stop event at destruction around launches of kernel `id`.
struct ProfScope {
    int slot = -1;
    hipStream_t s;
    ProfScope(int id, hipStream_t stream) : s(stream)
    {
        if ((g_prof.mask >> id) & 1u) {
            if (g_prof.used < g_prof.capacity) {
                slot = g_prof.used++;
                g_prof.kernel[slot] = id;
                (void)hipEventRecord(g_prof.start[slot], s);
            }
        }
    }
    ~ProfScope()
    {
        if (slot >= 0) (void)hipEventRecord(g_prof.stop[slot], s);
    }
};

}  // namespace pbdr
