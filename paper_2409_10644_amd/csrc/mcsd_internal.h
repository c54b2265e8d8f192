// Internal declarations shared by the library's translation units (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include "mcsd.h"

struct mcsd_mask {
    int32_t gamma_max;
    int32_t n_nodes_max;
    int32_t words_per_row;
    int32_t device;
    int32_t branching[MCSD_MAX_LEVELS];
    int32_t level_off[MCSD_MAX_LEVELS + 1];
    uint64_t *bits_host;
    int32_t *parent_host;
    int32_t *level_host;
    void *dev_block;       // one device allocation: bits, then parent
    uint64_t *bits_dev;
    int32_t *parent_dev;
};

// Tree shape passed to kernels by value.
struct McsdTreeDesc {
    int32_t gamma;
    int32_t b[MCSD_MAX_LEVELS];
    int32_t off[MCSD_MAX_LEVELS + 1];
};

static inline int mcsd_hip_status(hipError_t e) { return e == hipSuccess ? MCSD_OK : MCSD_EHIP; }

// Accelerator dies (each with its own L2) of `device` when the hardware deals workgroup i of a launch to die
// i % dies, as established by a probe launch in mcsd_build_mask; 0 when unknown or not so.  Defined in mask.cpp.
int mcsd_xcc_count(int device);

// One-shot profiling events per kernel (see mcsd_profile_next); defined in mask.cpp.  Arming stores `stop` and then
// `start`; a launch takes `start` with an atomic exchange, so exactly one launch consumes an armed pair even when
// several host threads launch the same kernel at once.
#include <atomic>
struct McsdProfileSlot { std::atomic<hipEvent_t> start, stop; };
extern McsdProfileSlot g_mcsd_profile[6];

// Launch `kernel` on `st`; if a profiling pair is armed for `which`, bracket the launch with it and disarm.
template <typename... Args, typename... Actual>
inline void mcsd_launch(int which, void (*kernel)(Args...), dim3 grid, dim3 block, hipStream_t st, Actual... args)
{
    McsdProfileSlot &slot = g_mcsd_profile[which];
    hipEvent_t start = slot.start.load(std::memory_order_relaxed);
    if (start) start = slot.start.exchange(nullptr, std::memory_order_acquire);
    if (start) {
        hipEvent_t stop = slot.stop.exchange(nullptr, std::memory_order_relaxed);
        hipExtLaunchKernelGGL(kernel, grid, block, 0, st, start, stop, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
    }
}
