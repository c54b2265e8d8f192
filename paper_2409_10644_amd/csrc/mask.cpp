// Topology-aware causal mask: host build at gamma_max, one upload, constant-time slices
// (Sec. 2.2; Sec. 3.2 and Fig. 2 of arXiv 2409.10644).
#include <cstdlib>
#include <cstring>
#include <new>

#include "mcsd_internal.h"

McsdProfileSlot g_mcsd_profile[6];      // static storage: both atomics of every slot start as null

// ---------------------------------------------------------------------------------------------------
// Which workgroups share a level-2 cache.  The GPU is made of several accelerator dies, each with its own L2;
// a launch deals its workgroups to the dies round-robin by workgroup id.  The tree-attention sweep folds the
// partial results of its key splits through the L2 when the workgroups of one (sequence, head) sit on one die,
// so the dealing is checked once per device, here, on the hardware: every workgroup of a small launch reports the
// id of its die.  Result: the number of dies when workgroup i runs on die (first + i) % dies for all i, whichever die
// the launch started with, else 0 (the sweep then leaves the fold to its second kernel).
// ---------------------------------------------------------------------------------------------------
namespace {
constexpr int XCC_PROBE_WGS = 256;
__global__ void xcc_probe_kernel(int32_t *out)
{
    unsigned x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)(x & 15u);
}
std::atomic<int> g_xcc_of_device[64];       // 0 = not probed yet, -1 = probed: dealing not as expected, else dies
}  // namespace

int mcsd_xcc_count(int device)
{
    if (device < 0 || device >= 64) return 0;
    const int v = g_xcc_of_device[device].load(std::memory_order_relaxed);
    return v > 0 ? v : 0;
}

// Called by mcsd_build_mask with `device` current (that call synchronises and allocates anyway).
static void probe_xcc_once(int device)
{
    if (device < 0 || device >= 64 || g_xcc_of_device[device].load(std::memory_order_relaxed) != 0) return;
    int result = -1;
    int32_t *dev = nullptr;
    int32_t host[XCC_PROBE_WGS];
    if (hipMalloc((void **)&dev, sizeof(host)) == hipSuccess) {
        bool ok = true;
        int dies = 0;
        for (int rep = 0; rep < 2 && ok; ++rep) {             // twice: the dealing must not depend on what ran before
            hipLaunchKernelGGL(xcc_probe_kernel, dim3(XCC_PROBE_WGS), dim3(64), 0, 0, dev);
            ok = hipGetLastError() == hipSuccess && hipMemcpy(host, dev, sizeof(host), hipMemcpyDeviceToHost) == hipSuccess;
            if (!ok) break;
            int mx = 0;
            for (int i = 0; i < XCC_PROBE_WGS; ++i) mx = host[i] > mx ? host[i] : mx;
            const int n = mx + 1;
            ok = (n == 1 || n == 2 || n == 4 || n == 8) && (rep == 0 || n == dies);
            // round-robin from whichever die is next: what the kernels rely on is that ids congruent modulo the number
            // of dies share a die
            for (int i = 0; i < XCC_PROBE_WGS && ok; ++i) ok = host[i] == (host[0] + i) % n;
            dies = n;
        }
        if (ok) result = dies;
        (void)hipFree(dev);
    }
    (void)hipGetLastError();
    g_xcc_of_device[device].store(result, std::memory_order_relaxed);
}

extern "C" int mcsd_profile_next(mcsd_kernel_t kernel, void *start_event, void *stop_event)
{
    if ((int)kernel < 0 || (int)kernel > 5) return MCSD_EINVAL;
    if ((start_event == nullptr) != (stop_event == nullptr)) return MCSD_EINVAL;
    // disarm first, then publish the stop event before the start event that launches look at
    McsdProfileSlot &slot = g_mcsd_profile[(int)kernel];
    slot.start.store(nullptr, std::memory_order_relaxed);
    slot.stop.store((hipEvent_t)stop_event, std::memory_order_relaxed);
    slot.start.store((hipEvent_t)start_event, std::memory_order_release);
    return MCSD_OK;
}

extern "C" const char *mcsd_strerror(int status)
{
    switch (status) {
    case MCSD_OK: return "ok";
    case MCSD_EINVAL: return "invalid argument";
    case MCSD_ENOMEM: return "out of memory";
    case MCSD_EHIP: return "HIP runtime error";
    case MCSD_EWORKSPACE: return "workspace missing or too small";
    case MCSD_EUNSUPPORTED: return "request outside the supported limits";
    default: return "unknown status";
    }
}

extern "C" int mcsd_build_mask(const int32_t *branching, int32_t gamma_max, mcsd_mask_t **out)
{
    if (!branching || !out || gamma_max < 1 || gamma_max > MCSD_MAX_LEVELS) return MCSD_EINVAL;
    *out = nullptr;
    int64_t level_size = 1, total = 0;
    int32_t level_off[MCSD_MAX_LEVELS + 1];
    for (int32_t l = 0; l < gamma_max; ++l) {
        if (branching[l] < 1 || branching[l] > MCSD_MAX_BRANCH) return MCSD_EINVAL;
        level_size *= branching[l];
        level_off[l] = (int32_t)total;
        total += level_size;
        if (total > MCSD_MAX_NODES) return MCSD_EUNSUPPORTED;
    }
    level_off[gamma_max] = (int32_t)total;
    const int32_t N = (int32_t)total;
    const int32_t W = (N + 63) / 64;

    mcsd_mask *m = new (std::nothrow) mcsd_mask();
    if (!m) return MCSD_ENOMEM;
    m->gamma_max = gamma_max;
    m->n_nodes_max = N;
    m->words_per_row = W;
    std::memcpy(m->branching, branching, sizeof(int32_t) * gamma_max);
    std::memcpy(m->level_off, level_off, sizeof(int32_t) * (gamma_max + 1));
    m->bits_host = (uint64_t *)std::calloc((size_t)N * W, sizeof(uint64_t));
    m->parent_host = (int32_t *)std::malloc(sizeof(int32_t) * N);
    m->level_host = (int32_t *)std::malloc(sizeof(int32_t) * N);
    m->dev_block = nullptr;
    if (!m->bits_host || !m->parent_host || !m->level_host) { mcsd_free_mask(m); return MCSD_ENOMEM; }

    // A row is its parent's row plus its own diagonal bit: level-major numbering puts every parent
    // before its children, so one forward pass fills the whole mask.
    for (int32_t l = 0; l < gamma_max; ++l) {
        const int32_t first = level_off[l], count = level_off[l + 1] - level_off[l];
        for (int32_t a = 0; a < count; ++a) {
            const int32_t i = first + a;
            const int32_t par = (l == 0) ? -1 : level_off[l - 1] + a / branching[l];
            m->parent_host[i] = par;
            m->level_host[i] = l + 1;
            uint64_t *row = m->bits_host + (size_t)i * W;
            if (par >= 0) std::memcpy(row, m->bits_host + (size_t)par * W, sizeof(uint64_t) * W);
            row[i >> 6] |= (uint64_t)1 << (i & 63);
        }
    }

    // No HIP device present: the handle carries the host copy only (device = -1, device pointers null);
    // it can be sliced and inspected, and the device entry points reject its views.
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev < 1) {
        (void)hipGetLastError();
        m->device = -1;
        m->bits_dev = nullptr;
        m->parent_dev = nullptr;
        *out = m;
        return MCSD_OK;
    }
    const size_t bits_bytes = ((size_t)N * W * sizeof(uint64_t) + 255) & ~(size_t)255;
    const size_t par_bytes = sizeof(int32_t) * (size_t)N;
    if (hipGetDevice(&m->device) != hipSuccess) { mcsd_free_mask(m); return MCSD_EHIP; }
    if (hipMalloc(&m->dev_block, bits_bytes + par_bytes) != hipSuccess) {
        m->dev_block = nullptr;
        (void)hipGetLastError();
        mcsd_free_mask(m);
        return MCSD_ENOMEM;
    }
    probe_xcc_once(m->device);
    m->bits_dev = (uint64_t *)m->dev_block;
    m->parent_dev = (int32_t *)((char *)m->dev_block + bits_bytes);
    if (hipMemcpy(m->bits_dev, m->bits_host, (size_t)N * W * sizeof(uint64_t), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(m->parent_dev, m->parent_host, par_bytes, hipMemcpyHostToDevice) != hipSuccess) {
        mcsd_free_mask(m);
        return MCSD_EHIP;
    }
    *out = m;
    return MCSD_OK;
}

extern "C" int mcsd_slice_mask(const mcsd_mask_t *full, int32_t gamma, mcsd_mask_view_t *out)
{
    if (!full || !out || gamma < 1 || gamma > full->gamma_max) return MCSD_EINVAL;
    out->gamma = gamma;
    out->n_nodes = full->level_off[gamma];   // rows below N(gamma) have no bits at columns >= N(gamma)
    out->gamma_max = full->gamma_max;
    out->n_nodes_max = full->n_nodes_max;
    out->words_per_row = full->words_per_row;
    out->device = full->device;
    out->bits_host = full->bits_host;
    out->bits_dev = full->bits_dev;
    out->parent_host = full->parent_host;
    out->parent_dev = full->parent_dev;
    out->level_host = full->level_host;
    out->level_off_host = full->level_off;
    out->branching_host = full->branching;
    return MCSD_OK;
}

extern "C" void mcsd_free_mask(mcsd_mask_t *m)
{
    if (!m) return;
    if (m->dev_block) (void)hipFree(m->dev_block);
    std::free(m->bits_host);
    std::free(m->parent_host);
    std::free(m->level_host);
    delete m;
}
