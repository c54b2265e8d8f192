// Measurement aid, not part of the method: a plain read-only streaming kernel.  Its bandwidth on a buffer much
// larger than the caches is what this machine's HBM delivers to the simplest possible reader, the yardstick
// next to the datasheet peak for the tree-attention sweep's achieved bandwidth.
#include "mcsd_internal.h"

namespace {

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// Every thread reads 16-byte words grid-strided, eight loads in flight, and folds them into one word that is
// stored only if it has an (impossible in practice) value, so the loads cannot be optimised away.  The loads are
// non-temporal, like the sweep's: read-once data that the caches need not keep.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4_t *__restrict__ src, size_t n16, u32x4_t *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4_t acc = {0, 0, 0, 0};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4_t v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc ^= v[k];
    }
    for (; i < n16; i += stride) {
        acc ^= __builtin_nontemporal_load(src + i);
    }
    if (acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u && acc.z == 0x85ebca6bu && acc.w == 0xc2b2ae35u) *sink = acc;
}

// Second measurement aid: how well this machine overlaps matrix instructions with vector work.  The kernel runs
// the arithmetic of the tree-attention inner loop for one 32-key block per iteration, with no memory traffic at all:
// a matrix phase (8 chained MFMA 32x32x16 bf16 for S^T = K Q^T, 8 for O^T += V^T P^T) and a vector phase (maximum,
// exponentials and bf16 packing of 16 scores per lane).  One workgroup per compute unit; `schedule` says how the
// phases of the wavefronts on a SIMD are arranged:
//   0  one wavefront per SIMD, phases one after the other (nothing overlaps)
//   1  two wavefronts per SIMD, free-running (what the sweep kernel relies on)
//   2  two per SIMD, a workgroup barrier after every phase: one does its matrix phase while the other does its vector phase
//   3  one per SIMD, the wavefront interleaves its own vector work with its own matrix instructions (software pipeline)
//   4  two per SIMD, both software-pipelined
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16_t;

__device__ inline void probe_matrix_phase(probe_f32x16_t (&o)[4], probe_f32x16_t &s, const probe_bf16x8_t (&a)[8],
                                          const probe_bf16x8_t (&b)[8], const probe_bf16x8_t (&p)[2])
{
    s = (probe_f32x16_t){0};
#pragma unroll
    for (int k = 0; k < 8; ++k) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k], b[k], s, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], p[i >> 2], o[i & 3], 0, 0, 0);
}

__device__ inline void probe_vector_phase(const probe_f32x16_t &s, probe_bf16x8_t (&p)[2], float &l, float &m, float c)
{
    float mx = m;
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[r]);
    m = mx;
    const float mc = mx * c;
    float ps = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float e = __builtin_amdgcn_exp2f(fmaf(s[r], c, -mc));
        ps += e;
        p[r >> 3][r & 7] = (__bf16)e;
    }
    l += ps;
}

// Both phases of one iteration in one instruction stream: the matrix instructions produce s_next and consume p_prev,
// the vector work turns s_cur into p_new; the scheduler is told to alternate one MFMA with a few vector instructions.
__device__ inline void probe_pipelined(probe_f32x16_t (&o)[4], probe_f32x16_t &s_next, const probe_f32x16_t &s_cur,
                                       const probe_bf16x8_t (&a)[8], const probe_bf16x8_t (&b)[8], const probe_bf16x8_t (&p_prev)[2],
                                       probe_bf16x8_t (&p_new)[2], float &l, float &m, float c)
{
    s_next = (probe_f32x16_t){0};
    float mx = m;
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_cur[r]);
    m = mx;
    const float mc = mx * c;
    float ps = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k], b[k], s_next, 0, 0, 0);
        const float e = __builtin_amdgcn_exp2f(fmaf(s_cur[k], c, -mc));
        ps += e;
        p_new[0][k] = (__bf16)e;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], p_prev[i >> 2], o[i & 3], 0, 0, 0);
        const float e = __builtin_amdgcn_exp2f(fmaf(s_cur[8 + i], c, -mc));
        ps += e;
        p_new[1][i] = (__bf16)e;
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);     // a few vector instructions
    }
    l += ps;
}

// 512 lanes per workgroup = two wavefronts per SIMD; schedules with one per SIMD retire the upper four at once.
// Every wavefront executes the same number of barriers (schedule 2: two per iteration), so none can be left waiting.
template <int SCHEDULE>
__global__ __launch_bounds__(512) void issue_probe_kernel(float *out, int iterations, float c)
{
    extern __shared__ unsigned char probe_lds[];            // only there to keep a second workgroup off the compute unit
    const int tid = threadIdx.x, wave = tid >> 6;
    if ((SCHEDULE == 0 || SCHEDULE == 3) && wave >= 4) return;
    probe_bf16x8_t a[8], b[8], p[2];
    for (int k = 0; k < 8; ++k)
        for (int e = 0; e < 8; ++e) {
            a[k][e] = (__bf16)(0.01f * ((tid + k + e) & 15));
            b[k][e] = (__bf16)(0.02f * ((tid * 3 + k + e) & 7));
        }
    for (int e = 0; e < 8; ++e) p[0][e] = p[1][e] = (__bf16)0.f;
    probe_f32x16_t o[4] = {(probe_f32x16_t){0}, (probe_f32x16_t){0}, (probe_f32x16_t){0}, (probe_f32x16_t){0}}, s = (probe_f32x16_t){0};
    float l = 0.f, m = -1e30f;
    if (SCHEDULE == 3 || SCHEDULE == 4) {
        probe_f32x16_t s2 = (probe_f32x16_t){0};
        probe_bf16x8_t p2[2] = {p[0], p[1]};
        for (int it = 0; it < iterations; it += 2) {
            probe_pipelined(o, s2, s, a, b, p, p2, l, m, c);
            __builtin_amdgcn_sched_barrier(0);
            probe_pipelined(o, s, s2, a, b, p2, p, l, m, c);
            __builtin_amdgcn_sched_barrier(0);
        }
    } else if (SCHEDULE == 2) {
        const bool second = wave >= 4;
        for (int it = 0; it < iterations; ++it) {
            if (!second) probe_matrix_phase(o, s, a, b, p);
            else probe_vector_phase(s, p, l, m, c);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            if (second) probe_matrix_phase(o, s, a, b, p);
            else probe_vector_phase(s, p, l, m, c);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        for (int it = 0; it < iterations; ++it) {
            probe_matrix_phase(o, s, a, b, p);
            __builtin_amdgcn_sched_barrier(0);
            probe_vector_phase(s, p, l, m, c);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float acc = l + m;
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) acc += o[i][r];
    out[(size_t)blockIdx.x * 512 + tid] = acc;
    if (tid == 0) probe_lds[0] = 1;
}

template <int SCHEDULE>
hipError_t launch_issue_probe(float *out, int workgroups, int iterations, hipStream_t st)
{
    const size_t lds = 100 * 1024;                          // one workgroup per compute unit
    hipError_t e = hipFuncSetAttribute((const void *)issue_probe_kernel<SCHEDULE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // (launched directly: the event hooks of mcsd_launch are for kernels without dynamic LDS)
    hipLaunchKernelGGL(issue_probe_kernel<SCHEDULE>, dim3(workgroups), dim3(512), lds, st, out, iterations, 0.01f);
    return hipGetLastError();
}

// Third measurement aid: where the workgroups of a sweep-shaped grid run.  256 lanes and 66 KiB of LDS per workgroup
// (two fit a compute unit, like the bf16 sweep's); every workgroup stays for `spin` iterations of a dependent
// arithmetic chain so that the whole grid is resident at once, then writes its die (XCC_ID) and its HW_ID word.
__global__ __launch_bounds__(256) void placement_probe_kernel(uint32_t *out, int spin)
{
    extern __shared__ unsigned char place_lds[];
    unsigned xcc, hw;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    float v = (float)threadIdx.x;
    for (int i = 0; i < spin; ++i) v = fmaf(v, 1.0000001f, 0.5f);
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = xcc & 15u;
        out[2 * blockIdx.x + 1] = hw;
        if (v == -1.f) place_lds[0] = 1;                     // (keeps the chain and the LDS allocation alive)
    }
}

}  // namespace

extern "C" int mcsd_placement_probe(int32_t workgroups, int32_t spin, void *out_dev, void *hip_stream)
{
    if (!out_dev || workgroups < 1 || workgroups > 65535 || spin < 0 || spin > (1 << 20)) return MCSD_EINVAL;
    const size_t lds = 66 * 1024;
    hipError_t e = hipFuncSetAttribute((const void *)placement_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return mcsd_hip_status(e);
    hipLaunchKernelGGL(placement_probe_kernel, dim3(workgroups), dim3(256), lds, (hipStream_t)hip_stream, (uint32_t *)out_dev, spin);
    return mcsd_hip_status(hipGetLastError());
}

extern "C" int mcsd_issue_probe(int32_t schedule, int32_t workgroups, int32_t iterations, void *out_dev, void *hip_stream)
{
    if (!out_dev || schedule < 0 || schedule > 4 || workgroups < 1 || workgroups > 65535 || iterations < 2 || iterations > (1 << 20) ||
        (iterations & 1))
        return MCSD_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    float *out = (float *)out_dev;
    hipError_t e;
    switch (schedule) {
    case 0: e = launch_issue_probe<0>(out, workgroups, iterations, st); break;
    case 1: e = launch_issue_probe<1>(out, workgroups, iterations, st); break;
    case 2: e = launch_issue_probe<2>(out, workgroups, iterations, st); break;
    case 3: e = launch_issue_probe<3>(out, workgroups, iterations, st); break;
    default: e = launch_issue_probe<4>(out, workgroups, iterations, st); break;
    }
    return mcsd_hip_status(e);
}

extern "C" int mcsd_stream_read(const void *src_dev, size_t bytes, void *sink_dev, int32_t workgroups, void *hip_stream)
{
    if (!src_dev || !sink_dev || bytes < 16 || ((uintptr_t)src_dev & 15) || ((uintptr_t)sink_dev & 15)) return MCSD_EINVAL;
    if (workgroups < 0 || workgroups > 65535) return MCSD_EINVAL;
    mcsd_launch(MCSD_KERNEL_STREAM_READ, stream_read_kernel, dim3(workgroups ? workgroups : 1024), dim3(256), (hipStream_t)hip_stream,
                (const u32x4_t *)src_dev, bytes / 16, (u32x4_t *)sink_dev);
    return mcsd_hip_status(hipGetLastError());
}
