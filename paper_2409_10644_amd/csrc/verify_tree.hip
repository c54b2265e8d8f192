// Multi-candidate verification for gfx950 (Sec. 2.1, Sec. 3.1 and Fig. 1 steps 4-6 of arXiv 2409.10644):
// recursive rejection sampling down the candidate tree, longest-path selection for target-initialised
// trees, and sampling of the new token(s).
//
// One workgroup of 1024 lanes walks one tree (draft-initialised) or one level-1 subtree (target-initialised).
// The residual r <- max(r - S*q, 0) is never stored: after j rejections an element is recomputed from p, q
// and the j previous sums (a chain of j fused multiply-adds), so a round is one coalesced sweep over the
// two vocabulary rows.  Sums over the vocabulary follow the balanced binary tree over the zero-padded
// index space that the header specifies: a lane adds its 4 consecutive elements pairwise, 64 lanes combine
// by butterfly (256 elements per wavefront load), and the 256-element block sums are reduced through a
// heap in LDS which is kept for the inverse-CDF descent.  All arithmetic is binary64 with explicit fma.
//
// Compiled with -ffp-contract=off.
#include "mcsd_internal.h"

namespace {

constexpr int VT = 1024;                 // threads per workgroup
constexpr int BLK = 256;                 // vocabulary elements per wavefront load
constexpr int MAX_NB = MCSD_MAX_VOCAB / BLK;

struct VerifyParams {
    McsdTreeDesc t;
    int32_t mode, B, V, n_nodes, n_new, R;
    int32_t NB;                          // power of two >= ceil(V / BLK)
    const int32_t *tokens;
    const float *p, *q;
    int64_t pbs, qbs;
    const float *ua, *us;
    int32_t *cand_path;                  // [B][R][gamma]
    int32_t *cand_len;                   // [B][R]
    int32_t *cand_new;                   // [B][R][n_new]
};

struct Shared {
    double heapB[2 * MAX_NB];            // heap over 256-element blocks: leaves at [NB, 2NB), root at 1
    double heapA[2 * BLK];               // heap inside one block, rebuilt for each descent
    double s_hist[MCSD_MAX_BRANCH + 1];  // S before each rejection round of the current context
    int lo_idx, hi_idx;
};

// Element t of the distribution after `rounds` rejections at a context with rows prow / qrow.
__device__ inline double residual_at(const float *prow, const float *qrow, const double *s_hist, int rounds,
                                     int t)
{
    double r = (double)prow[t];
    if (rounds > 0) {
        const double qv = (double)qrow[t];
        for (int k = 0; k < rounds; ++k) {
            const double d = __fma_rn(-s_hist[k], qv, r);
            r = d > 0.0 ? d : 0.0;
        }
    }
    return r;
}

// Builds heapB for the distribution (prow, qrow, rounds) and returns its total.  All threads call it.
// A wavefront handles GROUP blocks of 256 elements at a time: all their loads are issued before any is used, and
// the GROUP butterflies are independent instruction streams, so a round costs about one memory latency.
__device__ double block_tree_sum(Shared &sh, const VerifyParams &P, const float *prow, const float *qrow,
                                 int rounds)
{
    constexpr int GROUP = 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool vec = (((uintptr_t)prow | (uintptr_t)qrow) & 15) == 0;
    for (int blk0 = wave; blk0 < P.NB; blk0 += GROUP * (VT / 64)) {
        float pe[GROUP][4], qe[GROUP][4];
#pragma unroll
        for (int k = 0; k < GROUP; ++k) {
            const int blk = blk0 + k * (VT / 64);
            const int t0 = blk * BLK + lane * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) { pe[k][e] = 0.f; qe[k][e] = 0.f; }
            if (blk < P.NB) {
                if (vec && t0 + 3 < P.V) {
                    const float4 pv = *(const float4 *)(prow + t0);
                    pe[k][0] = pv.x; pe[k][1] = pv.y; pe[k][2] = pv.z; pe[k][3] = pv.w;
                    if (rounds > 0) {
                        const float4 qv = *(const float4 *)(qrow + t0);
                        qe[k][0] = qv.x; qe[k][1] = qv.y; qe[k][2] = qv.z; qe[k][3] = qv.w;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (t0 + e < P.V) {
                            pe[k][e] = prow[t0 + e];
                            if (rounds > 0) qe[k][e] = qrow[t0 + e];
                        }
                }
            }
        }
        double sblk[GROUP];
#pragma unroll
        for (int k = 0; k < GROUP; ++k) {
            double v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double r = (double)pe[k][e];                 // elements beyond V are 0 and stay 0
                const double qd = (double)qe[k][e];
                for (int j = 0; j < rounds; ++j) {
                    const double d = __fma_rn(-sh.s_hist[j], qd, r);
                    r = d > 0.0 ? d : 0.0;
                }
                v[e] = r;
            }
            sblk[k] = __dadd_rn(__dadd_rn(v[0], v[1]), __dadd_rn(v[2], v[3]));
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1)
#pragma unroll
            for (int k = 0; k < GROUP; ++k) sblk[k] = __dadd_rn(sblk[k], __shfl_xor(sblk[k], m, 64));
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < GROUP; ++k) {
                const int blk = blk0 + k * (VT / 64);
                if (blk < P.NB) sh.heapB[P.NB + blk] = sblk[k];
            }
        }
    }
    __syncthreads();
    for (int n = P.NB >> 1; n >= 1; n >>= 1) {
        if (tid < n) sh.heapB[n + tid] = __dadd_rn(sh.heapB[2 * (n + tid)], sh.heapB[2 * (n + tid) + 1]);
        __syncthreads();
    }
    return sh.heapB[1];
}

// Inverse-CDF draw from the distribution whose heapB is current.  All threads call it; all return the token.
__device__ int tree_sample(Shared &sh, const VerifyParams &P, const float *prow, const float *qrow, int rounds,
                           float u)
{
    const int tid = threadIdx.x;
    const double S = sh.heapB[1];
    double thr = __dmul_rn((double)u, S);
    int node = 1;
    while (node < P.NB) {
        const double left = sh.heapB[2 * node];
        if (thr < left) {
            node = 2 * node;
        } else {
            thr = __dsub_rn(thr, left);
            node = 2 * node + 1;
        }
    }
    const int blk = node - P.NB;
    __syncthreads();     // heapA may still be read by a previous descent
    if (tid < BLK) {
        const int t = blk * BLK + tid;
        sh.heapA[BLK + tid] = t < P.V ? residual_at(prow, qrow, sh.s_hist, rounds, t) : 0.0;
    }
    __syncthreads();
    for (int n = BLK >> 1; n >= 1; n >>= 1) {
        if (tid < n) sh.heapA[n + tid] = __dadd_rn(sh.heapA[2 * (n + tid)], sh.heapA[2 * (n + tid) + 1]);
        __syncthreads();
    }
    node = 1;
    while (node < BLK) {
        const double left = sh.heapA[2 * node];
        if (thr < left) {
            node = 2 * node;
        } else {
            thr = __dsub_rn(thr, left);
            node = 2 * node + 1;
        }
    }
    int t = blk * BLK + (node - BLK);
    const bool ok = t < P.V && sh.heapA[node] > 0.0;
    if (ok) return t;
    // Reached a zero-weight index (last-bit rounding of the subtraction, or an all-zero distribution):
    // nearest positive-weight index below, else nearest above, else 0.
    if (tid == 0) { sh.lo_idx = -1; sh.hi_idx = 0x7fffffff; }
    __syncthreads();
    int lo = -1, hi = 0x7fffffff;
    for (int e = tid; e < P.V; e += VT) {
        if (e == t) continue;
        if (residual_at(prow, qrow, sh.s_hist, rounds, e) > 0.0) {
            if (e < t) lo = e > lo ? e : lo;
            else hi = e < hi ? e : hi;
        }
    }
    if (lo >= 0) atomicMax(&sh.lo_idx, lo);
    if (hi != 0x7fffffff) atomicMin(&sh.hi_idx, hi);
    __syncthreads();
    t = sh.lo_idx >= 0 ? sh.lo_idx : (sh.hi_idx != 0x7fffffff ? sh.hi_idx : 0);
    __syncthreads();
    return t;
}

__global__ __launch_bounds__(VT) void verify_walk_kernel(const VerifyParams P)
{
    __shared__ Shared sh;
    const int tid = threadIdx.x;
    const int root = blockIdx.x, b = blockIdx.y;
    const int32_t *tokens = P.tokens + (int64_t)b * P.n_nodes;
    const float *p = P.p + (int64_t)b * P.pbs;
    const float *q = P.q + (int64_t)b * P.qbs;
    const float *ua = P.ua + (int64_t)b * P.n_nodes;
    int32_t *path_out = P.cand_path + ((int64_t)b * P.R + root) * P.t.gamma;

    int cur = -1, level = 0, n_acc = 0;      // context: node id (-1 = end of the prefix) and its level
    if (P.mode == MCSD_TARGET_INIT) {         // level-1 node `root` is accepted untested
        cur = root;
        level = 1;
        n_acc = 1;
        if (tid == 0) path_out[0] = root;
    }
    const float *term_p = nullptr, *term_q = nullptr;
    int term_rounds = 0;
    bool have_heap = false;
    while (level < P.t.gamma) {
        const float *prow = p + (int64_t)(cur + 1) * P.V;
        const float *qrow = q + (int64_t)(cur + 1) * P.V;
        const int cnt = P.t.b[level];
        const int first = cur < 0 ? 0 : P.t.off[level] + (cur - P.t.off[level - 1]) * cnt;
        int rounds = 0, accepted = -1;
        double S = 1.0;
        for (int c = 0; c < cnt; ++c) {
            const int node = first + c;
            int x = tokens[node];
            x = x < 0 ? 0 : (x >= P.V ? P.V - 1 : x);   // ids outside 0..V-1 are clamped, never dereferenced
            const double u = (double)ua[node];
            const double rx = residual_at(prow, qrow, sh.s_hist, rounds, x);
            if (__dmul_rn(u, __dmul_rn((double)qrow[x], S)) < rx) { accepted = node; break; }
            __syncthreads();                 // every lane has finished reading s_hist / heaps
            if (tid == 0) sh.s_hist[rounds] = S;
            __syncthreads();
            rounds += 1;
            S = block_tree_sum(sh, P, prow, qrow, rounds);
        }
        if (accepted < 0) {
            if (S > 0.0) { term_p = prow; term_q = qrow; term_rounds = rounds; have_heap = true; }
            else { term_p = prow; term_q = qrow; term_rounds = 0; have_heap = false; }
            break;
        }
        if (tid == 0) path_out[n_acc] = accepted;
        n_acc += 1;
        cur = accepted;
        level += 1;
    }
    if (term_p == nullptr) {                  // every level accepted: bonus from the row after the last node
        term_p = p + (int64_t)(cur + 1) * P.V;
        term_q = term_p;                      // never read: rounds == 0
        term_rounds = 0;
        have_heap = false;
    }
    if (tid == 0) {
        for (int l = n_acc; l < P.t.gamma; ++l) path_out[l] = -1;
        P.cand_len[(int64_t)b * P.R + root] = n_acc;
    }
    if (P.n_new > 0) {
        if (!have_heap) {
            __syncthreads();
            (void)block_tree_sum(sh, P, term_p, term_q, 0);
        }
        for (int k = 0; k < P.n_new; ++k) {
            const int t = tree_sample(sh, P, term_p, term_q, term_rounds, P.us[(int64_t)b * P.n_new + k]);
            if (tid == 0) P.cand_new[((int64_t)b * P.R + root) * P.n_new + k] = t;
        }
    }
}

// Target-initialised trees: the level-1 subtree with the longest accepted path wins, lowest id on ties.
__global__ void verify_select_kernel(const VerifyParams P, int32_t *out_path, int32_t *out_len, int32_t *out_new)
{
    const int b = blockIdx.x;
    __shared__ int best;
    if (threadIdx.x == 0) {
        int bi = 0, bl = -1;
        for (int r = 0; r < P.R; ++r) {
            const int len = P.cand_len[(int64_t)b * P.R + r];
            if (len > bl) { bl = len; bi = r; }
        }
        best = bi;
        out_len[b] = bl;
    }
    __syncthreads();
    const int64_t c = (int64_t)b * P.R + best;
    for (int l = threadIdx.x; l < P.t.gamma; l += blockDim.x) out_path[(int64_t)b * P.t.gamma + l] = P.cand_path[c * P.t.gamma + l];
    for (int k = threadIdx.x; k < P.n_new; k += blockDim.x) out_new[(int64_t)b * P.n_new + k] = P.cand_new[c * P.n_new + k];
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

extern "C" size_t mcsd_verify_tree_workspace(const mcsd_mask_view_t *mask, mcsd_mode_t mode, int32_t B, int32_t n_new)
{
    if (!mask || mode != MCSD_TARGET_INIT || B < 1 || n_new < 0) return 0;
    const size_t R = (size_t)mask->branching_host[0];
    return align256(sizeof(int32_t) * B * R * mask->gamma) + align256(sizeof(int32_t) * B * R) +
           align256(sizeof(int32_t) * B * R * (n_new > 0 ? n_new : 1));
}

extern "C" int mcsd_verify_tree(const mcsd_mask_view_t *mask, mcsd_mode_t mode, int32_t B, int32_t V,
                                const int32_t *tokens, const float *p_target, const float *q_draft,
                                int64_t p_batch_stride, int64_t q_batch_stride, const float *u_accept,
                                const float *u_sample, int32_t n_new, int32_t *out_path, int32_t *out_accept_len,
                                int32_t *out_new_tokens, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!mask || !tokens || !p_target || !u_accept || !out_path || !out_accept_len) return MCSD_EINVAL;
    if (mode != MCSD_DRAFT_INIT && mode != MCSD_TARGET_INIT) return MCSD_EINVAL;
    if (B < 1 || B > 65535 || V < 1 || n_new < 0 || n_new > 64) return MCSD_EINVAL;
    if (n_new > 0 && (!u_sample || !out_new_tokens)) return MCSD_EINVAL;
    if (mask->gamma < 1 || mask->gamma > MCSD_MAX_LEVELS) return MCSD_EINVAL;
    // draft rows are needed whenever some context has children to test
    const bool has_tests = mode == MCSD_DRAFT_INIT ? true : mask->gamma > 1;
    if (has_tests && !q_draft) return MCSD_EINVAL;
    if (V > MCSD_MAX_VOCAB) return MCSD_EUNSUPPORTED;
    if (p_batch_stride < (int64_t)(1 + mask->n_nodes) * V) return MCSD_EINVAL;
    if (has_tests && q_batch_stride < (int64_t)(1 + mask->level_off_host[mask->gamma - 1]) * V) return MCSD_EINVAL;

    VerifyParams P;
    P.t.gamma = mask->gamma;
    for (int l = 0; l < mask->gamma; ++l) P.t.b[l] = mask->branching_host[l];
    for (int l = 0; l <= mask->gamma; ++l) P.t.off[l] = mask->level_off_host[l];
    P.mode = mode; P.B = B; P.V = V; P.n_nodes = mask->n_nodes; P.n_new = n_new;
    P.R = mode == MCSD_TARGET_INIT ? mask->branching_host[0] : 1;
    int nb = 1;
    while (nb * BLK < V) nb <<= 1;
    P.NB = nb;
    P.tokens = tokens; P.p = p_target; P.q = q_draft ? q_draft : p_target;
    P.pbs = p_batch_stride; P.qbs = q_batch_stride;
    P.ua = u_accept; P.us = u_sample;
    hipStream_t st = (hipStream_t)hip_stream;
    if (mode == MCSD_DRAFT_INIT) {
        P.cand_path = out_path; P.cand_len = out_accept_len; P.cand_new = out_new_tokens;
        mcsd_launch(MCSD_KERNEL_VERIFY_WALK, verify_walk_kernel, dim3(1, B), dim3(VT), st, P);
        return mcsd_hip_status(hipGetLastError());
    }
    const size_t need = mcsd_verify_tree_workspace(mask, mode, B, n_new);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return MCSD_EWORKSPACE;
    const size_t R = (size_t)P.R;
    char *w = (char *)workspace;
    P.cand_path = (int32_t *)w;
    w += align256(sizeof(int32_t) * B * R * mask->gamma);
    P.cand_len = (int32_t *)w;
    w += align256(sizeof(int32_t) * B * R);
    P.cand_new = (int32_t *)w;
    mcsd_launch(MCSD_KERNEL_VERIFY_WALK, verify_walk_kernel, dim3(P.R, B), dim3(VT), st, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return MCSD_EHIP;
    hipLaunchKernelGGL(verify_select_kernel, dim3(B), dim3(64), 0, st, P, out_path, out_accept_len, out_new_tokens);
    return mcsd_hip_status(hipGetLastError());
}
