// Update after acceptance for gfx950 (Fig. 1 step 6 of arXiv 2409.10644): the tree K/V rows of the accepted path
// are appended to the prefix cache of every layer, the prefix lengths grow by the accepted length and the token
// ids that join the input are written out.
//
// A gather-scatter of at most gamma rows per sequence and layer (H * d elements each, for K and V): one
// workgroup per (path position, sequence, layer) moves the row of all heads with 16-byte accesses.  The lengths
// are read by every workgroup of the copy, so they are updated by a second, tiny kernel behind it.
#include "mcsd_internal.h"

namespace {

struct CommitParams {
    const void *kt[MCSD_COMMIT_MAX_LAYERS];
    const void *vt[MCSD_COMMIT_MAX_LAYERS];
    void *kp[MCSD_COMMIT_MAX_LAYERS];
    void *vp[MCSD_COMMIT_MAX_LAYERS];
    const int64_t *seq_base;
    const int32_t *path, *alen, *tokens, *new_tokens;
    int32_t *lens, *ids, *n_ids;
    int64_t node_stride, head_stride;
    int32_t B, H, d, elem_bytes, gamma, n_nodes, max_prefix, n_new, n_append;
};

__device__ inline int clamp_len(int L, int max_prefix) { return L < 0 ? 0 : (L > max_prefix ? max_prefix : L); }
__device__ inline int clamp_acc(int a, int gamma) { return a < 0 ? 0 : (a > gamma ? gamma : a); }

// grid (gamma, B, n_layers): cache row L_b + j of layer z <- tree row of node path[b][j], all heads, K and V
__global__ __launch_bounds__(256) void commit_copy_kernel(const CommitParams P)
{
    const int j = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
    if (j >= clamp_acc(P.alen[b], P.gamma)) return;
    const int node = P.path[(int64_t)b * P.gamma + j];
    if (node < 0 || node >= P.n_nodes) return;                             // never dereferenced
    const int64_t row = clamp_len(P.lens[b], P.max_prefix) + j;            // < capacity: the host checked max_prefix + gamma
    const int64_t eb = P.elem_bytes;
    const int chunks = (int)(P.d * eb) >> 4;                               // 16-byte chunks per row of one head
    const char *kt = (const char *)P.kt[layer], *vt = (const char *)P.vt[layer];
    char *kp = (char *)P.kp[layer], *vp = (char *)P.vp[layer];
    const int64_t dst0 = (P.seq_base[b] + row * P.d) * eb;
    for (int x = threadIdx.x; x < P.H * chunks; x += 256) {
        const int h = x / chunks, c = x - h * chunks;
        const int64_t src = ((((int64_t)b * P.H + h) * P.node_stride + node) * P.d) * eb + (int64_t)c * 16;
        const int64_t dst = dst0 + (int64_t)h * P.head_stride * eb + (int64_t)c * 16;
        const uint4 kv = *(const uint4 *)(kt + src);
        const uint4 vv = *(const uint4 *)(vt + src);
        *(uint4 *)(kp + dst) = kv;
        *(uint4 *)(vp + dst) = vv;
    }
}

// one thread per sequence: new length, token ids that join the input
__global__ void commit_finish_kernel(const CommitParams P)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= P.B) return;
    const int a = clamp_acc(P.alen[b], P.gamma);
    const int W = P.gamma + P.n_append;
    int32_t *ids = P.ids + (int64_t)b * W;
    int k = 0;
    for (int j = 0; j < a; ++j) {
        const int node = P.path[(int64_t)b * P.gamma + j];
        ids[k++] = (node >= 0 && node < P.n_nodes) ? P.tokens[(int64_t)b * P.n_nodes + node] : -1;
    }
    for (int j = 0; j < P.n_append; ++j) ids[k++] = P.new_tokens[(int64_t)b * P.n_new + j];
    P.n_ids[b] = k;
    for (; k < W; ++k) ids[k] = -1;
    P.lens[b] = clamp_len(P.lens[b], P.max_prefix) + a;
}

}  // namespace

extern "C" int mcsd_commit_path(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H, int32_t d,
                                int32_t n_layers, const void *const *k_tree, const void *const *v_tree,
                                int64_t node_stride, void *const *k_prefix, void *const *v_prefix,
                                const int64_t *seq_base_dev, int64_t head_stride, int32_t max_prefix,
                                int32_t capacity, const int32_t *out_path_dev, const int32_t *accept_len_dev,
                                const int32_t *tokens_dev, const int32_t *new_tokens_dev, int32_t n_new,
                                int32_t n_append, int32_t *prefix_lens_dev, int32_t *out_ids_dev,
                                int32_t *out_n_ids_dev, void *hip_stream)
{
    if (!mask || !k_tree || !v_tree || !k_prefix || !v_prefix || !seq_base_dev || !out_path_dev || !accept_len_dev ||
        !tokens_dev || !prefix_lens_dev || !out_ids_dev || !out_n_ids_dev)
        return MCSD_EINVAL;
    if (dtype != MCSD_F32 && dtype != MCSD_BF16) return MCSD_EINVAL;
    if (B < 1 || B > 65535 || H < 1 || H > 65535 || d < 1 || n_layers < 1) return MCSD_EINVAL;
    if (n_layers > MCSD_COMMIT_MAX_LAYERS) return MCSD_EUNSUPPORTED;
    if (mask->gamma < 1 || mask->gamma > MCSD_MAX_LEVELS || mask->n_nodes < 1) return MCSD_EINVAL;
    if (node_stride < mask->n_nodes || head_stride < 0 || max_prefix < 0) return MCSD_EINVAL;
    if ((int64_t)max_prefix + mask->gamma > (int64_t)capacity) return MCSD_EINVAL;
    if (n_new < 0 || n_append < 0 || n_append > n_new || (n_append > 0 && !new_tokens_dev)) return MCSD_EINVAL;
    const int eb = dtype == MCSD_BF16 ? 2 : 4;
    if (((int64_t)d * eb) & 15) return MCSD_EUNSUPPORTED;
    if (((node_stride * d) & 7) || (head_stride & 7)) return MCSD_EINVAL;

    CommitParams P;
    for (int l = 0; l < n_layers; ++l) {
        if (!k_tree[l] || !v_tree[l] || !k_prefix[l] || !v_prefix[l]) return MCSD_EINVAL;
        if (((uintptr_t)k_tree[l] | (uintptr_t)v_tree[l] | (uintptr_t)k_prefix[l] | (uintptr_t)v_prefix[l]) & 15) return MCSD_EINVAL;
        P.kt[l] = k_tree[l]; P.vt[l] = v_tree[l]; P.kp[l] = k_prefix[l]; P.vp[l] = v_prefix[l];
    }
    for (int l = n_layers; l < MCSD_COMMIT_MAX_LAYERS; ++l) { P.kt[l] = P.vt[l] = nullptr; P.kp[l] = P.vp[l] = nullptr; }
    P.seq_base = seq_base_dev;
    P.path = out_path_dev; P.alen = accept_len_dev; P.tokens = tokens_dev; P.new_tokens = new_tokens_dev;
    P.lens = prefix_lens_dev; P.ids = out_ids_dev; P.n_ids = out_n_ids_dev;
    P.node_stride = node_stride; P.head_stride = head_stride;
    P.B = B; P.H = H; P.d = d; P.elem_bytes = eb; P.gamma = mask->gamma; P.n_nodes = mask->n_nodes;
    P.max_prefix = max_prefix; P.n_new = n_new; P.n_append = n_append;

    hipStream_t st = (hipStream_t)hip_stream;
    mcsd_launch(MCSD_KERNEL_COMMIT_COPY, commit_copy_kernel, dim3(mask->gamma, B, n_layers), dim3(256), st, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return MCSD_EHIP;
    hipLaunchKernelGGL(commit_finish_kernel, dim3((B + 63) / 64), dim3(64), 0, st, P);
    return mcsd_hip_status(hipGetLastError());
}
