/*
 * libmcsd -- verification hot path of multi-candidate speculative decoding on AMD MI355X (gfx950).
 *
 * Implements, for "Improving Multi-candidate Speculative Decoding" (arXiv 2409.10644):
 *   - the topology-aware causal mask of a candidate token tree, built once for the longest draft length
 *     and sliced for every shorter one without rebuilding (Sec. 2.2, Sec. 3.2 and Fig. 2);
 *   - the target model's tree-attention pass: every tree node attends to the prefix KV cache and to its
 *     own ancestors in the tree (Sec. 2.2);
 *   - multi-candidate acceptance by recursive rejection sampling, longest-path selection for
 *     target-initialised trees and sampling of the new token(s) (Sec. 2.1, Sec. 3.1, Fig. 1 steps 4-6);
 *   - the update after acceptance: the accepted path's K/V rows join the prefix cache (Fig. 1 step 6).
 *   - the early-stop decision models that end a draft tree when no level-end node is likely to be accepted
 *     (Sec. 3.3), and the attention pass for the newest tree level only, grouped-query heads and an fp8 cache.
 *
 * Plain C ABI.  Every pointer is marked HOST or DEVICE.  The library owns only mask handles; every
 * tensor and workspace belongs to the caller.  Device work is enqueued on the caller's HIP stream and
 * the calls return without synchronising (mcsd_build_mask excepted).  Functions return MCSD_OK (0) or a
 * negative status; they never abort, throw or print.  Arguments are validated on the host before any
 * launch; on error nothing has been enqueued and no output has been touched.  The calls read no environment
 * variable and keep no mutable state besides the mask handles and the one-shot arming of mcsd_profile_next, so
 * calls on distinct streams (with distinct workspaces) may be made from several host threads at once.
 *
 * Tree convention.  A tree is the tuple of per-level branching factors (b_1 .. b_G), e.g. (4,2,2,1) or the
 * target-initialised (2,4,3,1,1) of Sec. 4.1.  Level l has N_l = b_1*...*b_l nodes; nodes are numbered
 * level by level, children of one parent next to each other, so node a of level l > 1 has parent a / b_l
 * of level l-1.  "gamma" below is the number of tree levels in use; N(gamma) = N_1 + ... + N_gamma.
 */
#ifndef MCSD_H
#define MCSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MCSD_OK = 0,
    MCSD_EINVAL = -1,       /* bad argument (null pointer, size out of range, gamma outside 1..gamma_max, ...) */
    MCSD_ENOMEM = -2,       /* host or device allocation failed (mcsd_build_mask only) */
    MCSD_EHIP = -3,         /* a HIP call or kernel launch reported an error */
    MCSD_EWORKSPACE = -4,   /* workspace missing or smaller than mcsd_*_workspace() says */
    MCSD_EUNSUPPORTED = -5  /* valid request outside the kernels' limits (see each function) */
};

enum { MCSD_MAX_LEVELS = 32, MCSD_MAX_NODES = 4096, MCSD_ATTN_MAX_NODES = 128, MCSD_MAX_BRANCH = 64,
       MCSD_MAX_VOCAB = 262144 };

typedef enum { MCSD_F32 = 0, MCSD_BF16 = 1 } mcsd_dtype_t;
typedef enum { MCSD_DRAFT_INIT = 0, MCSD_TARGET_INIT = 1 } mcsd_mode_t;

/* Static string for a status code.  HOST.  Never free it. */
const char *mcsd_strerror(int status);

/* ---------------------------------------------------------------------------------------------------
 * Mask (Sec. 2.2; Sec. 3.2, Fig. 2)
 * ------------------------------------------------------------------------------------------------- */

typedef struct mcsd_mask mcsd_mask_t; /* opaque, owned by the library */

/* A borrowed view of (a slice of) a mask.  Valid until mcsd_free_mask() of the handle it came from.
 * Bit j of row i (word i*words_per_row + j/64, bit j%64) is 1 iff tree node j is node i itself or an
 * ancestor of node i.  Rows of a slice keep the stride of the full mask. */
typedef struct {
    int32_t gamma;            /* levels in this slice */
    int32_t n_nodes;          /* N(gamma) */
    int32_t gamma_max;        /* levels of the full mask */
    int32_t n_nodes_max;      /* N(gamma_max) */
    int32_t words_per_row;    /* 64-bit words per row, that of the full mask */
    int32_t device;           /* HIP device that holds the *_dev arrays */
    const uint64_t *bits_host;      /* HOST   [n_nodes_max][words_per_row] */
    const uint64_t *bits_dev;       /* DEVICE same layout */
    const int32_t *parent_host;     /* HOST   [n_nodes_max], -1 for level-1 nodes */
    const int32_t *parent_dev;      /* DEVICE */
    const int32_t *level_host;      /* HOST   [n_nodes_max], 1-based */
    const int32_t *level_off_host;  /* HOST   [gamma_max+1], first node id of each level; last = n_nodes_max */
    const int32_t *branching_host;  /* HOST   [gamma_max] */
} mcsd_mask_view_t;

/* Build the mask for the whole tree (all gamma_max levels) on the host and upload it once to the current
 * HIP device.  Synchronises.  branching: HOST [gamma_max], every entry in 1..MCSD_MAX_BRANCH;
 * 1 <= gamma_max <= MCSD_MAX_LEVELS; N(gamma_max) <= MCSD_MAX_NODES.  *out receives a handle the caller
 * releases with mcsd_free_mask().  On a machine without a HIP device the handle holds the host copy only
 * (views have device = -1 and null *_dev pointers, which the device entry points reject). */
int mcsd_build_mask(const int32_t *branching, int32_t gamma_max, mcsd_mask_t **out);

/* The mask for draft length gamma (1..gamma_max): the upper-left N(gamma) x N(gamma) block of the full
 * mask (Sec. 3.2).  Constant time: fills *out (HOST) with pointers into the handle; no allocation, no
 * copy, no launch. */
int mcsd_slice_mask(const mcsd_mask_t *full, int32_t gamma, mcsd_mask_view_t *out);

/* Releases the handle's host and device memory.  NULL is allowed.  Views of it become invalid. */
void mcsd_free_mask(mcsd_mask_t *mask);

/* ---------------------------------------------------------------------------------------------------
 * Tree attention (Sec. 2.2)
 *
 * For every sequence b, head h and tree node i < n_nodes:
 *     out[b][h][i] = sum_j softmax_j(softmax_scale * <q_i, k_j>) * v_j
 * over all prefix keys j < prefix_lens[b] and all tree keys j whose mask bit (i, j) is set.
 *
 * q, k_tree, v_tree, out : DEVICE [B][H][node_stride][d]; the first n_nodes rows of each (b,h) are used /
 *                          written (node_stride >= n_nodes lets a gamma-slice be a view of gamma_max tensors).
 * k_prefix, v_prefix     : DEVICE; element (b,h,j,c) at seq_base[b] + h*head_stride + j*d + c.
 * seq_base_dev           : DEVICE int64 [B], element offsets.   prefix_lens_dev: DEVICE int32 [B], each in
 *                          0..max_prefix (larger values are clamped to max_prefix).
 * dtype                  : element type of q/k/v/out.  MCSD_BF16: bf16 in, fp32 accumulate on MFMA, bf16 out
 *                          (when the keys of a (sequence, head) are split over workgroups, each workgroup's
 *                          unnormalised partial output is exchanged as bf16 with fp32 maxima and denominators: one
 *                          more rounding of the output's own precision).  MCSD_F32: fp32 end to end on the vector ALU.
 * Limits: d in {64, 128}; 1 <= n_nodes <= MCSD_ATTN_MAX_NODES; softmax_scale finite and > 0; all tensor
 * base addresses 16-byte aligned; node_stride*d and head_stride and seq_base multiples of 8 elements.
 * workspace: DEVICE, at least mcsd_tree_attention_workspace(...) bytes (0 when the keys are not split: then it may
 * be NULL), 256-byte aligned; holds the partial results of the key splits and the arrival counters with which the
 * workgroup that finishes a (sequence, head) last folds them.  It must have been prepared with mcsd_workspace_init
 * once (and again after anything else wrote to it); every call leaves it prepared.  A call that finds a workspace
 * that was never prepared fills the output rows it owns with NaN.  Calls that share a workspace must be ordered on
 * one stream.  Inputs are never modified.
 * ------------------------------------------------------------------------------------------------- */

/* Prepares `workspace` (DEVICE, 256-byte aligned, workspace_bytes long) for the tree-attention entry points: one small
 * fill kernel on the stream (no memset node, so the call may be captured into a HIP graph).  Sizes too small to serve
 * any call that needs a workspace (below 66 KiB) are accepted and left alone. */
int mcsd_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream);

size_t mcsd_tree_attention_workspace(int32_t B, int32_t H, int32_t d, int32_t n_nodes, int32_t max_prefix);

int mcsd_tree_attention(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H, int32_t d,
                        const void *q, const void *k_tree, const void *v_tree, int64_t node_stride,
                        const void *k_prefix, const void *v_prefix, const int64_t *seq_base_dev,
                        const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                        float softmax_scale, void *out, void *workspace, size_t workspace_bytes,
                        void *hip_stream);

/* The same attention for the query rows row_begin .. n_nodes-1 only (0 <= row_begin < n_nodes); rows below
 * row_begin of q are not read and those of out are not written.  Keys are unchanged: the prefix and every tree
 * node j < n_nodes that the mask shows to the row.  This is the draft side of Fig. 1 step 3 and Sec. 3.2: the tree
 * grows level by level, each step takes the next slice of the mask built once and needs outputs only for the newest
 * level, row_begin = level_off_host[gamma-1].  Arguments, limits and workspace rules as above, with the workspace
 * sized by mcsd_tree_attention_rows_workspace (never more than mcsd_tree_attention_workspace of the same shape). */
size_t mcsd_tree_attention_rows_workspace(int32_t B, int32_t H, int32_t d, int32_t n_nodes, int32_t row_begin,
                                          int32_t max_prefix);

int mcsd_tree_attention_rows(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H, int32_t d,
                             int32_t row_begin, const void *q, const void *k_tree, const void *v_tree,
                             int64_t node_stride, const void *k_prefix, const void *v_prefix,
                             const int64_t *seq_base_dev, const int32_t *prefix_lens_dev, int64_t head_stride,
                             int32_t max_prefix, float softmax_scale, void *out, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* Grouped-query attention (beyond the paper's Llama-2-7B multi-head shape): H_q query heads share H_kv key/value
 * heads, H_q a multiple of H_kv; query head h uses key/value head h / (H_q / H_kv).
 * q, out         : DEVICE [B][H_q][node_stride][d]
 * k_tree, v_tree : DEVICE [B][H_kv][node_stride][d]
 * k_prefix, v_prefix : element (b,kvh,j,c) at seq_base[b] + kvh*head_stride + j*d + c
 * Everything else as mcsd_tree_attention_rows (which is the H_q == H_kv case).  On the bf16 path up to four query
 * blocks of one key/value head (4, 2 or 1 query heads, depending on the number of rows) are served by one
 * workgroup, so that head's K/V bytes leave HBM once for all of them. */
size_t mcsd_tree_attention_gqa_workspace(int32_t B, int32_t H_q, int32_t H_kv, int32_t d, int32_t n_nodes,
                                         int32_t row_begin, int32_t max_prefix);

int mcsd_tree_attention_gqa(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H_q, int32_t H_kv,
                            int32_t d, int32_t row_begin, const void *q, const void *k_tree, const void *v_tree,
                            int64_t node_stride, const void *k_prefix, const void *v_prefix,
                            const int64_t *seq_base_dev, const int32_t *prefix_lens_dev, int64_t head_stride,
                            int32_t max_prefix, float softmax_scale, void *out, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------------------------------
 * Tree attention over a quantised prefix cache (beyond the paper's bf16 setting; same operation, Sec. 2.2).
 *
 * As mcsd_tree_attention_gqa with dtype MCSD_BF16 and d = 128, except that the prefix K/V cache holds 8-bit
 * floating point: the OCP E4M3 format (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities,
 * S.1111.111 = NaN, largest finite value 448).  A stored key stands for stored * k_scale, a stored value for
 * stored * v_scale (one scale each per call; k_scale > 0).  q, k_tree, v_tree and out stay bf16: the tree's own
 * keys and values are fresh activations.  Conversion to bf16 is exact, so results differ from the bf16 entry point
 * on the same (representable) values only by the rounding of P * v_scale.
 *
 * k_prefix_fp8, v_prefix_fp8 : DEVICE uint8, element (b, kv head, j, c) at seq_base[b] + h*head_stride + j*128 + c,
 *                              in elements = bytes; head_stride and every seq_base[b] multiples of 16
 * workspace                  : DEVICE, mcsd_tree_attention_fp8kv_workspace(...) bytes, 256-byte aligned
 * Everything else as in mcsd_tree_attention_gqa.  Errors: the same, and MCSD_EINVAL for a scale that is not
 * finite or a k_scale <= 0.
 * ------------------------------------------------------------------------------------------------- */
size_t mcsd_tree_attention_fp8kv_workspace(int32_t B, int32_t H_q, int32_t H_kv, int32_t n_nodes, int32_t row_begin,
                                           int32_t max_prefix);

int mcsd_tree_attention_fp8kv(const mcsd_mask_view_t *mask, int32_t B, int32_t H_q, int32_t H_kv, int32_t row_begin,
                              const void *q, const void *k_tree, const void *v_tree, int64_t node_stride,
                              const void *k_prefix_fp8, const void *v_prefix_fp8, float k_scale, float v_scale,
                              const int64_t *seq_base_dev, const int32_t *prefix_lens_dev, int64_t head_stride,
                              int32_t max_prefix, float softmax_scale, void *out, void *workspace,
                              size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------------------------------
 * mcsd_tree_attention for callers that cannot allocate device memory or carry a workspace around: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * mcsd_tree_attention minus the workspace: the partial results and arrival counters of the key splits live in a
 * device array of MCSD_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until the process ends; its
 * address is looked up on the first call on a device, which also enqueues one small fill kernel on the stream).
 * The call allocates and frees nothing.  Shapes that need more than the array holds are MCSD_EUNSUPPORTED and nothing
 * is enqueued (the five headline configurations need 0 to 17.4 MB; larger batches of long prefixes under wide trees
 * need more and must bring a workspace).  All calls on one GPU share the array: calls that overlap in time on one GPU,
 * on whatever streams, race on it and must be ordered by the caller.
 * ------------------------------------------------------------------------------------------------- */
enum { MCSD_STATIC_SCRATCH_BYTES = 24 * 1024 * 1024 };

int mcsd_tree_attention_static(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H, int32_t d,
                               const void *q, const void *k_tree, const void *v_tree, int64_t node_stride,
                               const void *k_prefix, const void *v_prefix, const int64_t *seq_base_dev,
                               const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                               float softmax_scale, void *out, void *hip_stream);

/* ---------------------------------------------------------------------------------------------------
 * The same operation (Sec. 2.2) with the launch plan in the caller's hands, for measurement sweeps and tests; one entry
 * point covers what the four above do (prefix_fp8 != 0: the prefix cache holds E4M3 bytes and k_scale / v_scale
 * apply, d = 128, dtype MCSD_BF16; otherwise the scales are ignored).  The plan is a function of the shape arguments
 * and of *tuning only: the library reads no environment variable and keeps no state between the workspace query and
 * the call, so the same struct must be given to both.  tuning == NULL means all zeros.  Results do not depend on the
 * plan beyond the order in which partial results are added.  MCSD_EINVAL for values outside the ranges below.
 * ------------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t key_splits;     /* 0: the library chooses; 1..64: workgroups that share the prefix keys of one (sequence, head) */
    int32_t natural_order;  /* 0: the library chooses; 1: never reorder the workgroups of a ragged batch by length */
    int32_t fold;           /* 0: the library chooses; 1: always fold the key splits' partial results in a second kernel */
    int32_t stages;         /* 0: the library chooses; 2 or 4: LDS stages of the bf16 sweep's K/V ring (4 needs a compute
                               unit per workgroup and trees of more than 32 rows; ignored where it cannot apply) */
    int32_t tree_keys;      /* which workgroup of a (sequence, head) with split keys takes the tree's own keys: 0: the
                               library chooses; 1: one of their own; 2: the first split; 3: the last split that has keys */
} mcsd_attention_tuning_t;

size_t mcsd_tree_attention_tuned_workspace(const mcsd_attention_tuning_t *tuning, int32_t prefix_fp8, int32_t B,
                                           int32_t H_q, int32_t H_kv, int32_t d, int32_t n_nodes, int32_t row_begin,
                                           int32_t max_prefix);

int mcsd_tree_attention_tuned(const mcsd_attention_tuning_t *tuning, const mcsd_mask_view_t *mask, mcsd_dtype_t dtype,
                              int32_t prefix_fp8, float k_scale, float v_scale, int32_t B, int32_t H_q, int32_t H_kv,
                              int32_t d, int32_t row_begin, const void *q, const void *k_tree, const void *v_tree,
                              int64_t node_stride, const void *k_prefix, const void *v_prefix,
                              const int64_t *seq_base_dev, const int32_t *prefix_lens_dev, int64_t head_stride,
                              int32_t max_prefix, float softmax_scale, void *out, void *workspace,
                              size_t workspace_bytes, void *hip_stream);

/* The launch plan that a tree-attention call with these arguments would use on the current HIP device right now (it
 * depends on the device's compute units and, for fold_in_kernel, on a mask having been built on that device, which is
 * when the library learns how workgroups are dealt to the chip's dies).  HOST only, nothing is launched.  For
 * measurement: it names the kernel instantiation and grid that profiler output has to be matched with. */
typedef struct {
    int32_t mfma_path;          /* 1: bf16 sweep on the matrix cores; 0: fp32 kernels on the vector ALU */
    int32_t query_blocks;       /* 32-row query blocks per workgroup: 1, 2 or 4 */
    int32_t key_splits;         /* workgroups that share the prefix keys of one (sequence, head [chunk]) */
    int32_t workgroups;         /* grid of the sweep launch */
    int32_t stages;             /* LDS stages of the K/V ring (0 on the fp32 path) */
    int32_t fold_in_kernel;     /* 1: partial results are folded by the sweep itself; 0: a second kernel, or no splits */
    int32_t ordered_by_length;  /* 1: workgroups take their work in an order computed from the prefix lengths */
} mcsd_attention_plan_t;

int mcsd_tree_attention_plan(const mcsd_attention_tuning_t *tuning, mcsd_dtype_t dtype, int32_t prefix_fp8, int32_t B,
                             int32_t H_q, int32_t H_kv, int32_t d, int32_t n_nodes, int32_t row_begin,
                             int32_t max_prefix, mcsd_attention_plan_t *out);

/* ---------------------------------------------------------------------------------------------------
 * Verification (Sec. 2.1; Sec. 3.1; Fig. 1 steps 4-6)
 *
 * Recursive rejection sampling down the tree.  At a context with target row p and draft row q the
 * children are tried in node order: child c with token x is accepted iff  u_accept[c] * q(x) * S < r(x),
 * where r starts as p with S = 1 and after every rejection r <- max(r - S*q, 0), S <- sum(r) (the
 * unnormalised form of p <- norm(max(p - q, 0))).  The first accepted child becomes the context.  The walk
 * ends when all children of a context are rejected (new tokens come from r, or from p if r vanished) or
 * when level gamma is reached (new tokens come from the target row after the last node).
 * MCSD_DRAFT_INIT : one walk from the context that ends the prefix.
 * MCSD_TARGET_INIT: level-1 nodes were sampled from the target and are accepted untested; one walk per
 *                   level-1 node, the longest path wins (lowest node id on ties).
 * All arithmetic is binary64 with vocabulary sums taken as a balanced binary tree over the index space
 * padded with zeros to a power of two, and new tokens are drawn by descending that tree with threshold
 * u_sample * S; results are therefore reproducible bit for bit on any machine.
 *
 * tokens         : DEVICE int32 [B][n_nodes], each in 0..V-1
 * p_target       : DEVICE fp32; row r of sequence b at b*p_batch_stride + r*V; row 0 is the context that
 *                  ends the prefix, row 1+i the context after node i; rows 0..n_nodes
 * q_draft        : DEVICE fp32; same addressing with q_batch_stride; rows 0..N(gamma-1)
 * u_accept       : DEVICE fp32 [B][n_nodes] in [0,1), indexed by node
 * u_sample       : DEVICE fp32 [B][n_new] in [0,1);   0 <= n_new <= 64
 * out_path       : DEVICE int32 [B][gamma], accepted node ids from level 1 down, padded with -1
 * out_accept_len : DEVICE int32 [B]
 * out_new_tokens : DEVICE int32 [B][n_new], i.i.d. draws from the terminal distribution
 * workspace      : DEVICE, mcsd_verify_tree_workspace(...) bytes (0 for MCSD_DRAFT_INIT: may be NULL), 256-byte
 *                  aligned; need not be initialised.  Afterwards it holds the walks of all b_1 level-1 subtrees, for
 *                  inspection: int32 [B][b_1][gamma] paths (-1 padded), then int32 [B][b_1] accepted lengths, then
 *                  int32 [B][b_1][max(n_new,1)] new tokens, each block starting at a multiple of 256 bytes
 * Limits: 1 <= V <= MCSD_MAX_VOCAB.
 * ------------------------------------------------------------------------------------------------- */
size_t mcsd_verify_tree_workspace(const mcsd_mask_view_t *mask, mcsd_mode_t mode, int32_t B, int32_t n_new);

int mcsd_verify_tree(const mcsd_mask_view_t *mask, mcsd_mode_t mode, int32_t B, int32_t V,
                     const int32_t *tokens, const float *p_target, const float *q_draft,
                     int64_t p_batch_stride, int64_t q_batch_stride, const float *u_accept,
                     const float *u_sample, int32_t n_new, int32_t *out_path, int32_t *out_accept_len,
                     int32_t *out_new_tokens, void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same walk with the sampling scheme of the candidates stated (Sec. 2.2 leaves it open; mcsd_verify_tree is
 * MCSD_WITH_REPLACEMENT).  MCSD_WITHOUT_REPLACEMENT: the children of a context are distinct tokens, each drawn from
 * the draft row with the earlier ones removed; after a rejection the draft row therefore loses the rejected token as
 * well (q(x) <- 0, q <- norm(q)) before the next child is tested.  In the unnormalised arithmetic above, with q' the
 * draft row with zeros and Sq = 1 - (draft mass removed so far, subtracted in child order):
 *   test  u_accept[c] * q'(x) * S < r(x) * Sq,     update  r <- max(r * Sq - S * q', 0), then q'(x) <- 0.
 * For a chain (one child per context) both schemes are the same rule.  Arguments and errors as mcsd_verify_tree;
 * MCSD_EINVAL for an unknown scheme. */
typedef enum { MCSD_WITH_REPLACEMENT = 0, MCSD_WITHOUT_REPLACEMENT = 1 } mcsd_sampling_t;

int mcsd_verify_tree_sampling(const mcsd_mask_view_t *mask, mcsd_mode_t mode, mcsd_sampling_t sampling, int32_t B,
                              int32_t V, const int32_t *tokens, const float *p_target, const float *q_draft,
                              int64_t p_batch_stride, int64_t q_batch_stride, const float *u_accept,
                              const float *u_sample, int32_t n_new, int32_t *out_path, int32_t *out_accept_len,
                              int32_t *out_new_tokens, void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------------------------------
 * Update after acceptance (Fig. 1 step 6): the accepted path becomes part of the prefix.
 *
 * For every sequence b with a = accept_len[b] (0..gamma) and L = prefix_lens[b] (clamped to 0..max_prefix):
 * in each of the n_layers layers, cache row L + j of every head receives the tree K and V row of node
 * out_path[b][j], j = 0 .. a-1 (root side first); then prefix_lens[b] becomes L + a.  out_ids[b] receives the
 * accepted tokens tokens[b][out_path[b][j]] in that order followed by the first n_append new tokens
 * (draft-initialised decoding appends the one new token to the input, n_append = 1; with a target-initialised tree
 * the new tokens are the next tree's first level, n_append = 0), padded with -1; out_n_ids[b] counts the ids set.
 *
 * k_tree, v_tree     : HOST arrays [n_layers] of DEVICE pointers, each [B][H][node_stride][d] (read)
 * k_prefix, v_prefix : HOST arrays [n_layers] of DEVICE pointers to the caches, addressed as in
 *                      mcsd_tree_attention (seq_base_dev, head_stride shared by all layers); rows
 *                      L .. L+a-1 of every head are written, nothing else
 * capacity           : rows every (sequence, head) of the caches can hold; max_prefix + gamma <= capacity is
 *                      required, so a write can never leave the cache
 * out_path_dev, accept_len_dev, new_tokens_dev : as written by mcsd_verify_tree (DEVICE); tokens_dev as given to it
 * prefix_lens_dev    : DEVICE int32 [B], read and updated in place
 * out_ids_dev        : DEVICE int32 [B][gamma + n_append];  out_n_ids_dev: DEVICE int32 [B]
 * Node ids outside 0..n_nodes-1 and lengths outside 0..gamma are skipped / clamped, never dereferenced.
 * ONE call must cover all layers of the model: the call advances prefix_lens and writes the ids, so a second call
 * for further layers would append the same path again at the advanced lengths.  A model deeper than
 * MCSD_COMMIT_MAX_LAYERS layers is MCSD_EUNSUPPORTED rather than served in pieces.
 * Limits: 1 <= n_layers <= MCSD_COMMIT_MAX_LAYERS; d*sizeof(element) a multiple of 16; tensor base
 * addresses 16-byte aligned; node_stride*d, head_stride and seq_base multiples of 8 elements.
 * Two launches on the stream: the copies, then the lengths and ids (so prefix_lens is updated in place).
 * ------------------------------------------------------------------------------------------------- */
enum { MCSD_COMMIT_MAX_LAYERS = 64 };

int mcsd_commit_path(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H, int32_t d,
                     int32_t n_layers, const void *const *k_tree, const void *const *v_tree, int64_t node_stride,
                     void *const *k_prefix, void *const *v_prefix, const int64_t *seq_base_dev,
                     int64_t head_stride, int32_t max_prefix, int32_t capacity, const int32_t *out_path_dev,
                     const int32_t *accept_len_dev, const int32_t *tokens_dev, const int32_t *new_tokens_dev,
                     int32_t n_new, int32_t n_append, int32_t *prefix_lens_dev, int32_t *out_ids_dev,
                     int32_t *out_n_ids_dev, void *hip_stream);

/* ---------------------------------------------------------------------------------------------------
 * Early-stop decision models (Sec. 3.3; threshold beta = 0.4 in the caption of Fig. 2)
 *
 * After a draft-generation turn a small MLP predicts, for each of the W candidate sequences of each of B trees,
 * the probability that the target model accepts it; stop[b] = 1 iff every sequence of tree b is predicted below
 * beta (strictly), which ends draft generation for that tree before the maximum depth.
 *   mcsd_early_stop_distribution : type 2, input Concat(Topk(y), Ent(y)) of the draft model's output distribution
 *                                  y for the newest token: the k largest probabilities, largest first (values,
 *                                  duplicates kept, zeros when V < k), then the Shannon entropy in nats
 *                                  (0 ln 0 = 0); k + 1 inputs
 *   mcsd_early_stop_hidden       : type 1, input the draft model's hidden state of the newest token
 * An n-layer MLP is n affine maps with ReLU between them and a logistic sigmoid after the last (Sec. 3.3 gives the
 * layer counts, two for type 2 and three for type 1, and nothing else; weights are the caller's).  The networks
 * are evaluated in fp32: fused multiply-adds whose partial sums are combined as a tree, within about 1e-6 of an
 * evaluation in binary64 (a probability closer than that to beta may fall on the other side of it); the entropy
 * uses an fp32 logarithm per entry and a binary64 sum.
 *
 * mlp             : HOST struct; weight[l] / bias[l] are DEVICE fp32 arrays, weight[l] row-major
 *                   [width[l+1]][width[l]] (one row per output unit), width[0] = inputs, width[n_layers] = 1
 * draft_rows_dev  : DEVICE fp32; the distribution of sequence w of tree b starts at b*batch_stride + w*row_stride
 *                   (elements), V entries >= 0 (NaNs are ignored by Topk)
 * hidden_dev      : DEVICE fp32; same addressing, width[0] entries per row
 * features_dev    : DEVICE fp32 [B][W][k+1], the MLP's inputs rounded to fp32, or NULL
 * prob_dev        : DEVICE fp32 [B][W];   stop_dev : DEVICE int32 [B], decided from the fp32 values in prob_dev
 *                   (a NaN probability counts as not below beta)
 * Limits: 1 <= k <= MCSD_DECISION_MAX_K, 1 <= V <= MCSD_MAX_VOCAB, 1 <= n_layers <= MCSD_MLP_MAX_LAYERS, widths
 * after the first <= MCSD_MLP_MAX_WIDTH, hidden-state width <= MCSD_MLP_MAX_INPUTS.  B = 0 is a no-op.
 * Two launches on the stream (probabilities, then the stop flags); no workspace.
 * ------------------------------------------------------------------------------------------------- */
enum { MCSD_DECISION_MAX_K = 16, MCSD_MLP_MAX_LAYERS = 3, MCSD_MLP_MAX_WIDTH = 512, MCSD_MLP_MAX_INPUTS = 8192 };

typedef struct mcsd_mlp {
    int32_t n_layers;
    int32_t width[MCSD_MLP_MAX_LAYERS + 1];
    const float *weight[MCSD_MLP_MAX_LAYERS];
    const float *bias[MCSD_MLP_MAX_LAYERS];
} mcsd_mlp_t;

int mcsd_early_stop_distribution(const mcsd_mlp_t *mlp, int32_t B, int32_t W, int32_t V, int32_t k,
                                 const float *draft_rows_dev, int64_t batch_stride, int64_t row_stride, float beta,
                                 float *features_dev, float *prob_dev, int32_t *stop_dev, void *hip_stream);

int mcsd_early_stop_hidden(const mcsd_mlp_t *mlp, int32_t B, int32_t W, const float *hidden_dev,
                           int64_t batch_stride, int64_t row_stride, float beta, float *prob_dev, int32_t *stop_dev,
                           void *hip_stream);

/* ---------------------------------------------------------------------------------------------------
 * Measurement aid (not part of the method).  Arms a one-shot pair of HIP events (hipEvent_t, created by the
 * caller with timing enabled) for one of the library's kernels: the next launch of that kernel by the calling
 * process is bracketed by them, so hipEventElapsedTime(start, stop) is that kernel's own execution time on
 * the device.  The arming is consumed by exactly one launch, also when several host threads launch that kernel at
 * once (the slots are atomic); two threads arming the same kernel at the same time is the caller's to avoid.
 * Passing NULL events disarms.
 * ------------------------------------------------------------------------------------------------- */
typedef enum { MCSD_KERNEL_ATTN_SWEEP = 0, MCSD_KERNEL_ATTN_MERGE = 1, MCSD_KERNEL_VERIFY_WALK = 2,
               MCSD_KERNEL_COMMIT_COPY = 3, MCSD_KERNEL_STREAM_READ = 4, MCSD_KERNEL_DECISION = 5 } mcsd_kernel_t;
int mcsd_profile_next(mcsd_kernel_t kernel, void *start_event, void *stop_event);

/* Measurement aid (not part of the method).  Reads `bytes` (>= 16, rounded down to 16) from src_dev (DEVICE,
 * 16-byte aligned) with a plain grid-strided streaming kernel and discards them; sink_dev is 16 bytes of DEVICE
 * memory that is written only if the data has one particular value.  Timed on a buffer much larger than the caches
 * it gives the read bandwidth this machine's HBM delivers to the simplest reader.  workgroups: grid size in
 * workgroups of 256 lanes, 0 for the default of 1024. */
int mcsd_stream_read(const void *src_dev, size_t bytes, void *sink_dev, int32_t workgroups, void *hip_stream);

/* Measurement aid (not part of the method).  Runs the arithmetic of the tree-attention inner loop for one 32-key block
 * per iteration (16 MFMA 32x32x16 bf16 + maximum, 16 exponentials and bf16 packing per lane) with no memory traffic,
 * one workgroup per compute unit, under one of five arrangements of matrix and vector phases:
 *   0 one wavefront per SIMD, phases one after the other;  1 two per SIMD, free-running;  2 two per SIMD, alternating
 *   under workgroup barriers;  3 one per SIMD, software-pipelined within the wavefront;  4 two per SIMD, both pipelined.
 * Timed by the caller (events on the stream), it shows how far this machine overlaps matrix instructions with the
 * vector work of the same and of another wavefront.  out_dev: DEVICE, workgroups * 512 floats, overwritten.
 * iterations: even, 2 .. 2^20.  workgroups: 1 .. 65535. */
int mcsd_issue_probe(int32_t schedule, int32_t workgroups, int32_t iterations, void *out_dev, void *hip_stream);

/* Measurement aid (not part of the method).  Launches `workgroups` workgroups shaped like the bf16 sweep's (256 lanes,
 * 66 KiB of LDS: two per compute unit), keeps each busy for `spin` (0 .. 2^20) steps of a dependent multiply-add chain
 * so that the grid is resident together, and writes two words per workgroup to out_dev (DEVICE, workgroups * 2
 * uint32): the die it ran on (XCC_ID) and its hardware id word (HW_ID: compute unit in bits 8-11, shader array in
 * bit 12, shader engine in bits 13-15).  Shows how workgroup ids are dealt to dies and which ids share a compute
 * unit, the two facts the sweep's workgroup numbering is built on (nothing but speed depends on the second). */
int mcsd_placement_probe(int32_t workgroups, int32_t spin, void *out_dev, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MCSD_H */
