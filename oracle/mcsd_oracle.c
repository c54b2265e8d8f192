/*
 * CPU oracle for the verification hot path of multi-candidate speculative decoding
 * ("Improving Multi-candidate Speculative Decoding", arXiv 2409.10644).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the plain, slow definition that the tests, the smoke check
 * and the benchmark's CPU-baseline leg compare the GPU library against.  It shares no code with the
 * GPU library and must never be called from the product path.
 *
 * Everything is written for readability against the paper:
 *   O1  topology-aware causal mask of a token tree and its upper-left slices   (Sec. 2.2, Sec. 3.2, Fig. 2)
 *   O2  tree attention: every tree node attends to the whole prefix and to its own ancestors (Sec. 2.2)
 *   O3  multi-candidate verification: recursive rejection sampling over the tree, longest-path
 *       selection for target-initialised trees, sampling of the new token(s)    (Sec. 2.1, Sec. 3.1, Fig. 1 steps 4-6)
 *   O4  early-stop decision models: Topk/entropy features, the two MLPs, the stop rule   (Sec. 3.3)
 *
 * Arithmetic is IEEE-754 binary64 throughout (compile with -ffp-contract=off, never -ffast-math).
 * Where the paper is silent the reading is stated next to the code.
 *
 * Parity status: every function here is pinned by tests that do not re-use it (closed forms,
 * invariants, textbook special cases, brute-force enumeration); nothing is "parity unpinned".
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------------
 * Tree topology.
 *
 * A tree configuration is the tuple of per-level branching factors (b_1, ..., b_G), e.g. (4,2,2,1) or
 * the target-initialised (2,4,3,1,1) of Sec. 4.1.  Level l holds N_l = b_1*...*b_l nodes.  Nodes are
 * numbered level by level (this is the only numbering under which the mask of the first g levels is
 * the upper-left block of the full mask, as Sec. 3.2 / Fig. 2 require), and the children of one parent
 * are adjacent: the node with in-level index a at level l > 1 has the parent with in-level index
 * a / b_l at level l-1.  Level-1 nodes hang off the context that ends the prefix; their parent is -1.
 * ---------------------------------------------------------------------------------------------- */

/* Level sizes N_1..N_G into sizes[]; returns the node count N(G) = N_1 + ... + N_G, or -1 on bad input. */
int64_t mcsd_oracle_level_sizes(const int32_t *b, int32_t G, int64_t *sizes)
{
    int64_t total = 0, n = 1;
    if (!b || G < 1) return -1;
    for (int32_t l = 0; l < G; ++l) {
        if (b[l] < 1) return -1;
        n *= b[l];
        if (sizes) sizes[l] = n;
        total += n;
    }
    return total;
}

/* parent[i] and level[i] (1-based level) of every node. */
int mcsd_oracle_tree_tables(const int32_t *b, int32_t G, int32_t *parent, int32_t *level)
{
    int64_t N = mcsd_oracle_level_sizes(b, G, NULL);
    if (N < 0) return -1;
    int64_t off_prev = 0, off = 0, n = 1;
    for (int32_t l = 0; l < G; ++l) {
        n *= b[l];                                  /* N_l */
        for (int64_t a = 0; a < n; ++a) {
            level[off + a] = l + 1;
            parent[off + a] = (l == 0) ? -1 : (int32_t)(off_prev + a / b[l]);
        }
        off_prev = off;
        off += n;
    }
    return 0;
}

/* O1.  M is a dense N x N byte matrix, row-major: M[i][j] = 1 iff tree node j is node i itself or an
 * ancestor of node i (Sec. 2.2: a token may attend to the tokens on its own candidate path only).
 * The prefix is not part of the mask (Sec. 3.1: the mask side is the number of tree tokens). */
int mcsd_oracle_build_mask(const int32_t *b, int32_t G, uint8_t *M)
{
    int64_t N = mcsd_oracle_level_sizes(b, G, NULL);
    if (N < 0) return -1;
    int32_t *parent = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    int32_t *level = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    if (!parent || !level) { free(parent); free(level); return -2; }
    mcsd_oracle_tree_tables(b, G, parent, level);
    memset(M, 0, (size_t)N * (size_t)N);
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = i; j >= 0; j = parent[j])  /* i, parent(i), parent(parent(i)), ... */
            M[i * N + j] = 1;
    free(parent);
    free(level);
    return 0;
}

/* Sec. 3.2: the mask for a shorter draft length is the upper-left n x n block of the big mask. */
void mcsd_oracle_slice_mask(const uint8_t *M, int64_t n_full, int64_t n, uint8_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < n; ++j)
            out[i * n + j] = M[i * n_full + j];
}

/* ------------------------------------------------------------------------------------------------
 * O2.  Tree attention (plain definition, binary64).
 *
 * For sequence b, head h and tree node i:
 *     s_j = scale * <q_i, k_j>     over every prefix key j < L_b and every tree key j with M[i][j] = 1
 *     o_i = sum_j softmax(s)_j * v_j
 * Inputs are fp32 (dtype 0) or bfloat16 bit patterns (dtype 1); both convert to binary64 exactly.
 * Layouts: q, k_tree, v_tree [B][H][node_stride][d]; prefix K/V: element (b,h,j,c) at
 * seq_base[b] + h*head_stride + j*d + c.
 * A quantised prefix cache (beyond the paper's bf16 setting) stores 8-bit floating point, dtype 2: the OCP
 * "E4M3" format, 1 sign, 4 exponent (bias 7) and 3 mantissa bits, no infinities, S.1111.111 = NaN, largest
 * finite value 448; a stored value stands for stored * k_scale (keys) or stored * v_scale (values).
 * ---------------------------------------------------------------------------------------------- */
double mcsd_oracle_fp8_e4m3_value(uint8_t code)
{
    const int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);             /* subnormal: m/8 * 2^(1-bias) */
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

static double load_elem(const void *p, int64_t idx, int32_t dtype)
{
    if (dtype == 0) return (double)((const float *)p)[idx];
    if (dtype == 2) return mcsd_oracle_fp8_e4m3_value(((const uint8_t *)p)[idx]);
    uint32_t bits = (uint32_t)((const uint16_t *)p)[idx] << 16;   /* bfloat16 = upper half of a binary32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* One output row o_i (d values) for one (b, h, i); the prefix cache has its own element type and scales. */
static void attention_row(int32_t dtype, int32_t kv_dtype, double k_scale, double v_scale, int32_t H, int32_t d,
                          int32_t n, int64_t node_stride, const void *q, const void *k_tree, const void *v_tree,
                          const void *k_prefix, const void *v_prefix, const int64_t *seq_base, const int32_t *lens,
                          int64_t head_stride, double scale, const uint8_t *M, int64_t mask_stride, int32_t b,
                          int32_t h, int32_t i, double *out_row)
{
    const int64_t L = lens[b];
    const int64_t tree0 = ((int64_t)b * H + h) * node_stride * d;          /* (b,h,0,0) in q/k_tree/v_tree */
    const int64_t pre0 = seq_base[b] + (int64_t)h * head_stride;            /* (b,h,0,0) in the prefix cache */
    const int64_t total = L + n;
    double *s = (double *)malloc(sizeof(double) * (size_t)(total > 0 ? total : 1));
    uint8_t *vis = (uint8_t *)malloc((size_t)(total > 0 ? total : 1));

    for (int64_t j = 0; j < total; ++j) {
        const int tree = j >= L;
        const int64_t jj = tree ? j - L : j;
        vis[j] = tree ? M[(int64_t)i * mask_stride + jj] : 1;
        if (!vis[j]) continue;
        double dot = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            double qc = load_elem(q, tree0 + (int64_t)i * d + c, dtype);
            double kc = tree ? load_elem(k_tree, tree0 + jj * d + c, dtype)
                             : k_scale * load_elem(k_prefix, pre0 + jj * d + c, kv_dtype);
            dot += qc * kc;
        }
        s[j] = scale * dot;
    }
    double mx = -INFINITY;
    for (int64_t j = 0; j < total; ++j)
        if (vis[j] && s[j] > mx) mx = s[j];
    double denom = 0.0;
    for (int64_t j = 0; j < total; ++j)
        if (vis[j]) { s[j] = exp(s[j] - mx); denom += s[j]; }
    for (int32_t c = 0; c < d; ++c) out_row[c] = 0.0;
    for (int64_t j = 0; j < total; ++j) {
        if (!vis[j]) continue;
        const int tree = j >= L;
        const int64_t jj = tree ? j - L : j;
        const double w = s[j] / denom;
        for (int32_t c = 0; c < d; ++c) {
            double vc = tree ? load_elem(v_tree, tree0 + jj * d + c, dtype)
                             : v_scale * load_elem(v_prefix, pre0 + jj * d + c, kv_dtype);
            out_row[c] += w * vc;
        }
    }
    free(s);
    free(vis);
}

void mcsd_oracle_tree_attention_row(int32_t dtype, int32_t H, int32_t d, int32_t n, int64_t node_stride,
                                    const void *q, const void *k_tree, const void *v_tree,
                                    const void *k_prefix, const void *v_prefix,
                                    const int64_t *seq_base, const int32_t *lens, int64_t head_stride,
                                    double scale, const uint8_t *M, int64_t mask_stride,
                                    int32_t b, int32_t h, int32_t i, double *out_row)
{
    attention_row(dtype, dtype, 1.0, 1.0, H, d, n, node_stride, q, k_tree, v_tree, k_prefix, v_prefix, seq_base, lens,
                  head_stride, scale, M, mask_stride, b, h, i, out_row);
}

/* The same with an fp8 (E4M3) prefix cache: q, k_tree, v_tree are bfloat16. */
void mcsd_oracle_tree_attention_row_fp8kv(int32_t H, int32_t d, int32_t n, int64_t node_stride, const void *q,
                                          const void *k_tree, const void *v_tree, const void *k_prefix,
                                          const void *v_prefix, double k_scale, double v_scale, const int64_t *seq_base,
                                          const int32_t *lens, int64_t head_stride, double scale, const uint8_t *M,
                                          int64_t mask_stride, int32_t b, int32_t h, int32_t i, double *out_row)
{
    attention_row(1, 2, k_scale, v_scale, H, d, n, node_stride, q, k_tree, v_tree, k_prefix, v_prefix, seq_base, lens,
                  head_stride, scale, M, mask_stride, b, h, i, out_row);
}

void mcsd_oracle_tree_attention_fp8kv(int32_t B, int32_t H, int32_t d, int32_t n, int64_t node_stride, const void *q,
                                      const void *k_tree, const void *v_tree, const void *k_prefix, const void *v_prefix,
                                      double k_scale, double v_scale, const int64_t *seq_base, const int32_t *lens,
                                      int64_t head_stride, double scale, const uint8_t *M, int64_t mask_stride,
                                      double *out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < (int64_t)B * H; ++bh) {
        const int32_t b = (int32_t)(bh / H), h = (int32_t)(bh % H);
        for (int32_t i = 0; i < n; ++i)
            attention_row(1, 2, k_scale, v_scale, H, d, n, node_stride, q, k_tree, v_tree, k_prefix, v_prefix, seq_base,
                          lens, head_stride, scale, M, mask_stride, b, h, i, out + ((bh * n) + i) * d);
    }
}

/* All rows: out is binary64 [B][H][n][d].  (b,h) pairs are independent and may run on several threads;
 * each row is still computed by the routine above, in the same order. */
void mcsd_oracle_tree_attention(int32_t dtype, int32_t B, int32_t H, int32_t d, int32_t n, int64_t node_stride,
                                const void *q, const void *k_tree, const void *v_tree,
                                const void *k_prefix, const void *v_prefix,
                                const int64_t *seq_base, const int32_t *lens, int64_t head_stride,
                                double scale, const uint8_t *M, int64_t mask_stride, double *out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < (int64_t)B * H; ++bh) {
        const int32_t b = (int32_t)(bh / H), h = (int32_t)(bh % H);
        for (int32_t i = 0; i < n; ++i)
            mcsd_oracle_tree_attention_row(dtype, H, d, n, node_stride, q, k_tree, v_tree, k_prefix, v_prefix,
                                           seq_base, lens, head_stride, scale, M, mask_stride, b, h, i,
                                           out + ((bh * n) + i) * d);
    }
}

/* ------------------------------------------------------------------------------------------------
 * O3.  Verification.
 *
 * The paper inherits the acceptance rule from speculative sampling (Sec. 2.1) and its multi-candidate
 * extension (Sec. 2.2): a candidate x drawn from the draft distribution q is accepted with probability
 * min(1, p(x)/q(x)); after a rejection the target distribution is replaced by the normalised residual
 * norm(max(p - q, 0)) (both models' outputs are normalised distributions, Sec. 3.1) and the
 * next sibling is tried against it; when every sibling is rejected the new token is sampled from the
 * current residual.  Candidates of one context are i.i.d. draws from q (with replacement), so q is not
 * changed by a rejection.
 *
 * To make the result a deterministic function of the inputs on any machine, the residual is kept
 * UNNORMALISED together with its sum S:   r <- max(r - S*q, 0),  S <- sum(r),  test  u*q(x)*S < r(x)
 * (the same test as u < (r(x)/S)/q(x), without a division), and every sum over the vocabulary is taken
 * in one fixed order: a balanced binary tree over the index space zero-padded to a power of two.
 * ---------------------------------------------------------------------------------------------- */

static int64_t pow2_at_least(int64_t v)
{
    int64_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

/* Sum of a[lo .. lo+len) (len a power of two) as a balanced binary tree of binary64 additions. */
static double tree_node(const double *a, int64_t lo, int64_t len)
{
    if (len == 1) return a[lo];
    return tree_node(a, lo, len / 2) + tree_node(a, lo + len / 2, len / 2);
}

/* a has P entries (already zero-padded beyond the vocabulary). */
static double tree_sum(const double *a, int64_t P) { return tree_node(a, 0, P); }

/* Inverse-CDF sampling by descent through the same sum tree: go left when the threshold is below the
 * left subtree's sum, otherwise subtract it and go right.  A zero-weight index can only be reached by a
 * last-bit rounding of the subtraction (or when all weights are zero); then the nearest positive-weight
 * index below is taken, else the nearest above, else 0. */
static int32_t tree_sample(const double *a, int64_t P, int64_t V, float u)
{
    const double S = tree_sum(a, P);
    double thr = (double)u * S;
    int64_t lo = 0, len = P;
    while (len > 1) {
        const double left = tree_node(a, lo, len / 2);
        if (thr < left) {
            len /= 2;
        } else {
            thr = thr - left;
            lo += len / 2;
            len /= 2;
        }
    }
    int64_t t = lo;
    if (!(t < V && a[t] > 0.0)) {
        int64_t tt;
        for (tt = (t < V ? t : V) - 1; tt >= 0; --tt)
            if (a[tt] > 0.0) return (int32_t)tt;
        for (tt = t + 1; tt < V; ++tt)
            if (a[tt] > 0.0) return (int32_t)tt;
        return 0;
    }
    return (int32_t)t;
}

typedef struct {
    int32_t G;              /* levels in the slice */
    const int32_t *b;       /* branching */
    int64_t off[64];        /* off[l] = first node id of level l+1 ; off[G] = N */
    int64_t size[64];
} tree_t;

static int tree_init(tree_t *t, const int32_t *b, int32_t G)
{
    if (G < 1 || G > 62) return -1;
    if (mcsd_oracle_level_sizes(b, G, t->size) < 0) return -1;
    t->G = G;
    t->b = b;
    t->off[0] = 0;
    for (int32_t l = 0; l < G; ++l) t->off[l + 1] = t->off[l] + t->size[l];
    return 0;
}

/* Children of a context.  ctx = -1 is the context that ends the prefix (children: level 1);
 * ctx = node id at level l (1-based) has its b_{l+1} children at level l+1, next to each other. */
static void children_of(const tree_t *t, int64_t ctx, int32_t ctx_level, int64_t *first, int32_t *count)
{
    if (ctx < 0) { *first = 0; *count = t->b[0]; return; }
    const int64_t a = ctx - t->off[ctx_level - 1];          /* in-level index */
    *count = t->b[ctx_level];
    *first = t->off[ctx_level] + a * t->b[ctx_level];
}

/* Walk down from a context (row index `cur` in p/q: 0 = end of prefix, 1+i = after node i) whose
 * children are at level `lvl` (1-based).  Appends accepted node ids to path; on return `term` (P doubles)
 * holds the unnormalised distribution the new token(s) are drawn from. */
static int32_t traverse(const tree_t *t, int64_t start_node, int32_t start_level,
                        int32_t V, int64_t P, const int32_t *tokens,
                        const float *p, const float *q, const float *u_acc,
                        int32_t *path, double *r, double *term, int without_replacement, double *qz)
{
    int64_t cur = start_node;          /* node id of the current context, -1 for the prefix end */
    int32_t cur_level = start_level;   /* level of `cur` (0 for the prefix end) */
    int32_t n_acc = 0;
    while (cur_level < t->G) {
        const float *prow = p + (cur + 1) * (int64_t)V;
        const float *qrow = q + (cur + 1) * (int64_t)V;
        for (int64_t v = 0; v < P; ++v) r[v] = v < V ? (double)prow[v] : 0.0;
        double S = 1.0;                /* round 0 trusts the target row to be normalised */
        int64_t first; int32_t cnt; int64_t accepted = -1;
        children_of(t, cur, cur_level, &first, &cnt);
        if (!without_replacement) {
            for (int32_t c = 0; c < cnt; ++c) {
                const int64_t node = first + c;
                const int32_t x = tokens[node];
                const double u = (double)u_acc[node];
                if (u * ((double)qrow[x] * S) < r[x]) { accepted = node; break; }
                for (int64_t v = 0; v < V; ++v) {                 /* residual: r <- max(r - S*q, 0) */
                    double d = fma(-S, (double)qrow[v], r[v]);
                    r[v] = d > 0.0 ? d : 0.0;
                }
                S = tree_sum(r, P);
            }
        } else {
            /* Candidates drawn WITHOUT replacement (the siblings of a context are distinct tokens, each drawn from
             * the draft row with the earlier ones removed): after a rejection the draft row loses the rejected
             * token as well, q(x) <- 0, q <- norm(q).  Unnormalised: qz is the row with zeros, Sq its sum, kept as
             * 1 - (mass removed so far) since the row is trusted to be normalised like the target row;
             *   test   u * (qz(x)/Sq) < r(x)/S      <=>   u * qz(x) * S < r(x) * Sq
             *   update r <- max(r/S - qz/Sq, 0) * S * Sq = max(r*Sq - S*qz, 0),  then qz(x) <- 0, Sq <- Sq - qz(x). */
            for (int64_t v = 0; v < V; ++v) qz[v] = (double)qrow[v];
            double Sq = 1.0;
            for (int32_t c = 0; c < cnt; ++c) {
                const int64_t node = first + c;
                const int32_t x = tokens[node];
                const double u = (double)u_acc[node];
                if (u * (qz[x] * S) < r[x] * Sq) { accepted = node; break; }
                for (int64_t v = 0; v < V; ++v) {
                    double d = fma(-S, qz[v], r[v] * Sq);
                    r[v] = d > 0.0 ? d : 0.0;
                }
                Sq = Sq - qz[x];
                qz[x] = 0.0;
                S = tree_sum(r, P);
            }
        }
        if (accepted < 0) {
            /* all candidates rejected: new token(s) come from the residual; if the residual vanished
             * (p <= q everywhere after some round) fall back to the context's own target row */
            if (S > 0.0) memcpy(term, r, sizeof(double) * (size_t)P);
            else for (int64_t v = 0; v < P; ++v) term[v] = v < V ? (double)prow[v] : 0.0;
            return n_acc;
        }
        path[n_acc++] = (int32_t)accepted;
        cur = accepted;
        cur_level += 1;
    }
    /* every level accepted: the bonus token comes from the target row after the last node */
    const float *prow = p + (cur + 1) * (int64_t)V;
    for (int64_t v = 0; v < P; ++v) term[v] = v < V ? (double)prow[v] : 0.0;
    return n_acc;
}

/* mode 0 (draft-initialised): one walk from the prefix end; one new token is customary (n_new = 1).
 * mode 1 (target-initialised, Sec. 3.1): level-1 nodes were sampled from the target itself and need
 * no test; one walk per level-1 node, the longest accepted continuation wins (lowest node id on ties,
 * Fig. 1 step 5), and n_new tokens are drawn i.i.d. from the winner's terminal distribution to seed the
 * next tree (Fig. 1 step 6).
 *
 * tokens [B][N]; p [b*p_bstride + row*V + v], rows 0..N; q likewise, rows 0..N(G-1);
 * u_acc [B][N] (indexed by node); u_smp [B][n_new]; out_path [B][G] (-1 padded); out_len [B];
 * out_new [B][n_new].  Returns 0, or <0 on invalid arguments. */
static int verify_tree_impl(int32_t mode, int without_replacement, const int32_t *branching, int32_t G, int32_t B,
                            int32_t V, const int32_t *tokens, const float *p, const float *q, int64_t p_bstride,
                            int64_t q_bstride, const float *u_acc, const float *u_smp, int32_t n_new,
                            int32_t *out_path, int32_t *out_len, int32_t *out_new)
{
    tree_t t;
    if (tree_init(&t, branching, G) < 0 || V < 1 || B < 0 || n_new < 0 || (mode != 0 && mode != 1)) return -1;
    const int64_t N = t.off[G];
    const int64_t P = pow2_at_least(V);
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        double *r = (double *)malloc(sizeof(double) * (size_t)P);
        double *term = (double *)malloc(sizeof(double) * (size_t)P);
        double *best_term = (double *)malloc(sizeof(double) * (size_t)P);
        int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)(G + 1));
        int32_t *best_path = (int32_t *)malloc(sizeof(int32_t) * (size_t)(G + 1));
        double *qz = (double *)malloc(sizeof(double) * (size_t)P);
        if (!r || !term || !best_term || !path || !best_path || !qz) {
#pragma omp atomic write
            rc = -2;
            goto done;
        }
        const int32_t *tok_b = tokens + (int64_t)b * N;
        const float *p_b = p + (int64_t)b * p_bstride, *q_b = q + (int64_t)b * q_bstride;
        const float *ua_b = u_acc + (int64_t)b * N;
        int32_t best_len = -1;
        if (mode == 0) {
            best_len = traverse(&t, -1, 0, V, P, tok_b, p_b, q_b, ua_b, best_path, r, best_term, without_replacement, qz);
        } else {
            for (int32_t i = 0; i < branching[0]; ++i) {
                path[0] = i;                                   /* accepted by construction */
                int32_t len = 1 + traverse(&t, i, 1, V, P, tok_b, p_b, q_b, ua_b, path + 1, r, term, without_replacement, qz);
                if (len > best_len) {                          /* strict: lowest id wins ties */
                    best_len = len;
                    memcpy(best_path, path, sizeof(int32_t) * (size_t)len);
                    memcpy(best_term, term, sizeof(double) * (size_t)P);
                }
            }
        }
        out_len[b] = best_len;
        for (int32_t l = 0; l < G; ++l) out_path[(int64_t)b * G + l] = l < best_len ? best_path[l] : -1;
        for (int32_t k = 0; k < n_new; ++k)
            out_new[(int64_t)b * n_new + k] = tree_sample(best_term, P, V, u_smp[(int64_t)b * n_new + k]);
    done:
        free(r); free(term); free(best_term); free(path); free(best_path); free(qz);
    }
    return rc;
}

int mcsd_oracle_verify_tree(int32_t mode, const int32_t *branching, int32_t G, int32_t B, int32_t V,
                            const int32_t *tokens, const float *p, const float *q,
                            int64_t p_bstride, int64_t q_bstride,
                            const float *u_acc, const float *u_smp, int32_t n_new,
                            int32_t *out_path, int32_t *out_len, int32_t *out_new)
{
    return verify_tree_impl(mode, 0, branching, G, B, V, tokens, p, q, p_bstride, q_bstride, u_acc, u_smp, n_new,
                            out_path, out_len, out_new);
}

/* The same walk for candidates drawn without replacement (see traverse). */
int mcsd_oracle_verify_tree_without_replacement(int32_t mode, const int32_t *branching, int32_t G, int32_t B, int32_t V,
                                                const int32_t *tokens, const float *p, const float *q,
                                                int64_t p_bstride, int64_t q_bstride, const float *u_acc,
                                                const float *u_smp, int32_t n_new, int32_t *out_path,
                                                int32_t *out_len, int32_t *out_new)
{
    return verify_tree_impl(mode, 1, branching, G, B, V, tokens, p, q, p_bstride, q_bstride, u_acc, u_smp, n_new,
                            out_path, out_len, out_new);
}

/* ------------------------------------------------------------------------------------------------
 * Update after acceptance (Fig. 1 step 6): the accepted path becomes part of the prefix.
 * One layer's tensors.  For sequence b with accepted length a = accept_len[b] and old length L = lens[b]:
 * cache row L + j of every head receives the tree K and V row of node path[b][j] (j = 0 .. a-1, root side
 * first); the new length is L + a.  ids[b] lists the accepted tokens in that order followed by the first
 * n_append new tokens, padded with -1 up to gamma + n_append entries; n_ids[b] counts the entries that are set.
 * `lens_out` may be lens itself.  Elements are moved as raw storage (elem_bytes each).
 * ---------------------------------------------------------------------------------------------- */
int mcsd_oracle_commit_path(int32_t elem_bytes, int32_t B, int32_t H, int32_t d, int32_t gamma, int32_t n_nodes,
                            int64_t node_stride, const void *k_tree, const void *v_tree, void *k_prefix,
                            void *v_prefix, const int64_t *seq_base, int64_t head_stride, const int32_t *path,
                            const int32_t *accept_len, const int32_t *lens, int32_t *lens_out)
{
    const char *kt = (const char *)k_tree, *vt = (const char *)v_tree;
    char *kp = (char *)k_prefix, *vp = (char *)v_prefix;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t a = accept_len[b], L = lens[b];
        if (a < 0 || a > gamma || L < 0) return -1;
        for (int32_t j = 0; j < a; ++j) {
            const int32_t node = path[(int64_t)b * gamma + j];
            if (node < 0 || node >= n_nodes) return -1;
            for (int32_t h = 0; h < H; ++h) {
                const int64_t src = ((((int64_t)b * H + h) * node_stride + node) * d) * elem_bytes;
                const int64_t dst = (seq_base[b] + (int64_t)h * head_stride + (int64_t)(L + j) * d) * elem_bytes;
                memcpy(kp + dst, kt + src, (size_t)d * elem_bytes);
                memcpy(vp + dst, vt + src, (size_t)d * elem_bytes);
            }
        }
    }
    for (int32_t b = 0; b < B; ++b) lens_out[b] = lens[b] + accept_len[b];
    return 0;
}

/* The token ids that the accepted path adds to the input (Fig. 1 step 6). */
int mcsd_oracle_commit_ids(int32_t B, int32_t gamma, int32_t n_nodes, const int32_t *tokens, const int32_t *path,
                           const int32_t *accept_len, const int32_t *new_tokens, int32_t n_new, int32_t n_append,
                           int32_t *ids, int32_t *n_ids)
{
    if (n_append < 0 || n_append > n_new) return -1;
    const int32_t W = gamma + n_append;
    for (int32_t b = 0; b < B; ++b) {
        const int32_t a = accept_len[b];
        if (a < 0 || a > gamma) return -1;
        int32_t k = 0;
        for (int32_t j = 0; j < a; ++j) {
            const int32_t node = path[(int64_t)b * gamma + j];
            if (node < 0 || node >= n_nodes) return -1;
            ids[(int64_t)b * W + k++] = tokens[(int64_t)b * n_nodes + node];
        }
        for (int32_t j = 0; j < n_append; ++j) ids[(int64_t)b * W + k++] = new_tokens[(int64_t)b * n_new + j];
        n_ids[b] = k;
        for (; k < W; ++k) ids[(int64_t)b * W + k] = -1;
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------------
 * O4  Early-stop decision models (Sec. 3.3; threshold beta = 0.4 in the caption of Fig. 2).
 *
 * After every draft-generation turn a small MLP predicts, for each candidate sequence, the probability
 * that the target model will accept it; draft generation stops early iff every sequence of the tree is
 * predicted below beta.  Two models: type 1 is a three-layer MLP on the draft model's hidden state of the
 * newest token; type 2 is a two-layer MLP on Concat(Topk(y), Ent(y)) of the draft model's output
 * distribution y for that token.
 *
 * Readings where Sec. 3.3 is silent: an "n-layer MLP" is n affine maps with ReLU between them and a
 * logistic sigmoid after the last, so the output is a probability that can be compared with beta;
 * Topk(y) is the k largest probabilities in descending order (values, duplicates kept; zeros when the
 * row has fewer than k entries); Ent(y) is the Shannon entropy in nats with 0 ln 0 = 0; "lower than
 * the threshold" is strict.  Weights are inputs (the trained ones are not published).
 * ---------------------------------------------------------------------------------------------- */
static int cmp_float_desc(const void *a, const void *b)
{
    const float x = *(const float *)a, y = *(const float *)b;
    return (x < y) - (x > y);
}

/* x[0..k-1] = Topk(y), x[k] = Ent(y) for one distribution y[0..V-1]. */
int mcsd_oracle_decision_features(int64_t V, int32_t k, const float *y, double *x)
{
    if (V < 1 || k < 0) return -1;
    float *sorted = (float *)malloc(sizeof(float) * (size_t)V);
    memcpy(sorted, y, sizeof(float) * (size_t)V);
    qsort(sorted, (size_t)V, sizeof(float), cmp_float_desc);
    for (int32_t i = 0; i < k; ++i) x[i] = i < V ? (double)sorted[i] : 0.0;
    free(sorted);
    double h = 0.0;
    for (int64_t v = 0; v < V; ++v)
        if (y[v] > 0.0f) h -= (double)y[v] * log((double)y[v]);
    x[k] = h;
    return 0;
}

/* P = sigmoid(A_n(relu(... relu(A_1 x)))) with A_l z = weight[l] z + bias[l]; weight[l] is row-major
 * [width[l+1]][width[l]], width[0] inputs, width[n_layers] = 1. */
double mcsd_oracle_mlp(int32_t n_layers, const int32_t *width, const float *const *weight, const float *const *bias,
                       const double *x)
{
    int32_t wmax = 1;
    for (int32_t l = 0; l <= n_layers; ++l) if (width[l] > wmax) wmax = width[l];
    double *cur = (double *)malloc(sizeof(double) * (size_t)wmax);
    double *nxt = (double *)malloc(sizeof(double) * (size_t)wmax);
    memcpy(cur, x, sizeof(double) * (size_t)width[0]);
    for (int32_t l = 0; l < n_layers; ++l) {
        const int32_t n_in = width[l], n_out = width[l + 1];
        for (int32_t j = 0; j < n_out; ++j) {
            double s = (double)bias[l][j];
            for (int32_t i = 0; i < n_in; ++i) s += (double)weight[l][(int64_t)j * n_in + i] * cur[i];
            nxt[j] = (l + 1 < n_layers && s < 0.0) ? 0.0 : s;
        }
        double *t = cur; cur = nxt; nxt = t;
    }
    const double z = cur[0];
    free(cur);
    free(nxt);
    return 1.0 / (1.0 + exp(-z));
}

/* 1 iff all W candidate sequences of a tree are predicted below beta (then draft generation stops). */
int32_t mcsd_oracle_early_stop(const double *P, int32_t W, double beta)
{
    for (int32_t w = 0; w < W; ++w)
        if (!(P[w] < beta)) return 0;
    return 1;
}

/* Exposed for the tests that pin the summation order and the sampler on their own. */
double mcsd_oracle_tree_sum(const double *a, int64_t V)
{
    const int64_t P = pow2_at_least(V);
    double *pad = (double *)calloc((size_t)P, sizeof(double));
    memcpy(pad, a, sizeof(double) * (size_t)V);
    double s = tree_sum(pad, P);
    free(pad);
    return s;
}

int32_t mcsd_oracle_tree_sample(const double *a, int64_t V, float u)
{
    const int64_t P = pow2_at_least(V);
    double *pad = (double *)calloc((size_t)P, sizeof(double));
    memcpy(pad, a, sizeof(double) * (size_t)V);
    int32_t t = tree_sample(pad, P, V, u);
    free(pad);
    return t;
}

/* Expected improvement factor of speculative decoding, (1 - alpha^(gamma+1)) / ((1 - alpha)(c*gamma + 1))
 * (Sec. 3, unnumbered equation).  Reporting helper. */
double mcsd_oracle_improvement_factor(double alpha, double gamma, double c)
{
    return (1.0 - pow(alpha, gamma + 1.0)) / ((1.0 - alpha) * (c * gamma + 1.0));
}

/* Threads the (b,h) / per-sequence loops above will use (for reporting next to a timing). */
int32_t mcsd_oracle_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
