// Tree attention for gfx950 (Sec. 2.2 of arXiv 2409.10644): every node of the candidate tree attends
// to the prefix KV cache and to its own ancestors under the topology-aware mask.
//
// bf16 path.  One workgroup (4 wavefronts) owns one (sequence, head, key split).  The tree's queries are
// cut into blocks of 32 rows; a wavefront keeps one block of Q in registers for the whole sweep and the
// workgroup streams K/V tiles through LDS, so every K/V byte leaves HBM once and is used by all queries.
// Scores are computed transposed, S^T = K * Q^T, with v_mfma_f32_32x32x16_bf16: the accumulator then holds,
// per lane, 16 keys of ONE query, so the online-softmax reductions are in-lane plus one half-wave swap,
// and the exponentiated scores are already in the register layout of the B operand of O^T += V^T * P^T.
// V^T operands are read from the row-major V tile with the LDS transpose load (ds_read_b64_tr_b16).
// The tree's own keys are one or two extra tiles whose scores are masked with the packed bitmask slice.
//
// fp32 path: same split / online-softmax structure on the vector ALU (small reference-precision shapes).
#include <math.h>
#include <stdlib.h>

#include "mcsd_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;

struct AttnParams {
    const void *q, *kt, *vt, *kp, *vp;
    void *out;
    const int64_t *seq_base;
    const int32_t *lens;
    const uint64_t *mask_bits;
    int32_t mask_words;
    int32_t B, H, n;
    int32_t max_prefix;
    int64_t node_stride, head_stride;
    float c;          // softmax_scale * log2(e)
    int32_t S;        // key splits in the grid
    int32_t SP;       // partial results per (b,h): S * key groups per workgroup
    float *part_o;    // [B*H][SP][n][D]
    float *part_m;    // [B*H][SP][n]   running maximum of the raw scores
    float *part_l;    // [B*H][SP][n]   sum of exp2((s - m) * c)
};

struct AttnPlan {
    int QB, KG, T, S, SP;
};

__host__ __device__ inline int key_groups(int QB) { return QB <= 2 ? 2 : 1; }
__host__ __device__ inline int tile_keys_bf16(int) { return 64; }

AttnPlan make_plan(int dtype, int B, int H, int n, int max_prefix)
{
    AttnPlan pl;
    if (dtype == MCSD_BF16) {
        pl.QB = (n + 31) / 32;
        pl.KG = key_groups(pl.QB);
        pl.T = tile_keys_bf16(pl.QB);
    } else {
        pl.QB = 1;
        pl.KG = 1;
        pl.T = 32;
    }
    const long bh = (long)B * H;
    const int tiles_max = (max_prefix + pl.T - 1) / pl.T;
    long want = (512 + bh - 1) / bh;           // aim for >= 2 workgroups per compute unit
    long cap = tiles_max / 2;                   // at least two tiles per split
    long S = want < cap ? want : cap;
    if (S < 1) S = 1;
    if (S > 64) S = 64;
    if (const char *ov = getenv("MCSD_ATTN_SPLITS")) {     // tuning override: number of key splits
        const long v = atol(ov);
        if (v >= 1 && v <= 64) S = v;
    }
    pl.S = (int)S;
    pl.SP = pl.S * pl.KG;
    return pl;
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Swap the upper 32 lanes of one value with the lower 32 lanes of the other; with both arguments equal the
// pair (r0, r1) holds {own, partner} in some order on every lane, so max / sum across halves is r0 op r1.
__device__ inline float half_swap_max(float v)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_swap_sum(float v)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ inline s16x4_t lds_read_tr16(const unsigned char *p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3))) *)(p));
}

// ---------------------------------------------------------------------------------------------------
// bf16 / MFMA kernel
// ---------------------------------------------------------------------------------------------------
template <int D, int QB>
struct Bf16Cfg {
    static constexpr int KG = QB <= 2 ? 2 : 1;  // key groups: wavefronts that share a query block split the tile's keys
    static constexpr int T = 64;                // keys per tile
    static constexpr int KPW = T / 32 / KG;     // 32-key blocks per wavefront per tile
    static constexpr int SK = D * 2 + 16;       // LDS row stride of the K tile (bytes): 4 banks per row
    static constexpr int SV = D * 2 + 64;       // LDS row stride of the V tile (bytes): 16 banks per row
    static constexpr int CPR = D / 8;           // 16-byte chunks per K/V row
    static constexpr int RPP = 256 / CPR;       // rows per load pass of the workgroup
    static constexpr int NLD = T / RPP;         // load passes per tile
    static constexpr int KS = D / 16;           // k-steps of S^T = K Q^T
    static constexpr int CB = D / 32;           // 32-row blocks of O^T
};

// Log2-domain slack of the running reference maximum: the accumulators are rescaled only when a block's maximum
// exceeds the reference by more than this, so exponentiated scores stay below 2^RESCALE_SLACK.  The result is
// exact: numerator and denominator always share the same reference.
constexpr float RESCALE_SLACK = 6.f;

// One block of 32 keys against the wavefront's 32 queries.
// MODE 0: all keys visible; otherwise bit k of `bits` says whether key k of the block is visible to this lane's query.
template <int D, int QB, int MODE>
__device__ inline void attn_block(const unsigned char *ldsK, const unsigned char *ldsV, int kb, const bf16x8_t *qreg,
                                  f32x16_t *oacc, float &m_ref, float &l_run, float c, int g, int ln, uint32_t bits)
{
    using C = Bf16Cfg<D, QB>;
    // S^T[key][query] = K * Q^T : lane (query = ln, half g) gets keys 8*(r/4) + 4*g + r%4, r = 0..15
    f32x16_t sacc = {0};
    const unsigned char *krow = ldsK + (kb * 32 + ln) * C::SK + g * 16;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        bf16x8_t a = *(const bf16x8_t *)(krow + ks * 32);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc, 0, 0, 0);
    }
    if (MODE != 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 8 * (r / 4) + 4 * g + (r % 4);
            if (!((bits >> key) & 1u)) sacc[r] = -INFINITY;
        }
    }
    float mx = fmaxf(fmaxf(sacc[0], sacc[1]), sacc[2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) mx = fmaxf(fmaxf(mx, sacc[r]), sacc[r + 1]);
    mx = fmaxf(mx, sacc[15]);
    mx = half_swap_max(mx);
    // rescale only when the block maximum outgrows the reference by more than the slack (first block: -inf)
    const bool grow = (mx - m_ref) * c > RESCALE_SLACK;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        const float m_new = grow ? mx : m_ref;
        const float alpha = m_new == m_ref ? 1.f : fast_exp2((m_ref - m_new) * c);   // -inf reference: exp2(-inf) = 0
        m_ref = m_new;
        l_run *= alpha;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
    }
    const float mc = (m_ref == -INFINITY ? 0.f : m_ref) * c;
    float psum = 0.f;
    bf16x8_t pb[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float pv = fast_exp2(fmaf(sacc[r], c, -mc));
        psum += pv;
        pb[r / 8][r % 8] = (__bf16)pv;
    }
    l_run += psum;
    // O^T[c][query] += V^T[c][key] * P^T[key][query]; V^T operands via the LDS transpose load
    const int vcol = 16 * (ln >> 4) + 4 * (ln & 3);
    const int vkey = 4 * g + ((ln & 15) >> 2);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
        const unsigned char *vbase = ldsV + (kb * 32 + ks2 * 16 + vkey) * C::SV + vcol * 2;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb) {
            s16x4_t lo = lds_read_tr16(vbase + cb * 64);
            s16x4_t hi = lds_read_tr16(vbase + cb * 64 + 8 * C::SV);
            s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            bf16x8_t a = __builtin_bit_cast(bf16x8_t, both);
            oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[ks2], oacc[cb], 0, 0, 0);
        }
    }
}

// All key blocks of one tile that belong to this wavefront's key group.
// MODE 0: full prefix tile, 1: prefix tail (keys < valid exist), 2: tree tile (visibility from the mask row).
template <int D, int QB, int MODE>
__device__ inline void attn_tile(const unsigned char *ldsK, const unsigned char *ldsV, const bf16x8_t *qreg,
                                 f32x16_t *oacc, float &m_ref, float &l_run, float c, int kg, int g, int ln,
                                 int valid, const uint64_t *mrow, int tile_key0)
{
    using C = Bf16Cfg<D, QB>;
#pragma unroll
    for (int j = 0; j < C::KPW; ++j) {
        const int kb = kg * C::KPW + j;
        uint32_t bits = 0xffffffffu;
        if (MODE == 1) {
            const int left = valid - kb * 32;     // keys of this block that exist
            bits = left >= 32 ? 0xffffffffu : (left <= 0 ? 0u : ((1u << left) - 1u));
        } else if (MODE == 2) {
            const int col = tile_key0 + kb * 32;
            bits = (uint32_t)(((col >> 6) ? mrow[1] : mrow[0]) >> (col & 63));
        }
        attn_block<D, QB, MODE>(ldsK, ldsV, kb, qreg, oacc, m_ref, l_run, c, g, ln, bits);
    }
}

template <int D, int QB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void tree_attn_bf16_kernel(const AttnParams p)
{
    using C = Bf16Cfg<D, QB>;
    constexpr int TILE_BYTES = C::T * C::SK + C::T * C::SV;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * TILE_BYTES];     // two tiles: compute one, fill one

    const int s = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, ln = lane & 31;
    const int qb = wave % QB, kg = wave / QB;
    const bool computes = kg < C::KG;

    int L = p.lens[b];
    L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
    const int tiles_b = (L + C::T - 1) / C::T;
    const int tps = (tiles_b + p.S - 1) / p.S;
    const int t0 = min(s * tps, tiles_b), t1 = min(t0 + tps, tiles_b);
    const int n_tree_tiles = s == 0 ? (p.n + C::T - 1) / C::T : 0;
    const int n_pre = t1 - t0;
    if (n_pre + n_tree_tiles == 0) return;
    // leading tiles of this split that are full (only the sequence's last tile can be ragged)
    const int n_hot = (n_pre > 0 && t1 * C::T > L) ? n_pre - 1 : n_pre;

    const int64_t bh = (int64_t)b * p.H + h;
    const __bf16 *q = (const __bf16 *)p.q + bh * p.node_stride * D;
    const __bf16 *kt = (const __bf16 *)p.kt + bh * p.node_stride * D;
    const __bf16 *vt = (const __bf16 *)p.vt + bh * p.node_stride * D;
    const int64_t pre0 = p.seq_base[b] + (int64_t)h * p.head_stride;
    const __bf16 *kp = (const __bf16 *)p.kp + pre0;
    const __bf16 *vp = (const __bf16 *)p.vp + pre0;

    // Q block of this wavefront as B operands: lane holds Q[row][ks*16 + 8g .. +8]
    const int qrow = qb * 32 + ln;
    bf16x8_t qreg[C::KS];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (qrow < p.n) v = *(const uint4 *)(q + (int64_t)qrow * D + ks * 16 + g * 8);
        qreg[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
    // mask row of this lane's query (zero for padded rows)
    uint64_t mrow[2] = {0, 0};
    if (qrow < p.n) {
        mrow[0] = p.mask_bits[(int64_t)qrow * p.mask_words];
        if (p.mask_words > 1) mrow[1] = p.mask_bits[(int64_t)qrow * p.mask_words + 1];
    }

    f32x16_t oacc[C::CB];
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb) oacc[cb] = (f32x16_t){0};
    float m_ref = -INFINITY, l_run = 0.f;

    const int ld_row = tid / C::CPR, ld_chunk = tid % C::CPR;
    const int ld_off = ld_row * D + ld_chunk * 8;                  // element offset of this thread's first chunk
    uint4 kreg[C::NLD], vreg[C::NLD];

    auto stash = [&](int buf) {
        unsigned char *bk = lds + buf * TILE_BYTES, *bv = bk + C::T * C::SK;
#pragma unroll
        for (int i = 0; i < C::NLD; ++i) {
            const int row = i * C::RPP + ld_row;
            *(uint4 *)(bk + row * C::SK + ld_chunk * 16) = kreg[i];
            *(uint4 *)(bv + row * C::SV + ld_chunk * 16) = vreg[i];
        }
    };

    // ---- full prefix tiles: register prefetch one tile ahead of the LDS fill, LDS double-buffered ----
    if (n_hot > 0) {
        const __bf16 *ksrc = kp + (int64_t)t0 * C::T * D + ld_off;
        const __bf16 *vsrc = vp + (int64_t)t0 * C::T * D + ld_off;
        auto fetch_full = [&](int it) {
#pragma unroll
            for (int i = 0; i < C::NLD; ++i) {
                kreg[i] = *(const uint4 *)(ksrc + ((int64_t)it * C::T + i * C::RPP) * D);
                vreg[i] = *(const uint4 *)(vsrc + ((int64_t)it * C::T + i * C::RPP) * D);
            }
        };
        fetch_full(0);
        stash(0);
        if (n_hot > 1) fetch_full(1);
        __syncthreads();
        for (int it = 0; it < n_hot; ++it) {
            if (it + 1 < n_hot) stash((it + 1) & 1);          // tile it+1: registers -> the other LDS buffer
            if (it + 2 < n_hot) fetch_full(it + 2);           // tile it+2: HBM -> registers, lands during the MFMAs
            if (computes) {
                const unsigned char *ldsK = lds + (it & 1) * TILE_BYTES;
                attn_tile<D, QB, 0>(ldsK, ldsK + C::T * C::SK, qreg, oacc, m_ref, l_run, p.c, kg, g, ln, C::T, mrow, 0);
            }
            __syncthreads();                                   // tile it fully read, tile it+1 fully written
        }
    }

    // ---- ragged last prefix tile and the tree's own tiles: one at a time, rows beyond `valid` zero-filled ----
    const int n_rest = (n_pre - n_hot) + n_tree_tiles;
    for (int it = 0; it < n_rest; ++it) {
        const bool tail = it < n_pre - n_hot;
        const int tt = tail ? 0 : it - (n_pre - n_hot);
        const __bf16 *ksrc = tail ? kp + (int64_t)(t1 - 1) * C::T * D : kt + (int64_t)tt * C::T * D;
        const __bf16 *vsrc = tail ? vp + (int64_t)(t1 - 1) * C::T * D : vt + (int64_t)tt * C::T * D;
        const int valid = tail ? L - (t1 - 1) * C::T : min(C::T, p.n - tt * C::T);
#pragma unroll
        for (int i = 0; i < C::NLD; ++i) {
            const int row = i * C::RPP + ld_row;
            kreg[i] = make_uint4(0, 0, 0, 0);
            vreg[i] = make_uint4(0, 0, 0, 0);
            if (row < valid) {
                kreg[i] = *(const uint4 *)(ksrc + (int64_t)row * D + ld_chunk * 8);
                vreg[i] = *(const uint4 *)(vsrc + (int64_t)row * D + ld_chunk * 8);
            }
        }
        stash(0);
        __syncthreads();
        if (computes) {
            if (tail)
                attn_tile<D, QB, 1>(lds, lds + C::T * C::SK, qreg, oacc, m_ref, l_run, p.c, kg, g, ln, valid, mrow, 0);
            else
                attn_tile<D, QB, 2>(lds, lds + C::T * C::SK, qreg, oacc, m_ref, l_run, p.c, kg, g, ln, 0, mrow, tt * C::T);
        }
        __syncthreads();
    }
    if (!computes) return;

    const float l_tot = half_swap_sum(l_run);
    if (qrow >= p.n) return;
    if (p.SP == 1) {
        const float inv = 1.f / l_tot;
        __bf16 *o = (__bf16 *)p.out + (bh * p.node_stride + qrow) * D;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16x4_t v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (__bf16)(oacc[cb][4 * j + e] * inv);
                *(bf16x4_t *)(o + cb * 32 + 8 * j + 4 * g) = v;
            }
    } else {
        const int sp = s * C::KG + kg;
        const int64_t prow = (bh * p.SP + sp) * p.n + qrow;
        float *po = p.part_o + prow * D;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4_t v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = oacc[cb][4 * j + e];
                *(f32x4_t *)(po + cb * 32 + 8 * j + 4 * g) = v;
            }
        if (g == 0) {
            p.part_m[prow] = m_ref;
            p.part_l[prow] = l_tot;
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// fp32 / vector-ALU kernel (reference-precision shapes)
// ---------------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void tree_attn_f32_kernel(const AttnParams p)
{
    constexpr int T = 32;
    constexpr int NMAX = MCSD_ATTN_MAX_NODES;
    constexpr int RP = 256 / D;          // output rows per pass
    constexpr int NR = NMAX / RP;        // output rows per thread
    __shared__ float sQ[NMAX][D + 1];
    __shared__ float sK[T][D + 1];
    __shared__ float sV[T][D];
    __shared__ float sS[NMAX][T + 1];
    __shared__ float sAlpha[NMAX];
    __shared__ float sL[NMAX];
    __shared__ float sM[NMAX];

    const int s = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    int L = p.lens[b];
    L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
    const int tiles_b = (L + T - 1) / T;
    const int tps = (tiles_b + p.S - 1) / p.S;
    const int t0 = min(s * tps, tiles_b), t1 = min(t0 + tps, tiles_b);
    const int n_tree_tiles = s == 0 ? (p.n + T - 1) / T : 0;
    const int n_pre = t1 - t0;
    const int n_iter = n_pre + n_tree_tiles;
    if (n_iter == 0) return;

    const int64_t bh = (int64_t)b * p.H + h;
    const float *q = (const float *)p.q + bh * p.node_stride * D;
    const float *kt = (const float *)p.kt + bh * p.node_stride * D;
    const float *vt = (const float *)p.vt + bh * p.node_stride * D;
    const int64_t pre0 = p.seq_base[b] + (int64_t)h * p.head_stride;
    const float *kp = (const float *)p.kp + pre0;
    const float *vp = (const float *)p.vp + pre0;

    for (int idx = tid; idx < p.n * D; idx += 256) sQ[idx / D][idx % D] = q[idx];
    float acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;     // state of row `tid` (threads tid < n)
    const int oc = tid % D, oi0 = tid / D;

    for (int it = 0; it < n_iter; ++it) {
        const float *ksrc, *vsrc;
        int valid, tree_col0 = -1;
        if (it < n_pre) {
            const int t = t0 + it;
            ksrc = kp + (int64_t)t * T * D;
            vsrc = vp + (int64_t)t * T * D;
            valid = min(T, L - t * T);
        } else {
            const int tt = it - n_pre;
            ksrc = kt + (int64_t)tt * T * D;
            vsrc = vt + (int64_t)tt * T * D;
            valid = min(T, p.n - tt * T);
            tree_col0 = tt * T;
        }
        __syncthreads();
        for (int idx = tid; idx < T * D; idx += 256) {
            const int row = idx / D, col = idx % D;
            const bool ok = row < valid;
            sK[row][col] = ok ? ksrc[idx] : 0.f;
            sV[row][col] = ok ? vsrc[idx] : 0.f;
        }
        __syncthreads();
        {   // raw scores
            const int j = tid % T, i0 = tid / T;
            for (int i = i0; i < p.n; i += 256 / T) {
                float dot = 0.f;
#pragma unroll 8
                for (int cc = 0; cc < D; ++cc) dot = fmaf(sQ[i][cc], sK[j][cc], dot);
                bool vis = j < valid;
                if (tree_col0 >= 0) {
                    const int col = tree_col0 + j;
                    vis = vis && ((p.mask_bits[(int64_t)i * p.mask_words + (col >> 6)] >> (col & 63)) & 1ull);
                }
                sS[i][j] = vis ? dot : -INFINITY;
            }
        }
        __syncthreads();
        if (tid < p.n) {   // online softmax of row tid
            float mx = -INFINITY;
            for (int j = 0; j < T; ++j) mx = fmaxf(mx, sS[tid][j]);
            const float m_new = fmaxf(m_run, mx);
            const float mc = (m_new == -INFINITY ? 0.f : m_new) * p.c;
            const float alpha = exp2f(fmaf(m_run, p.c, -mc));
            float psum = 0.f;
            for (int j = 0; j < T; ++j) {
                const float pv = exp2f(fmaf(sS[tid][j], p.c, -mc));
                sS[tid][j] = pv;
                psum += pv;
            }
            l_run = l_run * alpha + psum;
            m_run = m_new;
            sAlpha[tid] = alpha;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = oi0 + RP * r;
            if (i < p.n) {
                float a = acc[r] * sAlpha[i];
#pragma unroll 8
                for (int j = 0; j < T; ++j) a = fmaf(sS[i][j], sV[j][oc], a);
                acc[r] = a;
            }
        }
    }
    __syncthreads();
    if (tid < p.n) { sL[tid] = l_run; sM[tid] = m_run; }
    __syncthreads();
    if (p.SP == 1) {
        float *o = (float *)p.out + bh * p.node_stride * D;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = oi0 + RP * r;
            if (i < p.n) o[(int64_t)i * D + oc] = acc[r] / sL[i];
        }
    } else {
        const int64_t prow0 = (bh * p.SP + s) * p.n;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = oi0 + RP * r;
            if (i < p.n) p.part_o[(prow0 + i) * D + oc] = acc[r];
        }
        if (tid < p.n) {
            p.part_m[prow0 + tid] = m_run;
            p.part_l[prow0 + tid] = l_run;
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// merge of the split partials:  out = sum_sp w_sp O_sp / sum_sp w_sp l_sp,  w_sp = exp2((m_sp - max m) c)
// ---------------------------------------------------------------------------------------------------
template <int D, bool OUT_BF16>
__global__ __launch_bounds__(256) void tree_attn_merge_kernel(const AttnParams p, int T, int KG)
{
    constexpr int TPR = D / 4;            // threads per output row (4 columns each)
    constexpr int ROWS = 256 / TPR;       // rows per workgroup
    const int h = blockIdx.y, b = blockIdx.z;
    const int i = blockIdx.x * ROWS + threadIdx.x / TPR, c4 = (threadIdx.x % TPR) * 4;
    if (i >= p.n) return;
    const int64_t bh = (int64_t)b * p.H + h;
    int L = p.lens[b];
    L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
    const int tiles_b = (L + T - 1) / T;
    const int tps = (tiles_b + p.S - 1) / p.S;
    // split s ran iff it had prefix tiles, or it is split 0 (which owns the tree tiles)
    const int n_active = tps > 0 ? min(p.S, (tiles_b + tps - 1) / tps) : 1;
    const int sp_active = max(n_active, 1) * KG;
    const int64_t row0 = bh * p.SP * p.n + i;          // partial sp of this row is at row0 + sp * n
    float M = -INFINITY;
    for (int sp = 0; sp < sp_active; ++sp) M = fmaxf(M, p.part_m[row0 + (int64_t)sp * p.n]);
    float den = 0.f;
    f32x4_t num = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int sp = 0; sp < sp_active; ++sp) {
        const int64_t prow = row0 + (int64_t)sp * p.n;
        const float w = exp2f((p.part_m[prow] - M) * p.c);     // exp2(-inf) = 0 for partials that saw no key
        const f32x4_t o = *(const f32x4_t *)(p.part_o + prow * D + c4);
        den = fmaf(w, p.part_l[prow], den);
        num += w * o;
    }
    const f32x4_t r = num / den;
    const int64_t off = (bh * p.node_stride + i) * D + c4;
    if (OUT_BF16) {
        bf16x4_t v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (__bf16)r[e];
        *(bf16x4_t *)((__bf16 *)p.out + off) = v;
    } else {
        *(f32x4_t *)((float *)p.out + off) = r;
    }
}

size_t workspace_bytes_for(const AttnPlan &pl, int B, int H, int d, int n)
{
    if (pl.SP == 1) return 0;
    const size_t rows = (size_t)B * H * pl.SP * n;
    size_t bytes = rows * d * sizeof(float);
    bytes = (bytes + 255) & ~(size_t)255;
    bytes += 2 * ((rows * sizeof(float) + 255) & ~(size_t)255);
    return bytes;
}

template <int D>
hipError_t launch_bf16(const AttnParams &p, const AttnPlan &pl, hipStream_t st)
{
    dim3 grid(pl.S, p.H, p.B), block(256);
    switch (pl.QB) {
    case 1: mcsd_launch(MCSD_KERNEL_ATTN_SWEEP, tree_attn_bf16_kernel<D, 1>, grid, block, st, p); break;
    case 2: mcsd_launch(MCSD_KERNEL_ATTN_SWEEP, tree_attn_bf16_kernel<D, 2>, grid, block, st, p); break;
    case 3: mcsd_launch(MCSD_KERNEL_ATTN_SWEEP, tree_attn_bf16_kernel<D, 3>, grid, block, st, p); break;
    default: mcsd_launch(MCSD_KERNEL_ATTN_SWEEP, tree_attn_bf16_kernel<D, 4>, grid, block, st, p); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.SP == 1) return e;
    mcsd_launch(MCSD_KERNEL_ATTN_MERGE, tree_attn_merge_kernel<D, true>, dim3((p.n + 1024 / D - 1) / (1024 / D), p.H, p.B), block, st, p, pl.T, pl.KG);
    return hipGetLastError();
}

template <int D>
hipError_t launch_f32(const AttnParams &p, const AttnPlan &pl, hipStream_t st)
{
    dim3 grid(pl.S, p.H, p.B), block(256);
    mcsd_launch(MCSD_KERNEL_ATTN_SWEEP, tree_attn_f32_kernel<D>, grid, block, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.SP == 1) return e;
    mcsd_launch(MCSD_KERNEL_ATTN_MERGE, tree_attn_merge_kernel<D, false>, dim3((p.n + 1024 / D - 1) / (1024 / D), p.H, p.B), block, st, p, pl.T, pl.KG);
    return hipGetLastError();
}

}  // namespace

extern "C" size_t mcsd_tree_attention_workspace(int32_t B, int32_t H, int32_t d, int32_t n_nodes, int32_t max_prefix)
{
    if (B < 1 || H < 1 || (d != 64 && d != 128) || n_nodes < 1 || n_nodes > MCSD_ATTN_MAX_NODES || max_prefix < 0)
        return 0;
    // the larger of the two dtypes' needs, so one buffer serves both
    const AttnPlan a = make_plan(MCSD_BF16, B, H, n_nodes, max_prefix);
    const AttnPlan f = make_plan(MCSD_F32, B, H, n_nodes, max_prefix);
    const size_t wa = workspace_bytes_for(a, B, H, d, n_nodes), wf = workspace_bytes_for(f, B, H, d, n_nodes);
    return wa > wf ? wa : wf;
}

extern "C" int mcsd_tree_attention(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H, int32_t d,
                                   const void *q, const void *k_tree, const void *v_tree, int64_t node_stride,
                                   const void *k_prefix, const void *v_prefix, const int64_t *seq_base_dev,
                                   const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                                   float softmax_scale, void *out, void *workspace, size_t workspace_bytes,
                                   void *hip_stream)
{
    if (!mask || !mask->bits_dev || !q || !k_tree || !v_tree || !out || !seq_base_dev || !prefix_lens_dev)
        return MCSD_EINVAL;
    if (dtype != MCSD_F32 && dtype != MCSD_BF16) return MCSD_EINVAL;
    if (B < 1 || H < 1 || B > 65535 || H > 65535 || max_prefix < 0) return MCSD_EINVAL;
    if (max_prefix > 0 && (!k_prefix || !v_prefix)) return MCSD_EINVAL;
    const int32_t n = mask->n_nodes;
    if (n < 1 || node_stride < n || head_stride < 0) return MCSD_EINVAL;
    if (!(softmax_scale > 0.f) || !isfinite(softmax_scale)) return MCSD_EINVAL;
    if (d != 64 && d != 128) return MCSD_EUNSUPPORTED;
    if (n > MCSD_ATTN_MAX_NODES) return MCSD_EUNSUPPORTED;
    if (mask->words_per_row > 2 && n > 128) return MCSD_EUNSUPPORTED;
    const uintptr_t align = (uintptr_t)q | (uintptr_t)k_tree | (uintptr_t)v_tree | (uintptr_t)out |
                            (uintptr_t)k_prefix | (uintptr_t)v_prefix;
    if (align & 15) return MCSD_EINVAL;
    if (((node_stride * d) & 7) || (head_stride & 7)) return MCSD_EINVAL;

    const AttnPlan pl = make_plan(dtype, B, H, n, max_prefix);
    const size_t need = workspace_bytes_for(pl, B, H, d, n);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return MCSD_EWORKSPACE;

    AttnParams p;
    p.q = q; p.kt = k_tree; p.vt = v_tree; p.kp = k_prefix; p.vp = v_prefix; p.out = out;
    p.seq_base = seq_base_dev; p.lens = prefix_lens_dev;
    p.mask_bits = mask->bits_dev; p.mask_words = mask->words_per_row;
    p.B = B; p.H = H; p.n = n; p.max_prefix = max_prefix;
    p.node_stride = node_stride; p.head_stride = head_stride;
    p.c = softmax_scale * 1.4426950408889634f;
    p.S = pl.S; p.SP = pl.SP;
    p.part_o = p.part_m = p.part_l = nullptr;
    if (need > 0) {
        const size_t rows = (size_t)B * H * pl.SP * n;
        const size_t o_bytes = (rows * d * sizeof(float) + 255) & ~(size_t)255;
        const size_t r_bytes = (rows * sizeof(float) + 255) & ~(size_t)255;
        p.part_o = (float *)workspace;
        p.part_m = (float *)((char *)workspace + o_bytes);
        p.part_l = (float *)((char *)workspace + o_bytes + r_bytes);
    }
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e;
    if (dtype == MCSD_BF16) e = d == 128 ? launch_bf16<128>(p, pl, st) : launch_bf16<64>(p, pl, st);
    else e = d == 128 ? launch_f32<128>(p, pl, st) : launch_f32<64>(p, pl, st);
    return mcsd_hip_status(e);
}
