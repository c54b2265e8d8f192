// Early-stop decision models (Sec. 3.3): after a draft-generation turn a small MLP predicts, per candidate
// sequence, the probability that the target model accepts it; the tree stops growing when every sequence is
// predicted below the threshold (caption of Fig. 2).
//
//   decision_distribution_kernel  type 2: Concat(Topk(y), Ent(y)) of one draft distribution y per workgroup (the
//                                 row is read once into registers, or streamed twice when it is too long), then
//                                 the MLP
//   decision_hidden_kernel        type 1: the MLP on the draft model's hidden states, four rows per workgroup
//   early_stop_kernel             stop[b] = every sequence of tree b below the threshold
//
// Type 2 is bound by reading each 128 kB vocabulary row once; type 1 by streaming the first layer's weights through
// a compute unit.  Topk values are selected, not computed, so they are exact; the entropy uses the hardware fp32
// logarithm with binary64 sums, the networks fp32 multiply-adds with tree-combined partial sums: the probabilities
// stay within ~1e-6 of a binary64 evaluation.
#include "mcsd_internal.h"

namespace {

constexpr int DT = 512;              // lanes per workgroup
constexpr int NW = DT / 64;          // wavefronts per workgroup
typedef float nt_f32x4_t __attribute__((ext_vector_type(4)));
constexpr int REG_F4 = 16;           // float4 a lane holds when the whole row fits in registers (V <= 32768)
constexpr int CAND_REG = 1024;       // candidates for the top-k kept in LDS: row in registers ...
constexpr int CAND_MEM = 8192;       // ... row streamed twice (any V up to MCSD_MAX_VOCAB)
constexpr int HROWS = 4;             // hidden-state rows per workgroup
static_assert(HROWS == 4, "the generic first layer of the hidden-state kernel names its four rows");
constexpr int K = MCSD_DECISION_MAX_K;

struct MlpDesc {
    int32_t n_layers;
    int32_t width[4];
    const float *w[3];
    const float *b[3];
};

// A value from another lane through the data-parallel-primitive path of the vector ALU (no LDS round trip).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes, result in every lane.  Partner lanes: l^1 and l^2 by quad permutation; the mirrored lane of
// the half row (row) stands in for l^4 (l^8) because groups of 4 (8) already agree; l^16 by swizzle; l^32 by the
// half-wave swap, which returns {own, partner} in an order a commutative operation ignores.
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_f64<0xB1>(v);
    v += dpp_f64<0x4E>(v);
    v += dpp_f64<0x141>(v);
    v += dpp_f64<0x140>(v);
    {
        const int lo = __builtin_amdgcn_ds_swizzle(__double2loint(v), 0x401F);
        const int hi = __builtin_amdgcn_ds_swizzle(__double2hiint(v), 0x401F);
        v += __hiloint2double(hi, lo);
    }
    const auto lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(v), (unsigned)__double2loint(v), false, false);
    const auto hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(v), (unsigned)__double2hiint(v), false, false);
    return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}

// The same for N independent fp32 values at once, level by level, so the N chains overlap.
template <int N>
__device__ __forceinline__ void wave_sum_f32_n(float (&v)[N])
{
    float t[N];
#pragma unroll
    for (int i = 0; i < N; ++i) t[i] = dpp_f32<0xB1>(v[i]);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] += t[i];
#pragma unroll
    for (int i = 0; i < N; ++i) t[i] = dpp_f32<0x4E>(v[i]);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] += t[i];
#pragma unroll
    for (int i = 0; i < N; ++i) t[i] = dpp_f32<0x141>(v[i]);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] += t[i];
#pragma unroll
    for (int i = 0; i < N; ++i) t[i] = dpp_f32<0x140>(v[i]);
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] += t[i];
#pragma unroll
    for (int i = 0; i < N; ++i) t[i] = __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v[i]), 0x401F));
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] += t[i];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const auto s = __builtin_amdgcn_permlane32_swap((unsigned)__float_as_int(v[i]), (unsigned)__float_as_int(v[i]), false, false);
        v[i] = __int_as_float((int)s[0]) + __int_as_float((int)s[1]);
    }
}

// Order-preserving map of a float to an unsigned key (larger value = larger key); 0 is below the key of every
// number, -inf included, and marks an absent value.
__device__ __forceinline__ unsigned order_key(float v)
{
    const unsigned b = __float_as_uint(v);
    return (b >> 31) ? ~b : b | 0x80000000u;
}
__device__ __forceinline__ float key_value(unsigned key)
{
    return __uint_as_float((key >> 31) ? key & 0x7fffffffu : ~key);
}

// Key of the k-th largest of the wave's two values per lane (0 if there are fewer than k): the key is built from
// the top bit down, keeping a bit whenever at least k keys are still at or above the candidate.  32 steps of two
// compares and two population counts, no data moves between lanes.
__device__ __forceinline__ unsigned wave_kth_key(unsigned ka, unsigned kb, int k)
{
    unsigned t = 0;
#pragma unroll 4
    for (int bit = 31; bit >= 0; --bit) {
        const unsigned c = t | (1u << bit);
        const int n = __popcll(__ballot(ka >= c)) + __popcll(__ballot(kb >= c));
        if (n >= k) t = c;
    }
    return t;
}

// One layer for R rows at once: out[r][j] = act(b[j] + sum_i W[j][i] * in(r, i)), fp32 multiply-adds.
// Narrow layers (<= 64 inputs, >= 64 outputs): a lane per output unit.  Otherwise a wavefront takes four output
// units per step, lanes over the inputs (coalesced weight reads), and the per-lane partial sums are combined as a
// balanced tree.  Weight loads are issued in batches ahead of their use.  Ends with a barrier.
template <int R, typename In>
__device__ __forceinline__ void mlp_layer(In in, int n_in, const float *W, const float *b, int n_out,
                                          float (*out)[MCSD_MLP_MAX_WIDTH], bool relu, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    if (n_in <= 64 && n_out >= 64) {
        for (int j = tid; j < n_out; j += DT) {
            float s[R];
            const float bj = b[j];
#pragma unroll
            for (int r = 0; r < R; ++r) s[r] = bj;
            const float *wr = W + (size_t)j * n_in;
            for (int i0 = 0; i0 < n_in; i0 += 16) {
                float w[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) w[u] = wr[min(i0 + u, n_in - 1)];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    if (i0 + u < n_in) {
#pragma unroll
                        for (int r = 0; r < R; ++r) s[r] = fmaf(w[u], in(r, i0 + u), s[r]);
                    }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) out[r][j] = (relu && s[r] < 0.0f) ? 0.0f : s[r];
        }
    } else {
        constexpr int JB = 4;
        for (int j0 = wave * JB; j0 < n_out; j0 += NW * JB) {
            float s[JB * R];
#pragma unroll
            for (int q = 0; q < JB * R; ++q) s[q] = 0.0f;
            for (int i0 = lane; i0 < n_in; i0 += 128) {
                float w[2][JB];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int jj = 0; jj < JB; ++jj)
                        w[u][jj] = W[(size_t)min(j0 + jj, n_out - 1) * n_in + min(i0 + 64 * u, n_in - 1)];
#pragma unroll
                for (int u = 0; u < 2; ++u)
                    if (i0 + 64 * u < n_in) {
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            const float xv = in(r, i0 + 64 * u);
#pragma unroll
                            for (int jj = 0; jj < JB; ++jj) s[jj * R + r] = fmaf(w[u][jj], xv, s[jj * R + r]);
                        }
                    }
            }
            wave_sum_f32_n<JB * R>(s);
            if (lane == 0) {
#pragma unroll
                for (int jj = 0; jj < JB; ++jj)
                    if (j0 + jj < n_out) {
                        const float bj = b[j0 + jj];
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            const float z = s[jj * R + r] + bj;
                            out[r][j0 + jj] = (relu && z < 0.0f) ? 0.0f : z;
                        }
                    }
            }
        }
    }
    __syncthreads();
}

// Layers first..n_layers-1 on activations already in act[cur]; returns the buffer index holding the logits.
template <int R>
__device__ __forceinline__ int mlp_tail(int n_layers, const int32_t *width, const float *const *w, const float *const *b,
                                        int first, float (*act)[R][MCSD_MLP_MAX_WIDTH], int cur, int tid)
{
    for (int l = first; l < n_layers; ++l) {
        float (*src)[MCSD_MLP_MAX_WIDTH] = act[cur];
        mlp_layer<R>([src](int r, int i) { return src[r][i]; }, width[l], w[l], b[l], width[l + 1], act[cur ^ 1],
                     l + 1 < n_layers, tid);
        cur ^= 1;
    }
    return cur;
}

__device__ __forceinline__ float logistic(float z) { return 1.0f / (1.0f + expf(-z)); }

// ---------------------------------------------------------------------------------------------- type 2
// MODE 0: the row lives in registers (V a multiple of 4, <= 32768, 16-byte aligned): one trip to HBM, all loads in
// flight at once.  MODE 1: float4 loads, MODE 2: scalar loads; both stream the row twice (the second pass is served
// by the cache).
template <int MODE>
__global__ __launch_bounds__(DT) void decision_distribution_kernel(MlpDesc mlp, int W, int V, int k,
                                                                   const float *__restrict__ rows, int64_t batch_stride,
                                                                   int64_t row_stride, float *__restrict__ features,
                                                                   float *__restrict__ prob)
{
    constexpr int CAP = MODE == 0 ? CAND_REG : CAND_MEM;
    __shared__ float s_cand[CAP];
    __shared__ float s_part[NW * K];
    __shared__ float s_top[K];
    __shared__ double s_ent[NW];
    __shared__ float s_act[2][1][MCSD_MLP_MAX_WIDTH];
    __shared__ int s_cnt;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = blockIdx.x;
    const float *y = rows + (int64_t)(m / W) * batch_stride + (int64_t)(m % W) * row_stride;

    float4 reg[MODE == 0 ? REG_F4 : 1];
    if (MODE == 0) {
#pragma unroll
        for (int j = 0; j < REG_F4; ++j) {
            const int i = tid * 4 + j * DT * 4;
            reg[j] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (i < V) {                                     // read exactly once: non-temporal, the caches need not keep it
                const nt_f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4_t *>(y + i));
                reg[j] = make_float4(t.x, t.y, t.z, t.w);
            }
        }
    }
    // every entry of the row, in the lane's own order (both passes must agree on nothing but the set)
    auto for_each = [&](auto f) {
        if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < REG_F4; ++j) { f(reg[j].x, j * 4); f(reg[j].y, j * 4 + 1); f(reg[j].z, j * 4 + 2); f(reg[j].w, j * 4 + 3); }
        } else if (MODE == 1) {
            for (int i = tid * 4; i < V; i += DT * 4) {
                const float4 v = *reinterpret_cast<const float4 *>(y + i);
                f(v.x, 0); f(v.y, 1); f(v.z, 2); f(v.w, 3);
            }
        } else {
            int n = 0;
            for (int i = tid; i < V; i += DT) f(y[i], n++);
        }
    };

    // pass 1: the lane's maximum and its share of -sum y log2 y.  The hardware logarithm (1 ulp) on normal numbers;
    // entries below the normal range contribute less than 1e-36 each and are skipped.  Four fp32 accumulators of
    // at most a quarter of the lane's entries each, combined in binary64.
    float tmax = -INFINITY;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    double hd = 0.0;                                            // streamed rows can be long: binary64 right away
    for_each([&](float p, int n) {
        tmax = fmaxf(tmax, p);
        const float t = (p >= 1.17549435e-38f) ? p * __log2f(p) : 0.0f;
        if (MODE == 0) acc[n & 3] -= t; else hd -= (double)t;
    });
    {
        if (MODE == 0) hd = ((double)acc[0] + (double)acc[1]) + ((double)acc[2] + (double)acc[3]);
        const double h = wave_sum(hd);
        if (lane == 0) s_ent[wave] = h;
    }
    if (tid == 0) s_cnt = 0;
    // tau = k-th largest lane maximum: at least k entries of the row are >= tau, and every entry above tau sits in
    // one of the at most k-1 lanes whose maximum is above it.  First the k largest of every wavefront (those above
    // its own k-th largest, then copies of that) ...
    {
        const unsigned key = order_key(tmax);
        const unsigned tw = wave_kth_key(key, 0u, k);
        const unsigned long long above = __ballot(key > tw);
        const int n_above = __popcll(above);
        if (key > tw) s_part[wave * K + __popcll(above & ((1ull << lane) - 1ull))] = tmax;
        if (lane >= n_above && lane < k) s_part[wave * K + lane] = key_value(tw);
    }
    __syncthreads();
    // ... then, in every wavefront for itself, the k-th largest of those 8 k values
    float tau;
    {
        const int ia = (lane / k) * K + lane % k, ib = ((lane + 64) / k) * K + (lane + 64) % k;
        const unsigned ka = lane < NW * k ? order_key(s_part[ia]) : 0u;
        const unsigned kb = lane + 64 < NW * k ? order_key(s_part[ib]) : 0u;
        tau = key_value(wave_kth_key(ka, kb, k));
    }

    // pass 2, only in the lanes that have any: the entries above tau, in any order
    if (tmax > tau) {
        int mine = 0;
        for_each([&](float p, int) { mine += p > tau ? 1 : 0; });
        int pos = atomicAdd(&s_cnt, mine);
        if (mine == 1) {                                        // the usual case: the lane's maximum and nothing else
            if (pos < CAP) s_cand[pos] = tmax;
        } else {
            for_each([&](float p, int) {
                if (p > tau) {
                    if (pos < CAP) s_cand[pos] = p;
                    ++pos;
                }
            });
        }
    }
    __syncthreads();

    // Topk = those candidates by rank (ties in list order), then copies of tau (entries equal to tau exist in
    // sufficient number), or zeros when the row has fewer than k entries
    {
        const int n = min(s_cnt, CAP);
        for (int i = tid; i < n; i += DT) {
            const float c = s_cand[i];
            int rank = 0;
            for (int j = 0; j < n; ++j) {
                const float o = s_cand[j];
                rank += (o > c || (o == c && j < i)) ? 1 : 0;
            }
            if (rank < k) s_top[rank] = c;
        }
        if (tid >= n && tid < k) s_top[tid] = tau > -INFINITY ? tau : 0.0f;
    }
    __syncthreads();
    if (tid < k) s_act[0][0][tid] = s_top[tid];
    if (tid == 0) {
        double e = 0.0;
        for (int w = 0; w < NW; ++w) e += s_ent[w];
        s_act[0][0][k] = (float)(e * 0.69314718055994530942);   // log2 -> nats
    }
    __syncthreads();
    if (features && tid <= k) features[(int64_t)m * (k + 1) + tid] = s_act[0][0][tid];

    const int cur = mlp_tail<1>(mlp.n_layers, mlp.width, mlp.w, mlp.b, 0, s_act, 0, tid);
    if (tid == 0) prob[m] = logistic(s_act[cur][0][0]);
}

// ---------------------------------------------------------------------------------------------- type 1
// First layer on HROWS hidden states of at most 256 NC entries (a multiple of 4, rows and weights 16-byte aligned):
// a lane keeps its slice of the four rows in registers (entries 4 lane + 256 c ..+3), a wavefront takes four output
// units per step and streams their weights once for all four rows; fp32 multiply-adds, per-lane partial sums combined as a
// balanced tree.  (A 768-wide row has 12 entries per lane: the products' rounding stays near 1e-7 of the sum.)
template <int NC>
__device__ __forceinline__ void hidden_first_layer(const float *const (&x)[HROWS], int n_in, const float *__restrict__ W,
                                   const float *__restrict__ b, int n_out, float (*out)[MCSD_MLP_MAX_WIDTH], bool relu,
                                   int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    float4 xr[HROWS][NC];
#pragma unroll
    for (int r = 0; r < HROWS; ++r)
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int i = lane * 4 + c * 256;               // loads are unconditional from a valid address
            const float4 t = *reinterpret_cast<const float4 *>(x[r] + min(i, n_in - 4));
            xr[r][c] = i < n_in ? t : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
    // JB output units per step; the next step's weights are requested before this step's arithmetic starts
    constexpr int JB = 4;
    auto load_weights = [&](float4 (&w)[JB][NC], int j0) {
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
            const float *wr = W + (size_t)min(j0 + jj, n_out - 1) * n_in;       // past the end: a valid row, unused
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int i = lane * 4 + c * 256;
                w[jj][c] = *reinterpret_cast<const float4 *>(wr + min(i, n_in - 4));    // beyond n_in: times zero

            }
        }
    };
    float4 wn[JB][NC];
    if (wave * JB < n_out) load_weights(wn, wave * JB);
    for (int j0 = wave * JB; j0 < n_out; j0 += NW * JB) {
        float4 w[JB][NC];
#pragma unroll
        for (int jj = 0; jj < JB; ++jj)
#pragma unroll
            for (int c = 0; c < NC; ++c) w[jj][c] = wn[jj][c];
        if (j0 + NW * JB < n_out) load_weights(wn, j0 + NW * JB);
        float s[JB * HROWS];
#pragma unroll
        for (int jj = 0; jj < JB; ++jj)
#pragma unroll
            for (int r = 0; r < HROWS; ++r) {
                float a = 0.0f;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    a = fmaf(w[jj][c].x, xr[r][c].x, a);
                    a = fmaf(w[jj][c].y, xr[r][c].y, a);
                    a = fmaf(w[jj][c].z, xr[r][c].z, a);
                    a = fmaf(w[jj][c].w, xr[r][c].w, a);
                }
                s[jj * HROWS + r] = a;
            }
        wave_sum_f32_n<JB * HROWS>(s);
        if (lane == 0) {
#pragma unroll
            for (int jj = 0; jj < JB; ++jj)
                if (j0 + jj < n_out) {
                    const float bj = b[j0 + jj];
#pragma unroll
                    for (int r = 0; r < HROWS; ++r) {
                        const float z = s[jj * HROWS + r] + bj;
                        out[r][j0 + jj] = (relu && z < 0.0f) ? 0.0f : z;
                    }
                }
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(DT) void decision_hidden_kernel(MlpDesc mlp, int M, int W, const float *__restrict__ hidden,
                                                             int64_t batch_stride, int64_t row_stride,
                                                             float *__restrict__ prob)
{
    __shared__ float s_act[2][HROWS][MCSD_MLP_MAX_WIDTH];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.x * HROWS;
    const float *x[HROWS];
#pragma unroll
    for (int r = 0; r < HROWS; ++r) {
        const int m = min(m0 + r, M - 1);                       // rows past the end repeat the last one, unwritten
        x[r] = hidden + (int64_t)(m / W) * batch_stride + (int64_t)(m % W) * row_stride;
    }
    const int n_in = mlp.width[0];
    const bool aligned = n_in % 4 == 0 && batch_stride % 4 == 0 && row_stride % 4 == 0 &&
                         (((uintptr_t)hidden | (uintptr_t)mlp.w[0]) & 15) == 0;
    if (aligned && n_in <= 256)
        hidden_first_layer<1>(x, n_in, mlp.w[0], mlp.b[0], mlp.width[1], s_act[0], mlp.n_layers > 1, tid);
    else if (aligned && n_in <= 512)
        hidden_first_layer<2>(x, n_in, mlp.w[0], mlp.b[0], mlp.width[1], s_act[0], mlp.n_layers > 1, tid);
    else if (aligned && n_in <= 768)
        hidden_first_layer<3>(x, n_in, mlp.w[0], mlp.b[0], mlp.width[1], s_act[0], mlp.n_layers > 1, tid);
    else if (aligned && n_in <= 1024)
        hidden_first_layer<4>(x, n_in, mlp.w[0], mlp.b[0], mlp.width[1], s_act[0], mlp.n_layers > 1, tid);
    else        // any width and alignment: straight from global memory
        mlp_layer<HROWS>([x0 = x[0], x1 = x[1], x2 = x[2], x3 = x[3]](int r, int i) {
                             return (r == 0 ? x0 : r == 1 ? x1 : r == 2 ? x2 : x3)[i];
                         }, n_in, mlp.w[0], mlp.b[0], mlp.width[1], s_act[0], mlp.n_layers > 1, tid);
    const int cur = mlp_tail<HROWS>(mlp.n_layers, mlp.width, mlp.w, mlp.b, 1, s_act, 0, tid);
    if (tid < HROWS && m0 + tid < M) prob[m0 + tid] = logistic(s_act[cur][tid][0]);
}

// ---------------------------------------------------------------------------------------------- stop rule
__global__ __launch_bounds__(256) void early_stop_kernel(const float *__restrict__ prob, int B, int W, float beta,
                                                         int32_t *__restrict__ stop)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    int all_below = 1;
    for (int w = 0; w < W; ++w)
        if (!(prob[(int64_t)b * W + w] < beta)) all_below = 0;
    stop[b] = all_below;
}

int check_mlp(const mcsd_mlp_t *mlp, int32_t n_in, MlpDesc *out)
{
    if (!mlp || mlp->n_layers < 1 || mlp->n_layers > MCSD_MLP_MAX_LAYERS) return MCSD_EINVAL;
    if (mlp->width[0] != n_in || mlp->width[mlp->n_layers] != 1) return MCSD_EINVAL;
    out->n_layers = mlp->n_layers;
    for (int l = 0; l <= mlp->n_layers; ++l) {
        if (mlp->width[l] < 1) return MCSD_EINVAL;
        if (l > 0 && mlp->width[l] > MCSD_MLP_MAX_WIDTH) return MCSD_EUNSUPPORTED;
        out->width[l] = mlp->width[l];
    }
    for (int l = 0; l < mlp->n_layers; ++l) {
        if (!mlp->weight[l] || !mlp->bias[l]) return MCSD_EINVAL;
        out->w[l] = mlp->weight[l];
        out->b[l] = mlp->bias[l];
    }
    for (int l = mlp->n_layers; l < 3; ++l) { out->w[l] = nullptr; out->b[l] = nullptr; out->width[l + 1] = 0; }
    return MCSD_OK;
}

int launch_stop(const float *prob, int32_t B, int32_t W, float beta, int32_t *stop, hipStream_t st)
{
    hipLaunchKernelGGL(early_stop_kernel, dim3((B + 255) / 256), dim3(256), 0, st, prob, (int)B, (int)W, beta, stop);
    return mcsd_hip_status(hipGetLastError());
}

}  // namespace

extern "C" int mcsd_early_stop_distribution(const mcsd_mlp_t *mlp, int32_t B, int32_t W, int32_t V, int32_t k,
                                            const float *draft_rows_dev, int64_t batch_stride, int64_t row_stride,
                                            float beta, float *features_dev, float *prob_dev, int32_t *stop_dev,
                                            void *hip_stream)
{
    if (B < 0 || W < 1 || V < 1 || k < 1 || batch_stride < 0 || row_stride < 0) return MCSD_EINVAL;
    if (k > MCSD_DECISION_MAX_K || V > MCSD_MAX_VOCAB) return MCSD_EUNSUPPORTED;
    MlpDesc d;
    if (int rc = check_mlp(mlp, k + 1, &d)) return rc;
    if (B == 0) return MCSD_OK;
    if (!draft_rows_dev || !prob_dev || !stop_dev) return MCSD_EINVAL;
    if ((int64_t)B * W > 0x7fffffff / (MCSD_DECISION_MAX_K + 1)) return MCSD_EUNSUPPORTED;
    // a lane holds at most ceil(V / (4 DT)) * 4 entries and at most k-1 lanes hold entries above the threshold
    static_assert((int64_t)(K - 1) * ((MCSD_MAX_VOCAB + 4 * DT - 1) / (4 * DT)) * 4 <= CAND_MEM, "candidate list too small");
    static_assert((K - 1) * REG_F4 * 4 <= CAND_REG, "candidate list too small");
    const bool vec = V % 4 == 0 && batch_stride % 4 == 0 && row_stride % 4 == 0 && ((uintptr_t)draft_rows_dev & 15) == 0;
    const int mode = !vec ? 2 : (V <= REG_F4 * 4 * DT ? 0 : 1);
    hipStream_t st = (hipStream_t)hip_stream;
    const dim3 grid((unsigned)(B * W)), block(DT);
    auto kernel = mode == 0 ? decision_distribution_kernel<0> : mode == 1 ? decision_distribution_kernel<1>
                                                                         : decision_distribution_kernel<2>;
    mcsd_launch(MCSD_KERNEL_DECISION, kernel, grid, block, st, d, (int)W, (int)V, (int)k, draft_rows_dev, batch_stride,
                row_stride, features_dev, prob_dev);
    if (int rc = mcsd_hip_status(hipGetLastError())) return rc;
    return launch_stop(prob_dev, B, W, beta, stop_dev, st);
}

extern "C" int mcsd_early_stop_hidden(const mcsd_mlp_t *mlp, int32_t B, int32_t W, const float *hidden_dev,
                                      int64_t batch_stride, int64_t row_stride, float beta, float *prob_dev,
                                      int32_t *stop_dev, void *hip_stream)
{
    if (B < 0 || W < 1 || batch_stride < 0 || row_stride < 0 || !mlp) return MCSD_EINVAL;
    if (mlp->width[0] > MCSD_MLP_MAX_INPUTS) return MCSD_EUNSUPPORTED;
    MlpDesc d;
    if (int rc = check_mlp(mlp, mlp->width[0], &d)) return rc;
    if (B == 0) return MCSD_OK;
    if (!hidden_dev || !prob_dev || !stop_dev) return MCSD_EINVAL;
    if ((int64_t)B * W > 0x7fffffff / 2) return MCSD_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)hip_stream;
    const int M = B * W;
    mcsd_launch(MCSD_KERNEL_DECISION, decision_hidden_kernel, dim3((M + HROWS - 1) / HROWS), dim3(DT), st, d, M, (int)W,
                hidden_dev, batch_stride, row_stride, prob_dev);
    if (int rc = mcsd_hip_status(hipGetLastError())) return rc;
    return launch_stop(prob_dev, B, W, beta, stop_dev, st);
}
