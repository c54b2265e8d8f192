// Multi-candidate verification for gfx950 (Sec. 2.1, Sec. 3.1 and Fig. 1 steps 4-6 of arXiv 2409.10644):
// recursive rejection sampling down the candidate tree, longest-path selection for target-initialised
// trees, and sampling of the new token(s).
//
// One workgroup of 1024 lanes walks one tree (draft-initialised) or one level-1 subtree (target-initialised).
// Sums over the vocabulary follow the balanced binary tree over the zero-padded index space that the header
// specifies; all arithmetic is binary64 with explicit fma, so results equal the oracle's recursion bit for bit.
//
// Vocabularies up to 32768 (verify_walk_fast_kernel): a context's two rows are read once, on its first rejection.
// Lane t of the workgroup owns the 32 CONSECUTIVE elements 32 t .. 32 t + 31: an aligned subtree of the sum tree, so
// a sum is 31 in-lane additions, one 6-level butterfly over the wavefront's 64 lanes and a 4-level tree over the 16
// wavefront sums (one barrier per rejection round).  The residual r <- max(r - S q, 0) lives in registers as
// binary64 and is updated in place; the draft row is parked in LDS.  Rows are fetched with coalesced 16-byte loads
// and handed to their owner lanes through LDS (a wavefront's 2048 elements stay inside the wavefront, so the
// hand-over needs no barrier); the LDS image is XOR-swizzled so that both sides are free of bank conflicts.
// New tokens are drawn by the wavefronts independently (wavefront k takes draws k, k + 16, ..): the 16 wavefront
// sums, then the heap of the chosen wavefront's lane sums (kept in LDS from the butterfly's levels), then the 32
// elements of the chosen lane, recomputed from the rows and the history of sums.
//
// Larger vocabularies (verify_walk_kernel): the residual is never stored; after j rejections an element is recomputed
// from p, q and the j previous sums (a chain of j fused multiply-adds), a round is one coalesced sweep over the two
// rows, 256-element blocks are reduced by butterflies and a tree over the block sums that every wavefront adds for
// itself; a heap over the blocks is built in LDS only for the inverse-CDF descent.
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

template <int NBMAX>
struct SharedT {
    double leaf[2][NBMAX];               // sums of the 256-element blocks, double-buffered over rejection rounds
    double heapB[2 * NBMAX];             // heap over the blocks: leaves at [NB, 2NB), root at 1 (built for the descent only)
    double heapA[2 * BLK];               // heap inside one block, rebuilt for each descent
    double s_hist[MCSD_MAX_BRANCH + 1];  // S before each rejection round of the current context
    double sq_hist[MCSD_MAX_BRANCH + 1]; // candidates without replacement: sum of the shrunken draft row before each round
    int x_hist[MCSD_MAX_BRANCH + 1];     // ... and the token rejected in that round (its draft mass is zero afterwards)
    int lo_idx, hi_idx;
};

// max(d, 0) as one instruction.  d is never NaN here, and the sign of a zero result never reaches a decision
// (zeros only enter sums, products and comparisons with 0), so this equals "d > 0 ? d : 0" for every use below.
__device__ inline double pos_part(double d) { return __builtin_fmax(d, 0.0); }

// One element of the distribution after `rounds` rejections, from its target value r and draft value qd.
// With replacement: r <- max(r - S q, 0) per round.  NOREP (candidates drawn without replacement): the draft row
// loses every rejected token, and with Sq the sum of what is left, r <- max(r Sq - S q', 0).
template <bool NOREP, class Shared>
__device__ inline double residual_chain(const Shared &sh, double r, double qd, int t, int rounds)
{
    for (int k = 0; k < rounds; ++k) {
        if (NOREP) {
            if (k > 0 && t == sh.x_hist[k - 1]) qd = 0.0;
            r = __dmul_rn(r, sh.sq_hist[k]);
        }
        const double d = __fma_rn(-sh.s_hist[k], qd, r);
        r = pos_part(d);
    }
    return r;
}

// Element t of the distribution after `rounds` rejections at a context with rows prow / qrow.
template <bool NOREP, class Shared>
__device__ inline double residual_at(const Shared &sh, const float *prow, const float *qrow, int rounds, int t)
{
    const double r = (double)prow[t];
    return rounds > 0 ? residual_chain<NOREP>(sh, r, (double)qrow[t], t, rounds) : r;
}

// A double from another lane of the row through the data-parallel-primitive path of the vector ALU (no LDS).
template <int CTRL>
__device__ inline double dpp_f64(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes in balanced-tree order (lane pairs, then pairs of pairs, ...); every lane gets the total.
// Partner lanes: l^1 and l^2 by quad permutation; then, since all lanes of a group of 4 (8) already hold the same
// value, the mirrored lane of the half row (row) stands in for l^4 (l^8); l^16 by swizzle; l^32 by the half-wave
// swap, whose two results are {own, partner} in an order that the commutative addition does not care about.
__device__ inline double wave_tree_sum(double v)
{
    v = __dadd_rn(v, dpp_f64<0xB1>(v));          // quad_perm [1,0,3,2]
    v = __dadd_rn(v, dpp_f64<0x4E>(v));          // quad_perm [2,3,0,1]
    v = __dadd_rn(v, dpp_f64<0x141>(v));         // row_half_mirror
    v = __dadd_rn(v, dpp_f64<0x140>(v));         // row_mirror
    {
        const int lo = __builtin_amdgcn_ds_swizzle(__double2loint(v), 0x401F);   // lane ^ 16 inside each 32
        const int hi = __builtin_amdgcn_ds_swizzle(__double2hiint(v), 0x401F);
        v = __dadd_rn(v, __hiloint2double(hi, lo));
    }
    {
        const auto lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(v), (unsigned)__double2loint(v), false, false);
        const auto hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(v), (unsigned)__double2hiint(v), false, false);
        v = __dadd_rn(__hiloint2double((int)hi[0], (int)lo[0]), __hiloint2double((int)hi[1], (int)lo[1]));
    }
    return v;
}

// Block sums of the distribution (prow, qrow, rounds) recomputed from memory into leaf[buf]; any NB.  No barrier
// at the end; s_hist[0 .. rounds) must be visible.
constexpr int SGROUP = 8;                // blocks a wavefront streams at a time
template <bool NOREP, class Shared>
__device__ void stream_block_sums(Shared &sh, const VerifyParams &P, const float *prow, const float *qrow,
                                  int rounds, int buf)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool vec = (((uintptr_t)prow | (uintptr_t)qrow) & 15) == 0;
    for (int blk0 = wave; blk0 < P.NB; blk0 += SGROUP * (VT / 64)) {
        float pe[SGROUP][4], qe[SGROUP][4];
#pragma unroll
        for (int k = 0; k < SGROUP; ++k) {
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
        double sblk[SGROUP];
#pragma unroll
        for (int k = 0; k < SGROUP; ++k) {
            double v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)                      // elements beyond V are 0 and stay 0
                v[e] = residual_chain<NOREP>(sh, (double)pe[k][e], (double)qe[k][e],
                                             (blk0 + k * (VT / 64)) * BLK + lane * 4 + e, rounds);
            sblk[k] = __dadd_rn(__dadd_rn(v[0], v[1]), __dadd_rn(v[2], v[3]));
        }
#pragma unroll
        for (int k = 0; k < SGROUP; ++k) sblk[k] = wave_tree_sum(sblk[k]);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < SGROUP; ++k) {
                const int blk = blk0 + k * (VT / 64);
                if (blk < P.NB) sh.leaf[buf][blk] = sblk[k];
            }
        }
    }
}

// Total of leaf[buf][0 .. NB) in balanced-tree order, computed by every wavefront for itself (no further barrier):
// a lane adds its NB/64 consecutive leaves as a small tree (zero-filled to PER: x + 0 is exact), then 64 lanes
// combine.  PER = largest NB / 64 the caller can have.
template <int PER, class Shared>
__device__ inline double top_tree_sum(const Shared &sh, const VerifyParams &P, int buf)
{
    const int lane = threadIdx.x & 63;
    const int per = P.NB >= 64 ? P.NB >> 6 : 1;                  // 1 .. PER
    double v[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int idx = lane * per + i;
        v[i] = (i < per && idx < P.NB) ? sh.leaf[buf][idx] : 0.0;
    }
#pragma unroll
    for (int w = PER / 2; w >= 1; w >>= 1)
#pragma unroll
        for (int i = 0; i < w; ++i) v[i] = __dadd_rn(v[2 * i], v[2 * i + 1]);
    return wave_tree_sum(v[0]);
}

// heapB from leaf[buf].  All threads call it; ends with a barrier.
template <class Shared>
__device__ void build_heap(Shared &sh, const VerifyParams &P, int buf)
{
    const int tid = threadIdx.x;
    for (int i = tid; i < P.NB; i += VT) sh.heapB[P.NB + i] = sh.leaf[buf][i];
    __syncthreads();
    for (int n = P.NB >> 1; n >= 1; n >>= 1) {
        for (int i = tid; i < n; i += VT) sh.heapB[n + i] = __dadd_rn(sh.heapB[2 * (n + i)], sh.heapB[2 * (n + i) + 1]);
        __syncthreads();
    }
}

// Inverse-CDF draw from the distribution whose heapB is current.  All threads call it; all return the token.
template <bool NOREP, class Shared>
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
        sh.heapA[BLK + tid] = t < P.V ? residual_at<NOREP>(sh, prow, qrow, rounds, t) : 0.0;
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
        if (residual_at<NOREP>(sh, prow, qrow, rounds, e) > 0.0) {
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

// Vocabularies beyond FAST_V: the rows are streamed again every round.
// NOREP: the candidates of a context were drawn without replacement (see residual_chain).
template <bool NOREP>
__global__ __launch_bounds__(VT) void verify_walk_kernel(const VerifyParams P)
{
    using Shared = SharedT<MAX_NB>;
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
    const int lane = tid & 63;
    const float *term_p = nullptr, *term_q = nullptr;
    int term_rounds = 0, term_buf = -1;       // term_buf >= 0: leaf[term_buf] holds the terminal distribution's block sums
    int buf = 0;
    while (level < P.t.gamma) {
        const float *prow = p + (int64_t)(cur + 1) * P.V;
        const float *qrow = q + (int64_t)(cur + 1) * P.V;
        const int cnt = P.t.b[level];
        const int first = cur < 0 ? 0 : P.t.off[level] + (cur - P.t.off[level - 1]) * cnt;
        // candidate `lane` of this context (in every wavefront): acceptance uniform, q(x) and the residual at x,
        // which is updated in place after every rejection
        double uc = 0.0, qc = 0.0, rc = 0.0;
        int xc = -1;
        if (lane < cnt) {
            int x = tokens[first + lane];
            x = x < 0 ? 0 : (x >= P.V ? P.V - 1 : x);   // ids outside 0..V-1 are clamped, never dereferenced
            xc = x;
            uc = (double)ua[first + lane];
            qc = (double)qrow[x];
            rc = (double)prow[x];
        }
        int rounds = 0, accepted = -1;
        double S = 1.0, Sq = 1.0;                        // both rows are trusted to be normalised in round 0
        // accept test of candidate c: the same value in every lane, read through one lane so that the walk is
        // scalar control flow
        auto accept = [&](int c) {
            const double u = __shfl(uc, c, 64), qx = __shfl(qc, c, 64), rx = __shfl(rc, c, 64);
            const double rhs = NOREP ? __dmul_rn(rx, Sq) : rx;
            return __builtin_amdgcn_readfirstlane((int)(__dmul_rn(u, __dmul_rn(qx, S)) < rhs)) != 0;
        };
        if (accept(0)) {
            accepted = first;
        } else {
            // First rejection at this context: from here on the residual is needed.
            for (int c = 0;;) {
                // candidate c was rejected: r <- max(r - S q, 0), S <- sum r
                const int xrej = NOREP ? __builtin_amdgcn_readfirstlane(__shfl(xc, c, 64)) : 0;
                const double qrej = NOREP ? __shfl(qc, c, 64) : 0.0;
                if (tid == 0) {
                    sh.s_hist[rounds] = S;
                    if (NOREP) { sh.sq_hist[rounds] = Sq; sh.x_hist[rounds] = xrej; }
                }
                buf ^= 1;
                {
                    __syncthreads();          // s_hist[rounds] (sq_hist, x_hist) visible
                    stream_block_sums<NOREP>(sh, P, prow, qrow, rounds + 1, buf);
                }
                {
                    const double d = __fma_rn(-S, qc, NOREP ? __dmul_rn(rc, Sq) : rc);
                    rc = pos_part(d);
                }
                if (NOREP) {
                    Sq = __dsub_rn(Sq, qrej);
                    if (xc == xrej) qc = 0.0;             // also a later duplicate of the rejected token
                }
                rounds += 1;
                __syncthreads();              // block sums (and s_hist) visible
                S = top_tree_sum<MAX_NB / 64>(sh, P, buf);
                if (++c == cnt) break;
                if (accept(c)) { accepted = first + c; break; }
            }
        }
        if (accepted < 0) {
            term_p = prow; term_q = qrow;
            if (S > 0.0) { term_rounds = rounds; term_buf = rounds > 0 ? buf : -1; }
            else { term_rounds = 0; term_buf = -1; }     // vanished residual: the context's own target row
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
        term_buf = -1;
    }
    if (tid == 0) {
        for (int l = n_acc; l < P.t.gamma; ++l) path_out[l] = -1;
        P.cand_len[(int64_t)b * P.R + root] = n_acc;
    }
    if (P.n_new > 0) {
        if (term_buf < 0) {
            buf ^= 1;
            __syncthreads();
            stream_block_sums<NOREP>(sh, P, term_p, term_q, 0, buf);
            term_buf = buf;
        }
        __syncthreads();
        build_heap(sh, P, term_buf);
        for (int k = 0; k < P.n_new; ++k) {
            const int t = tree_sample<NOREP>(sh, P, term_p, term_q, term_rounds, P.us[(int64_t)b * P.n_new + k]);
            if (tid == 0) P.cand_new[((int64_t)b * P.R + root) * P.n_new + k] = t;
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Vocabularies up to FAST_V: rows held by the workgroup, 32 consecutive elements per lane
// ---------------------------------------------------------------------------------------------------
constexpr int EPL = 32;                  // consecutive vocabulary elements per lane
constexpr int FAST_V = VT * EPL;         // 32768
constexpr int NWAVE = VT / 64;           // 16
constexpr int WCHUNKS = 64 * EPL / 4;    // 16-byte chunks of a wavefront's 2048 elements

struct FastShared {
    float qrow[FAST_V];                  // the context's draft row; wavefront w owns [2048 w, 2048 w + 2048), swizzled
    double wsum[2][NWAVE];               // sums of the wavefronts' 2048-element subtrees, double-buffered over rounds
    double heapw[NWAVE][128];            // per wavefront: heap over its 64 lane sums (root 1, leaves 64..127), for sampling
    double s_hist[MCSD_MAX_BRANCH + 1];  // S before each rejection round of the current context
    double sq_hist[MCSD_MAX_BRANCH + 1]; // candidates without replacement: sum of the shrunken draft row before each round
    int x_hist[MCSD_MAX_BRANCH + 1];     // ... and the token rejected in that round
};

// Position of chunk j (elements 4 j .. 4 j + 3 of the lane's 32) of lane l inside the wavefront's region, in 16-byte
// chunks.  The XOR makes the 16 lanes that LDS serves together hit 16 different 16-byte bank groups both when lanes
// read their own chunk j (lane stride 128 bytes) and when they write consecutive chunks of a row (see fast_load_row).
__device__ inline int fast_slot(int l, int j) { return l * 8 + (j ^ ((l >> 1) & 7)); }

// One row (V floats) from global memory into the wavefront's LDS region: coalesced 16-byte loads (lane i of load k
// fetches the wavefront's chunk 64 k + i), stored where the owner lane will look for it.  Elements beyond V are 0.
__device__ inline void fast_fetch_row(const VerifyParams &P, const float *row, float4 (&v)[8])
{
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));          // (offsets recomputed at every use instead of kept in registers for the whole walk)
    const int wave = t >> 6, lane = t & 63;
    if ((((uintptr_t)row & 15) | (P.V & 3)) == 0) {            // aligned rows: a chunk is inside V or outside as a whole
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int t0 = (wave * WCHUNKS + k * 64 + lane) * 4;
            v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (t0 < P.V) v[k] = *(const float4 *)(row + t0);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int t0 = (wave * WCHUNKS + k * 64 + lane) * 4;
            v[k].x = t0 + 0 < P.V ? row[t0 + 0] : 0.f;
            v[k].y = t0 + 1 < P.V ? row[t0 + 1] : 0.f;
            v[k].z = t0 + 2 < P.V ? row[t0 + 2] : 0.f;
            v[k].w = t0 + 3 < P.V ? row[t0 + 3] : 0.f;
        }
    }
}
__device__ inline void fast_park_row(float4 *region, const float4 (&v)[8])
{
    int lane = threadIdx.x & 63;
    asm volatile("" : "+v"(lane));       // (LDS addresses recomputed here, a few integer operations, instead of spilled)
#pragma unroll
    for (int k = 0; k < 8; ++k) region[fast_slot(k * 8 + (lane >> 3), lane & 7)] = v[k];   // chunk 64 k + lane: owner lane, its chunk
}

// Sum of the lane's 32 elements in tree order (pairs, pairs of pairs, ...).
__device__ inline double lane_tree_sum(const double (&r)[EPL])
{
    double q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) q[j] = __dadd_rn(__dadd_rn(r[4 * j], r[4 * j + 1]), __dadd_rn(r[4 * j + 2], r[4 * j + 3]));
    return __dadd_rn(__dadd_rn(__dadd_rn(q[0], q[1]), __dadd_rn(q[2], q[3])), __dadd_rn(__dadd_rn(q[4], q[5]), __dadd_rn(q[6], q[7])));
}

// The four tree levels over 16 values held by lanes 0..15 of every row of 16 lanes (partners l^1, l^2, then the
// mirrored lanes standing in for l^4 and l^8, as in wave_tree_sum).
__device__ inline double row16_tree_sum(double v)
{
    v = __dadd_rn(v, dpp_f64<0xB1>(v));
    v = __dadd_rn(v, dpp_f64<0x4E>(v));
    v = __dadd_rn(v, dpp_f64<0x141>(v));
    v = __dadd_rn(v, dpp_f64<0x140>(v));
    return v;
}

// Lane `src` (uniform) of a double.
__device__ inline double read_lane_f64(double v, int src)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), src), __builtin_amdgcn_readlane(__double2loint(v), src));
}

// One inverse-CDF draw from the terminal distribution by ONE wavefront (all 64 lanes call it; no barrier inside).
// wsum[buf] holds the wavefront sums and heapw the lane-sum heaps of that distribution; its elements are recomputed
// from the rows and the history (prow, qrow, rounds).  Returns the token in every lane.
template <bool NOREP>
__device__ int fast_sample(const FastShared &sh, const VerifyParams &P, int buf, const float *prow, const float *qrow,
                           int rounds, float u)
{
    const int lane = threadIdx.x & 63;
    // heap over the 16 wavefront sums, in registers: n[16 + w] = sum of wavefront w
    double n[32];
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) n[16 + w] = sh.wsum[buf][w];
#pragma unroll
    for (int i = 15; i >= 1; --i) n[i] = __dadd_rn(n[2 * i], n[2 * i + 1]);
    double thr = __dmul_rn((double)u, n[1]);
    int node = 1;
#pragma unroll
    for (int lvl = 0; lvl < 4; ++lvl) {
        double left = 0.0;
#pragma unroll
        for (int j = 0; j < (1 << lvl); ++j)
            if (node == (1 << lvl) + j) left = n[2 * ((1 << lvl) + j)];      // (selects: registers cannot be indexed at run time)
        if (thr < left) {
            node = 2 * node;
        } else {
            thr = __dsub_rn(thr, left);
            node = 2 * node + 1;
        }
    }
    const int w = node - 16;
    node = 1;
    while (node < 64) {
        const double left = sh.heapw[w][2 * node];
        if (thr < left) {
            node = 2 * node;
        } else {
            thr = __dsub_rn(thr, left);
            node = 2 * node + 1;
        }
    }
    const int t0 = (w * 64 + (node - 64)) * EPL;          // first element of the chosen lane
    // its 32 elements, one per lane of this wavefront (lanes 32..63 hold zeros), and the levels of their sum tree
    const int te = t0 + lane;
    double lv[6];
    lv[0] = (lane < EPL && te < P.V) ? residual_at<NOREP>(sh, prow, qrow, rounds, te) : 0.0;
    lv[1] = __dadd_rn(lv[0], dpp_f64<0xB1>(lv[0]));
    lv[2] = __dadd_rn(lv[1], dpp_f64<0x4E>(lv[1]));
    lv[3] = __dadd_rn(lv[2], dpp_f64<0x141>(lv[2]));
    lv[4] = __dadd_rn(lv[3], dpp_f64<0x140>(lv[3]));
    int lo = 0;
#pragma unroll
    for (int j = 5; j >= 1; --j) {                         // the node covers lanes lo .. lo + 2^j - 1
        const double left = read_lane_f64(lv[j - 1], lo);
        if (!(thr < left)) {
            thr = __dsub_rn(thr, left);
            lo += 1 << (j - 1);
        }
    }
    int t = t0 + lo;
    if (t < P.V && read_lane_f64(lv[0], lo) > 0.0) return t;
    // Reached a zero-weight index (last-bit rounding of the subtraction, or an all-zero distribution):
    // nearest positive-weight index below, else nearest above, else 0.
    int below = -1, above = 0x7fffffff;
    for (int e = lane; e < P.V; e += 64) {
        if (e == t) continue;
        if (residual_at<NOREP>(sh, prow, qrow, rounds, e) > 0.0) {
            if (e < t) below = e > below ? e : below;
            else above = e < above ? e : above;
        }
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) {
        const int ob = __shfl_xor(below, m, 64), oa = __shfl_xor(above, m, 64);
        below = ob > below ? ob : below;
        above = oa < above ? oa : above;
    }
    return below >= 0 ? below : (above != 0x7fffffff ? above : 0);
}

template <bool NOREP>
__global__ __launch_bounds__(VT) void verify_walk_fast_kernel(const VerifyParams P)
{
    __shared__ FastShared sh;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int root = blockIdx.x, b = blockIdx.y;
    const int32_t *tokens = P.tokens + (int64_t)b * P.n_nodes;
    const float *p = P.p + (int64_t)b * P.pbs;
    const float *q = P.q + (int64_t)b * P.qbs;
    const float *ua = P.ua + (int64_t)b * P.n_nodes;
    int32_t *path_out = P.cand_path + ((int64_t)b * P.R + root) * P.t.gamma;
    float4 *region = (float4 *)sh.qrow + wave * WCHUNKS;      // this wavefront's part of the parked row

    int cur = -1, level = 0, n_acc = 0;      // context: node id (-1 = end of the prefix) and its level
    if (P.mode == MCSD_TARGET_INIT) {         // level-1 node `root` is accepted untested
        cur = root;
        level = 1;
        n_acc = 1;
        if (tid == 0) path_out[0] = root;
    }
    double r[EPL];                            // this lane's 32 elements of the current residual
    const float *term_p = nullptr, *term_q = nullptr;
    int term_rounds = 0;
    bool term_in_regs = false;                // r holds the terminal distribution (a residual with positive sum)
    int buf = 0;

    // the target row `prow` into r: fetched coalesced, handed to the owner lanes through this wavefront's LDS region
    auto row_to_regs = [&](const float4 (&pv)[8]) {
        fast_park_row(region, pv);
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float4 v = region[fast_slot(ln, j)];
            r[4 * j] = (double)v.x; r[4 * j + 1] = (double)v.y; r[4 * j + 2] = (double)v.z; r[4 * j + 3] = (double)v.w;
        }
    };
    // sum of r over the vocabulary; with `heap` the levels of the wavefront's butterfly are kept for the sampler.
    // One barrier; wsum[buf] is written, the other buffer may still be read by slower wavefronts.
    auto total = [&](bool heap) {
        double v = lane_tree_sum(r);
        if (heap) sh.heapw[wave][64 + lane] = v;
        v = __dadd_rn(v, dpp_f64<0xB1>(v));
        if (heap && (lane & 1) == 0) sh.heapw[wave][32 + (lane >> 1)] = v;
        v = __dadd_rn(v, dpp_f64<0x4E>(v));
        if (heap && (lane & 3) == 0) sh.heapw[wave][16 + (lane >> 2)] = v;
        v = __dadd_rn(v, dpp_f64<0x141>(v));
        if (heap && (lane & 7) == 0) sh.heapw[wave][8 + (lane >> 3)] = v;
        v = __dadd_rn(v, dpp_f64<0x140>(v));
        if (heap && (lane & 15) == 0) sh.heapw[wave][4 + (lane >> 4)] = v;
        {
            const int lo = __builtin_amdgcn_ds_swizzle(__double2loint(v), 0x401F);   // lane ^ 16 inside each 32
            const int hi = __builtin_amdgcn_ds_swizzle(__double2hiint(v), 0x401F);
            v = __dadd_rn(v, __hiloint2double(hi, lo));
        }
        if (heap && (lane & 31) == 0) sh.heapw[wave][2 + (lane >> 5)] = v;
        {
            const auto lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(v), (unsigned)__double2loint(v), false, false);
            const auto hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(v), (unsigned)__double2hiint(v), false, false);
            v = __dadd_rn(__hiloint2double((int)hi[0], (int)lo[0]), __hiloint2double((int)hi[1], (int)lo[1]));
        }
        if (lane == 0) {
            sh.wsum[buf][wave] = v;
            if (heap) sh.heapw[wave][1] = v;
        }
        __syncthreads();
        return row16_tree_sum(sh.wsum[buf][lane & 15]);      // the same in every lane
    };

    while (level < P.t.gamma) {
        const float *prow = p + (int64_t)(cur + 1) * P.V;
        const float *qrow = q + (int64_t)(cur + 1) * P.V;
        const int cnt = P.t.b[level];
        const int first = cur < 0 ? 0 : P.t.off[level] + (cur - P.t.off[level - 1]) * cnt;
        // candidate `lane` of this context (in every wavefront): acceptance uniform, q(x) and the residual at x,
        // which is updated in place after every rejection
        double uc = 0.0, qc = 0.0, rc = 0.0;
        int xc = -1;
        if (lane < cnt) {
            int x = tokens[first + lane];
            x = x < 0 ? 0 : (x >= P.V ? P.V - 1 : x);   // ids outside 0..V-1 are clamped, never dereferenced
            xc = x;
            uc = (double)ua[first + lane];
            qc = (double)qrow[x];
            rc = (double)prow[x];
        }
        int rounds = 0, accepted = -1;
        double S = 1.0, Sq = 1.0;                        // both rows are trusted to be normalised in round 0
        auto accept = [&](int c) {
            const double u = __shfl(uc, c, 64), qx = __shfl(qc, c, 64), rx = __shfl(rc, c, 64);
            const double rhs = NOREP ? __dmul_rn(rx, Sq) : rx;
            return __builtin_amdgcn_readfirstlane((int)(__dmul_rn(u, __dmul_rn(qx, S)) < rhs)) != 0;
        };
        if (accept(0)) {
            accepted = first;
        } else {
            // First rejection at this context: from here on the residual is needed.  Both rows in flight at once
            // (one memory latency); the target row goes through the LDS region into r, then the draft row is parked
            // there.  The region is private to the wavefront, so none of this needs a barrier.
            {
                float4 pv[8], qv[8];
                fast_fetch_row(P, qrow, qv);
                fast_fetch_row(P, prow, pv);
                __builtin_amdgcn_sched_barrier(0);
                row_to_regs(pv);
                __builtin_amdgcn_sched_barrier(0);
                fast_park_row(region, qv);
            }
            for (int c = 0;;) {
                // candidate c was rejected: r <- max(r - S q, 0), S <- sum r
                const int xrej = NOREP ? __builtin_amdgcn_readfirstlane(__shfl(xc, c, 64)) : 0;
                const double qrej = NOREP ? __shfl(qc, c, 64) : 0.0;
                if (tid == 0) {
                    sh.s_hist[rounds] = S;
                    if (NOREP) { sh.sq_hist[rounds] = Sq; sh.x_hist[rounds] = xrej; }
                }
                buf ^= 1;
                // two chunks at a time, the next two read from LDS while these are updated
                float4 qv[2][2];
                qv[0][0] = region[fast_slot(lane, 0)];
                qv[0][1] = region[fast_slot(lane, 1)];
#pragma unroll
                for (int j0 = 0; j0 < 8; j0 += 2) {
                    if (j0 + 2 < 8) {
                        qv[(j0 / 2 + 1) & 1][0] = region[fast_slot(lane, j0 + 2)];
                        qv[(j0 / 2 + 1) & 1][1] = region[fast_slot(lane, j0 + 3)];
                    }
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        const float4 q4 = qv[(j0 / 2) & 1][jj];
                        const float qe[4] = {q4.x, q4.y, q4.z, q4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int i = 4 * (j0 + jj) + e;
                            r[i] = pos_part(__fma_rn(-S, (double)qe[e], NOREP ? __dmul_rn(r[i], Sq) : r[i]));
                        }
                    }
                }
                if (NOREP) {
                    // the rejected token leaves the draft row: its owner lane clears its LDS copy, after this round's
                    // update has used it
                    if (tid == (xrej >> 5)) ((float *)&region[fast_slot(lane, (xrej & 31) >> 2)])[xrej & 3] = 0.f;
                }
                {
                    const double d = __fma_rn(-S, qc, NOREP ? __dmul_rn(rc, Sq) : rc);
                    rc = pos_part(d);
                }
                if (NOREP) {
                    Sq = __dsub_rn(Sq, qrej);
                    if (xc == xrej) qc = 0.0;             // also a later duplicate of the rejected token
                }
                rounds += 1;
                S = total(false);
                if (++c == cnt) break;
                if (accept(c)) { accepted = first + c; break; }
            }
        }
        if (accepted < 0) {
            term_p = prow; term_q = qrow;
            if (S > 0.0) { term_rounds = rounds; term_in_regs = true; }
            else { term_rounds = 0; term_in_regs = false; }   // vanished residual: the context's own target row
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
        term_in_regs = false;
    }
    if (tid == 0) {
        for (int l = n_acc; l < P.t.gamma; ++l) path_out[l] = -1;
        P.cand_len[(int64_t)b * P.R + root] = n_acc;
    }
    if (P.n_new > 0) {
        if (!term_in_regs) {                  // the terminal distribution is a target row: bring it into r
            float4 pv[8];
            fast_fetch_row(P, term_p, pv);
            row_to_regs(pv);
        }
        buf ^= 1;
        (void)total(true);                    // wavefront sums and lane-sum heaps of the terminal distribution; one barrier
        for (int k = wave; k < P.n_new; k += NWAVE) {       // wavefronts draw independently from here on
            const int t = fast_sample<NOREP>(sh, P, buf, term_p, term_q, term_rounds, P.us[(int64_t)b * P.n_new + k]);
            if (lane == 0) P.cand_new[((int64_t)b * P.R + root) * P.n_new + k] = t;
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
    if (!mask || mode != MCSD_TARGET_INIT || B < 1 || n_new < 0 || mask->gamma < 1) return 0;
    const size_t R = (size_t)mask->branching_host[0];
    return align256(sizeof(int32_t) * B * R * mask->gamma) + align256(sizeof(int32_t) * B * R) +
           align256(sizeof(int32_t) * B * R * (n_new > 0 ? n_new : 1));
}

namespace {
void launch_walk(const VerifyParams &P, bool norep, dim3 grid, hipStream_t st)
{
    auto kernel = P.V <= FAST_V ? (norep ? verify_walk_fast_kernel<true> : verify_walk_fast_kernel<false>)
                                : (norep ? verify_walk_kernel<true> : verify_walk_kernel<false>);
    mcsd_launch(MCSD_KERNEL_VERIFY_WALK, kernel, grid, dim3(VT), st, P);
}
}  // namespace

extern "C" int mcsd_verify_tree(const mcsd_mask_view_t *mask, mcsd_mode_t mode, int32_t B, int32_t V,
                                const int32_t *tokens, const float *p_target, const float *q_draft,
                                int64_t p_batch_stride, int64_t q_batch_stride, const float *u_accept,
                                const float *u_sample, int32_t n_new, int32_t *out_path, int32_t *out_accept_len,
                                int32_t *out_new_tokens, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return mcsd_verify_tree_sampling(mask, mode, MCSD_WITH_REPLACEMENT, B, V, tokens, p_target, q_draft, p_batch_stride,
                                     q_batch_stride, u_accept, u_sample, n_new, out_path, out_accept_len,
                                     out_new_tokens, workspace, workspace_bytes, hip_stream);
}

extern "C" int mcsd_verify_tree_sampling(const mcsd_mask_view_t *mask, mcsd_mode_t mode, mcsd_sampling_t sampling,
                                         int32_t B, int32_t V, const int32_t *tokens, const float *p_target,
                                         const float *q_draft, int64_t p_batch_stride, int64_t q_batch_stride,
                                         const float *u_accept, const float *u_sample, int32_t n_new,
                                         int32_t *out_path, int32_t *out_accept_len, int32_t *out_new_tokens,
                                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (sampling != MCSD_WITH_REPLACEMENT && sampling != MCSD_WITHOUT_REPLACEMENT) return MCSD_EINVAL;
    const bool norep = sampling == MCSD_WITHOUT_REPLACEMENT;
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
        launch_walk(P, norep, dim3(1, B), st);
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
    launch_walk(P, norep, dim3(P.R, B), st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return MCSD_EHIP;
    hipLaunchKernelGGL(verify_select_kernel, dim3(B), dim3(64), 0, st, P, out_path, out_accept_len, out_new_tokens);
    return mcsd_hip_status(hipGetLastError());
}
