// Tree attention for gfx950 (Sec. 2.2 of arXiv 2409.10644): every node of the candidate tree attends
// to the prefix KV cache and to its own ancestors under the topology-aware mask.
//
// bf16 path.  One workgroup of 4 wavefronts (two workgroups per compute unit) owns one (sequence, head, key split).  The tree's
// queries are cut into blocks of 32 rows; a wavefront keeps one block of Q in registers for the whole sweep.  K/V
// tiles stream from HBM straight into a ring of LDS stages (global_load_lds, 16 bytes per lane, no registers
// in between), several tiles ahead of the one being computed, so every K/V byte leaves HBM once and is used by
// all queries.  The LDS image of a tile is XOR-swizzled at 16-byte granularity, which makes both read patterns
// below bank-conflict free without padding (direct-to-LDS loads can only write 1 KiB contiguous per instruction).
// Scores are computed transposed, S^T = K * Q^T, with v_mfma_f32_32x32x16_bf16: the accumulator then holds,
// per lane, 16 keys of ONE query, so the online-softmax reductions are in-lane plus one half-wave swap,
// and the exponentiated scores are already in the register layout of the B operand of O^T += V^T * P^T.
// V^T operands come from the row-major V tile through the LDS transpose load (ds_read_b64_tr_b16).
// Wavefronts that share a query block split each tile's keys (key groups) and are merged through LDS at the
// end; key splits across workgroups write partial results, which the workgroup of the (sequence, head) that arrives
// last folds at the end of the same kernel (a small second kernel when the splits do not share one die's L2).
// The tree's own keys are extra tiles whose scores are masked with the packed bitmask slice.
//
// fp32 path: split / online-softmax structure on the vector ALU (small reference-precision shapes).
#include <math.h>
#include <stdlib.h>

#include <atomic>
#include <type_traits>

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
    int32_t B, H, n;  // H: workgroup units per sequence (bf16 sweep: kv heads x chunks of query heads; fp32: query heads)
    int32_t Hq, Hkv;  // query heads, key/value heads (Hq = grp * Hkv)
    int32_t grp;      // query heads that share one key/value head
    int32_t hpw;      // query heads one workgroup of the bf16 sweep serves (they share its K/V stream)
    int32_t bph;      // 32-row query blocks per query head in a workgroup (1, 2 or 4); QBP = bph * hpw
    int32_t chunks;   // grp / hpw: workgroup units per key/value head
    int32_t pair_cus; // > 0: compute units; the grid has more workgroups than that and no separate tree workgroup (see the kernel)
    int32_t xcc;      // accelerator dies the hardware deals workgroup ids to round-robin (>= 1)
    int32_t fold;     // 1: the workgroup of a (sequence, unit) that finishes last folds the partial results itself
    int32_t tree_last; // 1 (no separate tree workgroup, no pairing): the last split that has keys takes the tree's keys, else split 0
    unsigned long long *ctr;   // fold == 1: arrival counter of unit u at ctr[u * CTR_STRIDE], zero before and after every launch
    const uint32_t *ws_tag;    // fold == 1: first word of the workspace, WS_TAG once prepared
    int32_t row0;     // first query row: rows row0 .. n-1 are computed (keys are always all n tree nodes)
    int32_t max_prefix;
    int64_t node_stride, head_stride;
    float c;          // softmax_scale * log2(e)
    float k_scale, v_scale;   // fp8 prefix cache: value = stored * scale
    int32_t S;        // key splits of the prefix
    int32_t G;        // workgroups per (b,h): S, plus one for the tree's own keys when the bf16 sweep splits the prefix
    int32_t tps;      // tiles per split (bf16 sweep): split s owns tiles [s*tps, (s+1)*tps) of every sequence
    int32_t SP;       // partial results per (b,h) (== G)
    float *part_o;    // [B*H][SP][n][D]; the bf16 sweep keeps its partial O there as bf16 (see the end of the sweep kernel)
    float *part_m;    // [B*H][SP][n]   reference maximum of the raw scores
    float *part_l;    // [B*H][SP][n]   sum of exp2((s - m) * c)
};

// Workspace of a call with split keys: [tag word, 256 bytes] [arrival counters, 64 KiB] [part_m] [part_l] [part_o].
// mcsd_workspace_init writes the tag and zeroes the counters; every launch leaves them as it found them.
constexpr uint32_t WS_TAG = 0x4d435344u;
constexpr size_t WS_HEADER = 256, WS_CTR_BYTES = 64 * 1024;
// One arrival counter per 128-byte line: atomics on one line are served one after the other (~85 ns each on this
// machine), so counters of different (sequence, unit) pairs that share a line would queue behind each other.
constexpr int CTR_STRIDE = 16;                          // in 8-byte counters
constexpr int FOLD_MAX_PARTIALS = 16;     // the in-kernel fold keeps one weight per partial result in registers

struct AttnPlan {
    int bph, hpw, chunks;  // bf16: query blocks per head, heads per workgroup, units per kv head (see AttnParams)
    int units;             // workgroup units per sequence: kv heads x chunks (bf16), query heads (fp32)
    int QBP;   // query blocks of 32 rows, rounded up to 1, 2 or 4 (bf16 path)
    int T;     // keys per tile
    int S;     // key splits of the prefix
    int G;     // workgroups per (b,h): S, or S + 1 when the bf16 sweep gives the tree's own keys a workgroup of their own
    int NS;    // LDS stages of the bf16 sweep
    int xcc;   // dies the workgroup ids are dealt to (1 when unknown: no renumbering)
    int pair_cus;  // see AttnParams
    int tree_last; // see AttnParams
    long grid_units; // (sequence, unit) slots of the grid: B * units, rounded up to a multiple of the dies where that lets the fold run in the kernel
    int fold;  // 1: folded inside the sweep kernel through the L2 its workgroups share
};

__host__ __device__ inline int tile_keys_bf16(int QBP) { return QBP == 1 ? 128 : 64; }   // == SweepCfg::T

// Compute units and accelerator dies of the current device (asked once per device; concurrent first calls store
// the same values).
void device_shape(int &n_cus, int &n_xcc)
{
    static std::atomic<int> cus_of_device[64];
    n_cus = -1;
    n_xcc = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return;
    n_cus = cus_of_device[dev].load(std::memory_order_relaxed);
    if (n_cus == 0) {
        int v = 0;
        n_cus = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0 ? v : -1;
        cus_of_device[dev].store(n_cus, std::memory_order_relaxed);
    }
    n_xcc = mcsd_xcc_count(dev);
}

AttnPlan make_plan(int dtype, int B, int Hq, int Hkv, int n_rows, int max_prefix, bool f8 = false,
                   const mcsd_attention_tuning_t *tune = nullptr)
{
    AttnPlan pl;
    const int grp = Hq / Hkv;
    if (dtype == MCSD_BF16) {
        const int qb = (n_rows + 31) / 32;
        pl.bph = qb <= 1 ? 1 : (qb == 2 ? 2 : 4);
        // the fp8 ring is sized for 64-key tiles: a single query block of one head runs as two, the second one empty
        if (f8 && pl.bph == 1 && grp % 2 != 0) pl.bph = 2;
        // grouped-query attention: as many query heads of one kv head as fit the workgroup's four query blocks
        // share its K/V stream (so those bytes leave HBM once for all of them)
        pl.hpw = 1;
        for (int c = 4 / pl.bph; c > 1; c >>= 1)
            if (grp % c == 0) { pl.hpw = c; break; }
        pl.QBP = pl.bph * pl.hpw;
        pl.chunks = grp / pl.hpw;
        pl.units = Hkv * pl.chunks;
        pl.T = tile_keys_bf16(pl.QBP);
    } else {
        pl.bph = pl.hpw = 1;
        pl.chunks = grp;
        pl.units = Hq;
        pl.QBP = 1;
        pl.T = 32;
    }
    const long bh = (long)B * pl.units;
    const long tiles_max = (max_prefix + pl.T - 1) / pl.T;
    // Key splits: enough workgroups for two per compute unit, at least four tiles per split (two of the 128-key
    // tiles of a single query block: the same bytes), at most 8 splits (6 with four query blocks, whose partial result
    // is twice the bytes: six splits and the tree's workgroup are what the seven-slot fold takes in one pass): every
    // split costs a partial result of n rows that is written, read back and folded.  Measured: one query block, 1024
    // keys: 14.3 -> 11.3 us per call with four splits instead of two; four query blocks, 1024 keys: 15.2 -> 13.2 us
    // with four instead of three; 2048 keys: 16.9 us with six, 17.8 us with seven.
    long S = (512 + bh - 1) / bh;
    // (the vector-ALU path is slow per tile: split it all the way)
    const long min_tiles = dtype == MCSD_BF16 ? (pl.QBP == 1 ? 2 : 4) : 1;
    if (S > tiles_max / min_tiles) S = tiles_max / min_tiles;
    if (dtype == MCSD_BF16 && S > (pl.QBP == 4 ? 6 : 8)) S = pl.QBP == 4 ? 6 : 8;
    if (S < 1) S = 1;
    if (S > 64) S = 64;
    // One split less when the streaming workgroups alone would have a compute unit each (256) but not together with
    // the tree's own workgroups: otherwise some compute units get two streaming workgroups and finish last
    // (measured on B*H = 32, 2048 keys, wide tree: step 0.80 -> 0.74 ms by giving the tree's workgroups the highest
    // ids instead, 0.69 ms with fewer splits).
    if (dtype == MCSD_BF16 && S > 2 && bh * S <= 256 && bh * (S + 1) > 256) --S;
    if (tune && tune->key_splits >= 1 && tune->key_splits <= 64) S = tune->key_splits;   // the caller's choice
    pl.NS = f8 ? 4 : 2;                                     // LDS stages (bf16: see below)
    pl.S = (int)S;
    // With split keys the tree's own tiles (masked, through registers) would lengthen one split's critical path:
    // they get a workgroup of their own, which costs one more partial result.  Only when all workgroups are
    // resident at once (two per compute unit): the hardware dispatcher does not rebalance long workgroups that
    // start behind short ones.
    pl.G = (dtype == MCSD_BF16 && S > 1 && bh * (S + 1) <= 512) ? (int)S + 1 : (int)S;
    pl.tree_last = 0;
    if (tune && dtype == MCSD_BF16 && S > 1 && tune->tree_keys != 0) {
        pl.G = tune->tree_keys == 1 ? (int)S + 1 : (int)S;
        pl.tree_last = tune->tree_keys == 3;
    }
    int n_cus, n_xcc;
    device_shape(n_cus, n_xcc);
    // Ragged grids larger than the chip are ordered by length inside the kernel (see there)
    pl.pair_cus = 0;
    if (dtype == MCSD_BF16 && pl.G == pl.S && (long)B * pl.S <= 256 && n_cus > 0 && bh * pl.S > n_cus &&
        !(tune && tune->natural_order) && !pl.tree_last)
        pl.pair_cus = n_cus;
    // bf16 tiles: two stages and two workgroups per compute unit.  Four stages (64-key tiles only: a 128-key tile is
    // 64 KB) exist for measurement: on launches that have a compute unit per workgroup anyway three tiles in flight
    // instead of one were expected to help and do not (cfg2: 7.5 against 6.2 us until the partial results are stored;
    // a bare ring of direct-to-LDS loads needs ~5 us for 128 KB per workgroup on 128 compute units at any depth: a
    // cold burst of this size is bound by the memory system's ramp-up, not by the bytes a compute unit has in flight).
    if (tune && !f8 && tune->stages == 4 && dtype == MCSD_BF16 && pl.QBP != 1) pl.NS = 4;
    pl.xcc = n_xcc > 0 ? n_xcc : 8;        // unknown: the renumbering is then only a guess that may help locality
    // The fold runs inside the sweep when all workgroups of one (sequence, unit) share a die's L2: the dealing of
    // workgroup ids to dies is known, and the kernel's numbering keeps a unit's workgroups at one id modulo dies.
    // A number of (sequence, unit) pairs that is no multiple of the dies is rounded up: the workgroups of the slots
    // beyond the last pair leave at once, and every real pair's workgroups still share a die.
    pl.grid_units = bh;
    bool same_die = n_xcc == 1;
    if (n_xcc > 1 && pl.pair_cus == 0) {
        same_die = true;
        if (dtype == MCSD_BF16 && pl.S > 1) pl.grid_units = (bh + n_xcc - 1) / n_xcc * n_xcc;
        else same_die = bh % n_xcc == 0;
    }
    if (pl.pair_cus > 0) same_die = n_xcc == 1 || (n_xcc > 1 && pl.units % n_xcc == 0 && pl.pair_cus % n_xcc == 0);
    pl.fold = dtype == MCSD_BF16 && pl.S > 1 && same_die && pl.G <= FOLD_MAX_PARTIALS &&
              (size_t)bh * CTR_STRIDE * sizeof(unsigned long long) <= WS_CTR_BYTES && !(tune && tune->fold == 1);
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
// 8-bit variant.  Within 16 lanes, lane i receives byte i%8 of the 8-byte words addressed by lanes 2e + i/8,
// e = 0..7 (checked on the hardware): lanes 2e and 2e+1 point at the two halves of a 16-byte piece of the row for
// slot e, and lane i ends up with column i of that piece from all eight rows.
typedef __attribute__((ext_vector_type(2))) int i32x2_t;
__device__ inline i32x2_t lds_read_tr8(const unsigned char *p)
{
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((i32x2_t __attribute__((address_space(3))) *)(p));
}

// 16 bytes per lane from global memory straight into LDS: lane l reads gbase + voff and lands at lds_base + 16*l
// (gbase and lds_base uniform).  Written as assembly on purpose: the compiler knows nothing about where such a
// load writes in LDS unless alias information happens to survive inlining, and otherwise makes the next LDS
// read wait for it (vmcnt(0)), which serialises the stream with the compute.  Here it is just an opaque
// instruction; the kernel waits for it itself (MCSD_WAIT_VMCNT + barrier) before anyone reads the stage.
// An untracked load can only make compiler-placed vmcnt waits longer, never shorter (loads retire in order).
// M0 carries the LDS address; nothing else in these kernels uses M0 (the toolchain rejects it as a clobber).
// NT marks the load non-temporal, for prefix K/V that exactly one workgroup reads: keeping a read-once stream out
// of the caches' retained set is worth 5-12 % of the sweep (measured; the coherence-scope bits make no
// difference).  Where several workgroups share a stream (grouped-query heads cut into several query chunks) the
// second reader needs the lines in L2 and the plain load is the faster one.
template <bool NT>
__device__ inline void load_to_lds16(const void *gbase, uint32_t voff, void *lds_base)
{
    const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)lds_base;
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                     :
                     : "s"(lds_addr), "v"(voff), "s"(gbase)
                     : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(lds_addr), "v"(voff), "s"(gbase)
                     : "memory");
}

// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt left at their maxima)
#define MCSD_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))

// ---------------------------------------------------------------------------------------------------
// bf16 / MFMA kernel
// ---------------------------------------------------------------------------------------------------
// F8: the prefix K/V cache holds fp8 (e4m3) elements; a ring stage is then a raw fp8 tile (half the bytes, twice
// the stages) that the operand reads convert to bf16 on their way into the matrix cores.
template <int D, int QBP, int NS_, bool F8 = false>
struct SweepCfg {
    static constexpr int WAVES = 4;
    static constexpr int KG = 4 / QBP;                 // key groups: wavefronts that share a query block and split the keys
    static constexpr int KPW = QBP == 4 ? 2 : 1;       // 32-key blocks per wavefront per tile
    static constexpr int THREADS = WAVES * 64;
    static constexpr int T = 32 * KG * KPW;            // keys per tile (64, 64, 128 for QBP = 4, 2, 1)
    static constexpr int RB = D * 2;                   // bytes per bf16 K/V row (tree tiles, register path)
    static constexpr int RBP = F8 ? D : D * 2;         // bytes per prefix K/V row (ring stages)
    static constexpr int CPR = RBP / 16;               // 16-byte chunks per prefix row
    static constexpr int RPI = 64 / CPR;               // rows covered by one direct-to-LDS instruction (1 KiB)
    static constexpr int TILE_K = T * RBP;             // bytes of the K half of a ring stage; V follows
    static constexpr int TILE = 2 * TILE_K;
    static constexpr int BTILE_K = T * RB;             // the same for a bf16 tile written through registers
    static constexpr int BCPR = RB / 16;
    static constexpr int NI = T / RPI / WAVES;         // direct-to-LDS instructions per wavefront for K (same for V)
    static constexpr int DPT = 2 * NI;                 // ... per tile
    static constexpr int NS = NS_;                     // LDS stages: one being computed, NS - 1 being filled
    static constexpr int KS = D / 16;                  // k-steps of S^T = K Q^T
    static constexpr int CB = D / 32;                  // 32-row blocks of O^T
    static constexpr int CPT = T * BCPR / THREADS;     // 16-byte bf16 chunks per thread for K (same for V), register path
    static constexpr int MSLOT = 32 * D * 4 + 256;     // LDS bytes to hand one query block's (O, m, l) to another wavefront
    static constexpr int RING = NS * TILE > 2 * BTILE_K ? NS * TILE : 2 * BTILE_K;
    static constexpr int LDS_BYTES = RING > (KG - 1) * QBP * MSLOT ? RING : (KG - 1) * QBP * MSLOT;
    static_assert(NI >= 1 && CPT >= 1 && (NS - 2) * DPT < 64 && LDS_BYTES <= 160 * 1024 - 64, "tile does not map onto the workgroup");
    static_assert(!F8 || D == 128, "fp8 tiles are laid out for 128-byte rows");
};

// XOR swizzle of the 16-byte chunk index inside row r.  With it, 16 consecutive rows read at the same logical
// chunk (K operand loads) and 4 consecutive rows read at 4 consecutive chunks (V transpose loads) both hit 16
// different 16-byte bank groups.
template <int D>
__device__ inline int swz(int r)
{
    return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
}

// The same for fp8 tiles (128-byte rows, 8 chunks): bijective on row bits 1-3, so 16 consecutive rows read at one
// chunk with 16-byte loads (K operands) hit 16 different bank groups together with the row's parity, and the rows
// {0..3, 8..11} + 4g read at two neighbouring chunks by the transpose loads (V operands) do as well.
__device__ inline int swz8(int r)
{
    return ((r >> 2) & 1) | (((r >> 1) & 1) << 1) | (((r >> 3) & 1) << 2);
}

// 8 fp8 (e4m3, OCP) values in two dwords -> 8 bf16, exact.
__device__ inline bf16x8_t fp8x8_to_bf16(unsigned lo, unsigned hi)
{
    typedef __attribute__((ext_vector_type(4))) unsigned u4;
    u4 w;
    w[0] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false));
    w[1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true));
    w[2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false));
    w[3] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true));
    return __builtin_bit_cast(bf16x8_t, w);
}

// Log2-domain slack of the running reference maximum: the accumulators are rescaled only when a block's maximum
// exceeds the reference by more than this, so exponentiated scores stay below 2^RESCALE_SLACK.  The result is
// exact: numerator and denominator always share the same reference.
constexpr float RESCALE_SLACK = 6.f;

// Per-lane LDS offsets of the two operand read patterns inside a stage (computed once).
struct LaneAddr {
    int k;   // K operand: row (kg*32 + ln), chunk g ^ swz; XOR ks*32 selects the k-step
    int v;   // V^T operand: row (kg*32 + 4g + j/4), chunk/sub of this lane; XOR ct*16 and an immediate select the rest
    int k8;  // the same inside an fp8 tile: row (kg*32 + ln), chunk g ^ swz8; XOR kp*32 selects the pair of k-steps
    int v8;  // fp8 V^T operand (8-bit transpose load): row of this lane's key slot, chunk (ln/16) ^ swz8, half ln & 1
};

// State of one 32-query block held by a wavefront.
template <int D>
struct QBlock {
    bf16x8_t q[D / 16];        // Q as B operands: lane holds Q[row][ks*16 + 8g .. +8]
    f32x16_t o[D / 32];        // O^T accumulators
    float m_ref, l_run;        // reference maximum (raw score units), per-lane part of the denominator
};

// Exponentials of one pair of scores: p = exp2(s*c - mc), added to the denominator and packed as bf16 into P^T
// (kept as dwords: pb[r/8] is one B operand).  The empty asm keeps the pair where it is written, between two MFMAs.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4_t;
// SCALED: the packed values carry the factor vs (the scale of an fp8 V tile); the denominator does not.
template <bool SCALED = false>
__device__ inline void softmax_exp2(const f32x16_t &sacc, int r, float c, float mc, float &psum, u32x4_t *pb, float vs = 1.f)
{
    const float p0 = fast_exp2(fmaf(sacc[r], c, -mc)), p1 = fast_exp2(fmaf(sacc[r + 1], c, -mc));
    psum += p0 + p1;
    bf16x2_t pk;
    pk[0] = (__bf16)(SCALED ? p0 * vs : p0);
    pk[1] = (__bf16)(SCALED ? p1 * vs : p1);
    unsigned u = __builtin_bit_cast(unsigned, pk);
    asm volatile("" : "+v"(u));
    pb[r / 8][(r % 8) / 2] = u;
}

// One tile: the wavefront's KPW blocks of 32 keys against its 32 queries.  With two blocks the instruction stream
// is laid out so that the matrix pipe and the vector ALU overlap inside the wavefront:
//     QK_0, QK_1 | block maxima, rare rescale | exp(0) | PV_0 with exp(1) in its shadow | PV_1
// Operand reads are issued ahead of their use.  MODE 0: all keys visible; otherwise bit k of bits[u] says whether
// key k of block u is visible to this lane's query.
// F8K: the kernel serves an fp8 prefix cache: the reference maximum is kept in log2 units (tiles of different
// scale share it) and P carries the V scale `vs` of the tile.  F8T: this stage is a raw fp8 tile.
template <int D, int QBP, int NS, int MODE, bool F8K = false, bool F8T = false>
__device__ inline void attn_tile(const unsigned char *stage, const LaneAddr la, QBlock<D> &qs, float c, int g,
                                 const uint32_t *bits, float vs = 1.f)
{
    using C = SweepCfg<D, QBP, NS, F8K>;
    constexpr int U = C::KPW;
    constexpr int ROWB = F8T ? C::RBP : C::RB;             // bytes per row of this stage
    constexpr int VOFF = F8T ? C::TILE_K : C::BTILE_K;     // where its V half starts
    // K rows of the blocks (A operands of S^T = K Q^T); block u sits 32*u rows below the lane's base row
    bf16x8_t kf[U][C::KS];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (F8T) {
            // one 16-byte read = the lane's share of two k-steps (see the column order in the kernel)
#pragma unroll
            for (int kp = 0; kp < C::KS / 2; ++kp) {
                const uint4 raw = *(const uint4 *)(stage + (la.k8 ^ (kp * 32)) + u * 32 * ROWB);
                kf[u][2 * kp] = fp8x8_to_bf16(raw.x, raw.y);
                kf[u][2 * kp + 1] = fp8x8_to_bf16(raw.z, raw.w);
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < C::KS; ++ks)
                kf[u][ks] = *(const bf16x8_t *)(stage + (la.k ^ ((F8K ? 4 * (ks >> 1) + (ks & 1) : 2 * ks) * 16)) + u * 32 * ROWB);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // S^T[key][query] : lane (query = ln, half g) gets keys 8*(r/4) + 4*g + r%4, r = 0..15
    f32x16_t sacc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        // The wavefront's runs of matrix instructions are issued at raised priority: the other wavefront of the SIMD,
        // busy with its soft-max, then does not delay them (measured: 2-3 % on the long sweeps; the opposite
        // assignment costs as much).
        if (u == 0) __builtin_amdgcn_s_setprio(2);
        sacc[u] = (f32x16_t){0};
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) sacc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[u][ks], qs.q[ks], sacc[u], 0, 0, 0);
    }
    __builtin_amdgcn_s_setprio(0);
    // V^T fragments via the LDS transpose load, issued ahead of their use: block 0's during the softmax, block 1's
    // before the first PV MFMA.  The reads of one k-step pair (ks2, e4) sit 16*ks2 + 8*e4 rows below the lane's
    // base row; the chunk select is cb*4 ^ e4*2.
    const unsigned char *vst = stage + VOFF;
    bf16x8_t vf[U][2][C::CB];
    auto read_v = [&](int u) {
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
            for (int cb = 0; cb < C::CB; ++cb) {
                if constexpr (F8T) {
                    // one 8-bit transpose load: the 8 key slots of this lane's column (slot e = key 8(e/4) + 4g + e%4)
                    const i32x2_t t = lds_read_tr8(vst + (la.v8 ^ ((cb * 2) * 16)) + (u * 32 + ks2 * 16) * ROWB);
                    vf[u][ks2][cb] = fp8x8_to_bf16((unsigned)t[0], (unsigned)t[1]);
                } else {
                    const s16x4_t lo = lds_read_tr16(vst + (la.v ^ (((cb * 4) ^ 0) * 16)) + (u * 32 + ks2 * 16) * ROWB);
                    const s16x4_t hi = lds_read_tr16(vst + (la.v ^ (((cb * 4) ^ 2) * 16)) + (u * 32 + ks2 * 16 + 8) * ROWB);
                    vf[u][ks2][cb] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
            }
    };
    read_v(0);
    // masking, maximum over the tile's blocks, rare rescale of the accumulators
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (MODE != 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = 8 * (r / 4) + 4 * g + (r % 4);
                if (!((bits[u] >> key) & 1u)) sacc[u][r] = -INFINITY;
            }
        }
        mx = fmaxf(fmaxf(mx, sacc[u][0]), sacc[u][1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, sacc[u][r]), sacc[u][r + 1]);
    }
    mx = half_swap_max(mx);
    if (F8K) mx *= c;                                       // log2 units from here on (c > 0)
    const float cm = F8K ? 1.f : c;                         // what turns a difference of reference maxima into log2 units
    // rescale only when the maximum outgrows the reference by more than the slack (first tile: -inf)
    const bool grow = (mx - qs.m_ref) * cm > RESCALE_SLACK;
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        const float m_new = grow ? mx : qs.m_ref;
        const float alpha = m_new == qs.m_ref ? 1.f : fast_exp2((qs.m_ref - m_new) * cm);   // -inf reference: exp2(-inf) = 0
        qs.m_ref = m_new;
        qs.l_run *= alpha;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) qs.o[cb][r] *= alpha;
    }
    const float mc = (qs.m_ref == -INFINITY ? 0.f : qs.m_ref) * cm;
    u32x4_t pb[U][2];
    float psum = 0.f;
    // With one block per wavefront the exponentials of its second half of keys (registers 8..15, the operand of the
    // second k-step pair) run in the shadow of the first half's PV MFMAs.
#pragma unroll
    for (int r = 0; r < (U == 1 ? 8 : 16); r += 2) softmax_exp2<F8K>(sacc[0], r, c, mc, psum, pb[0], vs);
    __builtin_amdgcn_sched_barrier(0);
    // O^T[c][query] += V^T[c][key] * P^T[key][query]
    if (U == 1) {
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb) {
            qs.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[0][0][cb], __builtin_bit_cast(bf16x8_t, pb[0][0]), qs.o[cb], 0, 0, 0);
            if (C::CB == 4) softmax_exp2<F8K>(sacc[0], 8 + 2 * cb, c, mc, psum, pb[0], vs);
            else { softmax_exp2<F8K>(sacc[0], 8 + 4 * cb, c, mc, psum, pb[0], vs); softmax_exp2<F8K>(sacc[0], 10 + 4 * cb, c, mc, psum, pb[0], vs); }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
            qs.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[0][1][cb], __builtin_bit_cast(bf16x8_t, pb[0][1]), qs.o[cb], 0, 0, 0);
        qs.l_run += psum;
        return;
    }
    if (U == 2) {
        read_v(1);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(2);
#pragma unroll
        for (int i = 0; i < 2 * C::CB; ++i) {
            const int ks2 = i / C::CB, cb = i % C::CB;
            qs.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[0][ks2][cb], __builtin_bit_cast(bf16x8_t, pb[0][ks2]), qs.o[cb], 0, 0, 0);
            if (C::CB == 4) softmax_exp2<F8K>(sacc[U - 1], 2 * i, c, mc, psum, pb[U - 1], vs);
            else { softmax_exp2<F8K>(sacc[U - 1], 4 * i, c, mc, psum, pb[U - 1], vs); softmax_exp2<F8K>(sacc[U - 1], 4 * i + 2, c, mc, psum, pb[U - 1], vs); }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
            qs.o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[U - 1][ks2][cb], __builtin_bit_cast(bf16x8_t, pb[U - 1][ks2]), qs.o[cb], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    qs.l_run += psum;
}

// The fold of the partial results of one query block by one wavefront of the workgroup that arrived last (see the
// end of the sweep kernel): rows = the wavefront's 32 queries (lane ln, half g), columns = the 32-column blocks
// kg, kg + KG, ..  ro / rm / rl describe the unit's partial O (fragment order), maxima and denominators and end after
// the last partial result in use: a load beyond it returns zero without touching memory, so nothing below branches
// on the number of partial results and all loads of a round are in flight together.
// A round: NSLOT partial results x the lane's two 16-byte chunks (jp = 0, 1: eight bf16 each = its float4 positions
// j = 2 jp, 2 jp + 1) of a column block.  The rounds of a column block are (first group), [(second group)]: an
// accumulator lives across the groups and its result is stored after every round (with two groups the first store
// of a position is overwritten by the complete one: same lane, same address, program order).  The loads of the next
// round are issued before this one is added up (two register buffers); a round beyond the last loads from beyond the
// end, i.e. nothing, and is not added up.
// Partial results are added in slot order whoever arrived last, so the result is reproducible.
// Nothing here may spill: a workgroup's scratch memory is cold at this point, every first touch a trip to HBM (a
// variant that spilled its weights took 9.7 us for five partial results, against 3).
template <int D, int QBP, int KG, int NSLOT>
__device__ __attribute__((always_inline)) inline void fold_partials(const __amdgpu_buffer_rsrc_t ro, const __amdgpu_buffer_rsrc_t rm,
                                     const __amdgpu_buffer_rsrc_t rl, const int n_active, const int kg, const int g,
                                     const int ln, const float cm, __bf16 *orow, f32x4_t *wlds)
{
    constexpr int CB = D / 32;
    constexpr int NW = NSLOT == 8 ? FOLD_MAX_PARTIALS : NSLOT;      // partial results this variant can hold
    constexpr int SLOT_BYTES = QBP * 32 * D * 2;
    float wgt[NW], lw[NW];
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        wgt[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rm, (i * QBP * 32 + ln) * 4, 0, 1));
        lw[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rl, (i * QBP * 32 + ln) * 4, 0, 1));
    }
    const int ngrp = NSLOT == 8 && n_active > NSLOT ? 2 : 1;
    const int rounds = ((CB - kg + KG - 1) / KG) * ngrp;
    typedef u32x4_t Round[NSLOT][2];
    auto issue = [&](Round &buf, int r) {
        const int grp = r % ngrp, cb = kg + (r / ngrp) * KG;
        int off = ((cb * 4 + g) * 32 + ln) * 16 + grp * NSLOT * SLOT_BYTES;
        if (r >= rounds) off = 0x40000000;                          // (uniform select) beyond every workspace
#pragma unroll
        for (int i = 0; i < NSLOT; ++i)
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) buf[i][jp] = __builtin_amdgcn_raw_buffer_load_b128(ro, off + jp * 1024 + i * SLOT_BYTES, 0, 1);
    };
    Round bufA, bufB;
    issue(bufA, 0);
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < NW; ++i) M = fmaxf(M, i < n_active ? wgt[i] : -INFINITY);
    float den = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        // 0 for a split that saw no visible key, and beyond the partial results in use
        wgt[i] = i < n_active ? fast_exp2((wgt[i] - M) * cm) : 0.f;
        den = fmaf(wgt[i], lw[i], den);
    }
    const float inv = 1.f / den;
    // Two groups: a round picks its group at run time, and registers cannot be indexed at run time, so the weights
    // go through LDS (the ring is free by now), written and read back by the same lane.
    if constexpr (NSLOT == 8) {
#pragma unroll
        for (int q4 = 0; q4 < NW / 4; ++q4)
            wlds[q4 * 256] = (f32x4_t){wgt[4 * q4], wgt[4 * q4 + 1], wgt[4 * q4 + 2], wgt[4 * q4 + 3]};
    }
    f32x4_t acc[4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    auto add_up = [&](Round &buf, int r) {
        const int grp = r % ngrp, cb = kg + (r / ngrp) * KG;
        float w[NSLOT];
        if constexpr (NSLOT == 8) {
            const f32x4_t wa = wlds[(2 * grp) * 256], wb = wlds[(2 * grp + 1) * 256];
#pragma unroll
            for (int i = 0; i < 4; ++i) { w[i] = wa[i]; w[4 + i] = wb[i]; }
        } else {
#pragma unroll
            for (int i = 0; i < NSLOT; ++i) w[i] = wgt[i];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {                               // the lane's float4 position j of this column block
            if (grp == 0) acc[j] = (f32x4_t){0.f, 0.f, 0.f, 0.f};   // a new position starts from zero (a select)
#pragma unroll
            for (int i = 0; i < NSLOT; ++i) {                       // slot order
                const unsigned d0 = buf[i][j >> 1][2 * (j & 1)], d1 = buf[i][j >> 1][2 * (j & 1) + 1];   // four bf16: exact as fp32 bit patterns
                const u32x4_t bits = {d0 << 16, d0 & 0xffff0000u, d1 << 16, d1 & 0xffff0000u};
                acc[j] += w[i] * __builtin_bit_cast(f32x4_t, bits);
            }
            bf16x4_t v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (__bf16)(acc[j][e] * inv);
            *(bf16x4_t *)(orow + cb * 32 + 8 * j + 4 * g) = v;
        }
    };
#pragma unroll 1
    for (int r = 0; r < rounds; r += 2) {
        issue(bufB, r + 1);
        __builtin_amdgcn_sched_barrier(0);
        add_up(bufA, r);
        __builtin_amdgcn_sched_barrier(0);
        issue(bufA, r + 2);
        __builtin_amdgcn_sched_barrier(0);
        if (r + 1 < rounds) add_up(bufB, r + 1);                    // (uniform)
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int D, int QBP, int NS, bool F8 = false>
__global__ __launch_bounds__((SweepCfg<D, QBP, NS, F8>::THREADS)) __attribute__((amdgpu_waves_per_eu(2, 2)))
void tree_attn_bf16_kernel(const AttnParams p)
{
    using C = SweepCfg<D, QBP, NS, F8>;
    __shared__ __attribute__((aligned(1024))) unsigned char ring[C::LDS_BYTES];

    // Workgroup ids are dealt round-robin to the accelerator dies (p.xcc of them, each with its own L2): renumber so
    // that the key splits of one (sequence, head), which read the same Q, tree K/V and mask rows, write neighbouring
    // partial results and fold them through that L2, share one die.
    const int total = gridDim.x;
    int wg = blockIdx.x;
    if (p.G > 1 && p.pair_cus == 0 && p.xcc > 1 && total % p.xcc == 0) wg = (wg % p.xcc) * (total / p.xcc) + wg / p.xcc;
    int s = wg % p.G;
    int bhi = wg / p.G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // the same in all lanes: keep it in a scalar register
    if (p.pair_cus > 0) {
        // More workgroups than compute units.  Up to two per compute unit they are all resident at once, and on this
        // machine workgroups i and i + #CUs of such a grid land on the same compute unit (measured; nothing but
        // speed depends on it): that pair gets a long and a short piece of work, so that every compute unit has
        // about the same number of keys to stream however ragged the batch is.  With more than two per compute unit
        // the hardware hands out workgroups in id order as slots free up: longest first.  The pieces are the
        // (sequence, key split) classes, p.H equal items each, ranked by their number of tiles here (B * S <= 256).
        __shared__ int32_t s_work[256], s_cls_at[256];
        const int n_cls = p.B * p.S;
        if (tid < n_cls) {
            const int Lt = p.lens[tid / p.S], sp = tid % p.S;
            const int Lc = Lt < 0 ? 0 : (Lt > p.max_prefix ? p.max_prefix : Lt);
            const int tl = (Lc + C::T - 1) / C::T - sp * p.tps;
            s_work[tid] = (tl < 0 ? 0 : (tl > p.tps ? p.tps : tl)) + (sp == 0 ? (p.n + C::T - 1) / C::T : 0);
        }
        __syncthreads();
        if (tid < n_cls) {
            int rank = 0;
            for (int o = 0; o < n_cls; ++o) rank += (s_work[o] > s_work[tid]) || (s_work[o] == s_work[tid] && o < tid);
            s_cls_at[rank] = tid;
        }
        __syncthreads();
        // rank i with rank total-1-i, in groups of p.xcc ids so that a rank keeps its id modulo the number of dies
        // (every key split of a (sequence, unit) then runs on the die of unit % dies)
        int r = wg;                                                              // longest first
        if (total <= 2 * p.pair_cus && wg >= p.pair_cus) {
            const int w2 = wg - p.pair_cus, cnt = total - p.pair_cus;
            r = (cnt % p.xcc == 0) ? p.pair_cus + (cnt / p.xcc - 1 - w2 / p.xcc) * p.xcc + w2 % p.xcc
                                   : total + p.pair_cus - 1 - wg;
        }
        const int cls = s_cls_at[r / p.H];
        s = cls % p.S;
        bhi = (cls / p.S) * p.H + r % p.H;
    }
    if (bhi >= p.B * p.H) return;                            // a slot of a grid rounded up to whole dies
    const int h = bhi % p.H, b = bhi / p.H;

    const int g = lane >> 5, ln = lane & 31;
    const int qb = wave % QBP, kg = wave / QBP;

    int L = p.lens[b];
    L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
    const uint32_t ws_tag = p.fold ? p.ws_tag[0] : WS_TAG;  // (read early: needed only at the very end)
    const int tiles_b = (L + C::T - 1) / C::T;
    const int tps = p.tps;                                  // fixed per call: short sequences use fewer splits
    const bool sep = p.G > p.S;                             // the tree's own keys have a workgroup of their own
    const int np = (tiles_b + tps - 1) / tps;               // prefix splits that have keys for this sequence (<= S)
    const bool tree_wg = sep ? s == p.S : s == (p.tree_last ? max(np, 1) - 1 : 0);
    const int t0 = (sep && tree_wg) ? tiles_b : min(s * tps, tiles_b), t1 = min(t0 + tps, tiles_b);
    const int n_tree_tiles = tree_wg ? (p.n + C::T - 1) / C::T : 0;
    const int n_pre = t1 - t0;
    if (n_pre + n_tree_tiles == 0) return;                  // this split has no keys
    const int n_active = sep ? np + 1 : max(1, np);         // partial results of this sequence: slots 0 .. n_active-1
    const int slot_id = (sep && tree_wg) ? np : s;
    // leading tiles of this split that are full (only the sequence's last tile can be ragged)
    const int n_hot = (n_pre > 0 && t1 * C::T > L) ? n_pre - 1 : n_pre;

    const int64_t bh = (int64_t)b * p.H + h;                 // workgroup unit: indexes the partial results
    const int kvh = h / p.chunks;                              // key/value head of this unit
    const int hq = kvh * p.grp + (h % p.chunks) * p.hpw + qb / p.bph;   // query head of this wavefront's block
    const int64_t bh_kv = (int64_t)b * p.Hkv + kvh, bh_q = (int64_t)b * p.Hq + hq;
    const __bf16 *q = (const __bf16 *)p.q + bh_q * p.node_stride * D;
    const __bf16 *kt = (const __bf16 *)p.kt + bh_kv * p.node_stride * D;
    const __bf16 *vt = (const __bf16 *)p.vt + bh_kv * p.node_stride * D;
    const int64_t pre0 = p.seq_base[b] + (int64_t)kvh * p.head_stride;     // in elements: 2 bytes each, 1 when fp8
    const unsigned char *kp = (const unsigned char *)p.kp + pre0 * (F8 ? 1 : 2);
    const unsigned char *vp = (const unsigned char *)p.vp + pre0 * (F8 ? 1 : 2);
    // softmax scale of a prefix tile and the factor its V values carry; the tree's own tiles use p.c and 1
    const float c_pre = F8 ? p.c * p.k_scale : p.c, vs_pre = F8 ? p.v_scale : 1.f;

    // query block of this wavefront; mask row of this lane's query (zero for padded rows)
    QBlock<D> qs;
    const int qrow = p.row0 + (qb % p.bph) * 32 + ln;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        uint4 v = make_uint4(0, 0, 0, 0);
        // Columns of k-step ks in lane half g: 16 ks + 8 g .. +7.  With an fp8 prefix cache the halves trade places
        // with the k-step's parity, 32 (ks/2) + 16 g + 8 (ks%2) .. +7, so that a lane's columns of two consecutive
        // k-steps are 16 consecutive bytes of an fp8 row (one conflict-free 16-byte LDS read); the contraction is
        // over all columns either way.
        const int col = F8 ? (ks >> 1) * 32 + g * 16 + (ks & 1) * 8 : ks * 16 + g * 8;
        if (qrow < p.n) v = *(const uint4 *)(q + (int64_t)qrow * D + col);
        qs.q[ks] = __builtin_bit_cast(bf16x8_t, v);
    }
    uint64_t mrow[2] = {0, 0};
    if (qrow < p.n) {
        mrow[0] = p.mask_bits[(int64_t)qrow * p.mask_words];
        if (p.mask_words > 1) mrow[1] = p.mask_bits[(int64_t)qrow * p.mask_words + 1];
    }
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb) qs.o[cb] = (f32x16_t){0};
    qs.m_ref = -INFINITY;
    qs.l_run = 0.f;

    // operand read offsets of this lane inside a stage; its first key block starts at row kg * KPW * 32
    LaneAddr la;
    {
        const int krow = kg * C::KPW * 32 + ln;
        la.k = krow * C::RB + (((F8 ? 2 * g : g) ^ swz<D>(krow)) * 16);     // bf16 chunk of (k-step 0, half g)
        const int j = ln & 15, grp = ln >> 4, jr = j >> 2;
        const int vrow = kg * C::KPW * 32 + 4 * g + jr;               // + 32*u + 16*ks2 + 8*e4 by immediate
        const int lchunk = grp * 2 + ((j & 3) >> 1);                   // + 4*cb
        // swz(vrow + 32*u + 16*ks2 + 8*e4) = swz(vrow) ^ (e4 << 1): the e4 part is folded into the compile-time XOR
        la.v = vrow * C::RB + ((lchunk ^ swz<D>(vrow)) * 16) + (j & 1) * 8;
        la.k8 = la.v8 = 0;
        if constexpr (F8) {
            la.k8 = krow * C::RBP + ((g ^ swz8(krow)) * 16);
            const int e = j >> 1;                                        // key slot this lane addresses
            const int row8 = kg * C::KPW * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
            la.v8 = row8 * C::RBP + ((grp ^ swz8(row8)) * 16) + (j & 1) * 8;
        }
    }
    uint32_t all_keys[C::KPW];
#pragma unroll
    for (int u = 0; u < C::KPW; ++u) all_keys[u] = 0xffffffffu;

    // ---- full prefix tiles: HBM -> LDS directly, one tile ahead of the compute ----
    if (n_hot > 0) {
        // lane's source offset inside a tile for instruction i: row G*RPI + lane/CPR, logical chunk (lane%CPR)^swz(row)
        uint32_t goff[C::NI];
#pragma unroll
        for (int i = 0; i < C::NI; ++i) {
            const int G = i * C::WAVES + wave;
            const int r = G * C::RPI + lane / C::CPR;
            goff[i] = (uint32_t)(r * C::RBP + (((lane % C::CPR) ^ (F8 ? swz8(r) : swz<D>(r))) * 16));
        }
        const unsigned char *ksrc = kp + (int64_t)t0 * C::TILE_K;
        const unsigned char *vsrc = vp + (int64_t)t0 * C::TILE_K;
        // Stage numbers are compile-time constants so that the compiler can tell the stage being filled from
        // the stage being read (otherwise it makes every LDS read wait for the loads just issued).
        // Every workgroup walks its full tiles in a rotated order (soft-max does not care): workgroups that start
        // together would otherwise sweep their equally aligned K/V streams in lock-step and crowd the same
        // memory channels.  `nxt` is the tile the next issue fetches.
        int nxt = (int)(((unsigned)wg * 37u) % (unsigned)n_hot);
        // load number i (0 .. DPT-1) of tile `nxt` into a stage: even i fetch K row groups, odd i the same of V
        // (uniform tile base + 32-bit lane offset: the load takes its base from scalar registers)
        const unsigned char *kbase = ksrc + (int64_t)nxt * C::TILE_K, *vbase = vsrc + (int64_t)nxt * C::TILE_K;
        auto issue_load = [&](int i, auto stage, auto read_once) {
            unsigned char *dst = ring + decltype(stage)::value * C::TILE + wave * 1024;
            static_assert(decltype(stage)::value < NS, "stage out of range");
            load_to_lds16<decltype(read_once)::value>((i & 1) ? vbase : kbase, goff[i >> 1],
                                                      dst + (i & 1) * C::TILE_K + (i >> 1) * C::WAVES * 1024);
        };
        auto advance = [&]() {
            nxt = nxt + 1 == n_hot ? 0 : nxt + 1;
            kbase = ksrc + (int64_t)nxt * C::TILE_K;
            vbase = vsrc + (int64_t)nxt * C::TILE_K;
        };
        const bool read_once = p.chunks == 1;               // no other workgroup streams these keys (uniform)
        auto issue_tile = [&](auto stage) {
            if (read_once) {
#pragma unroll
                for (int i = 0; i < C::DPT; ++i) issue_load(i, stage, std::true_type());
            } else {
#pragma unroll
                for (int i = 0; i < C::DPT; ++i) issue_load(i, stage, std::false_type());
            }
            advance();
        };
        if constexpr (NS == 2) {
        auto step = [&](int it, auto stage, auto prefetching) {
            constexpr int ST = decltype(stage)::value;
            constexpr bool PF = decltype(prefetching)::value;    // a later tile is fetched into the stage just freed
            // this wavefront's part of tile `it` has landed once at most NS-2 later tiles are outstanding
            MCSD_WAIT_VMCNT(0);
            __builtin_amdgcn_s_barrier();                     // ... and everyone's; the stage of tile it-1 is free again
            // (spreading these loads over the tile's MFMAs instead of issuing them in one burst was measured: no gain)
            if (PF) issue_tile(std::integral_constant<int, (ST + NS - 1) % NS>());
            attn_tile<D, QBP, NS, 0, false, false>(ring + ST * C::TILE, la, qs, p.c, g, all_keys);
        };
        static_assert(!F8, "fp8 tiles use the ring below");
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        issue_tile(S0());
        // all steps but the last fetch the next tile while they compute
        int it = 0;
        for (; it + 2 < n_hot; it += 2) {
            step(it, S0(), std::true_type());
            step(it + 1, S1(), std::true_type());
        }
        if (it + 1 < n_hot) {
            step(it, S0(), std::true_type());
            step(it + 1, S1(), std::false_type());
        } else {
            step(it, S0(), std::false_type());
        }
        } else {
        // A ring of NS stages keeps NS-1 tiles in flight: fp8 tiles (half the bytes); bf16 tiles only on request (it
        // needs a compute unit's LDS per workgroup and measured slower, see make_plan).  Tile t lives in stage
        // t % NS.  A step waits until exactly the tiles requested after its own are still outstanding: NS-2 of them in
        // the steady state, fewer at the end.
        auto step = [&](auto stage, int it) {
            constexpr int ST = decltype(stage)::value;
            const int later = min(n_hot - it - 1, NS - 2);        // uniform
            if (later >= 2) MCSD_WAIT_VMCNT(2 * C::DPT);
            else if (later == 1) MCSD_WAIT_VMCNT(C::DPT);
            else MCSD_WAIT_VMCNT(0);
            __builtin_amdgcn_s_barrier();
            if (it + NS - 1 < n_hot) issue_tile(std::integral_constant<int, (ST + NS - 1) % NS>());
            attn_tile<D, QBP, NS, 0, F8, F8>(ring + ST * C::TILE, la, qs, c_pre, g, all_keys, vs_pre);
        };
        static_assert(NS == 4, "the step sequence below is unrolled for four stages");
        // Q and the mask row must have arrived before the first direct-to-LDS load is issued: the steps below wait
        // with a non-zero count, and the compiler, which does not see those loads, would otherwise place its own
        // wait for Q at the first MFMA inside the loop, where it would also wait for the tiles in flight.
        MCSD_WAIT_VMCNT(0);
        if (0 < n_hot) issue_tile(std::integral_constant<int, 0>());
        if (1 < n_hot) issue_tile(std::integral_constant<int, 1 % NS>());
        if (2 < n_hot) issue_tile(std::integral_constant<int, 2 % NS>());
        for (int it = 0; it < n_hot; it += 4) {
            step(std::integral_constant<int, 0>(), it);
            if (it + 1 < n_hot) step(std::integral_constant<int, 1 % NS>(), it + 1);
            if (it + 2 < n_hot) step(std::integral_constant<int, 2 % NS>(), it + 2);
            if (it + 3 < n_hot) step(std::integral_constant<int, 3 % NS>(), it + 3);
        }
        }
        MCSD_WAIT_VMCNT(0);
    }
    __syncthreads();

    // ---- ragged last prefix tile and the tree's own tiles: through registers, rows beyond `valid` zero-filled ----
    const int n_rest = (n_pre - n_hot) + n_tree_tiles;
    for (int it = 0; it < n_rest; ++it) {
        const bool tail = it < n_pre - n_hot;
        const int tt = tail ? 0 : it - (n_pre - n_hot);
        const unsigned char *ksrc = tail ? kp + (int64_t)(t1 - 1) * C::TILE_K : (const unsigned char *)kt + (int64_t)tt * C::BTILE_K;
        const unsigned char *vsrc = tail ? vp + (int64_t)(t1 - 1) * C::TILE_K : (const unsigned char *)vt + (int64_t)tt * C::BTILE_K;
        const int valid = tail ? L - (t1 - 1) * C::T : min(C::T, p.n - tt * C::T);
#pragma unroll
        for (int i0 = 0; i0 < C::CPT; i0 += 4) {           // four chunks of K and V at a time keeps the staging small
            uint4 kreg[4], vreg[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int x = (i0 + i) * C::THREADS + tid, row = x / C::BCPR, ch = x % C::BCPR;
                kreg[i] = make_uint4(0, 0, 0, 0);
                vreg[i] = make_uint4(0, 0, 0, 0);
                if (i0 + i < C::CPT && row < valid) {
                    if (F8 && tail) {                      // 8 fp8 values become this 16-byte bf16 chunk
                        const uint2 k8 = *(const uint2 *)(ksrc + row * C::RBP + ch * 8);
                        const uint2 v8 = *(const uint2 *)(vsrc + row * C::RBP + ch * 8);
                        kreg[i] = __builtin_bit_cast(uint4, fp8x8_to_bf16(k8.x, k8.y));
                        vreg[i] = __builtin_bit_cast(uint4, fp8x8_to_bf16(v8.x, v8.y));
                    } else {
                        kreg[i] = *(const uint4 *)(ksrc + row * C::RB + ch * 16);
                        vreg[i] = *(const uint4 *)(vsrc + row * C::RB + ch * 16);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int x = (i0 + i) * C::THREADS + tid, row = x / C::BCPR, ch = x % C::BCPR;
                const int off = row * C::RB + ((ch ^ swz<D>(row)) * 16);
                if (i0 + i < C::CPT) {
                    *(uint4 *)(ring + off) = kreg[i];
                    *(uint4 *)(ring + C::BTILE_K + off) = vreg[i];
                }
            }
        }
        __syncthreads();
        uint32_t bits[C::KPW];
#pragma unroll
        for (int u = 0; u < C::KPW; ++u) {
            const int key0 = (kg * C::KPW + u) * 32;          // first key of this block inside the tile
            if (tail) {
                const int left = valid - key0;                 // keys of the block that exist
                bits[u] = left >= 32 ? 0xffffffffu : (left <= 0 ? 0u : ((1u << left) - 1u));
            } else {
                const int col = tt * C::T + key0;
                bits[u] = (uint32_t)(((col >> 6) ? mrow[1] : mrow[0]) >> (col & 63));
            }
        }
        attn_tile<D, QBP, NS, 1, F8, false>(ring, la, qs, tail ? c_pre : p.c, g, bits, tail ? vs_pre : 1.f);
        __syncthreads();
    }

    // ---- merge the key groups of each query block through LDS (layout [c/4][query] keeps lanes contiguous) ----
    float l_tot = half_swap_sum(qs.l_run);
    if (C::KG > 1) {
        if (kg > 0) {
            unsigned char *slot = ring + ((kg - 1) * QBP + qb) * C::MSLOT;
#pragma unroll
            for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    f32x4_t v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = qs.o[cb][4 * j + e];
                    *(f32x4_t *)(slot + (((cb * 4 + j) * 2 + g) * 32 + ln) * 16) = v;
                }
            if (g == 0) {
                ((float *)(slot + 32 * D * 4))[ln] = qs.m_ref;
                ((float *)(slot + 32 * D * 4))[32 + ln] = l_tot;
            }
        }
        __syncthreads();
    }
    // wavefronts of key group 0 now own one query block each; the others are done
    const float cm = F8 ? 1.f : p.c;                           // reference maxima are in log2 units already with fp8 tiles
    auto merge_from = [&](const float *src_o, float m_k, float l_k) {
        // (O, m, l) of the same query block from elsewhere, fragments in this lane's register layout
        const float m_new = fmaxf(qs.m_ref, m_k);
        const bool any = m_new != -INFINITY;                  // false: neither side has seen a key
        const float a = any ? fast_exp2((qs.m_ref - m_new) * cm) : 1.f, bsc = any ? fast_exp2((m_k - m_new) * cm) : 0.f;
        qs.m_ref = m_new;
        l_tot = l_tot * a + l_k * bsc;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const f32x4_t v = *(const f32x4_t *)(src_o + (((cb * 4 + j) * 2 + g) * 32 + ln) * 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) qs.o[cb][4 * j + e] = qs.o[cb][4 * j + e] * a + v[e] * bsc;
            }
    };
    if (kg == 0) {
#pragma unroll 1
        for (int k = 1; k < C::KG; ++k) {
            const unsigned char *slot = ring + ((k - 1) * QBP + qb) * C::MSLOT;
            merge_from((const float *)slot, ((const float *)(slot + 32 * D * 4))[ln], ((const float *)(slot + 32 * D * 4))[32 + ln]);
        }
    }
    auto store_out = [&]() {
        if (qrow >= p.n) return;
        const float inv = 1.f / l_tot;
        __bf16 *o = (__bf16 *)p.out + (bh_q * p.node_stride + qrow) * D;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16x4_t v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (__bf16)(qs.o[cb][4 * j + e] * inv);
                *(bf16x4_t *)(o + cb * 32 + 8 * j + 4 * g) = v;
            }
    };
    if (n_active == 1) {                                   // the only split of this sequence: no exchange needed
        if (kg == 0) store_out();
        return;
    }

    // ---- key splits: every split writes (O, m, l) in register-fragment order (fully coalesced) ----
    if (kg == 0 && qrow < p.n) {                           // padded query rows are never read back
        // O goes out rounded to bf16, the precision the output itself has (one more rounding of 2^-9 relative to the
        // partial's own magnitude; maxima and denominators stay fp32): half the bytes to write, acknowledge and fold.
        // A lane's 16-byte chunk (cb, jp) holds its accumulator registers 8 jp .. 8 jp + 7 of column block cb.
        __bf16 *po = (__bf16 *)p.part_o + ((bh * p.SP + slot_id) * (int64_t)(QBP * 32 * D)) + qb * 32 * D;
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                bf16x8_t v;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = (__bf16)qs.o[cb][8 * jp + e];
                *(bf16x8_t *)(po + (((cb * 2 + jp) * 2 + g) * 32 + ln) * 8) = v;
            }
        if (g == 0) {
            const int64_t prow = (bh * p.SP + slot_id) * (QBP * 32) + qb * 32 + ln;
            p.part_m[prow] = qs.m_ref;
            p.part_l[prow] = l_tot;
        }
    }
    if (!p.fold) return;                                   // a second kernel folds

    // ---- fold inside this kernel: the workgroup of this (sequence, unit) that arrives last does it ----
    // All workgroups of the unit run on one die (see the numbering above), so their partial results meet in that
    // die's L2: a store is there once it is acknowledged (the vector L1 writes through), and the loads below go past
    // the L1.  Nobody waits for anybody: a workgroup counts itself in and leaves unless it is the last.  The
    // counter also records, per die, how many of the arrivals ran there, so a launch that was not dealt to the
    // dies as the host established shows up here and poisons the output instead of folding stale data.
    auto store_nan = [&]() {
        if (kg != 0 || qrow >= p.n) return;
        __bf16 *o = (__bf16 *)p.out + (bh_q * p.node_stride + qrow) * D;
        bf16x4_t v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (__bf16)__builtin_nanf("");
#pragma unroll
        for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
            for (int j = 0; j < 4; ++j) *(bf16x4_t *)(o + cb * 32 + 8 * j + 4 * g) = v;
    };
    if (ws_tag != WS_TAG) {                                // workspace never prepared: its counters mean nothing
        store_nan();
        return;
    }
    __shared__ unsigned long long s_prev;
    unsigned die;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(die));
    die &= 7u;
    // This wavefront's partial stores have reached the L2 once the vector-memory counter is back at zero.  (A release
    // fence of workgroup scope does not wait for it: within a workgroup the shared L1 already orders them.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0)
        s_prev = __hip_atomic_fetch_add(p.ctr + bh * CTR_STRIDE, 1ull + (1ull << (8 + 7 * die)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const unsigned long long prev = s_prev;
    if ((int)(prev & 0xffu) + 1 != n_active) return;       // someone else arrives later
    if (tid == 0) __hip_atomic_store(p.ctr + bh * CTR_STRIDE, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // as it was found
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    if ((int)((prev >> (8 + 7 * die)) & 0x7fu) + 1 != n_active) {   // an arrival from another die
        store_nan();
        return;
    }
    if (qrow >= p.n) return;
    // Every wavefront folds its query block's rows for its share of the columns (32-column blocks kg, kg + KG, ..),
    // all partial results read back in slot order, its own included: the result does not depend on who came last.
    // Loads go through buffer descriptors that end after the last partial result in use (see fold_partials).
    const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(
        (void *)((__bf16 *)p.part_o + (bh * p.SP) * (int64_t)(QBP * 32 * D) + qb * 32 * D), 0, (int)(n_active * QBP * 32 * D * 2), 0x00027000);
    const __amdgpu_buffer_rsrc_t rm = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(p.part_m + bh * p.SP * (QBP * 32) + qb * 32), 0, (int)(n_active * QBP * 32 * 4), 0x00027000);
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(p.part_l + bh * p.SP * (QBP * 32) + qb * 32), 0, (int)(n_active * QBP * 32 * 4), 0x00027000);
    __bf16 *orow = (__bf16 *)p.out + (bh_q * p.node_stride + qrow) * D;
    // as few slots per round as hold the partial results: a load beyond the end still costs its turn in the L1
    if (n_active <= 3) fold_partials<D, QBP, C::KG, 3>(ro, rm, rl, n_active, kg, g, ln, cm, orow, (f32x4_t *)ring + tid);
    else if (n_active <= 5) fold_partials<D, QBP, C::KG, 5>(ro, rm, rl, n_active, kg, g, ln, cm, orow, (f32x4_t *)ring + tid);
    else if (n_active <= 7) fold_partials<D, QBP, C::KG, 7>(ro, rm, rl, n_active, kg, g, ln, cm, orow, (f32x4_t *)ring + tid);
    else fold_partials<D, QBP, C::KG, 8>(ro, rm, rl, n_active, kg, g, ln, cm, orow, (f32x4_t *)ring + tid);
}

// Folds the partial results of the key splits of the bf16 sweep.  One thread per 4 output columns of one query;
// fragment order makes the loads of a wavefront contiguous.  Partials are folded in split order.
template <int D, int QBP>
__global__ __launch_bounds__(256) void tree_attn_merge_bf16_kernel(const AttnParams p, int T)
{
    constexpr int POS = D * 8;                                // float4 positions per (b, h, query block)
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int pos = (int)(idx % POS);
    const int qb = (int)((idx / POS) % QBP);
    const int64_t bh = idx / ((int64_t)POS * QBP);
    if (bh >= (int64_t)p.B * p.H) return;
    const int ln = pos & 31, g = (pos >> 5) & 1, f = pos >> 6;
    const int lrow = qb * 32 + ln;                            // row of the partial results
    const int row = p.row0 + (qb % p.bph) * 32 + ln;          // tree node
    if (row >= p.n) return;
    const int unit = (int)(bh % p.H);
    const int64_t bh_q = (bh / p.H) * p.Hq + (unit / p.chunks) * p.grp + (unit % p.chunks) * p.hpw + qb / p.bph;
    int L = p.lens[bh / p.H];
    L = L < 0 ? 0 : (L > p.max_prefix ? p.max_prefix : L);
    const int tiles_b = (L + T - 1) / T;
    const int np = (tiles_b + p.tps - 1) / p.tps;
    const int n_active = p.G > p.S ? np + 1 : max(1, np);
    if (n_active == 1) return;                                // the sweep wrote this sequence's output itself
    // eight partials at a time, all loads issued before the first use; folded in slot order
    float M = -INFINITY, den = 0.f;
    f32x4_t num = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < n_active; s0 += 8) {
        float m[8], l[8];
        f32x4_t o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            m[i] = -INFINITY;
            l[i] = 0.f;
            o[i] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
            if (s0 + i < n_active) {
                const int64_t prow = (bh * p.SP + s0 + i) * (QBP * 32) + lrow;
                m[i] = p.part_m[prow];
                l[i] = p.part_l[prow];
                const bf16x4_t ob = *(const bf16x4_t *)((const __bf16 *)p.part_o + ((bh * p.SP + s0 + i) * (int64_t)(QBP * 32 * D)) +
                                                        qb * 32 * D + ((((f >> 2) * 2 + ((f >> 1) & 1)) * 2 + g) * 32 + ln) * 8 + (f & 1) * 4);
                o[i] = (f32x4_t){(float)ob[0], (float)ob[1], (float)ob[2], (float)ob[3]};
            }
        }
        float Mn = M;
#pragma unroll
        for (int i = 0; i < 8; ++i) Mn = fmaxf(Mn, m[i]);
        if (Mn == -INFINITY) continue;                        // nothing visible so far
        const float a = fast_exp2((M - Mn) * p.c);            // exp2(-inf) = 0 on the first group
        den *= a;
        num *= a;
        M = Mn;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float w = fast_exp2((m[i] - M) * p.c);      // 0 for a split that saw no visible key
            den = fmaf(w, l[i], den);
            num += w * o[i];
        }
    }
    const f32x4_t r = num / den;
    bf16x4_t v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (__bf16)r[e];
    const int c = (f / 4) * 32 + 8 * (f % 4) + 4 * g;
    *(bf16x4_t *)((__bf16 *)p.out + (bh_q * p.node_stride + row) * D + c) = v;
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

    const int64_t bh = (int64_t)b * p.H + h;                 // query head
    const int kvh = h / p.grp;
    const int64_t bh_kv = (int64_t)b * p.Hkv + kvh;
    const float *q = (const float *)p.q + bh * p.node_stride * D;
    const float *kt = (const float *)p.kt + bh_kv * p.node_stride * D;
    const float *vt = (const float *)p.vt + bh_kv * p.node_stride * D;
    const int64_t pre0 = p.seq_base[b] + (int64_t)kvh * p.head_stride;
    const float *kp = (const float *)p.kp + pre0;
    const float *vp = (const float *)p.vp + pre0;

    for (int idx = p.row0 * D + tid; idx < p.n * D; idx += 256) sQ[idx / D][idx % D] = q[idx];   // rows below row0 are not read
    if (tid < NMAX) { sM[tid] = -INFINITY; sL[tid] = 0.f; }     // running maximum / denominator of every row
    float acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.f;
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
        {   // scores and online soft-max: the 32 lanes of a half wavefront own one row at a time, one key each
            const int j = tid % T, i0 = tid / T;
            for (int i = p.row0 + i0; i < p.n; i += 256 / T) {
                float dot = 0.f;
#pragma unroll 8
                for (int cc = 0; cc < D; ++cc) dot = fmaf(sQ[i][cc], sK[j][cc], dot);
                bool vis = j < valid;
                if (tree_col0 >= 0) {
                    const int col = tree_col0 + j;
                    vis = vis && ((p.mask_bits[(int64_t)i * p.mask_words + (col >> 6)] >> (col & 63)) & 1ull);
                }
                const float sc = vis ? dot : -INFINITY;
                float mx = sc;
#pragma unroll
                for (int m = 1; m < T; m <<= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
                const float m_old = sM[i];
                const float m_new = fmaxf(m_old, mx);
                const float mc = (m_new == -INFINITY ? 0.f : m_new) * p.c;
                const float pv = exp2f(fmaf(sc, p.c, -mc));
                float psum = pv;
#pragma unroll
                for (int m = 1; m < T; m <<= 1) psum += __shfl_xor(psum, m, 64);
                sS[i][j] = pv;
                if (j == 0) {
                    const float alpha = exp2f(fmaf(m_old, p.c, -mc));
                    sAlpha[i] = alpha;
                    sL[i] = sL[i] * alpha + psum;
                    sM[i] = m_new;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = oi0 + RP * r;
            if (i >= p.row0 && i < p.n) {
                float a = acc[r] * sAlpha[i];
#pragma unroll 8
                for (int j = 0; j < T; ++j) a = fmaf(sS[i][j], sV[j][oc], a);
                acc[r] = a;
            }
        }
    }
    __syncthreads();
    if (p.SP == 1) {
        float *o = (float *)p.out + bh * p.node_stride * D;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = oi0 + RP * r;
            if (i >= p.row0 && i < p.n) o[(int64_t)i * D + oc] = acc[r] / sL[i];
        }
    } else {
        const int64_t prow0 = (bh * p.SP + s) * p.n;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const int i = oi0 + RP * r;
            if (i >= p.row0 && i < p.n) p.part_o[(prow0 + i) * D + oc] = acc[r];
        }
        if (tid >= p.row0 && tid < p.n) {
            p.part_m[prow0 + tid] = sM[tid];
            p.part_l[prow0 + tid] = sL[tid];
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
    if (i >= p.n || i < p.row0) return;
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


size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// workspace: [tag] [counters] [part_m] [part_l] [part_o]; nothing when the keys are not split
size_t partial_rows(const AttnPlan &pl, int dtype, int B, int n)
{
    // per workgroup unit and split; bf16 path: whole 32-row query blocks in register-fragment order; fp32 path: n rows
    return (size_t)B * pl.units * pl.G * (dtype == MCSD_BF16 ? (size_t)pl.QBP * 32 : (size_t)n);
}

size_t workspace_bytes_for(const AttnPlan &pl, int dtype, int B, int d, int n)
{
    if (pl.S == 1) return 0;
    const size_t rows = partial_rows(pl, dtype, B, n);
    return WS_HEADER + WS_CTR_BYTES + 2 * align256(rows * sizeof(float)) + align256(rows * d * (dtype == MCSD_BF16 ? 2 : sizeof(float)));
}

// Prepares a workspace: tag word, zero counters.  One thread per 16 bytes of the header and counter area.
__global__ __launch_bounds__(256) void workspace_init_kernel(uint4 *ws)
{
    const unsigned i = blockIdx.x * 256 + threadIdx.x;
    if (i < (WS_HEADER + WS_CTR_BYTES) / 16) ws[i] = make_uint4(i == 0 ? WS_TAG : 0u, 0u, 0u, 0u);
}

template <int D, int QBP, int NS, bool F8 = false>
void launch_sweep(const AttnParams &p, const AttnPlan &pl, hipStream_t st)
{
    const dim3 grid((unsigned)((size_t)pl.G * pl.grid_units));
    mcsd_launch(MCSD_KERNEL_ATTN_SWEEP, tree_attn_bf16_kernel<D, QBP, NS, F8>, grid, dim3(SweepCfg<D, QBP, NS, F8>::THREADS), st, p);
}

template <int D, int QBP>
void launch_merge(const AttnParams &p, const AttnPlan &pl, hipStream_t st)
{
    const size_t threads = (size_t)p.B * p.H * QBP * D * 8;
    mcsd_launch(MCSD_KERNEL_ATTN_MERGE, tree_attn_merge_bf16_kernel<D, QBP>, dim3((unsigned)((threads + 255) / 256)), dim3(256), st, p, pl.T);
}

template <int D>
hipError_t launch_bf16(const AttnParams &p, const AttnPlan &pl, hipStream_t st)
{
    if (pl.QBP == 1) launch_sweep<D, 1, 2>(p, pl, st);
    else if (pl.QBP == 2) { if (pl.NS == 4) launch_sweep<D, 2, 4>(p, pl, st); else launch_sweep<D, 2, 2>(p, pl, st); }
    else { if (pl.NS == 4) launch_sweep<D, 4, 4>(p, pl, st); else launch_sweep<D, 4, 2>(p, pl, st); }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.S == 1 || pl.fold) return e;
    if (pl.QBP == 1) launch_merge<D, 1>(p, pl, st);
    else if (pl.QBP == 2) launch_merge<D, 2>(p, pl, st);
    else launch_merge<D, 4>(p, pl, st);
    return hipGetLastError();
}

// fp8 prefix cache (d = 128): four-stage ring; reference maxima reach the fold in log2 units
hipError_t launch_fp8kv(const AttnParams &p, const AttnPlan &pl, hipStream_t st)
{
    if (pl.QBP == 2) launch_sweep<128, 2, 4, true>(p, pl, st);
    else launch_sweep<128, 4, 4, true>(p, pl, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.S == 1 || pl.fold) return e;
    AttnParams pm = p;
    pm.c = 1.f;
    if (pl.QBP == 2) launch_merge<128, 2>(pm, pl, st);
    else launch_merge<128, 4>(pm, pl, st);
    return hipGetLastError();
}

template <int D>
hipError_t launch_f32(const AttnParams &p, const AttnPlan &pl, hipStream_t st)
{
    dim3 grid(pl.S, p.H, p.B), block(256);
    mcsd_launch(MCSD_KERNEL_ATTN_SWEEP, tree_attn_f32_kernel<D>, grid, block, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.S == 1) return e;
    mcsd_launch(MCSD_KERNEL_ATTN_MERGE, tree_attn_merge_kernel<D, false>, dim3((p.n + 1024 / D - 1) / (1024 / D), p.H, p.B), block, st, p, pl.T, 1);
    return hipGetLastError();
}

size_t workspace_query(const mcsd_attention_tuning_t *tune, bool f8, int32_t B, int32_t H_q, int32_t H_kv, int32_t d,
                       int32_t n_nodes, int32_t row_begin, int32_t max_prefix)
{
    if (B < 1 || H_q < 1 || H_kv < 1 || H_q % H_kv != 0 || (d != 64 && d != 128) || n_nodes < 1 ||
        n_nodes > MCSD_ATTN_MAX_NODES || max_prefix < 0 || row_begin < 0 || row_begin >= n_nodes || (f8 && d != 128))
        return 0;
    const AttnPlan a = make_plan(MCSD_BF16, B, H_q, H_kv, n_nodes - row_begin, max_prefix, f8, tune);
    const size_t wa = workspace_bytes_for(a, MCSD_BF16, B, d, n_nodes);
    if (f8) return wa;
    // the larger of the two dtypes' needs, so one buffer serves both
    const AttnPlan f = make_plan(MCSD_F32, B, H_q, H_kv, n_nodes - row_begin, max_prefix, false, tune);
    const size_t wf = workspace_bytes_for(f, MCSD_F32, B, d, n_nodes);
    return wa > wf ? wa : wf;
}

int attention_call(const mcsd_attention_tuning_t *tune, const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, bool f8,
                   float k_scale, float v_scale, int32_t B,
                   int32_t H_q, int32_t H_kv, int32_t d, int32_t row_begin, const void *q, const void *k_tree,
                   const void *v_tree, int64_t node_stride, const void *k_prefix, const void *v_prefix,
                   const int64_t *seq_base_dev, const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                   float softmax_scale, void *out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const int32_t H = H_q;
    if (H_kv < 1 || H_q < 1 || H_q % H_kv != 0) return MCSD_EINVAL;
    if (!mask || !mask->bits_dev || !q || !k_tree || !v_tree || !out || !seq_base_dev || !prefix_lens_dev)
        return MCSD_EINVAL;
    if (dtype != MCSD_F32 && dtype != MCSD_BF16) return MCSD_EINVAL;
    if (B < 1 || H < 1 || B > 65535 || H > 65535 || max_prefix < 0) return MCSD_EINVAL;
    if (max_prefix > 0 && (!k_prefix || !v_prefix)) return MCSD_EINVAL;
    if (tune && (tune->key_splits < 0 || tune->key_splits > 64 || tune->fold < 0 || tune->fold > 1 ||
                 tune->tree_keys < 0 || tune->tree_keys > 3 ||
                 (tune->stages != 0 && tune->stages != 2 && tune->stages != 4)))
        return MCSD_EINVAL;
    const int32_t n = mask->n_nodes;
    if (n < 1 || node_stride < n || head_stride < 0) return MCSD_EINVAL;
    if (row_begin < 0 || row_begin >= n) return MCSD_EINVAL;
    if (!(softmax_scale > 0.f) || !isfinite(softmax_scale)) return MCSD_EINVAL;
    if (d != 64 && d != 128) return MCSD_EUNSUPPORTED;
    if (n > MCSD_ATTN_MAX_NODES) return MCSD_EUNSUPPORTED;
    if (f8 && (d != 128 || dtype != MCSD_BF16)) return MCSD_EUNSUPPORTED;
    if (f8 && (!(k_scale > 0.f) || !isfinite(k_scale) || !isfinite(v_scale))) return MCSD_EINVAL;
    const uintptr_t align = (uintptr_t)q | (uintptr_t)k_tree | (uintptr_t)v_tree | (uintptr_t)out |
                            (uintptr_t)k_prefix | (uintptr_t)v_prefix;
    if (align & 15) return MCSD_EINVAL;
    if (((node_stride * d) & 7) || (head_stride & (f8 ? 15 : 7))) return MCSD_EINVAL;   // 16-byte rows and heads

    const AttnPlan pl = make_plan(dtype, B, H_q, H_kv, n - row_begin, max_prefix, f8, tune);
    if ((int64_t)pl.G * pl.grid_units > 0x7fffffff) return MCSD_EUNSUPPORTED;           // one-dimensional grid
    const size_t need = workspace_bytes_for(pl, dtype, B, d, n);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return MCSD_EWORKSPACE;

    AttnParams p;
    p.q = q; p.kt = k_tree; p.vt = v_tree; p.kp = k_prefix; p.vp = v_prefix; p.out = out;
    p.seq_base = seq_base_dev; p.lens = prefix_lens_dev;
    p.mask_bits = mask->bits_dev; p.mask_words = mask->words_per_row;
    p.B = B; p.H = pl.units; p.n = n; p.row0 = row_begin; p.max_prefix = max_prefix;
    p.Hq = H_q; p.Hkv = H_kv; p.grp = H_q / H_kv; p.hpw = pl.hpw; p.bph = pl.bph; p.chunks = pl.chunks;
    p.node_stride = node_stride; p.head_stride = head_stride;
    p.c = softmax_scale * 1.4426950408889634f;
    p.k_scale = f8 ? k_scale : 1.f;
    p.v_scale = f8 ? v_scale : 1.f;
    p.S = pl.S; p.G = pl.G; p.SP = pl.G;
    p.pair_cus = pl.pair_cus;
    p.tree_last = pl.tree_last;
    p.xcc = pl.xcc;
    p.fold = pl.fold;
    p.tps = (int32_t)((((int64_t)max_prefix + pl.T - 1) / pl.T + pl.S - 1) / pl.S);
    if (p.tps < 1) p.tps = 1;
    char *w = (char *)workspace;
    p.part_o = p.part_m = p.part_l = nullptr;
    p.ctr = nullptr;
    p.ws_tag = nullptr;
    if (pl.S > 1) {
        const size_t rows = partial_rows(pl, dtype, B, n);
        p.ws_tag = (const uint32_t *)w;
        p.ctr = (unsigned long long *)(w + WS_HEADER);
        w += WS_HEADER + WS_CTR_BYTES;
        p.part_m = (float *)w;
        w += align256(rows * sizeof(float));
        p.part_l = (float *)w;
        w += align256(rows * sizeof(float));
        p.part_o = (float *)w;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e;
    if (f8) e = launch_fp8kv(p, pl, st);
    else if (dtype == MCSD_BF16) e = d == 128 ? launch_bf16<128>(p, pl, st) : launch_bf16<64>(p, pl, st);
    else e = d == 128 ? launch_f32<128>(p, pl, st) : launch_f32<64>(p, pl, st);
    return mcsd_hip_status(e);
}

}  // namespace

// ---------------------------------------------------------------------------------------------------
// Entry point that allocates nothing: the workspace is a file-scope device array.  Each GPU the library runs on
// holds its own copy at its own address; the array's name is a host-side stand-in only, so the device address is
// asked for once per device with hipGetSymbolAddress and that pointer, never the name, is what the kernels get.
// ---------------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[MCSD_STATIC_SCRATCH_BYTES];

namespace {
std::atomic<void *> g_scratch_of_device[64];        // device address of `scratch`, null until the first call there
std::atomic<int> g_scratch_prepared[64];            // 1 once the tag word has been written on that device

// Device address of this device's copy of `scratch`; the first call on a device also enqueues the fill kernel that
// writes the workspace tag (the counters start as zeros like all of the array, and every launch leaves them zero).
int static_scratch(hipStream_t st, void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MCSD_EHIP;
    void *ptr = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return MCSD_EHIP;
        }
        g_scratch_of_device[dev].store(ptr, std::memory_order_release);
    }
    if (g_scratch_prepared[dev].load(std::memory_order_acquire) == 0) {
        const unsigned n16 = (unsigned)((WS_HEADER + WS_CTR_BYTES) / 16);
        hipLaunchKernelGGL(workspace_init_kernel, dim3((n16 + 255) / 256), dim3(256), 0, st, (uint4 *)ptr);
        if (hipGetLastError() != hipSuccess) return MCSD_EHIP;
        g_scratch_prepared[dev].store(1, std::memory_order_release);
    }
    *out = ptr;
    return MCSD_OK;
}
}  // namespace

extern "C" int mcsd_tree_attention_static(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H,
                                          int32_t d, const void *q, const void *k_tree, const void *v_tree,
                                          int64_t node_stride, const void *k_prefix, const void *v_prefix,
                                          const int64_t *seq_base_dev, const int32_t *prefix_lens_dev,
                                          int64_t head_stride, int32_t max_prefix, float softmax_scale, void *out,
                                          void *hip_stream)
{
    if (!mask || B < 1 || H < 1 || max_prefix < 0 || (d != 64 && d != 128) || mask->n_nodes < 1 ||
        mask->n_nodes > MCSD_ATTN_MAX_NODES || (dtype != MCSD_F32 && dtype != MCSD_BF16))
        return attention_call(nullptr, mask, dtype, false, 1.f, 1.f, B, H, H, d, 0, q, k_tree, v_tree, node_stride, k_prefix,
                              v_prefix, seq_base_dev, prefix_lens_dev, head_stride, max_prefix, softmax_scale, out, nullptr,
                              0, hip_stream);          // (reports the argument error; nothing is launched)
    // the shape's need against the array's size, before anything is enqueued
    const AttnPlan pl = make_plan(dtype, B, H, H, mask->n_nodes, max_prefix);
    if (workspace_bytes_for(pl, dtype, B, d, mask->n_nodes) > (size_t)MCSD_STATIC_SCRATCH_BYTES) return MCSD_EUNSUPPORTED;
    void *ws = nullptr;
    const int rc = static_scratch((hipStream_t)hip_stream, &ws);
    if (rc != MCSD_OK) return rc;
    return attention_call(nullptr, mask, dtype, false, 1.f, 1.f, B, H, H, d, 0, q, k_tree, v_tree, node_stride, k_prefix,
                          v_prefix, seq_base_dev, prefix_lens_dev, head_stride, max_prefix, softmax_scale, out, ws,
                          (size_t)MCSD_STATIC_SCRATCH_BYTES, hip_stream);
}

extern "C" int mcsd_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!workspace && workspace_bytes > 0) return MCSD_EINVAL;
    if ((uintptr_t)workspace & 255) return MCSD_EINVAL;
    if (workspace_bytes < WS_HEADER + WS_CTR_BYTES) return MCSD_OK;    // too small to serve a call that needs one
    const unsigned n16 = (unsigned)((WS_HEADER + WS_CTR_BYTES) / 16);
    hipLaunchKernelGGL(workspace_init_kernel, dim3((n16 + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream, (uint4 *)workspace);
    return mcsd_hip_status(hipGetLastError());
}

extern "C" size_t mcsd_tree_attention_gqa_workspace(int32_t B, int32_t H_q, int32_t H_kv, int32_t d, int32_t n_nodes,
                                                    int32_t row_begin, int32_t max_prefix)
{
    return workspace_query(nullptr, false, B, H_q, H_kv, d, n_nodes, row_begin, max_prefix);
}

extern "C" size_t mcsd_tree_attention_rows_workspace(int32_t B, int32_t H, int32_t d, int32_t n_nodes,
                                                     int32_t row_begin, int32_t max_prefix)
{
    return workspace_query(nullptr, false, B, H, H, d, n_nodes, row_begin, max_prefix);
}

extern "C" size_t mcsd_tree_attention_workspace(int32_t B, int32_t H, int32_t d, int32_t n_nodes, int32_t max_prefix)
{
    return workspace_query(nullptr, false, B, H, H, d, n_nodes, 0, max_prefix);
}

extern "C" size_t mcsd_tree_attention_fp8kv_workspace(int32_t B, int32_t H_q, int32_t H_kv, int32_t n_nodes,
                                                      int32_t row_begin, int32_t max_prefix)
{
    return workspace_query(nullptr, true, B, H_q, H_kv, 128, n_nodes, row_begin, max_prefix);
}

extern "C" size_t mcsd_tree_attention_tuned_workspace(const mcsd_attention_tuning_t *tuning, int32_t prefix_fp8, int32_t B,
                                                      int32_t H_q, int32_t H_kv, int32_t d, int32_t n_nodes,
                                                      int32_t row_begin, int32_t max_prefix)
{
    if (tuning && (tuning->key_splits < 0 || tuning->key_splits > 64)) return 0;
    return workspace_query(tuning, prefix_fp8 != 0, B, H_q, H_kv, d, n_nodes, row_begin, max_prefix);
}

extern "C" int mcsd_tree_attention_plan(const mcsd_attention_tuning_t *tuning, mcsd_dtype_t dtype, int32_t prefix_fp8,
                                        int32_t B, int32_t H_q, int32_t H_kv, int32_t d, int32_t n_nodes, int32_t row_begin,
                                        int32_t max_prefix, mcsd_attention_plan_t *out)
{
    if (!out || B < 1 || H_q < 1 || H_kv < 1 || H_q % H_kv != 0 || (d != 64 && d != 128) || n_nodes < 1 ||
        n_nodes > MCSD_ATTN_MAX_NODES || max_prefix < 0 || row_begin < 0 || row_begin >= n_nodes ||
        (dtype != MCSD_F32 && dtype != MCSD_BF16) || (prefix_fp8 && (d != 128 || dtype != MCSD_BF16)))
        return MCSD_EINVAL;
    if (tuning && (tuning->key_splits < 0 || tuning->key_splits > 64 || tuning->fold < 0 || tuning->fold > 1 ||
                   tuning->tree_keys < 0 || tuning->tree_keys > 3 ||
                   (tuning->stages != 0 && tuning->stages != 2 && tuning->stages != 4)))
        return MCSD_EINVAL;
    const AttnPlan pl = make_plan(dtype, B, H_q, H_kv, n_nodes - row_begin, max_prefix, prefix_fp8 != 0, tuning);
    out->mfma_path = dtype == MCSD_BF16;
    out->query_blocks = pl.QBP;
    out->key_splits = pl.S;
    out->workgroups = (int32_t)((int64_t)pl.G * (dtype == MCSD_BF16 ? pl.grid_units : (long)pl.units * B));
    out->stages = dtype == MCSD_BF16 ? pl.NS : 0;
    out->fold_in_kernel = pl.fold;
    out->ordered_by_length = pl.pair_cus > 0;
    return MCSD_OK;
}

extern "C" int mcsd_tree_attention(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H, int32_t d,
                                   const void *q, const void *k_tree, const void *v_tree, int64_t node_stride,
                                   const void *k_prefix, const void *v_prefix, const int64_t *seq_base_dev,
                                   const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                                   float softmax_scale, void *out, void *workspace, size_t workspace_bytes,
                                   void *hip_stream)
{
    return attention_call(nullptr, mask, dtype, false, 1.f, 1.f, B, H, H, d, 0, q, k_tree, v_tree, node_stride, k_prefix,
                          v_prefix, seq_base_dev, prefix_lens_dev, head_stride, max_prefix, softmax_scale, out, workspace,
                          workspace_bytes, hip_stream);
}

extern "C" int mcsd_tree_attention_rows(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H,
                                        int32_t d, int32_t row_begin, const void *q, const void *k_tree,
                                        const void *v_tree, int64_t node_stride, const void *k_prefix,
                                        const void *v_prefix, const int64_t *seq_base_dev,
                                        const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                                        float softmax_scale, void *out, void *workspace, size_t workspace_bytes,
                                        void *hip_stream)
{
    return attention_call(nullptr, mask, dtype, false, 1.f, 1.f, B, H, H, d, row_begin, q, k_tree, v_tree, node_stride,
                          k_prefix, v_prefix, seq_base_dev, prefix_lens_dev, head_stride, max_prefix, softmax_scale, out,
                          workspace, workspace_bytes, hip_stream);
}

extern "C" int mcsd_tree_attention_gqa(const mcsd_mask_view_t *mask, mcsd_dtype_t dtype, int32_t B, int32_t H_q,
                                       int32_t H_kv, int32_t d, int32_t row_begin, const void *q, const void *k_tree,
                                       const void *v_tree, int64_t node_stride, const void *k_prefix,
                                       const void *v_prefix, const int64_t *seq_base_dev,
                                       const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                                       float softmax_scale, void *out, void *workspace, size_t workspace_bytes,
                                       void *hip_stream)
{
    return attention_call(nullptr, mask, dtype, false, 1.f, 1.f, B, H_q, H_kv, d, row_begin, q, k_tree, v_tree,
                          node_stride, k_prefix, v_prefix, seq_base_dev, prefix_lens_dev, head_stride, max_prefix,
                          softmax_scale, out, workspace, workspace_bytes, hip_stream);
}

extern "C" int mcsd_tree_attention_fp8kv(const mcsd_mask_view_t *mask, int32_t B, int32_t H_q, int32_t H_kv,
                                         int32_t row_begin, const void *q, const void *k_tree, const void *v_tree,
                                         int64_t node_stride, const void *k_prefix_fp8, const void *v_prefix_fp8,
                                         float k_scale, float v_scale, const int64_t *seq_base_dev,
                                         const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                                         float softmax_scale, void *out, void *workspace, size_t workspace_bytes,
                                         void *hip_stream)
{
    return attention_call(nullptr, mask, MCSD_BF16, true, k_scale, v_scale, B, H_q, H_kv, 128, row_begin, q, k_tree,
                          v_tree, node_stride, k_prefix_fp8, v_prefix_fp8, seq_base_dev, prefix_lens_dev, head_stride,
                          max_prefix, softmax_scale, out, workspace, workspace_bytes, hip_stream);
}

extern "C" int mcsd_tree_attention_tuned(const mcsd_attention_tuning_t *tuning, const mcsd_mask_view_t *mask,
                                         mcsd_dtype_t dtype, int32_t prefix_fp8, float k_scale, float v_scale, int32_t B,
                                         int32_t H_q, int32_t H_kv, int32_t d, int32_t row_begin, const void *q,
                                         const void *k_tree, const void *v_tree, int64_t node_stride,
                                         const void *k_prefix, const void *v_prefix, const int64_t *seq_base_dev,
                                         const int32_t *prefix_lens_dev, int64_t head_stride, int32_t max_prefix,
                                         float softmax_scale, void *out, void *workspace, size_t workspace_bytes,
                                         void *hip_stream)
{
    return attention_call(tuning, mask, dtype, prefix_fp8 != 0, k_scale, v_scale, B, H_q, H_kv, d, row_begin, q, k_tree,
                          v_tree, node_stride, k_prefix, v_prefix, seq_base_dev, prefix_lens_dev, head_stride, max_prefix,
                          softmax_scale, out, workspace, workspace_bytes, hip_stream);
}
