"""Seeded synthetic inputs for the MCSD verification hot path.

This module only *produces inputs* (tensors, probabilities, tree tokens, uniforms).  It holds
none of the method's arithmetic: no mask, no attention, no acceptance rule.  The CPU oracle and
the HIP library are both fed from here, with bit-identical buffers, and neither of them is
imported here.

The five workloads stand in for the paper's experimental setting (Llama-2-7B-Chat target, 68M
draft, tree configurations such as (4,2,2,1) and target-initialised wide roots; Sec. 4.1), whose
model weights and prompt sets are not available: the shapes are Llama-2-7B's attention
(32 heads x 128, bf16), the vocabulary is 32000, and the draft distribution is the target's
logits plus Gaussian noise whose sigma controls the acceptance rate.

Random streams: numpy Generator(PCG64(SeedSequence([seed, cfg_id, tensor_id]))).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

DRAFT_INIT = 0
TARGET_INIT = 1

# tensor ids for the random streams
_T_LENS, _T_Q, _T_KT, _T_VT, _T_KP, _T_VP, _T_PL, _T_QL, _T_TOK, _T_UA, _T_US, _T_MLP, _T_HID = range(13)


@dataclass(frozen=True)
class Workload:
    cfg_id: int
    name: str
    B: int
    H: int
    d: int
    dtype: str                       # "f32" | "bf16": storage type of q/k/v and of the output
    prefix_min: int
    prefix_max: int                  # lens ~ integer U[min, max]; equal -> fixed length
    branching: Tuple[int, ...]       # per-level branching factors b_1..b_Gamma
    V: int
    target_sigma: float              # target logits ~ N(0, sigma^2)
    draft_noise_sigma: Optional[float]  # draft = target + N(0, s^2); None -> independent N(0, target_sigma^2)
    mode: int                        # primary verification mode

    @property
    def gamma_max(self) -> int:
        return len(self.branching)

    def level_sizes(self) -> Tuple[int, ...]:
        out, n = [], 1
        for b in self.branching:
            n *= b
            out.append(n)
        return tuple(out)

    def n_nodes(self, gamma: Optional[int] = None) -> int:
        g = self.gamma_max if gamma is None else gamma
        return int(sum(self.level_sizes()[:g]))


WORKLOADS: Dict[str, Workload] = {
    # tiny CPU-checkable case
    "cfg1": Workload(1, "cfg1", B=1, H=4, d=64, dtype="f32", prefix_min=128, prefix_max=128,
                     branching=(2, 2, 2), V=1000, target_sigma=2.0, draft_noise_sigma=None,
                     mode=DRAFT_INIT),
    # Llama-2-7B attention shape, MCSD tree (4,2,2,1)
    "cfg2": Workload(2, "cfg2", B=1, H=32, d=128, dtype="bf16", prefix_min=1024, prefix_max=1024,
                     branching=(4, 2, 2, 1), V=32000, target_sigma=3.0, draft_noise_sigma=1.0,
                     mode=DRAFT_INIT),
    # dynamic-gamma sweep: mask built once at gamma_max = 8
    "cfg3": Workload(3, "cfg3", B=1, H=32, d=128, dtype="bf16", prefix_min=2048, prefix_max=2048,
                     branching=(3, 2, 2, 1, 1, 1, 1, 1), V=32000, target_sigma=3.0,
                     draft_noise_sigma=1.0, mode=DRAFT_INIT),
    # batched ragged prefixes
    "cfg4": Workload(4, "cfg4", B=16, H=32, d=128, dtype="bf16", prefix_min=512, prefix_max=4096,
                     branching=(4, 2, 2, 2), V=32000, target_sigma=3.0, draft_noise_sigma=1.5,
                     mode=DRAFT_INIT),
    # long context, target-initialised wide root
    "cfg5": Workload(5, "cfg5", B=8, H=32, d=128, dtype="bf16", prefix_min=16384, prefix_max=16384,
                     branching=(8, 2, 2, 1, 1), V=32000, target_sigma=3.0, draft_noise_sigma=2.0,
                     mode=TARGET_INIT),
    # the ragged batch of cfg4 four times over: more workgroups than the chip holds at once (not one of the five
    # benchmark configurations; a serving-size batch for the attention sweep)
    "cfg4_b64": Workload(7, "cfg4_b64", B=64, H=32, d=128, dtype="bf16", prefix_min=512, prefix_max=4096,
                         branching=(4, 2, 2, 2), V=32000, target_sigma=3.0, draft_noise_sigma=1.5,
                         mode=DRAFT_INIT),
    # the paper's dynamic setting (Sec. 4.1: depth D = 5, width W = 16): a fork-shaped tree, 16 chains of 5 tokens,
    # temperature 1; one of the "next" workloads, not one of the five benchmark configurations
    "fork": Workload(6, "fork", B=1, H=32, d=128, dtype="bf16", prefix_min=1024, prefix_max=1024,
                     branching=(16, 1, 1, 1, 1), V=32000, target_sigma=3.0, draft_noise_sigma=1.0,
                     mode=DRAFT_INIT),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (reduced sizes for CPU-checkable cases)."""
    return replace(w, **kw)


def _rng(seed: int, cfg_id: int, tensor_id: int, extra: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, cfg_id, tensor_id, extra])))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def e4m3_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Numbers that 8-bit E4M3 codes stand for (OCP format: bias 7, no infinities, S.1111.111 = NaN)."""
    b = np.asarray(b, dtype=np.uint8).astype(np.int32)
    e, m = (b >> 3) & 15, b & 7
    mag = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(b >> 7 == 1, -mag, mag).astype(np.float32)


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to 8-bit E4M3 (round-to-nearest-even, values beyond +-448 saturate) and return the codes."""
    x = np.asarray(x, dtype=np.float32)
    grid = e4m3_bits_to_f32(np.arange(127, dtype=np.uint8)).astype(np.float64)      # 0 .. 448, ascending
    mids = (grid[:-1] + grid[1:]) / 2.0
    a = np.abs(x.astype(np.float64))
    lo = np.searchsorted(mids, a, side="left")                  # a <= mids[lo]: candidates lo (and lo+1 on a tie)
    tie = (lo < mids.size) & (a == mids[np.minimum(lo, mids.size - 1)])
    code = np.where(tie & (lo % 2 == 1), lo + 1, lo).astype(np.uint8)
    code = np.where(np.isnan(x), np.uint8(0x7F), code)
    return (code | (np.signbit(x).astype(np.uint8) << 7)).astype(np.uint8)


def _normal(rng: np.random.Generator, shape, dtype: str, mult: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    if mult != 1.0:
        x *= np.float32(mult)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def prefix_lens(w: Workload, seed: int = 0) -> np.ndarray:
    if w.prefix_min == w.prefix_max:
        return np.full(w.B, w.prefix_min, dtype=np.int32)
    return _rng(seed, w.cfg_id, _T_LENS).integers(w.prefix_min, w.prefix_max + 1, size=w.B).astype(np.int32)


def attention_inputs(w: Workload, seed: int = 0, lens: Optional[Sequence[int]] = None,
                     tensor_mult: float = 1.0, kv_capacity: Optional[int] = None,
                     variant: int = 0, kv_fp8: Optional[Tuple[float, float]] = None) -> dict:
    """q / k_tree / v_tree of shape [B][H][Nmax][d] and a prefix KV cache [B][H][cap][d].

    Storage is fp32 arrays (dtype "f32") or uint16 arrays holding bfloat16 bit patterns ("bf16").
    The cache has room for `cap` keys per (sequence, head); only the first lens[b] rows of each are
    meaningful, the rest is zero.  `seq_base[b]` is the element offset of sequence b in the cache and
    `head_stride` the element distance between heads.  `variant` selects a different random
    stream of the same recipe (distinct KV buffers for the layers of one step).
    kv_fp8 = (k_scale, v_scale): the prefix cache is stored as 8-bit E4M3 codes (uint8 arrays) of value / scale,
    from the same random stream as the bf16 cache (dtype must be "bf16"); the tree tensors stay bf16.
    """
    lens_a = prefix_lens(w, seed) if lens is None else np.asarray(lens, dtype=np.int32)
    assert lens_a.shape == (w.B,)
    nmax = w.n_nodes()
    cap = int(kv_capacity) if kv_capacity is not None else max(int(lens_a.max()), 1)
    assert cap >= int(lens_a.max())
    store = np.float32 if w.dtype == "f32" else np.uint16
    if kv_fp8 is not None:
        assert w.dtype == "bf16"
        store = np.uint8
    shape_t = (w.B, w.H, nmax, w.d)
    q = _normal(_rng(seed, w.cfg_id, _T_Q, variant), shape_t, w.dtype, tensor_mult)
    kt = _normal(_rng(seed, w.cfg_id, _T_KT, variant), shape_t, w.dtype, tensor_mult)
    vt = _normal(_rng(seed, w.cfg_id, _T_VT, variant), shape_t, w.dtype, tensor_mult)
    kp = np.zeros((w.B, w.H, cap, w.d), dtype=store)
    vp = np.zeros((w.B, w.H, cap, w.d), dtype=store)
    rk, rv = _rng(seed, w.cfg_id, _T_KP, variant), _rng(seed, w.cfg_id, _T_VP, variant)
    for b in range(w.B):
        L = int(lens_a[b])
        if L and kv_fp8 is None:
            kp[b, :, :L] = _normal(rk, (w.H, L, w.d), w.dtype, tensor_mult)
            vp[b, :, :L] = _normal(rv, (w.H, L, w.d), w.dtype, tensor_mult)
        elif L:
            kp[b, :, :L] = f32_to_e4m3_bits(_normal(rk, (w.H, L, w.d), "f32", tensor_mult) / np.float32(kv_fp8[0]))
            vp[b, :, :L] = f32_to_e4m3_bits(_normal(rv, (w.H, L, w.d), "f32", tensor_mult) / np.float32(kv_fp8[1]))
    head_stride = cap * w.d
    seq_base = (np.arange(w.B, dtype=np.int64) * (w.H * head_stride)).astype(np.int64)
    out = dict(q=q, k_tree=kt, v_tree=vt, k_prefix=kp, v_prefix=vp, lens=lens_a, seq_base=seq_base,
               head_stride=head_stride, node_stride=nmax, scale=float(1.0 / np.sqrt(w.d)), dtype=w.dtype)
    if kv_fp8 is not None:
        out.update(k_scale=float(np.float32(kv_fp8[0])), v_scale=float(np.float32(kv_fp8[1])))
    return out


def _softmax_rows_f32(logits: np.ndarray) -> np.ndarray:
    z = logits.astype(np.float64)
    z -= z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)


def _draw(rng: np.random.Generator, probs_row: np.ndarray, count: int) -> np.ndarray:
    """`count` i.i.d. token ids from a probability row (plain cumulative-sum inversion)."""
    cdf = np.cumsum(probs_row.astype(np.float64))
    u = rng.random(count) * cdf[-1]
    return np.minimum(np.searchsorted(cdf, u, side="right"), probs_row.size - 1).astype(np.int32)


def _draw_distinct(rng: np.random.Generator, probs_row: np.ndarray, count: int) -> np.ndarray:
    """`count` token ids drawn one after the other, each from the row with the earlier ones removed."""
    w = probs_row.astype(np.float64).copy()
    out = np.empty(count, dtype=np.int32)
    for i in range(count):
        if not (w > 0).any():                    # fewer tokens with mass than candidates: repeat the last one
            out[i] = out[i - 1] if i else 0
            continue
        out[i] = _draw(rng, w, 1)[0]
        while w[out[i]] == 0.0:                  # the inversion's last-bit landing on an emptied slot
            out[i] = _draw(rng, w, 1)[0]
        w[out[i]] = 0.0
    return out


def verify_inputs(w: Workload, seed: int = 0, gamma: Optional[int] = None, mode: Optional[int] = None,
                  n_new: Optional[int] = None, replacement: bool = True) -> dict:
    """Target / draft next-token distributions, tree tokens and uniforms for one verification call.

    p_target: fp32 [B][1+N][V]   (row 0: the context that ends the prefix; row 1+i: after tree node i)
    q_draft : fp32 [B][1+Nin][V] (Nin = nodes of levels < gamma: the contexts that have children)
    tokens  : int32 [B][N]       child tokens of context c are i.i.d. draws from q_draft[c]; in
                                 target-initialised mode the level-1 tokens are draws from p_target[0]
    u_accept: fp32 [B][N] in [0,1);  u_sample: fp32 [B][n_new] in [0,1)
    Nodes are numbered level by level, children of one parent next to each other.
    replacement=False: the children of a context are distinct tokens (drawn without replacement).
    """
    g = w.gamma_max if gamma is None else int(gamma)
    md = w.mode if mode is None else int(mode)
    sizes = w.level_sizes()[:g]
    N = int(sum(sizes))
    Nin = int(sum(sizes[:-1]))
    if n_new is None:
        n_new = 1 if md == DRAFT_INIT else int(w.branching[0])
    rp, rq = _rng(seed, w.cfg_id, _T_PL, g), _rng(seed, w.cfg_id, _T_QL, g)
    p = np.empty((w.B, 1 + N, w.V), dtype=np.float32)
    q = np.empty((w.B, 1 + Nin, w.V), dtype=np.float32)
    for b in range(w.B):
        tl = rp.standard_normal((1 + N, w.V), dtype=np.float32) * np.float32(w.target_sigma)
        p[b] = _softmax_rows_f32(tl)
        if w.draft_noise_sigma is None:
            dl = rq.standard_normal((1 + Nin, w.V), dtype=np.float32) * np.float32(w.target_sigma)
        else:
            dl = tl[: 1 + Nin] + rq.standard_normal((1 + Nin, w.V), dtype=np.float32) * np.float32(w.draft_noise_sigma)
        q[b] = _softmax_rows_f32(dl)
    rt = _rng(seed, w.cfg_id, _T_TOK, g * 2 + md)
    tokens = np.empty((w.B, N), dtype=np.int32)
    for b in range(w.B):
        # grow the tree level by level, as a draft model would
        level_nodes = [-1]            # node ids of the previous level (-1: the context before the tree)
        nxt = 0
        for lv, bf in enumerate(w.branching[:g]):
            new_nodes = []
            for par in level_nodes:
                ctx = 1 + par         # row of the context whose children are drawn
                row = p[b, 0] if (md == TARGET_INIT and lv == 0) else q[b, ctx]
                tokens[b, nxt:nxt + bf] = _draw(rt, row, bf) if replacement else _draw_distinct(rt, row, bf)
                new_nodes.extend(range(nxt, nxt + bf))
                nxt += bf
            level_nodes = new_nodes
        assert nxt == N
    ua = _rng(seed, w.cfg_id, _T_UA, g).random((w.B, N), dtype=np.float32)
    us = _rng(seed, w.cfg_id, _T_US, g).random((w.B, n_new), dtype=np.float32)
    return dict(p_target=p, q_draft=q, tokens=tokens, u_accept=ua, u_sample=us, gamma=g, mode=md,
                n_new=int(n_new), N=N, Nin=Nin)


def mlp_weights(widths: Sequence[int], seed: int = 0, stream: int = 0, gain: float = 2.0,
                out_bias: float = 0.0) -> Tuple[list, list]:
    """Random stand-ins for the trained weights of an early-stop decision model (Sec. 3.3; the trained ones are
    not published).  widths = (inputs, hidden..., 1); layer l gets weight fp32 [widths[l+1]][widths[l]] ~
    N(0, gain / fan_in) and bias ~ N(0, 0.1^2); `out_bias` is added to the last bias (it moves the outputs
    relative to the threshold)."""
    assert len(widths) >= 2 and widths[-1] == 1
    rng = _rng(seed, 100, _T_MLP, stream)
    ws, bs = [], []
    for l in range(len(widths) - 1):
        fan_in, fan_out = int(widths[l]), int(widths[l + 1])
        ws.append(rng.standard_normal((fan_out, fan_in), dtype=np.float32) * np.float32(np.sqrt(gain / fan_in)))
        bs.append(rng.standard_normal(fan_out, dtype=np.float32) * np.float32(0.1))
    bs[-1] = bs[-1] + np.float32(out_bias)
    return ws, bs


def hidden_states(B: int, W: int, width: int, seed: int = 0, stream: int = 0) -> np.ndarray:
    """Stand-in for the draft model's last hidden state of the newest token of each of the W candidate
    sequences of B trees: fp32 [B][W][width] ~ N(0, 1)."""
    return _rng(seed, 100, _T_HID, stream).standard_normal((B, W, width), dtype=np.float32)
