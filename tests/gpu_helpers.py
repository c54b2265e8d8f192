"""Helpers for the GPU parity tests: move seeded inputs to the device, call the C ABI through the binding,
bring results back as numpy.  No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

from workloads import bf16_bits_to_f32

BF16_RTOL, BF16_ATOL = 2e-2, 1e-2        # tolerance of the bf16 path against the binary64 oracle
F32_RTOL, F32_ATOL = 1e-5, 1e-5          # tolerance of the fp32 path


def dev(a: np.ndarray, dtype: str | None = None) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


class AttnDevice:
    """Device copies of one attention input dict (as made by workloads.attention_inputs)."""

    def __init__(self, inp: dict):
        dt = inp["dtype"]
        self.dtype = dt
        self.code = 1 if dt == "bf16" else 0
        self.q, self.kt, self.vt = (dev(inp[k], dt) for k in ("q", "k_tree", "v_tree"))
        self.kp, self.vp = (dev(inp[k], dt) for k in ("k_prefix", "v_prefix"))
        self.lens = dev(np.ascontiguousarray(inp["lens"], dtype=np.int32))
        self.base = dev(np.ascontiguousarray(inp["seq_base"], dtype=np.int64))
        self.B, self.H, self.node_stride, self.d = inp["q"].shape
        self.head_stride = int(inp["head_stride"])
        self.max_prefix = int(max(int(np.max(inp["lens"])), 0))
        self.scale = float(np.float32(inp["scale"]))
        self.out = torch.zeros_like(self.q)


def run_attention(binding, view, ad: AttnDevice, max_prefix: int | None = None, fill: float | None = None) -> np.ndarray:
    """Calls mcsd_tree_attention; returns the first n_nodes rows as float64 [B][H][n][d]."""
    n = view.n_nodes
    mp = ad.max_prefix if max_prefix is None else max_prefix
    ws_bytes = binding.tree_attention_workspace(ad.B, ad.H, ad.d, n, mp)
    ws = binding.new_workspace(ws_bytes)
    if fill is not None:
        ad.out.fill_(fill)
    binding.tree_attention(view, ad.code, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp,
                           ad.base, ad.lens, ad.head_stride, mp, ad.scale, ad.out, ws)
    torch.cuda.synchronize()
    out = ad.out[:, :, :n].float().cpu().numpy().astype(np.float64)
    return out


def assert_close(got: np.ndarray, want: np.ndarray, dtype: str, what: str = ""):
    rtol, atol = (BF16_RTOL, BF16_ATOL) if dtype == "bf16" else (F32_RTOL, F32_ATOL)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - want)
    lim = atol + rtol * np.abs(want)
    bad = err > lim
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} elements out of tolerance; worst err "
                           f"{float(err.max()):.3e} at {np.unravel_index(int(np.argmax(err - lim)), err.shape)}")


def run_verify(binding, view, mode: int, vi: dict):
    """Calls mcsd_verify_tree on one verify input dict; returns (path, accept_len, new_tokens) as numpy."""
    p, q = dev(vi["p_target"]), dev(vi["q_draft"])
    tokens, ua, us = dev(vi["tokens"]), dev(vi["u_accept"]), dev(vi["u_sample"])
    B, rows_p, V = vi["p_target"].shape
    rows_q = vi["q_draft"].shape[1]
    n_new = vi["u_sample"].shape[1]
    g = view.gamma
    path = torch.full((B, g), -7, dtype=torch.int32, device="cuda")
    alen = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    new = torch.full((B, max(n_new, 1)), -7, dtype=torch.int32, device="cuda")
    ws_bytes = binding.verify_tree_workspace(view, mode, B, n_new)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda") if ws_bytes else None
    binding.verify_tree(view, mode, B, V, tokens, p, q, rows_p * V, rows_q * V, ua, us if n_new else None, n_new,
                        path, alen, new if n_new else None, ws)
    torch.cuda.synchronize()
    return path.cpu().numpy(), alen.cpu().numpy(), new.cpu().numpy()[:, :n_new]
