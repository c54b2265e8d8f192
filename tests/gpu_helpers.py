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


class DynamicIteration:
    """Device state and calls of one iteration of the paper's dynamic setting (Sec. 3.2, Sec. 3.3) for one workload:
    per level g the draft model's attention for the newest rows under the slice for g and the stop decision on the
    newest contexts' draft distributions; at the decided draft length the target's attention, the verification and the
    update after acceptance.  The mask is built once for the deepest tree; everything else works on slices of it.
    `w` is the target's attention shape, `w_draft` the draft model's (same tree, batch, vocabulary)."""

    BETA, K = 0.4, 10                    # threshold of Fig. 2's caption; top-10 values + entropy feed the decision model

    def __init__(self, binding, w, w_draft, n_draft_layers, n_target_layers, seed, out_bias, mode=0):
        from workloads import attention_inputs, mlp_weights, verify_inputs
        assert w.branching == w_draft.branching and w.B == w_draft.B and mode == 0
        self.b, self.w, self.mode = binding, w, mode
        self.D = w.gamma_max
        self.off = [0] + [int(x) for x in np.cumsum(w.level_sizes())]
        self.W = w.branching[0]
        L = int(w.prefix_max)
        self.cap, self.max_prefix = L + self.D + 3, L
        self.draft_host = [attention_inputs(w_draft, seed=seed, kv_capacity=self.cap, variant=100 + l) for l in range(n_draft_layers)]
        self.target_host = [attention_inputs(w, seed=seed, kv_capacity=self.cap, variant=l) for l in range(n_target_layers)]
        self.draft = [AttnDevice(i) for i in self.draft_host]
        self.target = [AttnDevice(i) for i in self.target_host]
        self.vi = vi = verify_inputs(w, seed=seed, gamma=self.D, mode=mode)
        self.p, self.q, self.us = dev(vi["p_target"]), dev(vi["q_draft"]), dev(vi["u_sample"])
        levels = range(1, self.D + 1)
        self.tok = {g: dev(np.ascontiguousarray(vi["tokens"][:, :self.off[g]])) for g in levels}
        self.ua = {g: dev(np.ascontiguousarray(vi["u_accept"][:, :self.off[g]])) for g in levels}
        self.ws_host, self.bs_host = mlp_weights((self.K + 1, 64, 1), seed=seed, out_bias=out_bias)
        self.mlp = binding.make_mlp([torch.from_numpy(a).cuda() for a in self.ws_host],
                                    [torch.from_numpy(a).cuda() for a in self.bs_host])
        self.mask = binding.build_mask(w.branching)                    # once, for the deepest tree
        self.views = {g: binding.slice_mask(self.mask, g) for g in levels}
        n = self.off[self.D]
        ws_bytes = max(binding.tree_attention_workspace(a.B, a.H, a.d, n, L) for a in (self.draft[0], self.target[0]))
        self.ws = binding.new_workspace(ws_bytes)
        vb = max(binding.verify_tree_workspace(self.views[g], mode, w.B, 1) for g in levels)
        self.vws = torch.empty(max(vb, 256), dtype=torch.uint8, device="cuda")
        i32 = dict(dtype=torch.int32, device="cuda")
        self.prob = torch.zeros((w.B, self.W), dtype=torch.float32, device="cuda")
        self.stop = torch.zeros((w.B,), **i32)
        self.stop_host = torch.zeros((w.B,), dtype=torch.int32, pin_memory=True)   # where the host reads the decision
        self.path = {g: torch.full((w.B, g), -9, **i32) for g in levels}
        self.ids = {g: torch.full((w.B, g + 1), -9, **i32) for g in levels}
        self.alen, self.new, self.n_ids = torch.full((w.B,), -9, **i32), torch.full((w.B, 1), -9, **i32), torch.full((w.B,), -9, **i32)
        self.lens0 = self.target[0].lens.clone()
        self.lens = self.target[0].lens.clone()
        self.cache0 = [(a.kp.clone(), a.vp.clone()) for a in self.target]

    def reset(self, caches=True):
        """Back to the state before the iteration (the update after acceptance moves lengths and cache rows)."""
        self.lens.copy_(self.lens0)
        if caches:
            for a, (k0, v0) in zip(self.target, self.cache0):
                a.kp.copy_(k0)
                a.vp.copy_(v0)
            for a in self.draft + self.target:
                a.out.fill_(float("nan"))
        self.stop.fill_(-9)
        self.prob.fill_(-9.0)

    def draft_level(self, g):
        """The draft model's attention for the newest level g under the slice for g, then the stop decision."""
        b, v, rb = self.b, self.views[g], self.off[g - 1]
        for a in self.draft:
            b.tree_attention_rows(v, a.code, a.B, a.H, a.d, rb, a.q, a.kt, a.vt, a.node_stride, a.kp, a.vp, a.base, a.lens,
                                  a.head_stride, self.max_prefix, a.scale, a.out, self.ws)
        if g < self.D:      # the newest contexts' draft distributions: rows 1 + off[g-1] .. of q_draft
            V, rows_q = self.w.V, self.vi["q_draft"].shape[1]
            b.early_stop_distribution(self.mlp, self.w.B, self.W, V, self.K, self.q[:, 1 + rb:], rows_q * V, V, self.BETA, None,
                                      self.prob, self.stop)

    def target_step(self, g):
        """At draft length g: the target's tree attention, verification, update after acceptance."""
        b, v, w, V = self.b, self.views[g], self.w, self.w.V
        for a in self.target:
            b.tree_attention(v, a.code, a.B, a.H, a.d, a.q, a.kt, a.vt, a.node_stride, a.kp, a.vp, a.base, self.lens0,
                             a.head_stride, self.max_prefix, a.scale, a.out, self.ws)
        b.verify_tree(v, self.mode, w.B, V, self.tok[g], self.p, self.q, self.vi["p_target"].shape[1] * V,
                      self.vi["q_draft"].shape[1] * V, self.ua[g], self.us, 1, self.path[g], self.alen, self.new, self.vws)
        T, a0 = self.target, self.target[0]
        b.commit_path(v, a0.code, a0.B, a0.H, a0.d, [a.kt for a in T], [a.vt for a in T], a0.node_stride,
                      [a.kp for a in T], [a.vp for a in T], a0.base, a0.head_stride, self.max_prefix, self.cap, self.path[g],
                      self.alen, self.tok[g], self.new, 1, 1, self.lens, self.ids[g], self.n_ids)

    def capture(self):
        """One HIP graph per level and one per draft length; returns (level graphs, target graphs) keyed by g."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                       # every piece once on a side stream before its capture
            for g in range(1, self.D + 1):
                self.reset(caches=False)
                self.draft_level(g)
                self.target_step(g)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        levels, targets = {}, {}
        for g in range(1, self.D + 1):
            levels[g] = torch.cuda.CUDAGraph()
            with torch.cuda.graph(levels[g]):
                self.draft_level(g)
            targets[g] = torch.cuda.CUDAGraph()
            with torch.cuda.graph(targets[g]):
                self.target_step(g)
        return levels, targets

    def run(self, level_fn, target_fn, force_gamma=None, caches=True):
        """Levels until the device says stop for every tree (or the deepest level; or `force_gamma` levels whatever the
        flags say), then the target step.  The host reads the flag after each level.  Returns (gamma, flags read)."""
        self.reset(caches)
        flags, gamma = [], self.D if force_gamma is None else force_gamma
        for g in range(1, gamma + 1):
            level_fn(g)
            if g < self.D:
                self.stop_host.copy_(self.stop, non_blocking=True)    # the decision the loop waits for
                torch.cuda.current_stream().synchronize()
                flags.append(self.stop_host.numpy().copy())
                if force_gamma is None and bool(flags[-1].all()):
                    gamma = g
                    break
        target_fn(gamma)
        return gamma, flags

    def snapshot(self, g):
        torch.cuda.synchronize()
        n = self.off[g]
        return dict(path=self.path[g].cpu().numpy(), alen=self.alen.cpu().numpy(), new=self.new.cpu().numpy(),
                    ids=self.ids[g].cpu().numpy(), n_ids=self.n_ids.cpu().numpy(), lens=self.lens.cpu().numpy(),
                    caches=[(a.kp.view(torch.int16).cpu().numpy(), a.vp.view(torch.int16).cpu().numpy()) for a in self.target],
                    target_out=[a.out[:, :, :n].float().cpu().numpy() for a in self.target],
                    draft_out=[a.out[:, :, :n].float().cpu().numpy() for a in self.draft])
