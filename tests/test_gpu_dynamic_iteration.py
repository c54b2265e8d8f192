"""One whole iteration of the paper's dynamic setting (Sec. 3.2, Sec. 3.3, Fig. 1 steps 3-6) composed from the library's
entry points on the fork-shaped tree (16 chains, depth 5), against the same sequence composed from the oracle's
functions:

    for every level g: mcsd_slice_mask(g) -> mcsd_tree_attention_rows for the newest level over the draft model's
    caches -> mcsd_early_stop_distribution (beta = 0.4) on the newest contexts' draft distributions, whose flag on
    the device decides the draft length gamma;
    then, at that gamma: the target's mcsd_tree_attention -> mcsd_verify_tree -> mcsd_commit_path.

The mask is built once for the deepest tree; every level and the verification use slices of it.  The pieces are
captured per level / per gamma as HIP graphs, replayed in the order the stop flags dictate, and every replayed result
must equal the eager one bit for bit.  Integer results (stop flags, paths, lengths, tokens, ids, cache rows) must match
the oracle exactly, attention within the bf16 tolerance."""
import numpy as np
import pytest
import torch

from workloads import DRAFT_INIT, WORKLOADS, attention_inputs, mlp_weights, scaled, verify_inputs

pytestmark = pytest.mark.gpu

BETA, K = 0.4, 10
N_DRAFT_LAYERS, N_TARGET_LAYERS = 2, 2


@pytest.fixture(scope="module")
def binding():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2409_10644_amd import binding as b
    return b


@pytest.fixture(scope="module")
def H():
    import gpu_helpers
    return gpu_helpers


class Iteration:
    """Device state of one tree and the calls of one iteration, level by level."""

    def __init__(self, binding, H, w, seed, out_bias):
        self.b, self.H, self.w = binding, H, w
        self.D = w.gamma_max
        self.off = [0] + list(np.cumsum(w.level_sizes()))
        self.W = w.branching[0]
        L = int(w.prefix_max)
        self.cap = L + self.D + 3
        self.max_prefix = L
        self.draft_host = [attention_inputs(w, seed=seed, kv_capacity=self.cap, variant=10 + l) for l in range(N_DRAFT_LAYERS)]
        self.target_host = [attention_inputs(w, seed=seed, kv_capacity=self.cap, variant=20 + l) for l in range(N_TARGET_LAYERS)]
        self.draft = [H.AttnDevice(i) for i in self.draft_host]
        self.target = [H.AttnDevice(i) for i in self.target_host]
        self.vi = vi = verify_inputs(w, seed=seed, gamma=self.D, mode=DRAFT_INIT)
        self.p, self.q = H.dev(vi["p_target"]), H.dev(vi["q_draft"])
        self.ua, self.us = H.dev(vi["u_accept"]), H.dev(vi["u_sample"])
        self.tok = {g: H.dev(np.ascontiguousarray(vi["tokens"][:, :self.off[g]])) for g in range(1, self.D + 1)}
        self.uag = {g: H.dev(np.ascontiguousarray(vi["u_accept"][:, :self.off[g]])) for g in range(1, self.D + 1)}
        self.ws_host, self.bs_host = mlp_weights((K + 1, 64, 1), seed=seed, out_bias=out_bias)
        self.mlp = binding.make_mlp([torch.from_numpy(a).cuda() for a in self.ws_host], [torch.from_numpy(a).cuda() for a in self.bs_host])
        self.mask = binding.build_mask(w.branching)                    # once, for the deepest tree
        self.views = {g: binding.slice_mask(self.mask, g) for g in range(1, self.D + 1)}
        a = self.draft[0]
        self.ws = binding.new_workspace(binding.tree_attention_workspace(a.B, a.H, a.d, self.off[self.D], self.max_prefix))
        self.prob = torch.zeros((w.B, self.W), dtype=torch.float32, device="cuda")
        self.stop = torch.zeros((w.B,), dtype=torch.int32, device="cuda")
        self.path = {g: torch.full((w.B, g), -9, dtype=torch.int32, device="cuda") for g in range(1, self.D + 1)}
        self.alen = torch.full((w.B,), -9, dtype=torch.int32, device="cuda")
        self.new = torch.full((w.B, 1), -9, dtype=torch.int32, device="cuda")
        self.ids = {g: torch.full((w.B, g + 1), -9, dtype=torch.int32, device="cuda") for g in range(1, self.D + 1)}
        self.n_ids = torch.full((w.B,), -9, dtype=torch.int32, device="cuda")
        vb = max(binding.verify_tree_workspace(self.views[g], DRAFT_INIT, w.B, 1) for g in self.views)
        self.vws = torch.empty(max(vb, 256), dtype=torch.uint8, device="cuda")
        self.lens0 = self.target[0].lens.clone()
        self.lens = self.target[0].lens.clone()
        self.cache0 = [(a.kp.clone(), a.vp.clone()) for a in self.target]

    def reset(self):
        self.lens.copy_(self.lens0)
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
            b.early_stop_distribution(self.mlp, self.w.B, self.W, V, K, self.q[:, 1 + rb:], rows_q * V, V, BETA, None,
                                      self.prob, self.stop)

    def target_step(self, g):
        """At draft length g: the target's tree attention, verification, update after acceptance."""
        b, v, w = self.b, self.views[g], self.w
        for a in self.target:
            b.tree_attention(v, a.code, a.B, a.H, a.d, a.q, a.kt, a.vt, a.node_stride, a.kp, a.vp, a.base, self.lens0,
                             a.head_stride, self.max_prefix, a.scale, a.out, self.ws)
        V = w.V
        b.verify_tree(v, DRAFT_INIT, w.B, V, self.tok[g], self.p, self.q, self.vi["p_target"].shape[1] * V,
                      self.vi["q_draft"].shape[1] * V, self.uag[g], self.us, 1, self.path[g], self.alen, self.new, self.vws)
        a0 = self.target[0]
        b.commit_path(v, a0.code, a0.B, a0.H, a0.d, [a.kt for a in self.target], [a.vt for a in self.target], a0.node_stride,
                      [a.kp for a in self.target], [a.vp for a in self.target], a0.base, a0.head_stride, self.max_prefix,
                      self.cap, self.path[g], self.alen, self.tok[g], self.new, 1, 1, self.lens, self.ids[g], self.n_ids)

    def snapshot(self, g):
        torch.cuda.synchronize()
        return dict(path=self.path[g].cpu().numpy(), alen=self.alen.cpu().numpy(), new=self.new.cpu().numpy(),
                    ids=self.ids[g].cpu().numpy(), n_ids=self.n_ids.cpu().numpy(), lens=self.lens.cpu().numpy(),
                    caches=[(a.kp.view(torch.int16).cpu().numpy(), a.vp.view(torch.int16).cpu().numpy()) for a in self.target],
                    target_out=[a.out[:, :, :self.off[g]].float().cpu().numpy() for a in self.target],
                    draft_out=[a.out[:, :, :self.off[g]].float().cpu().numpy() for a in self.draft])


def _run(it, level_fn, target_fn):
    """Levels until the device says stop (or the deepest level), then the target step; returns gamma, flags, results."""
    it.reset()
    flags, gamma = [], it.D
    for g in range(1, it.D + 1):
        level_fn(g)
        if g < it.D:
            torch.cuda.synchronize()
            flags.append(it.stop.cpu().numpy().copy())
            if bool(flags[-1].all()):
                gamma = g
                break
    target_fn(gamma)
    return gamma, flags, it.snapshot(gamma)


# (seed, bias added to the decision model's output, draft length at which the oracle's decisions stop the drafting):
# the biases sit between the levels' largest outputs, at least 5e-3 in the logit away from each
CASES = [(1, 0.5, 1), (4, -5.05, 2), (0, -0.87, 3), (7, 1.9, 4), (2, 0.0, 5)]


@pytest.mark.parametrize("seed,out_bias,gamma_expected", CASES)
def test_dynamic_iteration_matches_the_oracle_and_its_graph_replays(binding, oracle, H, seed, out_bias, gamma_expected):
    w = scaled(WORKLOADS["fork"], B=1, H=4, prefix_min=333, prefix_max=333, cfg_id=120)
    it = Iteration(binding, H, w, seed, out_bias)
    gamma, flags, eager = _run(it, it.draft_level, it.target_step)

    # ---- the same sequence from the oracle's functions ----
    vi, off, V = it.vi, it.off, w.V
    M = oracle.build_mask(w.branching)
    want_gamma = it.D
    for g in range(1, it.D):
        rows = vi["q_draft"][:, 1 + off[g - 1]:1 + off[g]]                       # [B][W][V]
        pr = oracle.mlp(it.ws_host, it.bs_host, oracle.decision_features(rows.reshape(-1, V), K)).reshape(w.B, it.W)
        assert np.abs(pr - BETA).min() > 1e-5, "a probability too close to the threshold for fp32 and binary64 to agree"
        st = oracle.early_stop(pr, BETA)
        assert np.array_equal(flags[g - 1], st), f"stop flags of level {g}"
        if st.all():
            want_gamma = g
            break
    assert gamma == want_gamma == gamma_expected
    n = off[gamma]
    # draft attention of every level walked: the newest rows of each level came from the slice for that level
    for l, inp in enumerate(it.draft_host):
        H.assert_close(eager["draft_out"][l].astype(np.float64), oracle.tree_attention(inp, M, n), "bf16", f"draft layer {l}")
    for l, inp in enumerate(it.target_host):
        H.assert_close(eager["target_out"][l].astype(np.float64), oracle.tree_attention(inp, M, n), "bf16", f"target layer {l}")
    tokens = np.ascontiguousarray(vi["tokens"][:, :n])
    want = oracle.verify_tree(DRAFT_INIT, w.branching[:gamma], tokens, np.ascontiguousarray(vi["p_target"][:, :1 + n]),
                              np.ascontiguousarray(vi["q_draft"][:, :1 + off[gamma - 1]]),
                              np.ascontiguousarray(vi["u_accept"][:, :n]), vi["u_sample"])
    assert np.array_equal(eager["path"], want[0]) and np.array_equal(eager["alen"], want[1]) and np.array_equal(eager["new"], want[2])
    for l, inp in enumerate(it.target_host):
        kp, vp, new_lens = oracle.commit_path(inp, gamma, n, want[0], want[1])
        assert np.array_equal(eager["caches"][l][0].view(kp.dtype), kp) and np.array_equal(eager["caches"][l][1].view(vp.dtype), vp)
        assert np.array_equal(eager["lens"], new_lens)
    want_ids, want_n = oracle.commit_ids(gamma, tokens, want[0], want[1], want[2], 1)
    assert np.array_equal(eager["ids"], want_ids) and np.array_equal(eager["n_ids"], want_n)

    # ---- the pieces captured as HIP graphs, one per level and one per draft length, replayed in the same order ----
    side = torch.cuda.Stream()
    graphs_level, graphs_target = {}, {}
    it.reset()
    with torch.cuda.stream(side):                           # warm-up of every piece on the capture stream
        for g in range(1, it.D + 1):
            it.reset()                                      # the update after acceptance moves the lengths
            it.draft_level(g)
            it.target_step(g)
    torch.cuda.synchronize()
    for g in range(1, it.D + 1):
        graphs_level[g] = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graphs_level[g]):
            it.draft_level(g)
        graphs_target[g] = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graphs_target[g]):
            it.target_step(g)
    for rep in range(2):                                    # replayed twice, with eager resets in between
        g2, flags2, replayed = _run(it, lambda g: graphs_level[g].replay(), lambda g: graphs_target[g].replay())
        assert g2 == gamma and all(np.array_equal(a, b) for a, b in zip(flags, flags2))
        for key in ("path", "alen", "new", "ids", "n_ids", "lens"):
            assert np.array_equal(eager[key], replayed[key]), (key, rep)
        for (k0, v0), (k1, v1) in zip(eager["caches"], replayed["caches"]):
            assert np.array_equal(k0, k1) and np.array_equal(v0, v1)
        for key in ("target_out", "draft_out"):
            for a, b_ in zip(eager[key], replayed[key]):
                assert np.array_equal(a, b_, equal_nan=True), (key, rep)
