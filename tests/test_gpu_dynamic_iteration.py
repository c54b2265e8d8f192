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

from workloads import DRAFT_INIT, WORKLOADS, scaled

pytestmark = pytest.mark.gpu

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


# (seed, bias added to the decision model's output, draft length at which the oracle's decisions stop the drafting):
# the biases sit between the levels' largest outputs, at least 5e-3 in the logit away from each
CASES = [(1, 0.5, 1), (4, -5.05, 2), (0, -0.87, 3), (7, 1.9, 4), (2, 0.0, 5)]


@pytest.mark.parametrize("seed,out_bias,gamma_expected", CASES)
def test_dynamic_iteration_matches_the_oracle_and_its_graph_replays(binding, oracle, H, seed, out_bias, gamma_expected):
    w = scaled(WORKLOADS["fork"], B=1, H=4, prefix_min=333, prefix_max=333, cfg_id=120)
    it = H.DynamicIteration(binding, w, w, N_DRAFT_LAYERS, N_TARGET_LAYERS, seed, out_bias)
    BETA, K = it.BETA, it.K
    gamma, flags = it.run(it.draft_level, it.target_step)
    eager = it.snapshot(gamma)

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
    graphs_level, graphs_target = it.capture()
    for rep in range(2):                                    # replayed twice, with eager resets in between
        g2, flags2 = it.run(lambda g: graphs_level[g].replay(), lambda g: graphs_target[g].replay())
        replayed = it.snapshot(g2)
        assert g2 == gamma and all(np.array_equal(a, b) for a, b in zip(flags, flags2))
        for key in ("path", "alen", "new", "ids", "n_ids", "lens"):
            assert np.array_equal(eager[key], replayed[key]), (key, rep)
        for (k0, v0), (k1, v1) in zip(eager["caches"], replayed["caches"]):
            assert np.array_equal(k0, k1) and np.array_equal(v0, v1)
        for key in ("target_out", "draft_out"):
            for a, b_ in zip(eager[key], replayed[key]):
                assert np.array_equal(a, b_, equal_nan=True), (key, rep)
