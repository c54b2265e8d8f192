"""GPU parity of mcsd_verify_tree_sampling(MCSD_WITHOUT_REPLACEMENT) against the CPU oracle: accepted paths, lengths
and new tokens bit for bit, on trees whose sibling tokens were drawn without replacement and on inputs that break
that promise (duplicate siblings, tokens the draft row cannot produce), where the rule is still a fixed function."""
import numpy as np
import pytest
import torch

from workloads import DRAFT_INIT, TARGET_INIT, WORKLOADS, scaled, verify_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2409_10644_amd import binding as b
    return b


@pytest.fixture(scope="module")
def H():
    import gpu_helpers
    return gpu_helpers


def run(binding, H, view, mode, vi, sampling):
    p, q = H.dev(vi["p_target"]), H.dev(vi["q_draft"])
    tokens, ua, us = H.dev(vi["tokens"]), H.dev(vi["u_accept"]), H.dev(vi["u_sample"])
    B, rows_p, V = vi["p_target"].shape
    rows_q, n_new, g = vi["q_draft"].shape[1], vi["u_sample"].shape[1], view.gamma
    path = torch.full((B, g), -7, dtype=torch.int32, device="cuda")
    alen = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    new = torch.full((B, max(n_new, 1)), -7, dtype=torch.int32, device="cuda")
    ws_bytes = binding.verify_tree_workspace(view, mode, B, n_new)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda") if ws_bytes else None
    binding.verify_tree_sampling(view, mode, sampling, B, V, tokens, p, q, rows_p * V, rows_q * V, ua,
                                 us if n_new else None, n_new, path, alen, new if n_new else None, ws)
    torch.cuda.synchronize()
    return path.cpu().numpy(), alen.cpu().numpy(), new.cpu().numpy()[:, :n_new]


def check(binding, oracle, H, w, mode, gamma=None, seed=0, n_new=None, distinct=True, vi=None):
    g = w.gamma_max if gamma is None else gamma
    if vi is None:
        vi = verify_inputs(w, seed=seed, gamma=g, mode=mode, n_new=n_new, replacement=not distinct)
    v = binding.slice_mask(binding.build_mask(w.branching), g)
    got = run(binding, H, v, mode, vi, binding.MCSD_WITHOUT_REPLACEMENT)
    want = oracle.verify_tree(mode, w.branching[:g], vi["tokens"], vi["p_target"], vi["q_draft"], vi["u_accept"],
                              vi["u_sample"], replacement=False)
    for a, b in zip(got, want):
        assert np.array_equal(a, b), (a, b)
    # the plain entry point is the with-replacement scheme of the same call
    same = run(binding, H, v, mode, vi, binding.MCSD_WITH_REPLACEMENT)
    plain = H.run_verify(binding, v, mode, vi)
    for a, b in zip(same, plain):
        assert np.array_equal(a, b)
    return got, oracle.verify_tree(mode, w.branching[:g], vi["tokens"], vi["p_target"], vi["q_draft"], vi["u_accept"],
                                   vi["u_sample"])


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4", "cfg5", "fork"])
def test_configurations_bit_exact(binding, oracle, H, name, mode):
    check(binding, oracle, H, WORKLOADS[name], mode)


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_cfg3_every_gamma(binding, oracle, H, mode):
    for g in range(1, 9):
        check(binding, oracle, H, WORKLOADS["cfg3"], mode, gamma=g)


@pytest.mark.parametrize("V", [5, 255, 257, 1000, 4099, 32768, 50001])
@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_vocabulary_sizes_both_kernel_paths(binding, oracle, H, V, mode):
    """Rows in registers (V <= 32768) and streamed rows (beyond), aligned and unaligned."""
    w = scaled(WORKLOADS["cfg1"], B=6, V=V, branching=(3, 2, 2), cfg_id=62, target_sigma=1.5)
    check(binding, oracle, H, w, mode, seed=V, n_new=3)


def test_deep_rejection_chains_differ_from_the_with_replacement_rule(binding, oracle, H):
    """Independent draft and target (low acceptance), wide levels: many rounds with a shrinking draft row."""
    w = scaled(WORKLOADS["cfg1"], B=64, V=777, branching=(8, 6), cfg_id=63, target_sigma=3.0)
    got, with_rep = check(binding, oracle, H, w, DRAFT_INIT, n_new=2)
    assert (got[1] == 0).any() and (got[1] > 0).any()
    assert any(not np.array_equal(a, b) for a, b in zip(got, with_rep))       # the schemes are different rules here
    w2 = scaled(WORKLOADS["cfg1"], B=16, V=40000, branching=(8, 3), cfg_id=64, target_sigma=3.0)
    check(binding, oracle, H, w2, DRAFT_INIT, n_new=2)
    check(binding, oracle, H, w2, TARGET_INIT, n_new=4)


@pytest.mark.parametrize("V", [300, 40000])
def test_inputs_that_break_the_promise_still_follow_the_rule(binding, oracle, H, V):
    """Siblings drawn WITH replacement (duplicates) and random tokens (draft mass may be tiny or zero)."""
    w = scaled(WORKLOADS["cfg1"], B=32, V=V, branching=(6, 4), cfg_id=65, target_sigma=4.0)
    check(binding, oracle, H, w, DRAFT_INIT, n_new=2, distinct=False)
    vi = verify_inputs(w, seed=5, mode=DRAFT_INIT, n_new=2)
    rng = np.random.default_rng(5)
    vi["tokens"] = rng.integers(0, V, size=vi["tokens"].shape).astype(np.int32)
    vi["tokens"][:, 1] = vi["tokens"][:, 0]                      # a duplicate right away
    vi["q_draft"][:, :, : V // 2] = 0                             # half the vocabulary has no draft mass
    vi["q_draft"] /= vi["q_draft"].sum(-1, keepdims=True)
    check(binding, oracle, H, w, DRAFT_INIT, vi=vi)


def test_unknown_scheme_is_an_error(binding, H):
    w = WORKLOADS["cfg1"]
    vi = verify_inputs(w, seed=0)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    with pytest.raises(binding.McsdError) as e:
        run(binding, H, v, DRAFT_INIT, vi, 2)
    assert e.value.status == binding.MCSD_EINVAL
