"""GPU parity of the early-stop decision models (Sec. 3.3): mcsd_early_stop_distribution / mcsd_early_stop_hidden
through the C ABI against the CPU oracle on the same seeded inputs.

Topk values must match bit for bit (they are selected, not computed); the entropy within 2e-6 relative (fp32
logarithm per entry on the GPU, binary64 in the oracle); probabilities within 1e-5 absolute; stop flags must be
exactly the rule applied to the GPU's own fp32 probabilities, and equal to the oracle's wherever no probability lies
within 1e-5 of the threshold (the only place where the two precisions can decide differently)."""
import os

import numpy as np
import pytest
import torch

from workloads import DRAFT_INIT, WORKLOADS, hidden_states, mlp_weights, scaled, verify_inputs

pytestmark = pytest.mark.gpu

BETA = 0.4                      # caption of Fig. 2
P_ATOL = 1e-5
ENT_RTOL = 2e-6


@pytest.fixture(scope="module")
def binding():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2409_10644_amd import binding as b
    return b


def _dev_mlp(binding, ws, bs):
    return binding.make_mlp([torch.from_numpy(w).cuda() for w in ws], [torch.from_numpy(b).cuda() for b in bs])


def _run_distribution(binding, mlp, rows_t, B, W, V, k, batch_stride, row_stride, beta=BETA, features=True):
    feat = torch.full((B, W, k + 1), -7.0, dtype=torch.float32, device="cuda") if features else None
    prob = torch.full((B, W), -7.0, dtype=torch.float32, device="cuda")
    stop = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    binding.early_stop_distribution(mlp, B, W, V, k, rows_t, batch_stride, row_stride, beta, feat, prob, stop)
    torch.cuda.synchronize()
    return (feat.cpu().numpy() if features else None), prob.cpu().numpy(), stop.cpu().numpy()


def _check_against_oracle(oracle, rows, ws, bs, k, feat, prob, stop, beta=BETA):
    """rows: numpy fp32 [B][W][V] (what the GPU read)."""
    B, W, V = rows.shape
    want_f = oracle.decision_features(rows.reshape(B * W, V), k)
    want_p = oracle.mlp(ws, bs, want_f).reshape(B, W)
    if feat is not None:
        got_f = feat.reshape(B * W, k + 1).astype(np.float64)
        assert np.array_equal(got_f[:, :k], want_f[:, :k]), "Topk values differ"
        np.testing.assert_allclose(got_f[:, k], want_f[:, k], rtol=ENT_RTOL, atol=1e-9)
    assert np.all(np.isfinite(prob))
    assert np.abs(prob.astype(np.float64) - want_p).max() <= P_ATOL
    assert stop.tolist() == [int(np.all(prob[b] < np.float32(beta))) for b in range(B)]
    clear = np.abs(want_p - beta).min(axis=1) > P_ATOL
    want_s = oracle.early_stop(want_p, beta)
    assert np.array_equal(stop[clear], want_s[clear])
    return want_p, clear


# ---------------------------------------------------------------------------------------------------- type 2
@pytest.mark.parametrize("k", [1, 10, 16])
def test_distribution_model_on_every_level_of_the_fork_workload(binding, oracle, k):
    """Sec. 4.1's dynamic setting: width 16, depth 5; after each turn the 16 newest contexts' draft rows are judged."""
    w = WORKLOADS["fork"]
    vi = verify_inputs(w, seed=0, mode=DRAFT_INIT)
    q = vi["q_draft"]                                   # [1][1 + 64][V]
    qd = torch.from_numpy(q).cuda()
    ws, bs = mlp_weights((k + 1, 64, 1), seed=k, out_bias=-0.3)
    mlp = _dev_mlp(binding, ws, bs)
    Wd, V = w.branching[0], w.V
    seen = []
    for level in range(1, w.gamma_max):                 # contexts after the nodes of this level
        first = 1 + (level - 1) * Wd
        rows_t = qd[:, first:first + Wd]
        feat, prob, stop = _run_distribution(binding, mlp, rows_t, 1, Wd, V, k, q.shape[1] * V, V)
        want_p, clear = _check_against_oracle(oracle, q[:, first:first + Wd], ws, bs, k, feat, prob, stop)
        assert clear.all()
        seen.append(want_p)
    assert np.std(np.concatenate(seen)) > 1e-3          # the stand-in network is not constant


VOCABS = [1, 3, 17, 255, 1000, 2048, 4099, 32000, 50001, 262144]


@pytest.mark.parametrize("V", VOCABS)
def test_distribution_model_vocabulary_sizes_and_special_rows(binding, oracle, V):
    rng = np.random.default_rng(V)
    k, B, W = 10, 2, 5
    rows = np.zeros((B, W, V), dtype=np.float32)
    z = rng.standard_normal((V,)) * 3.0
    rows[0, 0] = (np.exp(z - z.max()) / np.exp(z - z.max()).sum()).astype(np.float32)      # peaked soft-max row
    rows[0, 1] = 1.0 / V                                                                    # all entries tie
    rows[0, 2, rng.integers(V)] = 1.0                                                       # point mass
    rows[0, 3] = rows[0, 0]
    rows[0, 3, rng.integers(0, V, size=max(V // 3, 1))] = rows[0, 0].max()                  # the maximum many times
    rows[0, 4, : max(V // 2, 1)] = rng.random(max(V // 2, 1)).astype(np.float32) * np.float32(2.0 / V)   # zeros in the tail
    # the 16 largest values all in one lane of the vectorised layout (entries 20..23 + 2048 j), every other lane small
    rows[1, 0] = rng.random(V).astype(np.float32) * np.float32(1e-6)
    lane_idx = [i for j in range(64) for i in range(20 + 2048 * j, 24 + 2048 * j) if i < V][:16]
    rows[1, 0, lane_idx] = np.float32(0.01) + np.arange(len(lane_idx), dtype=np.float32) * np.float32(1e-3)
    rows[1, 1] = np.float32(2.0) ** -12                                                     # exactly representable ties
    rows[1, 2] = rng.random(V).astype(np.float32)                                           # not a distribution: still defined
    rows[1, 3] = 0.0                                                                        # empty row
    rows[1, 4] = rows[0, 0][::-1]
    ws, bs = mlp_weights((k + 1, 32, 1), seed=3)
    mlp = _dev_mlp(binding, ws, bs)
    feat, prob, stop = _run_distribution(binding, mlp, torch.from_numpy(rows).cuda(), B, W, V, k, W * V, V)
    _check_against_oracle(oracle, rows, ws, bs, k, feat, prob, stop)


@pytest.mark.parametrize("offset,pad", [(0, 0), (1, 0), (0, 3), (4, 8), (2, 6)])
def test_distribution_model_strides_and_alignment(binding, oracle, offset, pad):
    """Rows inside a larger buffer: padded rows, a gap between the trees, a base that is not 16-byte aligned."""
    rng = np.random.default_rng(offset * 10 + pad)
    B, W, V, k = 3, 4, 1000, 7
    row_stride, batch_stride = V + pad, W * (V + pad) + 2 * pad + 4
    buf = np.full(offset + B * batch_stride + 16, np.float32(99.0), dtype=np.float32)        # poison between the rows
    rows = np.empty((B, W, V), dtype=np.float32)
    for b in range(B):
        for wv in range(W):
            r = rng.random(V).astype(np.float32)
            r /= r.sum()
            rows[b, wv] = r
            o = offset + b * batch_stride + wv * row_stride
            buf[o:o + V] = r
    ws, bs = mlp_weights((k + 1, 48, 1), seed=5)
    mlp = _dev_mlp(binding, ws, bs)
    t = torch.from_numpy(buf).cuda()
    feat, prob, stop = _run_distribution(binding, mlp, t[offset:], B, W, V, k, batch_stride, row_stride)
    _check_against_oracle(oracle, rows, ws, bs, k, feat, prob, stop)


def test_distribution_model_many_trees_three_layers_no_feature_output(binding, oracle):
    w = scaled(WORKLOADS["fork"], B=40, V=4000, branching=(16, 1), cfg_id=61)
    vi = verify_inputs(w, seed=2, mode=DRAFT_INIT)
    q = vi["q_draft"]                                   # [40][1 + 16][V]
    k = 12
    ws, bs = mlp_weights((k + 1, 128, 16, 1), seed=8, out_bias=-0.2)
    mlp = _dev_mlp(binding, ws, bs)
    qd = torch.from_numpy(q).cuda()
    _, prob, stop = _run_distribution(binding, mlp, qd[:, 1:], w.B, 16, w.V, k, q.shape[1] * w.V, w.V, features=False)
    want_p, clear = _check_against_oracle(oracle, q[:, 1:], ws, bs, k, None, prob, stop)
    assert clear.sum() >= w.B - 2
    binding.early_stop_distribution(mlp, 0, 16, w.V, k, None, 0, 0, BETA, None, None, None)    # B = 0: nothing to do


# ---------------------------------------------------------------------------------------------------- type 1
@pytest.mark.parametrize("widths,B,W", [((768, 256, 64, 1), 1, 16), ((2048, 512, 128, 1), 3, 5), ((5, 3, 2, 1), 2, 2),
                                        ((8192, 512, 1), 1, 7), ((16, 1), 4, 4), ((768, 256, 64, 1), 33, 16),
                                        ((100, 37, 1), 1, 1)])
def test_hidden_state_model(binding, oracle, widths, B, W):
    ws, bs = mlp_weights(widths, seed=len(widths) + widths[0], out_bias=-0.4)
    x = hidden_states(B, W, widths[0], seed=widths[0])
    mlp = _dev_mlp(binding, ws, bs)
    prob = torch.full((B, W), -7.0, dtype=torch.float32, device="cuda")
    stop = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    binding.early_stop_hidden(mlp, B, W, torch.from_numpy(x).cuda(), W * widths[0], widths[0], BETA, prob, stop)
    torch.cuda.synchronize()
    prob, stop = prob.cpu().numpy(), stop.cpu().numpy()
    want = oracle.mlp(ws, bs, x.reshape(B * W, -1).astype(np.float64)).reshape(B, W)
    assert np.abs(prob - want).max() <= 1e-6            # fp32 multiply-adds with tree-combined partial sums against the binary64 oracle
    assert stop.tolist() == [int(np.all(prob[b] < np.float32(BETA))) for b in range(B)]
    clear = np.abs(want - BETA).min(axis=1) > P_ATOL
    assert np.array_equal(stop[clear], oracle.early_stop(want, BETA)[clear])
    assert want.std() > 1e-3 or B * W == 1


def test_hidden_state_model_padded_rows(binding, oracle):
    B, W, n_in, pad = 2, 3, 40, 5
    ws, bs = mlp_weights((n_in, 16, 8, 1), seed=11)
    x = hidden_states(B, W, n_in + pad, seed=4)          # the last `pad` entries of every row are not inputs
    mlp = _dev_mlp(binding, ws, bs)
    prob = torch.zeros((B, W), dtype=torch.float32, device="cuda")
    stop = torch.zeros((B,), dtype=torch.int32, device="cuda")
    binding.early_stop_hidden(mlp, B, W, torch.from_numpy(x).cuda(), W * (n_in + pad), n_in + pad, BETA, prob, stop)
    torch.cuda.synchronize()
    want = oracle.mlp(ws, bs, x[:, :, :n_in].reshape(B * W, n_in).astype(np.float64)).reshape(B, W)
    assert np.abs(prob.cpu().numpy() - want).max() <= 1e-6


def test_networks_evaluated_by_hand_on_the_gpu(binding):
    from test_oracle_decision import _read_cases
    for case in _read_cases():
        n = len(case["widths"]) - 1
        ws = [np.array(case["W"][l + 1], dtype=np.float32) for l in range(n)]
        bs = [np.array(case["b"][l + 1], dtype=np.float32) for l in range(n)]
        mlp = _dev_mlp(binding, ws, bs)
        x = torch.tensor([case["x"]], dtype=torch.float32, device="cuda")
        prob = torch.zeros((1, 1), dtype=torch.float32, device="cuda")
        stop = torch.zeros((1,), dtype=torch.int32, device="cuda")
        binding.early_stop_hidden(mlp, 1, 1, x, len(case["x"]), len(case["x"]), BETA, prob, stop)
        torch.cuda.synchronize()
        assert abs(float(prob[0, 0]) - case["P"]) <= 2e-7, case["name"]
        assert int(stop[0]) == int(case["P"] < BETA)


def test_stop_rule_including_a_probability_exactly_at_the_threshold(binding):
    """One input, weight 1, bias 0: P = sigmoid(x); x = 0 gives exactly 1/2."""
    mlp = _dev_mlp(binding, [np.ones((1, 1), dtype=np.float32)], [np.zeros(1, dtype=np.float32)])
    x = torch.tensor([[-2.0, -3.0, -1.0],        # all below 1/2: stop
                      [-2.0, 0.0, -1.0],         # one exactly at the threshold is not below it
                      [-2.0, 4.0, -1.0],
                      [-9.0, -9.0, -9.0]], dtype=torch.float32, device="cuda")
    prob = torch.zeros((4, 3), dtype=torch.float32, device="cuda")
    stop = torch.full((4,), -7, dtype=torch.int32, device="cuda")
    binding.early_stop_hidden(mlp, 4, 3, x, 3, 1, 0.5, prob, stop)
    torch.cuda.synchronize()
    assert float(prob[1, 1]) == 0.5
    assert stop.tolist() == [1, 0, 0, 1]
