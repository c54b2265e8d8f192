"""Pins for the oracle's early-stop decision models (Sec. 3.3 of arXiv 2409.10644; threshold in the caption of
Fig. 2).  None of them re-uses the oracle's own code: entropies with closed forms, top-k by exhaustive extraction,
networks small enough to evaluate by hand (tests/golden/decision_mlp_by_hand.txt), networks whose ReLUs never clip
(they collapse into one affine map, evaluated with a library matrix product), and the symmetry of the logistic."""
import os

import numpy as np
import pytest

from workloads import hidden_states, mlp_weights

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "decision_mlp_by_hand.txt")


# ---------------------------------------------------------------------------------------------------- features
def test_entropy_closed_forms(oracle):
    V, k = 1024, 4
    rows = np.zeros((4, V), dtype=np.float32)
    rows[0, 17] = 1.0                                   # a point mass: 0 nats
    rows[1, ::2] = 2.0 ** -9                            # uniform on 512 entries: ln 512
    rows[2, [3, 500, 999]] = (0.5, 0.25, 0.25)          # dyadic: 1.5 ln 2
    rows[3, :976] = 2.0 ** -10                          # 976 entries of 2^-10 (a row that does not sum to one):
    f = oracle.decision_features(rows, k)               #   -sum p ln p = 976/1024 * 10 ln 2
    assert f.shape == (4, k + 1)
    assert f[0, k] == 0.0
    assert f[1, k] == pytest.approx(9 * np.log(2.0), rel=1e-13)
    assert f[2, k] == pytest.approx(1.5 * np.log(2.0), rel=1e-14)
    assert f[3, k] == pytest.approx(976 / 1024 * 10 * np.log(2.0), rel=1e-13)
    # entropy is the LAST feature and the probabilities come first, largest first
    assert f[2, :k].tolist() == [0.5, 0.25, 0.25, 0.0]
    assert f[0, :k].tolist() == [1.0, 0.0, 0.0, 0.0]


def test_entropy_is_below_ln_n_and_additive_over_independent_parts(oracle):
    rng = np.random.default_rng(5)
    a = rng.random(16); a /= a.sum()
    b = rng.random(32); b /= b.sum()
    joint = np.outer(a, b).reshape(1, -1)               # H(a x b) = H(a) + H(b)
    k = 1
    Ha = oracle.decision_features(a.astype(np.float32)[None], k)[0, k]
    Hb = oracle.decision_features(b.astype(np.float32)[None], k)[0, k]
    Hj = oracle.decision_features(joint.astype(np.float32), k)[0, k]
    assert Hj == pytest.approx(Ha + Hb, rel=1e-6)       # fp32 rounding of the inputs only
    assert Ha < np.log(16.0) and Hb < np.log(32.0)


def _topk_by_extraction(row, k):
    """k times: take the largest remaining entry out of the row."""
    rest = [float(x) for x in row]
    out = []
    for _ in range(k):
        if not rest:
            out.append(0.0)
            continue
        best = 0
        for i in range(1, len(rest)):
            if rest[i] > rest[best]:
                best = i
        out.append(rest.pop(best))
    return out


@pytest.mark.parametrize("V,k", [(1, 1), (3, 5), (7, 7), (50, 10), (257, 16), (1000, 1)])
def test_topk_against_exhaustive_extraction(oracle, V, k):
    rng = np.random.default_rng(V * 31 + k)
    rows = rng.random((3, V)).astype(np.float32)
    rows[1, rng.integers(0, V, size=max(V // 2, 1))] = rows[1, 0]        # many duplicates
    rows[2] = 0.0
    rows[2, : max(V // 3, 1)] = 0.125                                    # fewer distinct values than k, zeros
    f = oracle.decision_features(rows, k)
    for m in range(3):
        assert f[m, :k].tolist() == _topk_by_extraction(rows[m], k)


def test_features_do_not_depend_on_token_order(oracle):
    rng = np.random.default_rng(9)
    row = rng.random(4096).astype(np.float32)
    row /= row.sum()
    perm = rng.permutation(row.size)
    a = oracle.decision_features(row[None], 10)
    b = oracle.decision_features(row[perm][None], 10)
    assert a[0, :10].tolist() == b[0, :10].tolist()
    assert a[0, 10] == pytest.approx(b[0, 10], rel=1e-13)


# ---------------------------------------------------------------------------------------------------- networks
def _read_cases():
    """Blocks of the golden file: `case NAME`, `widths a b c`, `W<l>` rows, `b<l>` row, `x` row, `P value`."""
    cases, cur = [], None
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, *rest = line.split()
            if key == "case":
                cur = dict(name=rest[0], W={}, b={})
                cases.append(cur)
            elif key == "widths":
                cur["widths"] = [int(t) for t in rest]
            elif key.startswith("W"):
                cur["W"].setdefault(int(key[1:]), []).append([float(t) for t in rest])
            elif key.startswith("b"):
                cur["b"][int(key[1:])] = [float(t) for t in rest]
            elif key == "x":
                cur["x"] = [float(t) for t in rest]
            elif key == "P":
                cur["P"] = float(rest[0])
    return cases


@pytest.mark.parametrize("case", _read_cases(), ids=lambda c: c["name"])
def test_networks_evaluated_by_hand(oracle, case):
    n = len(case["widths"]) - 1
    ws = [np.array(case["W"][l + 1], dtype=np.float32) for l in range(n)]
    bs = [np.array(case["b"][l + 1], dtype=np.float32) for l in range(n)]
    for l in range(n):
        assert ws[l].shape == (case["widths"][l + 1], case["widths"][l])
    P = oracle.mlp(ws, bs, np.array([case["x"]], dtype=np.float64))
    assert P[0] == pytest.approx(case["P"], abs=1e-7)       # ln 3 is written with 8 digits in the file


@pytest.mark.parametrize("widths", [(11, 64, 1), (768, 256, 64, 1), (5, 3, 2, 1)])
def test_network_without_clipping_is_one_affine_map(oracle, widths):
    """Positive inputs, positive weights and biases: no ReLU ever clips, so the network is sigmoid(a.x + c) with
    a, c from plain matrix products of the layers."""
    rng = np.random.default_rng(len(widths) * 1000 + widths[0])
    ws = [(rng.random((widths[l + 1], widths[l])) / widths[l]).astype(np.float32) for l in range(len(widths) - 1)]
    bs = [rng.random(widths[l + 1]).astype(np.float32) * np.float32(0.1) for l in range(len(widths) - 1)]
    ws[-1] = -ws[-1]                                        # only the output may be negative
    X = rng.random((6, widths[0]))
    A, c = np.eye(widths[0]), np.zeros(widths[0])
    for w, b in zip(ws, bs):
        A, c = w.astype(np.float64) @ A, w.astype(np.float64) @ c + b.astype(np.float64)
    z = X @ A[0] + c[0]
    assert np.all(z < 0)                                    # the case is not trivial: outputs differ from 1/2 downwards
    np.testing.assert_allclose(oracle.mlp(ws, bs, X), 1.0 / (1.0 + np.exp(-z)), rtol=1e-12)


def test_negating_the_last_layer_mirrors_the_probability(oracle):
    ws, bs = mlp_weights((17, 32, 8, 1), seed=1)
    X = hidden_states(1, 9, 17, seed=1)[0].astype(np.float64)
    P = oracle.mlp(ws, bs, X)
    Q = oracle.mlp(ws[:-1] + [-ws[-1]], bs[:-1] + [-bs[-1]], X)
    assert np.all((P > 0) & (P < 1)) and P.std() > 1e-3
    np.testing.assert_allclose(P + Q, 1.0, rtol=0, atol=1e-15)


def test_dead_hidden_layer_leaves_the_output_bias(oracle):
    ws, bs = mlp_weights((6, 10, 1), seed=2)
    bs[0] = np.full(10, -1e6, dtype=np.float32)             # every hidden unit is clipped to 0
    bs[1] = np.array([np.log(3.0)], dtype=np.float32)
    P = oracle.mlp(ws, bs, np.ones((2, 6)))
    assert P[0] == pytest.approx(0.75, abs=1e-7) and P[1] == P[0]      # sigmoid(ln 3) = 3/4


# ---------------------------------------------------------------------------------------------------- stop rule
def test_stop_only_when_every_sequence_is_below_the_threshold(oracle):
    beta = 0.4
    P = np.array([[0.1, 0.39, 0.2],          # all below: stop
                  [0.1, 0.4, 0.2],           # one AT the threshold is not "lower than" it: go on
                  [0.9, 0.0, 0.0],           # one confident sequence keeps the tree growing
                  [0.0, 0.0, 0.0]])
    assert oracle.early_stop(P, beta).tolist() == [1, 0, 0, 1]
    assert oracle.early_stop(np.array([[0.39999]]), beta).tolist() == [1]
    assert oracle.early_stop(np.array([[0.5]]), beta).tolist() == [0]
