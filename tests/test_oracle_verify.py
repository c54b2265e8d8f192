"""Pins for the oracle's multi-candidate verification (no GPU).

The expectations come from: exact rational arithmetic (fractions.Fraction) on dyadic inputs where every
floating-point operation of the oracle is exact, the textbook single-candidate rule, hand-derived closed
forms for the output law, and brute-force enumeration over token assignments with seeded Monte-Carlo
integration over the uniforms (error bound computed, 6 sigma).
"""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

DRAFT, TARGET = 0, 1


# ----------------------------------------------------------------------------------------------
# summation order and sampler
# ----------------------------------------------------------------------------------------------
def test_tree_sum_is_the_balanced_tree_not_a_linear_scan(oracle):
    e = 2.0 ** -53
    # balanced: (1 + e) + (e + e) = 1 + 2^-52 (first add ties to even -> 1.0); linear scan gives 1.0
    assert oracle.tree_sum(np.array([1.0, e, e, e])) == 1.0 + 2.0 ** -52
    # padding to a power of two happens on the right: [1, e, e] -> (1 + e) + (e + 0) = 1.0 (tie to even)
    assert oracle.tree_sum(np.array([1.0, e, e])) == 1.0
    # (e + e) + (1 + 0) is exact
    assert oracle.tree_sum(np.array([e, e, 1.0])) == 1.0 + 2.0 ** -52


def test_tree_sum_exact_on_integers(oracle):
    rng = np.random.default_rng(1)
    for V in (1, 2, 3, 7, 1000, 1024, 1025):
        a = rng.integers(0, 1000, size=V).astype(np.float64)
        assert oracle.tree_sum(a) == float(a.sum())


def _linear_cdf_sample(weights, u_frac):
    """Smallest t with u*S < w_0 + ... + w_t, exact rational arithmetic."""
    S = sum(weights)
    thr = u_frac * S
    acc = Fraction(0)
    for t, w in enumerate(weights):
        acc += w
        if thr < acc:
            return t
    raise AssertionError("u must be < 1")


def test_tree_sample_equals_linear_cdf_on_integer_weights(oracle):
    rng = np.random.default_rng(2)
    for V in (1, 2, 5, 8, 37, 64, 100):
        w = rng.integers(0, 6, size=V)
        if w.sum() == 0:
            w[V // 2] = 3
        a = w.astype(np.float64)
        fr = [Fraction(int(x)) for x in w]
        for u in np.concatenate([rng.random(40, dtype=np.float32), np.float32([0.0, 0.5, 1 - 2.0 ** -24])]):
            uf = Fraction(float(u))               # a float32 is an exact dyadic rational
            got = oracle.tree_sample(a, float(u))
            assert got == _linear_cdf_sample(fr, uf)
            assert w[got] > 0                      # zero-weight entries are never returned


def test_tree_sample_extremes(oracle):
    a = np.array([0.0, 0.0, 0.25, 0.0, 0.5, 0.25, 0.0])
    assert oracle.tree_sample(a, 0.0) == 2
    assert oracle.tree_sample(a, float(np.float32(1 - 2.0 ** -24))) == 5
    assert oracle.tree_sample(np.zeros(5), 0.3) == 0          # all-zero: index 0 by convention


# ----------------------------------------------------------------------------------------------
# exact rational model of the textbook rule (normalised residuals, division allowed)
# ----------------------------------------------------------------------------------------------
def _children(br, ctx, lvl):
    """ctx = -1 (prefix end, lvl 0) or node id at 1-based level lvl.  Independent of the oracle: uses
    explicit (level, in-level index) pairs."""
    sizes, n = [], 1
    for b in br:
        n *= b
        sizes.append(n)
    off = [0]
    for s in sizes:
        off.append(off[-1] + s)
    if ctx < 0:
        return list(range(br[0]))
    a = ctx - off[lvl - 1]
    return [off[lvl] + a * br[lvl] + c for c in range(br[lvl])]


def _textbook_walk(br, start, start_lvl, tokens, p, q, ua):
    """Recursive rejection sampling with exact fractions.  Returns (path, terminal distribution)."""
    cur, lvl, path = start, start_lvl, []
    G = len(br)
    while lvl < G:
        dist = list(p[cur + 1])
        qq = q[cur + 1]
        acc = None
        for c in _children(br, cur, lvl):
            x = tokens[c]
            if qq[x] == 0:
                ok = dist[x] > 0
            else:
                ok = ua[c] < min(Fraction(1), dist[x] / qq[x])
            if ok:
                acc = c
                break
            res = [max(a - b, Fraction(0)) for a, b in zip(dist, qq)]
            tot = sum(res)
            if tot == 0:
                # residual vanished: further candidates cannot be accepted; fall back to the target row
                dist = None
                break
            dist = [r / tot for r in res]
        if acc is None:
            if dist is None:
                return path, list(p[cur + 1])
            return path, dist
        path.append(acc)
        cur, lvl = acc, lvl + 1
    return path, list(p[cur + 1])


def _textbook_verify(mode, br, tokens, p, q, ua, us):
    if mode == DRAFT:
        path, term = _textbook_walk(br, -1, 0, tokens, p, q, ua)
    else:
        best = None
        for i in range(br[0]):
            pth, term_i = _textbook_walk(br, i, 1, tokens, p, q, ua)
            if best is None or 1 + len(pth) > len(best[0]):
                best = ([i] + pth, term_i)
        path, term = best
    return path, [_linear_cdf_sample(term, u) for u in us]


def _dyadic_rows(rng, rows, V, denom=64):
    """Probability rows whose entries are multiples of 1/denom (exact in fp32), some of them zero."""
    out = np.zeros((rows, V), dtype=np.float32)
    for r in range(rows):
        cuts = np.sort(rng.integers(0, denom + 1, size=V - 1))
        parts = np.diff(np.concatenate([[0], cuts, [denom]]))
        out[r] = rng.permutation(parts) / denom
    return out


@pytest.mark.parametrize("mode", [DRAFT, TARGET])
@pytest.mark.parametrize("br", [(1, 1, 1), (2, 2), (3, 2, 1), (2, 1, 2), (4,)])
def test_exact_agreement_with_rational_textbook_rule(oracle, mode, br):
    """On dyadic inputs every oracle operation is exact, so the unnormalised-residual formulation must
    reproduce the normalised textbook rule decision for decision, and the tree sampler the linear CDF."""
    rng = np.random.default_rng(hash((mode,) + tuple(br)) % (2 ** 32))
    V, G = 8, len(br)
    sizes = np.cumprod(br)
    N, Nin = int(sizes.sum()), int(sizes[:-1].sum())
    B, n_new = 300, 2
    p = np.stack([_dyadic_rows(rng, 1 + N, V, 64) for _ in range(B)])
    q = np.stack([_dyadic_rows(rng, 1 + Nin, V, 16) for _ in range(B)])
    tokens = rng.integers(0, V, size=(B, N)).astype(np.int32)
    ua = (rng.integers(0, 256, size=(B, N)) / 256).astype(np.float32)
    us = (rng.integers(0, 4096, size=(B, n_new)) / 4096).astype(np.float32)
    path, alen, new = oracle.verify_tree(mode, br, tokens, p, q, ua, us)
    lens_seen = set()
    for b in range(B):
        pf = [[Fraction(float(x)) for x in row] for row in p[b]]
        qf = [[Fraction(float(x)) for x in row] for row in q[b]]
        want_path, want_new = _textbook_verify(mode, br, tokens[b].tolist(), pf, qf,
                                               [Fraction(float(x)) for x in ua[b]],
                                               [Fraction(float(x)) for x in us[b]])
        assert alen[b] == len(want_path)
        assert path[b, :alen[b]].tolist() == want_path
        assert np.all(path[b, alen[b]:] == -1)
        assert new[b].tolist() == want_new
        lens_seen.add(int(alen[b]))
    if not (mode == TARGET and G == 1):
        assert len(lens_seen) >= 2      # the cases exercise both acceptance and rejection


def test_single_candidate_chain_is_textbook_speculative_sampling(oracle):
    """k = 1 (Sec. 2.1): accept while u < p(x)/q(x); at the first rejection sample from norm(max(p-q,0));
    after gamma accepts sample the bonus token from the target row.  Real-valued (non-dyadic) inputs:
    round 0 of every context uses S = 1, so accept/reject decisions are exact comparisons in binary64."""
    rng = np.random.default_rng(5)
    G, V, B = 4, 50, 400
    br = (1,) * G
    logits_p = rng.standard_normal((B, 1 + G, V)) * 2
    logits_q = logits_p[:, :G] + rng.standard_normal((B, G, V))
    sm = lambda z: (np.exp(z - z.max(-1, keepdims=True)) / np.exp(z - z.max(-1, keepdims=True)).sum(-1, keepdims=True))
    p = sm(logits_p).astype(np.float32)
    q = sm(logits_q).astype(np.float32)
    tokens = np.stack([[rng.choice(V, p=q[b, l].astype(np.float64) / q[b, l].astype(np.float64).sum())
                        for l in range(G)] for b in range(B)]).astype(np.int32)
    ua = rng.random((B, G), dtype=np.float32)
    us = rng.random((B, 1), dtype=np.float32)
    path, alen, new = oracle.verify_tree(DRAFT, br, tokens, p, q, ua, us)
    mismatched_tokens = 0
    for b in range(B):
        n = 0
        while n < G:
            x = tokens[b, n]
            # textbook test with a division, in binary64
            if not (float(ua[b, n]) * float(q[b, n, x]) < float(p[b, n, x])):
                break
            n += 1
        assert alen[b] == n
        assert path[b, :n].tolist() == list(range(n))
        if n < G:
            res = np.maximum(p[b, n].astype(np.float64) - q[b, n].astype(np.float64), 0)
        else:
            res = p[b, G].astype(np.float64)
        cdf = np.cumsum(res)
        t = int(np.searchsorted(cdf, float(us[b, 0]) * cdf[-1], side="right"))
        mismatched_tokens += int(t != new[b, 0])
        assert res[new[b, 0]] > 0
    # the linear scan and the tree descent round differently; they may disagree only when u*S falls within
    # rounding distance of a CDF step (probability ~ V * 2^-52 per draw)
    assert mismatched_tokens == 0
    assert 0 < alen.mean() < G


def test_p_equals_q_accepts_everything_and_disjoint_rejects_everything(oracle):
    rng = np.random.default_rng(6)
    br, V, B = (2, 2), 16, 50
    N, Nin = 6, 2
    rows = _dyadic_rows(rng, B * (1 + N), V, 64).reshape(B, 1 + N, V)
    tokens = np.zeros((B, N), dtype=np.int32)
    for b in range(B):
        for node in range(N):
            ctx = 0 if node < 2 else 1 + (node - 2) // 2
            tokens[b, node] = rng.choice(np.nonzero(rows[b, ctx])[0])
    ua = rng.random((B, N), dtype=np.float32)
    us = rng.random((B, 1), dtype=np.float32)
    path, alen, _ = oracle.verify_tree(DRAFT, br, tokens, rows, rows[:, :1 + Nin].copy(), ua, us)
    assert np.all(alen == 2) and np.all(path[:, 0] == 0) and np.all(path[:, 1] == 2)   # first child every time
    # disjoint supports: p on even tokens, q on odd tokens -> every candidate rejected, new token ~ p
    p = np.zeros((B, 1 + N, V), dtype=np.float32)
    q = np.zeros((B, 1 + Nin, V), dtype=np.float32)
    p[:, :, 0::2] = 1 / 8
    q[:, :, 1::2] = 1 / 8
    tokens = (2 * rng.integers(0, 8, size=(B, N)) + 1).astype(np.int32)
    path, alen, new = oracle.verify_tree(DRAFT, br, tokens, p, q, ua, us)
    assert np.all(alen == 0) and np.all(path == -1)
    want = 2 * np.floor(us[:, 0].astype(np.float64) * 8).astype(int)     # inverse CDF of uniform over evens
    assert np.array_equal(new[:, 0], want)


def test_vanished_residual_falls_back_to_target_row(oracle):
    """A rejected candidate leaves max(p - q, 0); when that is identically zero the remaining siblings are
    rejected as well and the new token is drawn from the context's unmodified target row."""
    V = 4
    p = np.array([[[0.5, 0.5, 0.0, 0.0], [0.25, 0.25, 0.25, 0.25]]], dtype=np.float32)      # rows 0, 1
    q = np.array([[[0.5, 0.25, 0.25, 0.0]]], dtype=np.float32)
    # candidate token 2: p(2) = 0 -> rejected; residual = max(p - q, 0) = [0, .25, 0, 0] -> new token is 1
    path, alen, new = oracle.verify_tree(DRAFT, (1,), np.array([[2]], np.int32), p, q,
                                         np.array([[0.0]], np.float32), np.array([[0.99]], np.float32))
    assert alen[0] == 0 and new[0, 0] == 1
    # p <= q everywhere on a rejected candidate: p == q on {0,1} but candidate 3 has q(3) > 0 = p(3)
    p2 = np.array([[[0.5, 0.25, 0.0, 0.0], [0.25] * 4, [0.25] * 4]], dtype=np.float32)     # row 0 unnormalised on purpose
    q2 = np.array([[[0.5, 0.25, 0.0, 0.25]]], dtype=np.float32)
    path, alen, new = oracle.verify_tree(DRAFT, (2,), np.array([[3, 0]], np.int32), p2, q2,
                                         np.array([[0.0, 0.0]], np.float32), np.array([[0.7]], np.float32))
    # residual is identically zero: the second candidate (token 0) is rejected too (0 < 0 is false) and the
    # new token comes from the unmodified target row: CDF .5/.75 of total .75 -> u = 0.7 -> index 1
    assert alen[0] == 0 and new[0, 0] == 1


# ----------------------------------------------------------------------------------------------
# output law: exact enumeration over token assignments, seeded Monte-Carlo integration over uniforms
# ----------------------------------------------------------------------------------------------
def _law_of_first_emitted(oracle, mode, br, p_fn, q_fn, V, M, first_two=False, seed=0, replacement=True):
    """Enumerate every token assignment, weighted by its probability under the generation process, and
    integrate over the uniforms with M seeded random draws per assignment.  Rows are functions of the
    token history, so equal histories have equal distributions.  Returns (law of the first emitted token,
    joint law of the first two when at least one node was accepted, 6-sigma bound of the sampling error)."""
    sizes = np.cumprod(br)
    N, Nin = int(sizes.sum()), int(sizes[:-1].sum())
    off = np.concatenate([[0], np.cumsum(sizes)])
    parent = [-1] * N
    for l in range(1, len(br)):
        for a in range(sizes[l]):
            parent[off[l] + a] = off[l - 1] + a // br[l]
    n_new = 2 if first_two else 1
    rng = np.random.default_rng(seed)
    law1 = np.zeros(V)
    law2 = np.zeros((V, V))
    var = 0.0
    for toks in product(range(V), repeat=N):
        hist = []
        for i in range(N):
            h, j = [], i
            while j >= 0:
                h.append(toks[j])
                j = parent[j]
            hist.append(tuple(h[::-1]))
        p_rows = np.stack([p_fn(())] + [p_fn(hist[i]) for i in range(N)]).astype(np.float32)
        q_rows = np.stack([q_fn(())] + [q_fn(hist[i]) for i in range(Nin)]).astype(np.float32)
        weight = 1.0
        gone = {}                                  # without replacement: mass already drawn by earlier siblings
        for i in range(N):
            src = p_fn(()) if (mode == TARGET and parent[i] < 0) else q_fn(hist[i][:-1])
            if replacement:
                weight *= float(np.float32(src[toks[i]]))
            else:
                taken = gone.setdefault(parent[i], [])
                if toks[i] in taken:
                    weight = 0.0
                    break
                left = 1.0 - sum(float(np.float32(src[t])) for t in taken)
                weight *= float(np.float32(src[toks[i]])) / left if left > 0 else 0.0
                taken.append(toks[i])
        if weight == 0.0:
            continue
        ua = rng.random((M, N), dtype=np.float32)
        us = rng.random((M, n_new), dtype=np.float32)
        path, alen, new = oracle.verify_tree(mode, br, np.tile(np.int32(toks), (M, 1)),
                                             np.tile(p_rows, (M, 1, 1)), np.tile(q_rows, (M, 1, 1)), ua, us,
                                             replacement=replacement)
        tok_arr = np.int32(toks)
        first = np.where(alen > 0, tok_arr[np.maximum(path[:, 0], 0)], new[:, 0])
        np.add.at(law1, first, weight / M)
        var += 0.25 * weight * weight / M
        if first_two:
            second = np.where(alen > 1, tok_arr[np.maximum(path[:, 1], 0)], new[:, 0])
            ok = alen >= 1
            np.add.at(law2, (first[ok], second[ok]), weight / M)
    return law1, law2, 6.0 * np.sqrt(var) + 1e-6


def _rows_by_history(V, seed):
    cache = {}

    def fn(hist):
        if hist not in cache:
            r = np.random.default_rng([seed, len(hist)] + [int(t) for t in hist])
            w = r.random(V) + 0.05
            if r.random() < 0.5:
                w[r.integers(V)] = 0.0
            cache[hist] = (w / w.sum()).astype(np.float32)
        return cache[hist]
    return fn


@pytest.mark.parametrize("br", [(1,), (2,), (3,), (4,), (1, 1), (2, 2)])
def test_draft_init_first_token_law_is_the_target_law(oracle, br):
    """Losslessness (Sec. 2.1): the first emitted token is distributed as the target row of the prefix end,
    for any number of candidates per context and any depth."""
    V = 3
    p_fn, q_fn = _rows_by_history(V, 11), _rows_by_history(V, 12)
    N = int(np.cumprod(br).sum())
    M = {1: 1000000, 2: 300000}.get(N, 60000 if N <= 4 else 6000)
    law, _, tol = _law_of_first_emitted(oracle, DRAFT, br, p_fn, q_fn, V, M)
    target = p_fn(()).astype(np.float64)
    assert tol < 5e-3
    assert abs(law.sum() - 1.0) < 1e-5
    assert np.max(np.abs(law - target / target.sum())) < tol


def test_the_law_pin_can_tell_wrong_rules():
    """Sanity of the pin itself, on the same rows: two plausible mistakes -- drawing the new token from the
    plain target row after a rejection, or never updating the residual between siblings -- move the
    first-token law of a one-level tree by far more than the sampling tolerance (5e-3)."""
    V = 3
    p_fn, q_fn = _rows_by_history(V, 11), _rows_by_history(V, 12)
    p0, q0 = p_fn(()).astype(np.float64), q_fn(()).astype(np.float64)
    acc = np.minimum(p0, q0)                          # P(candidate = x and accepted)
    wrong1 = acc + (1 - acc.sum()) * p0               # k = 1, new token ~ p instead of the residual
    assert np.max(np.abs(wrong1 - p0)) > 0.02
    res = np.maximum(p0 - q0, 0)
    res /= res.sum()
    rej = 1 - acc.sum()
    wrong2 = acc + rej * acc + rej * rej * res        # k = 2, second sibling tested against p, not the residual
    assert np.max(np.abs(wrong2 - p0)) > 0.02


def test_chain_first_two_tokens_follow_the_target_chain_rule(oracle):
    """(1,1) chain: the first token has law p(.); when the first draft token x1 is accepted the next emitted
    token is ~ p(. | x1):  P(x1 accepted, second = x2) = min(p, q)(x1) * p(x2 | x1)."""
    V = 3
    p_fn, q_fn = _rows_by_history(V, 21), _rows_by_history(V, 22)
    law1, law2, tol = _law_of_first_emitted(oracle, DRAFT, (1, 1), p_fn, q_fn, V, 200000, first_two=True)
    p0, q0 = p_fn(()).astype(np.float64), q_fn(()).astype(np.float64)
    assert np.max(np.abs(law1 - p0)) < tol
    for x1 in range(V):
        want = min(p0[x1], q0[x1]) * p_fn((x1,)).astype(np.float64)
        assert np.max(np.abs(law2[x1] - want)) < tol


def test_target_init_width_one_is_lossless_width_two_is_biased(oracle):
    """Sec. 3.1 / Sec. 4.1: with one target-initialised token the output law stays the target's; with two,
    picking the root with the longest accepted continuation tilts it towards roots whose continuation is
    accepted more often.  For the tree (2,1) the tilt has a closed form derived by hand:
        P_out(t) = p(t) * (1 - Abar + A(t)),   A(t) = sum_x min(p_t(x), q_t(x)),   Abar = sum_t p(t) A(t)
    (root 0 wins unless its child is rejected and root 1's child is accepted)."""
    V = 3
    p_fn, q_fn = _rows_by_history(V, 31), _rows_by_history(V, 32)
    p0 = p_fn(()).astype(np.float64)
    law_w1, _, tol1 = _law_of_first_emitted(oracle, TARGET, (1, 1), p_fn, q_fn, V, 200000)
    assert np.max(np.abs(law_w1 - p0)) < tol1
    law_w2, _, tol2 = _law_of_first_emitted(oracle, TARGET, (2, 1), p_fn, q_fn, V, 60000)
    A = np.array([np.minimum(p_fn((t,)).astype(np.float64), q_fn((t,)).astype(np.float64)).sum() for t in range(V)])
    Abar = float((p0 * A).sum())
    want = p0 * (1 - Abar + A)
    assert tol2 < 5e-3
    assert np.max(np.abs(law_w2 - want)) < tol2
    assert np.max(np.abs(want - p0)) > 0.02           # the bias is real on these rows ...
    assert np.max(np.abs(law_w2 - p0)) > 0.015        # ... and the oracle exhibits it


def test_target_init_tie_goes_to_the_lowest_root(oracle):
    V = 4
    br = (3, 1)
    N = 6
    p = np.full((1, 1 + N, V), 0.25, dtype=np.float32)
    q = np.full((1, 1 + 3, V), 0.25, dtype=np.float32)
    tokens = np.array([[0, 1, 2, 3, 3, 3]], dtype=np.int32)
    us = np.array([[0.1, 0.6, 0.9]], dtype=np.float32)
    # p == q: every child is accepted -> three paths of length 2 -> root 0 wins
    path, alen, new = oracle.verify_tree(TARGET, br, tokens, p, q, np.full((1, N), 0.5, np.float32), us)
    assert alen[0] == 2 and path[0].tolist() == [0, 3]
    assert new[0].tolist() == [0, 2, 3]               # i.i.d. draws from the uniform target row after node 3
    # make root 0's child unacceptable (p(3) = 0 in root 0's context): roots 1 and 2 tie -> root 1
    p2 = p.copy()
    p2[0, 1] = [1 / 3, 1 / 3, 1 / 3, 0.0]
    path, alen, _ = oracle.verify_tree(TARGET, br, tokens, p2, q, np.full((1, N), 0.5, np.float32), us)
    assert alen[0] == 2 and path[0].tolist() == [1, 4]
    # gamma = 1: nothing to test, root 0, new tokens from the row after it
    path, alen, new = oracle.verify_tree(TARGET, (3,), tokens[:, :3], p[:, :4], q[:, :1],
                                         np.full((1, 3), 0.5, np.float32), us)
    assert alen[0] == 1 and path[0].tolist() == [0] and new[0].tolist() == [0, 2, 3]


def test_workload_generator_shapes_and_acceptance(oracle):
    from workloads import WORKLOADS, scaled, verify_inputs
    w = scaled(WORKLOADS["cfg2"], V=2000, B=8)
    vi = verify_inputs(w, seed=0)
    assert vi["p_target"].shape == (8, 45, 2000) and vi["q_draft"].shape == (8, 29, 2000)
    path, alen, new = oracle.verify_tree(vi["mode"], w.branching, vi["tokens"], vi["p_target"], vi["q_draft"],
                                         vi["u_accept"], vi["u_sample"])
    assert alen.min() >= 0 and alen.max() <= 4 and new.min() >= 0 and new.max() < 2000
    for b in range(8):
        assert np.all(path[b, :alen[b]] >= 0) and np.all(path[b, alen[b]:] == -1)


def test_one_hot_target_rows_reduce_to_arg_max_matching(oracle):
    """Greedy decoding (temperature 0, Sec. 4.1): with one-hot target rows the rejection rule accepts a candidate
    exactly when it is the target's arg-max, whatever the draft row and the uniform, and the new token is the
    arg-max of the row the walk ends on."""
    rng = np.random.default_rng(21)
    br, V, B = (3, 2, 2), 50, 40
    parent, level = oracle.tree_tables(br)
    N, Nin = len(parent), int((level < 3).sum())
    top = rng.integers(0, V, size=(B, 1 + N))
    p = np.zeros((B, 1 + N, V), dtype=np.float32)
    np.put_along_axis(p, top[..., None], 1.0, axis=-1)
    q = rng.random((B, 1 + Nin, V)).astype(np.float32)
    q /= q.sum(-1, keepdims=True)
    tokens = rng.integers(0, V, size=(B, N)).astype(np.int32)
    for b in range(B):
        for node in range(N):
            if rng.random() < 0.5:
                tokens[b, node] = top[b, 1 + parent[node]]
    ua = rng.random((B, N), dtype=np.float32)
    us = rng.random((B, 1), dtype=np.float32)
    path, alen, new = oracle.verify_tree(0, br, tokens, p, q.astype(np.float32), ua, us)
    for b in range(B):
        # textbook greedy walk: first child (in node order) whose token is the arg-max of its context
        cur, want = -1, []
        for lv in range(3):
            kids = [n for n in range(N) if parent[n] == cur and level[n] == lv + 1]
            hit = [n for n in kids if tokens[b, n] == top[b, 1 + cur]]
            if not hit:
                break
            cur = hit[0]
            want.append(cur)
        assert alen[b] == len(want) and path[b, :len(want)].tolist() == want
        assert new[b, 0] == top[b, 1 + cur]
    assert len(set(alen.tolist())) >= 3


# ----------------------------------------------------------------------------------------------
# candidates drawn without replacement (a variant next to the paper's setting; the rule is the one of
# multi-candidate speculative sampling: after a rejection the draft row also loses the rejected token)
# ----------------------------------------------------------------------------------------------
def _textbook_walk_distinct(br, start, start_lvl, tokens, p, q, ua):
    """The normalised rule in exact fractions: accept with probability min(1, p(x)/q(x)); after a rejection
    p <- norm(max(p - q, 0)), q(x) <- 0, q <- norm(q)."""
    cur, lvl, path = start, start_lvl, []
    while lvl < len(br):
        dist, qq = list(p[cur + 1]), list(q[cur + 1])
        acc = None
        for c in _children(br, cur, lvl):
            x = tokens[c]
            assert qq[x] > 0                            # valid input: a token the current draft row can produce
            if ua[c] < min(Fraction(1), dist[x] / qq[x]):
                acc = c
                break
            res = [max(a - b, Fraction(0)) for a, b in zip(dist, qq)]
            tot = sum(res)
            assert tot > 0
            dist = [r / tot for r in res]
            qq[x] = Fraction(0)
            left = sum(qq)
            qq = [v / left for v in qq]
        if acc is None:
            return path, dist
        path.append(acc)
        cur, lvl = acc, lvl + 1
    return path, list(p[cur + 1])


@pytest.mark.parametrize("mode", [DRAFT, TARGET])
@pytest.mark.parametrize("br", [(2, 2), (3, 2, 1), (2, 1, 3), (4,)])
def test_without_replacement_exact_agreement_with_rational_textbook_rule(oracle, mode, br):
    rng = np.random.default_rng(hash((7, mode) + tuple(br)) % (2 ** 32))
    V, G = 8, len(br)
    sizes = np.cumprod(br)
    N, Nin = int(sizes.sum()), int(sizes[:-1].sum())
    B, n_new = 300, 2
    p = np.stack([_dyadic_rows(rng, 1 + N, V, 64) for _ in range(B)])
    # draft rows with full support: 1/32 everywhere plus dyadic extra mass (so distinct siblings always exist)
    q = np.stack([(_dyadic_rows(rng, 1 + Nin, V, 24) * 24 + 1) / 32 for _ in range(B)]).astype(np.float32)
    assert np.all(q.sum(axis=-1) == 1.0)
    tokens = np.empty((B, N), dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(sizes)])
    for b in range(B):                                       # distinct tokens inside every sibling group
        for l, bf in enumerate(br):
            for grp in range(sizes[l] // bf):
                tokens[b, off[l] + grp * bf: off[l] + (grp + 1) * bf] = rng.permutation(V)[:bf]
    ua = (rng.integers(0, 256, size=(B, N)) / 256).astype(np.float32)
    us = (rng.integers(0, 4096, size=(B, n_new)) / 4096).astype(np.float32)
    path, alen, new = oracle.verify_tree(mode, br, tokens, p, q, ua, us, replacement=False)
    lens_seen, differs = set(), 0
    with_rep = oracle.verify_tree(mode, br, tokens, p, q, ua, us)
    for b in range(B):
        pf = [[Fraction(float(x)) for x in row] for row in p[b]]
        qf = [[Fraction(float(x)) for x in row] for row in q[b]]
        uaf = [Fraction(float(x)) for x in ua[b]]
        if mode == DRAFT:
            want_path, term = _textbook_walk_distinct(br, -1, 0, tokens[b].tolist(), pf, qf, uaf)
        else:
            best = None
            for i in range(br[0]):
                pth, term_i = _textbook_walk_distinct(br, i, 1, tokens[b].tolist(), pf, qf, uaf)
                if best is None or 1 + len(pth) > len(best[0]):
                    best = ([i] + pth, term_i)
            want_path, term = best
        want_new = [_linear_cdf_sample(term, Fraction(float(u))) for u in us[b]]
        assert alen[b] == len(want_path) and path[b, :alen[b]].tolist() == want_path
        assert new[b].tolist() == want_new
        lens_seen.add(int(alen[b]))
        differs += int(alen[b] != with_rep[1][b] or new[b].tolist() != with_rep[2][b].tolist())
    if not (mode == TARGET and G == 1):
        assert len(lens_seen) >= 2
    if max((br[1:] if mode == TARGET else br) + (1,)) > 1:
        assert differs > 0          # the two rules are not the same rule on these inputs


@pytest.mark.parametrize("br", [(2,), (3,), (2, 2)])
def test_without_replacement_first_token_law_is_the_target_law(oracle, br):
    """Losslessness of the without-replacement rule: distinct siblings drawn one after the other from the
    renormalised draft row, verified with the draft row shrinking after every rejection."""
    V = 3
    p_fn, q_fn = _rows_by_history(V, 41), _rows_by_history(V, 42)
    N = int(np.cumprod(br).sum())
    M = {2: 300000, 3: 150000}.get(N, 6000)
    law, _, tol = _law_of_first_emitted(oracle, DRAFT, br, p_fn, q_fn, V, M, replacement=False)
    target = p_fn(()).astype(np.float64)
    assert tol < 5e-3
    assert abs(law.sum() - 1.0) < 1e-5
    assert np.max(np.abs(law - target / target.sum())) < tol


def test_without_replacement_is_the_same_rule_for_single_candidates(oracle):
    """No siblings, nothing to remove: a chain gives identical results under both rules."""
    rng = np.random.default_rng(3)
    br, V, B = (1, 1, 1, 1), 50, 200
    p = rng.random((B, 5, V)).astype(np.float32); p /= p.sum(-1, keepdims=True)
    q = rng.random((B, 4, V)).astype(np.float32); q /= q.sum(-1, keepdims=True)
    tokens = rng.integers(0, V, size=(B, 4)).astype(np.int32)
    ua, us = rng.random((B, 4), dtype=np.float32), rng.random((B, 1), dtype=np.float32)
    a = oracle.verify_tree(DRAFT, br, tokens, p, q, ua, us)
    b = oracle.verify_tree(DRAFT, br, tokens, p, q, ua, us, replacement=False)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
