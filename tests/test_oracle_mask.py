"""Pins for the oracle's tree topology, mask and slices (no GPU).

Nothing here re-uses the oracle's parent-walk: the expectations are the node counts the paper prints,
a closed form over in-level indices, structural invariants, and "slice == rebuild".
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_tree_counts.txt")

TREES = [(2, 2, 2), (4, 2, 2, 1), (3, 2, 2, 1, 1, 1, 1, 1), (4, 2, 2, 2), (8, 2, 2, 1, 1),
         (2, 4, 3, 1, 1), (3, 1, 1), (1, 1, 1, 1), (1,), (5,), (16, 1, 1, 1, 1), (1, 3, 1, 2)]


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            br, sizes, total, leaves, _cite = [s.strip() for s in line.split(";")]
            rows.append((tuple(int(x) for x in br.split(",")), tuple(int(x) for x in sizes.split(",")),
                         int(total), int(leaves)))
    return rows


@pytest.mark.parametrize("row", _golden_rows())
def test_node_counts_printed_in_the_paper(oracle, row):
    br, sizes, total, leaves = row
    got = oracle.level_sizes(br)
    assert tuple(int(x) for x in got) == sizes
    assert oracle.n_nodes(br) == total
    assert int(got[-1]) == leaves
    M = oracle.build_mask(br)
    assert M.shape == (total, total)            # mask side = number of tree tokens; no prefix columns


def test_target_init_example_40_draft_tokens_per_root(oracle):
    # Sec. 4.1: 4 + 4*3 + 4*3*1 + 4*3*1*1 = 40 draft tokens under each of the 2 target-sampled tokens
    M = oracle.build_mask((2, 4, 3, 1, 1))
    for root in (0, 1):
        descendants = int(M[:, root].sum()) - 1
        assert descendants == 40


def test_workload_node_counts():
    from workloads import WORKLOADS
    assert WORKLOADS["cfg1"].n_nodes() == 14
    assert WORKLOADS["cfg2"].n_nodes() == 44
    assert WORKLOADS["cfg4"].n_nodes() == 60
    assert [WORKLOADS["cfg3"].n_nodes(g) for g in range(1, 9)] == [3, 9, 21, 33, 45, 57, 69, 81]
    assert WORKLOADS["cfg5"].n_nodes(4) == 88 and WORKLOADS["cfg5"].n_nodes(5) == 120


def _closed_form_mask(br):
    """M[i][j] = 1 iff level(j) <= level(i) and a_i // prod(b[level(j)+1 .. level(i)]) == a_j."""
    sizes, n = [], 1
    for b in br:
        n *= b
        sizes.append(n)
    off = np.concatenate([[0], np.cumsum(sizes)])
    N = int(off[-1])
    lvl = np.zeros(N, dtype=int)
    idx = np.zeros(N, dtype=int)
    for l, s in enumerate(sizes):
        lvl[off[l]:off[l + 1]] = l
        idx[off[l]:off[l + 1]] = np.arange(s)
    M = np.zeros((N, N), dtype=np.uint8)
    for i in range(N):
        for j in range(N):
            if lvl[j] <= lvl[i]:
                div = 1
                for m in range(lvl[j] + 1, lvl[i] + 1):
                    div *= br[m]
                M[i, j] = 1 if idx[i] // div == idx[j] else 0
    return M, lvl + 1, sizes


@pytest.mark.parametrize("br", TREES)
def test_mask_equals_closed_form_and_invariants(oracle, br):
    M = oracle.build_mask(br)
    want, lvl, sizes = _closed_form_mask(br)
    assert np.array_equal(M, want)
    N = M.shape[0]
    assert np.array_equal(np.triu(M, 1), np.zeros_like(M))          # lower triangular
    assert np.all(np.diag(M) == 1)                                   # a node sees itself
    assert np.array_equal(M.sum(axis=1), lvl)                        # one ancestor per level
    assert int(M.sum()) == sum((l + 1) * s for l, s in enumerate(sizes))
    n1 = sizes[0]
    assert np.array_equal(M[:n1, :n1], np.eye(n1, dtype=np.uint8))   # siblings at level 1 are different paths
    parent, level = oracle.tree_tables(br)
    assert np.array_equal(level, lvl)
    assert np.all(parent[:n1] == -1)
    for i in range(n1, N):
        assert M[i, parent[i]] == 1 and level[parent[i]] == level[i] - 1
    # children of one parent are adjacent and there are b_l of them
    for l in range(1, len(br)):
        lo, hi = sum(sizes[:l]), sum(sizes[:l + 1])
        par = parent[lo:hi]
        assert np.all(np.diff(par) >= 0)
        assert np.all(np.bincount(par - par.min()) == br[l])


def test_fork_tree_rows(oracle):
    # fork (3,1,1): node i sees i, i-3, i-6, ... (Fig. 2's 9 x 9 mask)
    M = oracle.build_mask((3, 1, 1))
    for i in range(9):
        cols = set(np.nonzero(M[i])[0].tolist())
        assert cols == set(range(i % 3, i + 1, 3))
    # the three slices named in Sec. 3.2 are the upper-left 3x3, 6x6 and 9x9 blocks
    assert np.array_equal(oracle.slice_mask(M, 3), np.eye(3, dtype=np.uint8))
    assert np.array_equal(oracle.slice_mask(M, 6), oracle.build_mask((3, 1)))
    assert np.array_equal(oracle.slice_mask(M, 9), M)


def test_chain_is_causal(oracle):
    M = oracle.build_mask((1, 1, 1, 1, 1))
    assert np.array_equal(M, np.tril(np.ones((5, 5), dtype=np.uint8)))


@pytest.mark.parametrize("br", TREES)
def test_slice_equals_rebuild_for_every_gamma(oracle, br):
    M = oracle.build_mask(br)
    sizes = oracle.level_sizes(br)
    for g in range(1, len(br) + 1):
        n = int(sizes[:g].sum())
        sl = oracle.slice_mask(M, n)
        assert np.array_equal(sl, oracle.build_mask(br[:g]))
        assert not M[:n, n:].any()        # rows of the slice have no bits outside it


def test_bad_branching_rejected(oracle):
    with pytest.raises(ValueError):
        oracle.build_mask((2, 0, 1))


def test_improvement_factor_closed_form(oracle):
    # Sec. 3: IF = (1 - a^(g+1)) / ((1 - a)(c g + 1));  a = 0.5, g = 4, c = 0  ->  (1 - 1/32) / 0.5
    assert oracle.improvement_factor(0.5, 4, 0.0) == pytest.approx(1.9375, rel=1e-15)
    assert oracle.improvement_factor(0.5, 4, 0.1) == pytest.approx(1.9375 / 1.4, rel=1e-15)
