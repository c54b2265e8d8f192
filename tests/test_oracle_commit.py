"""Pins for the oracle's update after acceptance (Fig. 1 step 6 of arXiv 2409.10644): the accepted path becomes
part of the prefix.  The fixed fact used: once a root-to-leaf path has been appended to the KV cache it is an ordinary
causal sequence, so plain soft-max attention of an accepted node's query over the cache up to and including its own
row must equal that node's tree-attention output under the topology-aware mask."""
import numpy as np
import pytest

from workloads import WORKLOADS, attention_inputs, bf16_bits_to_f32, scaled


def _chain(parent, leaf):
    out = []
    while leaf >= 0:
        out.append(int(leaf))
        leaf = int(parent[leaf])
    return out[::-1]


def _plain_attention(q, K, V, scale):
    """Textbook soft-max attention of one query over all rows of K / V, binary64."""
    s = (K @ q) * scale
    w = np.exp(s - s.max())
    return (w / w.sum()) @ V


def _as_f64(a, dtype):
    return a.astype(np.float64) if dtype == "f32" else bf16_bits_to_f32(a).astype(np.float64)


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("bf16", 128)])
def test_committed_path_is_a_plain_causal_sequence(oracle, dtype, d):
    br = (3, 2, 2)
    w = scaled(WORKLOADS["cfg1"], B=3, H=2, d=d, dtype=dtype, branching=br, cfg_id=60)
    lens = (5, 9, 0)
    inp = attention_inputs(w, seed=3, lens=lens, kv_capacity=12)
    parent, level = oracle.tree_tables(br)
    n = len(parent)
    M = oracle.build_mask(br)
    # three different situations: a full path, a path that stops at level 2, nothing accepted
    leaves = [int(np.where(level == 3)[0][7]), int(np.where(level == 2)[0][1]), 0]
    path = np.full((3, 3), -1, dtype=np.int32)
    alen = np.array([3, 2, 0], dtype=np.int32)
    for b in range(2):
        c = _chain(parent, leaves[b])
        assert len(c) == alen[b]
        path[b, :len(c)] = c
    kp, vp, new_lens = oracle.commit_path(inp, 3, n, path, alen)
    assert new_lens.tolist() == [8, 11, 0]
    scale = float(np.float32(inp["scale"]))
    K, V, Q = _as_f64(kp, dtype), _as_f64(vp, dtype), _as_f64(inp["q"], dtype)
    for b in range(2):
        for j in range(alen[b]):
            node = path[b, j]
            for h in range(2):
                rows = lens[b] + j + 1
                got = _plain_attention(Q[b, h, node], K[b, h, :rows], V[b, h, :rows], scale)
                want = oracle.tree_attention_row(inp, M, n, b, h, int(node))
                np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_commit_touches_only_the_appended_rows(oracle):
    br = (2, 2)
    w = scaled(WORKLOADS["cfg1"], B=2, H=3, branching=br, cfg_id=61)
    inp = attention_inputs(w, seed=5, lens=(4, 7), kv_capacity=10)
    path = np.array([[1, 4], [0, -1]], dtype=np.int32)          # node 4 = second child of node 1
    alen = np.array([2, 1], dtype=np.int32)
    kp, vp, new_lens = oracle.commit_path(inp, 2, 6, path, alen)
    assert new_lens.tolist() == [6, 8]
    for old, new, tree in ((inp["k_prefix"], kp, inp["k_tree"]), (inp["v_prefix"], vp, inp["v_tree"])):
        expect = old.copy()
        expect[0, :, 4] = tree[0, :, 1]
        expect[0, :, 5] = tree[0, :, 4]
        expect[1, :, 7] = tree[1, :, 0]
        assert np.array_equal(new, expect)
    # nothing accepted: nothing changes
    kp0, vp0, lens0 = oracle.commit_path(inp, 2, 6, np.full((2, 2), -1, dtype=np.int32), np.zeros(2, dtype=np.int32))
    assert np.array_equal(kp0, inp["k_prefix"]) and np.array_equal(vp0, inp["v_prefix"]) and lens0.tolist() == [4, 7]
    with pytest.raises(ValueError):
        oracle.commit_path(inp, 2, 6, np.array([[6, 0], [0, 0]], dtype=np.int32), alen)      # node id out of range


def test_commit_ids_worked_example(oracle):
    # tree (2,2): nodes 0,1 | 2,3 (children of 0), 4,5 (children of 1)
    tokens = np.array([[100, 101, 102, 103, 104, 105], [200, 201, 202, 203, 204, 205]], dtype=np.int32)
    path = np.array([[1, 5], [0, -1]], dtype=np.int32)
    alen = np.array([2, 1], dtype=np.int32)
    new = np.array([[7, 8], [9, 10]], dtype=np.int32)
    ids, n_ids = oracle.commit_ids(2, tokens, path, alen, new, n_append=1)
    assert ids.tolist() == [[101, 105, 7], [200, 9, -1]] and n_ids.tolist() == [3, 2]
    ids, n_ids = oracle.commit_ids(2, tokens, path, alen, new, n_append=0)       # target-initialised: candidates, not input
    assert ids.tolist() == [[101, 105], [200, -1]] and n_ids.tolist() == [2, 1]
    ids, n_ids = oracle.commit_ids(2, tokens, path, np.zeros(2, dtype=np.int32), new, n_append=2)
    assert ids.tolist() == [[7, 8, -1, -1], [9, 10, -1, -1]] and n_ids.tolist() == [2, 2]
