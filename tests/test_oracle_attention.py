"""Pins for the oracle's tree attention (no GPU).

Independent references: torch's scaled_dot_product_attention on CPU (library routine), and a few lines of
numpy softmax attention applied to explicitly gathered root-to-node paths.
"""
import numpy as np
import pytest
import torch

from workloads import WORKLOADS, attention_inputs, bf16_bits_to_f32, scaled


def _as_f64(a, dtype):
    return a.astype(np.float64) if dtype == "f32" else bf16_bits_to_f32(a).astype(np.float64)


def _plain_attention(q, K, V, scale):
    """Textbook softmax attention of one query over explicit keys/values (numpy, fp64)."""
    s = (K @ q) * scale
    w = np.exp(s - s.max())
    w /= w.sum()
    return w @ V


def _small(dtype, branching, B=2, H=2, d=64, lens=(5, 0), seed=3):
    w = scaled(WORKLOADS["cfg1"], B=B, H=H, d=d, dtype=dtype, branching=tuple(branching), cfg_id=77)
    return w, attention_inputs(w, seed=seed, lens=lens, kv_capacity=max(max(lens), 1) + 3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("br", [(2, 2, 2), (4, 2, 2, 1), (3, 1, 1), (2, 3)])
def test_per_path_equivalence(oracle, dtype, br):
    """Sec. 2.2: tree attention computes, for every node, ordinary attention over prefix + its own path."""
    w, inp = _small(dtype, br, lens=(7, 0))
    n = w.n_nodes()
    M = oracle.build_mask(br)
    out = oracle.tree_attention(inp, M, n)
    parent, _ = oracle.tree_tables(br)
    q, kt, vt = (_as_f64(inp[k], dtype) for k in ("q", "k_tree", "v_tree"))
    kp, vp = (_as_f64(inp[k], dtype) for k in ("k_prefix", "v_prefix"))
    scale = float(np.float32(inp["scale"]))
    for b in range(w.B):
        L = int(inp["lens"][b])
        for h in range(w.H):
            for i in range(n):
                path, j = [], i
                while j >= 0:
                    path.append(j)
                    j = parent[j]
                path = path[::-1]
                K = np.concatenate([kp[b, h, :L], kt[b, h, path]])
                V = np.concatenate([vp[b, h, :L], vt[b, h, path]])
                want = _plain_attention(q[b, h, i], K, V, scale)
                np.testing.assert_allclose(out[b, h, i], want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_tree_is_causal_attention_sdpa(oracle, dtype):
    """k = 1 chain: the tree pass is ordinary causal attention over [prefix ; tree] (library routine)."""
    br = (1, 1, 1, 1, 1, 1)
    w, inp = _small(dtype, br, B=1, H=3, lens=(9,))
    n = w.n_nodes()
    out = oracle.tree_attention(inp, oracle.build_mask(br), n)
    L = 9
    q, kt, vt = (_as_f64(inp[k], dtype) for k in ("q", "k_tree", "v_tree"))
    kp, vp = (_as_f64(inp[k], dtype)[:, :, :L] for k in ("k_prefix", "v_prefix"))
    K = torch.from_numpy(np.concatenate([kp, kt], axis=2))
    V = torch.from_numpy(np.concatenate([vp, vt], axis=2))
    # queries for all L+n positions; only the last n are the tree's
    Q = torch.from_numpy(np.concatenate([np.zeros_like(kp), q], axis=2))
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True,
                                                           scale=float(np.float32(inp["scale"])))
    np.testing.assert_allclose(out, ref[:, :, L:].numpy(), rtol=1e-10, atol=1e-12)


def test_equal_values_give_that_value(oracle):
    br = (4, 2, 2, 1)
    w, inp = _small("f32", br, lens=(11, 3))
    row = np.linspace(-1, 1, w.d, dtype=np.float32)
    inp["v_tree"][...] = row
    inp["v_prefix"][...] = row
    out = oracle.tree_attention(inp, oracle.build_mask(br), w.n_nodes())
    np.testing.assert_allclose(out, np.broadcast_to(row.astype(np.float64), out.shape), rtol=1e-13, atol=1e-14)


def test_empty_prefix_root_nodes_return_their_own_value(oracle):
    """L = 0: a level-1 node sees only itself, so its output is its own value row."""
    br = (3, 2)
    w, inp = _small("f32", br, lens=(0, 0))
    out = oracle.tree_attention(inp, oracle.build_mask(br), w.n_nodes())
    np.testing.assert_allclose(out[:, :, :3], inp["v_tree"][:, :, :3].astype(np.float64), rtol=1e-14)


def test_mask_is_honoured_one_hot_value_probe(oracle):
    """With v_tree = one-hot(node id) and zero prefix values, output column j is the weight put on tree key j:
    it must be positive exactly where the closed-form ancestor relation holds."""
    br = (2, 3, 2)
    w, inp = _small("f32", br, B=1, H=1, d=64, lens=(4,))
    n = w.n_nodes()
    inp["v_prefix"][...] = 0
    inp["v_tree"][...] = 0
    for j in range(n):
        inp["v_tree"][0, 0, j, j] = 1.0
    M = oracle.build_mask(br)
    out = oracle.tree_attention(inp, M, n)[0, 0]
    assert np.array_equal((out[:, :n] > 0).astype(np.uint8), M)


def test_slice_uses_node_stride_views(oracle):
    """A gamma-slice reads the first N(gamma) rows of gamma_max-sized tensors (node_stride stays N_max)."""
    br = (3, 2, 2)
    w, inp = _small("bf16", br, lens=(6, 2))
    M = oracle.build_mask(br)
    full = oracle.tree_attention(inp, M, w.n_nodes())
    for g in (1, 2):
        n = w.n_nodes(g)
        part = oracle.tree_attention(inp, M, n)        # same buffers, same big mask, fewer nodes
        # a node's visible set lies in its own slice, so the first n rows do not change
        np.testing.assert_array_equal(part, full[:, :, :n])


def test_row_entry_matches_full(oracle):
    br = (2, 2, 2)
    w, inp = _small("bf16", br, lens=(8, 1))
    M = oracle.build_mask(br)
    full = oracle.tree_attention(inp, M, w.n_nodes())
    row = oracle.tree_attention_row(inp, M, w.n_nodes(), 1, 0, 9)
    np.testing.assert_array_equal(row, full[1, 0, 9])


def test_bf16_bits_decode_like_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(1000).astype(np.float32)
    from workloads import f32_to_bf16_bits
    bits = f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), t.view(torch.int16).numpy())
    assert np.array_equal(bf16_bits_to_f32(bits), t.to(torch.float32).numpy())
