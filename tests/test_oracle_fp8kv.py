"""Pins for the oracle's fp8 (E4M3) prefix cache: the element format against what the OCP 8-bit floating point
specification fixes (bias 7, no infinities, one NaN pattern per sign, largest finite value 448, subnormals down to
2^-9), against an independently written decoder and encoder, and the attention routine against the bf16 routine on
values both formats hold exactly (where the two must agree bit for bit, scales included)."""
import numpy as np
import pytest

from workloads import (WORKLOADS, attention_inputs, bf16_bits_to_f32, e4m3_bits_to_f32, f32_to_bf16_bits,
                       f32_to_e4m3_bits, scaled)


def test_e4m3_values_fixed_by_the_format(oracle):
    val = [oracle.fp8_e4m3_value(c) for c in range(256)]
    assert val[0x38] == 1.0 and val[0x40] == 2.0 and val[0x30] == 0.5 and val[0x39] == 1.125
    assert val[0x7E] == 448.0                               # S.1111.110: the largest finite value
    assert val[0x01] == 2.0 ** -9 and val[0x07] == 7 * 2.0 ** -9          # subnormals: m/8 * 2^-6
    assert val[0x08] == 2.0 ** -6                           # smallest normal
    assert val[0x00] == 0.0 and val[0x80] == 0.0 and np.signbit(val[0x80])
    assert [c for c in range(256) if np.isnan(val[c])] == [0x7F, 0xFF]      # no infinities, one NaN per sign
    pos = val[:0x7F]
    assert all(a < b for a, b in zip(pos, pos[1:]))         # codes order like the numbers
    assert all(val[c + 128] == -val[c] for c in range(0x7F))
    assert all(float(v * 512).is_integer() for v in pos)    # every value is a multiple of 2^-9
    for e in range(1, 15):                                  # 8 equally spaced values per binade
        steps = {pos[8 * e + m + 1] - pos[8 * e + m] for m in range(7)}
        assert steps == {2.0 ** (e - 7) / 8}


def test_e4m3_decoder_against_an_independent_one_and_encoder_round_trip(oracle):
    codes = np.arange(256, dtype=np.uint8)
    mine = e4m3_bits_to_f32(codes)
    for c in range(256):
        o = oracle.fp8_e4m3_value(c)
        assert (np.isnan(o) and np.isnan(mine[c])) or o == float(mine[c])
    finite = np.array([c for c in range(256) if not np.isnan(mine[c]) and c != 0x80], dtype=np.uint8)
    assert np.array_equal(f32_to_e4m3_bits(mine[finite]), finite)
    # nearest, ties to even, saturation
    x = np.array([1.0625, 1.1875, 1.06, 1.07, 447.0, 480.0, 1e9, -1e9, 2.0 ** -10, 1.5 * 2.0 ** -9], dtype=np.float32)
    assert f32_to_e4m3_bits(x).tolist() == [0x38, 0x3A, 0x38, 0x39, 0x7E, 0x7E, 0x7E, 0xFE, 0x00, 0x02]
    rng = np.random.default_rng(0)
    y = (rng.standard_normal(20000) * 3).astype(np.float32)
    q = e4m3_bits_to_f32(f32_to_e4m3_bits(y)).astype(np.float64)
    grid = np.array(sorted({float(v) for v in mine if not np.isnan(v)}))
    best = np.abs(grid[None, :] - y[:, None].astype(np.float64)).min(axis=1)
    assert np.array_equal(np.abs(q - y), best)              # nothing on the grid is nearer


def _both_caches(w, lens, k_scale, v_scale, seed):
    """The same prefix values once as bf16 and once as E4M3 codes of value / scale; values on a grid both hold."""
    inp = attention_inputs(w, seed=seed, lens=lens)
    rng = np.random.default_rng(seed + 100)
    shape = inp["k_prefix"].shape
    kv = rng.integers(-8, 9, size=shape).astype(np.float32) * np.float32(0.25)     # multiples of 1/4 in [-2, 2]
    vv = rng.integers(-8, 9, size=shape).astype(np.float32) * np.float32(0.25)
    for b, L in enumerate(lens):
        kv[b, :, L:] = 0
        vv[b, :, L:] = 0
    bf = dict(inp, k_prefix=f32_to_bf16_bits(kv), v_prefix=f32_to_bf16_bits(vv))
    f8 = dict(inp, k_prefix=f32_to_e4m3_bits(kv / np.float32(k_scale)), v_prefix=f32_to_e4m3_bits(vv / np.float32(v_scale)),
              k_scale=k_scale, v_scale=v_scale)
    assert np.array_equal(bf16_bits_to_f32(bf["k_prefix"]), kv)
    assert np.array_equal(e4m3_bits_to_f32(f8["k_prefix"]) * np.float32(k_scale), kv)
    assert np.array_equal(e4m3_bits_to_f32(f8["v_prefix"]) * np.float32(v_scale), vv)
    return bf, f8


@pytest.mark.parametrize("k_scale,v_scale", [(1.0, 1.0), (0.5, 0.125), (2.0, 0.25)])
def test_fp8_cache_equals_bf16_cache_on_values_both_hold_exactly(oracle, k_scale, v_scale):
    br = (3, 2, 2)
    w = scaled(WORKLOADS["cfg2"], B=2, H=2, branching=br, cfg_id=71)
    lens = (37, 5)
    bf, f8 = _both_caches(w, lens, k_scale, v_scale, seed=4)
    M = oracle.build_mask(br)
    n = M.shape[0]
    a = oracle.tree_attention(bf, M, n)
    b = oracle.tree_attention_fp8kv(f8, M, n)
    assert np.array_equal(a, b)                             # powers of two: every product is the same number
    row = oracle.tree_attention_row_fp8kv(f8, M, n, 1, 1, n - 1)
    assert np.array_equal(row, b[1, 1, n - 1])
    # the two scales are not interchangeable: swapping them changes the result unless they are equal
    swapped = oracle.tree_attention_fp8kv(dict(f8, k_scale=v_scale, v_scale=k_scale), M, n)
    assert (k_scale == v_scale) == bool(np.array_equal(swapped, b))


def test_fp8_cache_value_scale_is_linear_and_key_scale_acts_inside_the_softmax(oracle):
    br = (2, 2)
    w = scaled(WORKLOADS["cfg2"], B=1, H=1, branching=br, cfg_id=72)
    inp = attention_inputs(w, seed=1, lens=(50,), kv_fp8=(0.5, 0.25))
    M = oracle.build_mask(br)
    n = M.shape[0]
    zero_tree = dict(inp, v_tree=np.zeros_like(inp["v_tree"]))                 # only prefix values contribute
    a = oracle.tree_attention_fp8kv(zero_tree, M, n)
    b = oracle.tree_attention_fp8kv(dict(zero_tree, v_scale=0.75), M, n)
    np.testing.assert_allclose(b, a * 3.0, rtol=1e-12, atol=1e-14)
    # halving k_scale equals halving the softmax scale for a prefix-only context (no tree keys visible: impossible,
    # a node always sees itself, so compare through a tree whose keys are zero instead: their scores are 0 either way)
    zk = dict(inp, k_tree=np.zeros_like(inp["k_tree"]))
    c = oracle.tree_attention_fp8kv(dict(zk, k_scale=0.25), M, n)
    d = oracle.tree_attention_fp8kv(dict(zk, scale=inp["scale"] / 2), M, n)
    np.testing.assert_allclose(c, d, rtol=1e-12, atol=1e-14)
