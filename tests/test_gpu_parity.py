"""GPU parity: libmcsd.so (through the C ABI) against the CPU oracle on the same seeded inputs.

Masks, accepted paths, lengths and sampled tokens must match bit for bit; attention within 2e-2 relative /
1e-2 absolute (bf16 path) or 1e-5 (fp32 path) of the binary64 oracle.
"""
import numpy as np
import pytest
import torch

from workloads import DRAFT_INIT, TARGET_INIT, WORKLOADS, attention_inputs, prefix_lens, scaled, verify_inputs

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


# ------------------------------------------------------------------------------------------------
# masks on the device
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_device_mask_bits_match_oracle_for_every_gamma(binding, oracle, name):
    w = WORKLOADS[name]
    m = binding.build_mask(w.branching)
    full = oracle.build_mask(w.branching)
    for g in range(1, w.gamma_max + 1):
        v = binding.slice_mask(m, g)
        assert v.device >= 0 and v.bits_dev
        n, W = v.n_nodes, v.words_per_row
        host = np.empty(v.n_nodes_max * W, dtype=np.uint64)
        torch.cuda.synchronize()
        binding.HipRuntime().memcpy_dtoh(host.ctypes.data, v.bits_dev, host.nbytes)   # the library's own buffer
        host = host.reshape(v.n_nodes_max, W)
        got = np.zeros((n, n), dtype=np.uint8)
        for j in range(n):
            got[:, j] = (host[:n, j >> 6] >> np.uint64(j & 63)) & np.uint64(1)
        assert np.array_equal(got, oracle.build_mask(w.branching[:g]))
        assert np.array_equal(got, oracle.slice_mask(full, n))


# ------------------------------------------------------------------------------------------------
# attention: the five configurations
# ------------------------------------------------------------------------------------------------
def test_cfg1_fp32_every_gamma(binding, oracle, H):
    w = WORKLOADS["cfg1"]
    inp = attention_inputs(w, seed=0)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)
    M = oracle.build_mask(w.branching)
    for g in (1, 2, 3):
        v = binding.slice_mask(m, g)
        got = H.run_attention(binding, v, ad)
        want = oracle.tree_attention(inp, M, v.n_nodes)
        H.assert_close(got, want, "f32", f"cfg1 gamma={g}")


def test_cfg2_full(binding, oracle, H):
    w = WORKLOADS["cfg2"]
    inp = attention_inputs(w, seed=0)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)
    v = binding.slice_mask(m, w.gamma_max)
    got = H.run_attention(binding, v, ad, fill=float("nan"))
    want = oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes)
    H.assert_close(got, want, "bf16", "cfg2")
    # rows beyond n_nodes of the output buffer are not touched (node_stride == n here, so nothing to check);
    # determinism: a second call gives the same bits
    again = H.run_attention(binding, v, ad)
    assert np.array_equal(got, again)


@pytest.mark.parametrize("B,Hh,L", [(1, 32, 2048), (2, 16, 2048), (1, 30, 2048), (1, 32, 2000)])
def test_grids_around_one_workgroup_per_compute_unit(binding, oracle, H, B, Hh, L):
    """32 (sequence, head) units and 2048 keys: the plan takes 7 key splits + 1 tree workgroup per unit (256
    workgroups) rather than 8 + 1; unit counts that are and are not multiples of 8; a ragged last tile."""
    w = scaled(WORKLOADS["cfg2"], B=B, H=Hh, prefix_min=L, prefix_max=L, cfg_id=66)
    inp = attention_inputs(w, seed=4)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    got = H.run_attention(binding, v, ad, fill=float("nan"))
    want = oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes)
    H.assert_close(got, want, "bf16", f"B{B} H{Hh} L{L}")


def test_cfg2_tensors_scaled_variant(binding, oracle, H):
    """Second reading of the recipe: tensors themselves scaled by 1/sqrt(128) (flat softmax)."""
    w = WORKLOADS["cfg2"]
    inp = attention_inputs(w, seed=1, tensor_mult=float(1 / np.sqrt(128)))
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)
    v = binding.slice_mask(m, w.gamma_max)
    got = H.run_attention(binding, v, ad)
    want = oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes)
    H.assert_close(got, want, "bf16", "cfg2 scaled tensors")


def test_cfg3_gamma_sweep_by_slicing_only(binding, oracle, H):
    w = WORKLOADS["cfg3"]
    inp = attention_inputs(w, seed=0)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)           # built once at gamma_max = 8
    M = oracle.build_mask(w.branching)
    for g in range(1, 9):
        v = binding.slice_mask(m, g)
        got = H.run_attention(binding, v, ad, fill=123.0)
        want = oracle.tree_attention(inp, M, v.n_nodes)
        H.assert_close(got, want, "bf16", f"cfg3 gamma={g}")
        # rows of the gamma_max-sized output beyond N(gamma) keep the fill value: padded queries are never stored
        rest = ad.out[:, :, v.n_nodes:].float().cpu().numpy()
        assert np.all(rest == 123.0)


def test_cfg4_ragged_batch_full_tensor(binding, oracle, H):
    """Every (sequence, head, node, column) of the ragged batch: the output starts as NaN, so a unit that the
    length-ranked grid skipped, or wrote for the wrong (sequence, head), cannot pass."""
    w = WORKLOADS["cfg4"]
    lens = prefix_lens(w, 0)
    assert lens.min() >= 512 and lens.max() <= 4096 and len(set(lens.tolist())) > 8
    inp = attention_inputs(w, seed=0, kv_capacity=4096)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)
    v = binding.slice_mask(m, w.gamma_max)
    got = H.run_attention(binding, v, ad, max_prefix=4096, fill=float("nan"))
    want = oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes)
    H.assert_close(got, want, "bf16", "cfg4 full tensor")


def test_cfg5_long_context_full_tensor(binding, oracle, H):
    """gamma = 5 (120 nodes) and its gamma = 4 slice (88 nodes) over the same buffers, every output element; rows of
    the buffer beyond N(gamma) keep the NaN they were filled with."""
    w = WORKLOADS["cfg5"]
    inp = attention_inputs(w, seed=0)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)
    M = oracle.build_mask(w.branching)
    for g in (5, 4):
        v = binding.slice_mask(m, g)
        assert v.n_nodes == (120 if g == 5 else 88)
        got = H.run_attention(binding, v, ad, fill=float("nan"))
        want = oracle.tree_attention(inp, M, v.n_nodes)
        H.assert_close(got, want, "bf16", f"cfg5 gamma={g} full tensor")
        rest = ad.out[:, :, v.n_nodes:].float()
        assert bool(torch.isnan(rest).all()), "rows beyond N(gamma) were written"
    del ad
    torch.cuda.empty_cache()


def test_cfg4_batch64_full_tensor(binding, oracle, H):
    """cfg4's recipe with 64 sequences (2048 workgroups handed out longest first): every output element."""
    w = WORKLOADS["cfg4_b64"]
    inp = attention_inputs(w, seed=0, kv_capacity=4096)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    got = H.run_attention(binding, v, ad, max_prefix=4096, fill=float("nan"))
    want = oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes)
    H.assert_close(got, want, "bf16", "cfg4_b64 full tensor")
    del ad
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------------------
# attention: edge cases, every topology with short / empty prefixes (mask errors are visible there)
# ------------------------------------------------------------------------------------------------
TOPOLOGIES = [(2, 2, 2), (4, 2, 2, 1), (3, 2, 2, 1, 1, 1, 1, 1), (4, 2, 2, 2), (8, 2, 2, 1, 1), (2, 4, 3, 1, 1),
              (16, 1, 1, 1, 1), (1,), (1, 1, 1), (8, 3, 4), (33,), (5, 5)]


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
@pytest.mark.parametrize("br", TOPOLOGIES)
def test_short_and_empty_prefix_every_topology(binding, oracle, H, br, dtype, d):
    w = scaled(WORKLOADS["cfg2"], B=3, H=2, d=d, dtype=dtype, branching=tuple(br), cfg_id=50)
    inp = attention_inputs(w, seed=7, lens=(0, 1, 5), kv_capacity=8)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(br)
    M = oracle.build_mask(br)
    for g in sorted({1, len(br)}):
        v = binding.slice_mask(m, g)
        got = H.run_attention(binding, v, ad, max_prefix=8)
        want = oracle.tree_attention(inp, M, v.n_nodes)
        H.assert_close(got, want, dtype, f"tree {br} gamma={g}")


@pytest.mark.parametrize("L", [63, 64, 65, 127, 128, 129, 200, 1000])
@pytest.mark.parametrize("br", [(4, 2, 2, 1), (8, 2, 2, 1, 1), (3, 2)])
def test_ragged_tails_and_split_boundaries(binding, oracle, H, br, L):
    """Prefix lengths around the tile size; with B*H small the sweep is split over several workgroups."""
    w = scaled(WORKLOADS["cfg2"], B=2, H=2, branching=tuple(br), cfg_id=51)
    inp = attention_inputs(w, seed=L, lens=(L, max(L - 37, 0)), kv_capacity=L + 3)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(br)
    v = binding.slice_mask(m, len(br))
    got = H.run_attention(binding, v, ad, max_prefix=L + 3)
    want = oracle.tree_attention(inp, oracle.build_mask(br), v.n_nodes)
    H.assert_close(got, want, "bf16", f"L={L} tree {br}")


# The split plan is made on the host from B * H and the longest allowed prefix alone, so the actual lengths can be
# anything below it: far shorter than planned for, empty, or wildly different between sequences.  `max_prefix` may
# exceed the cache capacity: only lens[b] keys are ever read.
PLAN_VS_LENGTH_CASES = [
    # (tree, B, H, d, lens, max_prefix, note)
    ((4, 2, 2, 1), 3, 2, 128, (0, 9000, 130), 65536, "one long sequence, a short and an empty one"),
    ((8, 2, 2, 1, 1), 4, 4, 128, (0, 70, 1000, 3000), 16384, "two tree tiles, lengths far below the plan"),
    ((3, 2), 4, 4, 128, (5, 64, 129, 700), 32768, "one query block, 128-key tiles"),
    ((4, 2, 2, 2), 40, 4, 64, None, 2048, "many short sequences"),
    ((4, 2, 2, 2), 8, 8, 128, (2000, 4000, 2500, 3100, 3999, 2048, 2111, 3333), 4096, "ragged long sequences"),
]


@pytest.mark.parametrize("case", PLAN_VS_LENGTH_CASES, ids=[c[-1] for c in PLAN_VS_LENGTH_CASES])
def test_lengths_unlike_the_plan(binding, oracle, H, case):
    br, B, Hh, d, lens, max_prefix, note = case
    w = scaled(WORKLOADS["cfg4"], B=B, H=Hh, d=d, branching=tuple(br), cfg_id=52)
    if lens is None:
        lens = np.random.default_rng(9).integers(0, 600, size=B)
        lens[3] = 0
    inp = attention_inputs(w, seed=11, lens=tuple(int(x) for x in lens))
    ad = H.AttnDevice(inp)
    m = binding.build_mask(br)
    M = oracle.build_mask(br)
    v = binding.slice_mask(m, len(br))
    got = H.run_attention(binding, v, ad, max_prefix=max_prefix, fill=77.0)
    want = oracle.tree_attention(inp, M, v.n_nodes)
    H.assert_close(got, want, "bf16", note)
    again = H.run_attention(binding, v, ad, max_prefix=max_prefix)
    assert np.array_equal(got, again), "two runs differ"


def test_lengths_are_clamped_to_max_prefix(binding, oracle, H):
    br = (4, 2, 2, 1)
    w = scaled(WORKLOADS["cfg4"], B=16, H=32, branching=br, cfg_id=53)
    lens = [300] * 16
    inp = attention_inputs(w, seed=3, lens=lens, kv_capacity=640)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(br), 4)
    ad.lens.copy_(torch.tensor([300, 5000, -3, 640] * 4, dtype=torch.int32))       # the device sees other lengths
    got = H.run_attention(binding, v, ad, max_prefix=640, fill=float("nan"))
    seen = dict(inp, lens=np.asarray([300, 640, 0, 640] * 4, dtype=np.int32))       # ... clamped to 0 .. max_prefix
    H.assert_close(got, oracle.tree_attention(seen, oracle.build_mask(br), v.n_nodes), "bf16", "clamped lengths")


def test_boosted_tree_keys_make_mask_errors_visible(binding, oracle, H):
    """Long prefix, but every tree key is aligned with every query, so the visible tree keys share most of the
    softmax weight equally: one wrong mask bit moves the output far beyond the tolerance."""
    br = (4, 2, 2, 1)
    w = scaled(WORKLOADS["cfg2"], B=1, H=4, branching=br, cfg_id=52)
    inp = attention_inputs(w, seed=9, lens=(777,))
    from workloads import bf16_bits_to_f32, f32_to_bf16_bits
    q0 = bf16_bits_to_f32(inp["q"])[:, :, :1]                       # one query vector per head
    inp["q"] = f32_to_bf16_bits(np.broadcast_to(q0, inp["q"].shape).copy())
    inp["k_tree"] = f32_to_bf16_bits(np.broadcast_to(0.7 * q0, inp["q"].shape).copy())
    ad = H.AttnDevice(inp)
    m = binding.build_mask(br)
    v = binding.slice_mask(m, 4)
    got = H.run_attention(binding, v, ad)
    M = oracle.build_mask(br)
    want = oracle.tree_attention(inp, M, v.n_nodes)
    H.assert_close(got, want, "bf16", "boosted tree keys")
    # the same inputs under a wrong mask (plain causal over node ids) differ by far more than the tolerance
    wrong = oracle.tree_attention(inp, np.tril(np.ones_like(M)), v.n_nodes)
    assert np.max(np.abs(wrong - want)) > 0.2
    # ... and so does a single flipped bit
    M1 = M.copy()
    M1[5, 1] ^= 1
    assert np.max(np.abs(oracle.tree_attention(inp, M1, v.n_nodes) - want)) > 0.1


def test_maximum_node_count_and_limits(binding, oracle, H):
    br = (8, 3, 4)                                     # 8 + 24 + 96 = 128 nodes: the kernel's maximum
    w = scaled(WORKLOADS["cfg2"], B=1, H=3, branching=br, cfg_id=53)
    inp = attention_inputs(w, seed=3, lens=(300,))
    ad = H.AttnDevice(inp)
    m = binding.build_mask(br)
    v = binding.slice_mask(m, 3)
    assert v.n_nodes == 128
    got = H.run_attention(binding, v, ad)
    H.assert_close(got, oracle.tree_attention(inp, oracle.build_mask(br), 128), "bf16", "128 nodes")
    big = binding.build_mask((8, 3, 4, 2))             # 320 nodes: mask is fine, attention refuses
    vb = binding.slice_mask(big, 4)
    with pytest.raises(binding.McsdError) as e:
        H.run_attention(binding, vb, ad)
    assert e.value.status in (binding.MCSD_EUNSUPPORTED, binding.MCSD_EINVAL)


def test_workspace_too_small_is_an_error_not_a_fault(binding, H):
    w = WORKLOADS["cfg2"]
    inp = attention_inputs(w, seed=0)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)
    v = binding.slice_mask(m, 4)
    need = binding.tree_attention_workspace(ad.B, ad.H, ad.d, v.n_nodes, ad.max_prefix)
    assert need > 256                                  # 32 (b,h) pairs over 1024 keys: the keys are split
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.McsdError) as e:
        binding.tree_attention(v, 1, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp, ad.base,
                               ad.lens, ad.head_stride, ad.max_prefix, ad.scale, ad.out, ws)
    assert e.value.status == binding.MCSD_EWORKSPACE


def _tuned_attention(binding, view, ad, tuning, ws=None, max_prefix=None):
    mp = ad.max_prefix if max_prefix is None else max_prefix
    if ws is None:
        ws = binding.new_workspace(binding.tree_attention_tuned_workspace(tuning, 0, ad.B, ad.H, ad.H, ad.d, view.n_nodes, 0, mp))
    binding.tree_attention_tuned(tuning, view, ad.code, 0, 1.0, 1.0, ad.B, ad.H, ad.H, ad.d, 0, ad.q, ad.kt, ad.vt,
                                 ad.node_stride, ad.kp, ad.vp, ad.base, ad.lens, ad.head_stride, mp, ad.scale, ad.out, ws)
    torch.cuda.synchronize()
    return ad.out[:, :, :view.n_nodes].float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("fold", [0, 1])
@pytest.mark.parametrize("splits", [1, 2, 3, 4, 5, 6, 8, 9, 15, 16])
def test_every_split_count_folds_to_the_same_attention(binding, oracle, H, splits, fold):
    """cfg2 with the number of key splits in the caller's hands, folded by the workgroup that finishes last
    (fold = 0 leaves the choice to the library: that path, up to 16 partial results) and by the second kernel
    (fold = 1); the workspace is reused for a second call, which must give the same bits."""
    w = WORKLOADS["cfg2"]
    inp = attention_inputs(w, seed=2)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    tuning = binding.AttentionTuning(key_splits=splits, fold=fold)
    ws = binding.new_workspace(binding.tree_attention_tuned_workspace(tuning, 0, ad.B, ad.H, ad.H, ad.d, v.n_nodes, 0, ad.max_prefix))
    ad.out.fill_(float("nan"))
    got = _tuned_attention(binding, v, ad, tuning, ws)
    H.assert_close(got, oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes), "bf16", f"{splits} splits")
    ad.out.fill_(float("nan"))
    again = _tuned_attention(binding, v, ad, tuning, ws)
    assert np.array_equal(got, again), "the second call on the same workspace differs"


@pytest.mark.parametrize("splits", [1, 2, 3])
@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("branching", [(8, 2, 2, 1, 1), (4, 2, 2, 2), (3, 2, 2, 1, 1, 1, 1, 1)])
def test_the_four_stage_ring_matches_the_oracle(binding, oracle, H, branching, d, splits):
    """stages = 4: the four-stage ring of the bf16 sweep (a measurement option), for two and four query blocks and both
    head dimensions.  Prefix lengths from no full tile to more tiles than stages, with and without a ragged last
    tile, in one ragged batch; every element against the oracle."""
    lens = (0, 63, 64, 65, 128, 200, 256, 321, 384, 449, 512, 600, 1024, 1087)
    w = scaled(WORKLOADS["cfg5"], B=len(lens), H=2, d=d, branching=branching, prefix_min=0, prefix_max=max(lens), cfg_id=69)
    inp = attention_inputs(w, seed=7, lens=lens)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(branching), len(branching))
    tuning = binding.AttentionTuning(key_splits=splits, stages=4)
    ad.out.fill_(float("nan"))
    got = _tuned_attention(binding, v, ad, tuning)
    H.assert_close(got, oracle.tree_attention(inp, oracle.build_mask(branching), v.n_nodes), "bf16", f"stages 4, {splits} splits, d {d}")


@pytest.mark.parametrize("tree_keys", [1, 2, 3])
@pytest.mark.parametrize("splits", [2, 3, 6, 7])
def test_the_trees_own_keys_may_go_to_any_workgroup(binding, oracle, H, splits, tree_keys):
    """The tree's keys with a workgroup of their own, with the first split, or with the last split that has keys
    (ragged batch: a different split per sequence; one sequence without any prefix)."""
    w = scaled(WORKLOADS["cfg2"], B=4, H=8, cfg_id=68)
    inp = attention_inputs(w, seed=3, lens=(1024, 0, 130, 577))
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    tuning = binding.AttentionTuning(key_splits=splits, tree_keys=tree_keys)
    ad.out.fill_(float("nan"))
    got = _tuned_attention(binding, v, ad, tuning)
    H.assert_close(got, oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes), "bf16", f"{splits} splits, tree keys {tree_keys}")


@pytest.mark.parametrize("B,Hh,d,lens", [(1, 32, 128, (1024,)), (1, 12, 64, (1024,)), (5, 8, 128, (1024, 0, 130, 577, 900))])
def test_two_hundred_calls_on_one_workspace_give_the_same_bits(binding, H, B, Hh, d, lens):
    """The fold inside the sweep hands the partial results over through arrival counters that every call must leave
    at zero, and whichever workgroup arrives last folds: 200 back-to-back calls on one workspace, without the host
    in between, must all give the bits of the first (whole head counts, one that is rounded up to whole dies, a ragged
    batch)."""
    w = scaled(WORKLOADS["cfg2"], B=B, H=Hh, d=d, cfg_id=70)
    ad = H.AttnDevice(attention_inputs(w, seed=1, lens=lens))
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    ws = binding.new_workspace(binding.tree_attention_workspace(ad.B, ad.H, ad.d, v.n_nodes, ad.max_prefix))
    outs = []
    for i in range(200):
        ad.out.fill_(float("nan"))
        binding.tree_attention(v, ad.code, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp, ad.base, ad.lens,
                               ad.head_stride, ad.max_prefix, ad.scale, ad.out, ws)
        outs.append(ad.out[:, :, :v.n_nodes].clone())
    torch.cuda.synchronize()
    assert bool(torch.isfinite(outs[0].float()).all())
    assert all(torch.equal(o.view(torch.int16), outs[0].view(torch.int16)) for o in outs[1:])


@pytest.mark.parametrize("B,Hh,lens", [(1, 8, (1000,)), (3, 8, (0, 70, 700)), (2, 12, (513, 64)), (1, 3, (900,)), (5, 7, (300,) * 5)])
def test_folds_for_head_counts_that_do_and_do_not_divide_over_the_dies(binding, oracle, H, B, Hh, lens):
    """The in-kernel fold needs all workgroups of a (sequence, head) on one die; with head counts that do not divide
    over the dies the library must take the second kernel instead.  Either way every element matches."""
    br = (4, 2, 2, 1)
    w = scaled(WORKLOADS["cfg2"], B=B, H=Hh, cfg_id=67)
    inp = attention_inputs(w, seed=5, lens=lens)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(br), 4)
    got = H.run_attention(binding, v, ad, fill=float("nan"))
    H.assert_close(got, oracle.tree_attention(inp, oracle.build_mask(br), v.n_nodes), "bf16", f"B{B} H{Hh}")


def test_a_workspace_that_was_never_prepared_poisons_the_output(binding, H):
    """The arrival counters of the fold live in the workspace; one that mcsd_workspace_init never saw must not give
    plausible numbers: the rows come back NaN."""
    w = WORKLOADS["cfg2"]
    ad = H.AttnDevice(attention_inputs(w, seed=0))
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    need = binding.tree_attention_workspace(ad.B, ad.H, ad.d, v.n_nodes, ad.max_prefix)
    ws = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda")
    ad.out.fill_(1.0)
    binding.tree_attention(v, ad.code, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp, ad.base,
                           ad.lens, ad.head_stride, ad.max_prefix, ad.scale, ad.out, ws)
    torch.cuda.synchronize()
    assert bool(torch.isnan(ad.out[:, :, :v.n_nodes].float()).all())
    binding.workspace_init(ws)                              # prepared: the same buffer now serves
    binding.tree_attention(v, ad.code, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp, ad.base,
                           ad.lens, ad.head_stride, ad.max_prefix, ad.scale, ad.out, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(ad.out[:, :, :v.n_nodes].float()).all())


def test_tuning_out_of_range_is_rejected(binding, H):
    w = WORKLOADS["cfg2"]
    ad = H.AttnDevice(attention_inputs(w, seed=0))
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    ws = binding.new_workspace(1 << 24)
    for bad in (binding.AttentionTuning(key_splits=65), binding.AttentionTuning(key_splits=-1), binding.AttentionTuning(tree_keys=4), binding.AttentionTuning(fold=2)):
        with pytest.raises(binding.McsdError) as e:
            _tuned_attention(binding, v, ad, bad, ws)
        assert e.value.status == binding.MCSD_EINVAL


# ------------------------------------------------------------------------------------------------
# verification: bit-exact paths, lengths and tokens
# ------------------------------------------------------------------------------------------------
def _check_verify(binding, oracle, H, w, mode, gamma=None, seed=0, n_new=None):
    g = w.gamma_max if gamma is None else gamma
    vi = verify_inputs(w, seed=seed, gamma=g, mode=mode, n_new=n_new)
    m = binding.build_mask(w.branching)
    v = binding.slice_mask(m, g)
    path, alen, new = H.run_verify(binding, v, mode, vi)
    want_path, want_len, want_new = oracle.verify_tree(mode, w.branching[:g], vi["tokens"], vi["p_target"],
                                                       vi["q_draft"], vi["u_accept"], vi["u_sample"])
    assert np.array_equal(alen, want_len), (alen, want_len)
    assert np.array_equal(path, want_path)
    assert np.array_equal(new, want_new), (new, want_new)
    return alen


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4", "cfg5"])
def test_verify_configs_bit_exact(binding, oracle, H, name, mode):
    w = WORKLOADS[name]
    alen = _check_verify(binding, oracle, H, w, mode)
    assert alen.min() >= (1 if mode == TARGET_INIT else 0)


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_verify_cfg3_every_gamma(binding, oracle, H, mode):
    w = WORKLOADS["cfg3"]
    for g in range(1, 9):
        _check_verify(binding, oracle, H, w, mode, gamma=g)


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_verify_cfg5_gamma4_slice(binding, oracle, H, mode):
    _check_verify(binding, oracle, H, WORKLOADS["cfg5"], mode, gamma=4)


@pytest.mark.parametrize("V", [1, 2, 3, 5, 255, 256, 257, 1000, 1023, 4099, 50001])
@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_verify_vocabulary_sizes(binding, oracle, H, V, mode):
    """Sizes around the 256-element blocks, not multiples of 4 (unaligned rows), and a large odd vocabulary."""
    w = scaled(WORKLOADS["cfg1"], B=6, V=V, branching=(3, 2, 2), cfg_id=60, target_sigma=1.5)
    _check_verify(binding, oracle, H, w, mode, seed=V, n_new=3)


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_verify_largest_vocabulary(binding, oracle, H, mode):
    """V = MCSD_MAX_VOCAB (262144): 1024 blocks, the streamed-row path at its largest; one entry more is refused."""
    V = 262144
    w = scaled(WORKLOADS["cfg1"], B=2, V=V, branching=(3, 2), cfg_id=63, target_sigma=1.5)
    _check_verify(binding, oracle, H, w, mode, seed=5, n_new=3)
    vi = verify_inputs(scaled(w, V=8), seed=0, gamma=2, mode=mode, n_new=3)
    v = binding.slice_mask(binding.build_mask(w.branching), 2)
    dev = {k: H.dev(vi[k]) for k in ("tokens", "p_target", "q_draft", "u_accept", "u_sample")}
    out = [torch.zeros(n, dtype=torch.int32, device="cuda") for n in (2 * 2, 2, 2 * 3)]
    with pytest.raises(binding.McsdError) as e:
        binding.verify_tree(v, mode, 2, V + 1, dev["tokens"], dev["p_target"], dev["q_draft"], 10 * (V + 1), 10 * (V + 1),
                            dev["u_accept"], dev["u_sample"], 3, out[0], out[1], out[2],
                            torch.empty(4096, dtype=torch.uint8, device="cuda"))
    assert e.value.status == binding.MCSD_EUNSUPPORTED


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_verify_deepest_tree(binding, oracle, H, mode):
    """gamma = MCSD_MAX_LEVELS (32): two chains of 32 tokens; high agreement so that walks go deep."""
    br = (2,) + (1,) * 31
    w = scaled(WORKLOADS["cfg1"], B=8, V=300, branching=br, cfg_id=64, target_sigma=1.0, draft_noise_sigma=0.05)
    alen = _check_verify(binding, oracle, H, w, mode, seed=2, n_new=2)
    assert alen.max() >= 8, alen                               # some walk really goes deep
    for g in (1, 17, 31):
        _check_verify(binding, oracle, H, w, mode, gamma=g, seed=3, n_new=2)


def test_verify_many_sequences_and_deep_rejection_chains(binding, oracle, H):
    """Independent draft and target (low acceptance) with wide levels: long chains of residual updates."""
    w = scaled(WORKLOADS["cfg1"], B=64, V=777, branching=(8, 6), cfg_id=61, target_sigma=3.0)
    alen = _check_verify(binding, oracle, H, w, DRAFT_INIT, n_new=2)
    assert (alen == 0).any() and (alen > 0).any()
    _check_verify(binding, oracle, H, w, TARGET_INIT, n_new=5)


def test_verify_special_rows(binding, oracle, H):
    """p == q (everything accepted, bonus from the leaf's row), disjoint supports (everything rejected,
    residual == p), vanished residual (fallback to the target row), all on the device."""
    rng = np.random.default_rng(8)
    br, V, B = (2, 2), 64, 5
    N, Nin = 6, 2
    m = binding.build_mask(br)
    v = binding.slice_mask(m, 2)
    p = rng.random((B, 1 + N, V)).astype(np.float32)
    p /= p.sum(-1, keepdims=True)
    p = p.astype(np.float32)
    ua = rng.random((B, N), dtype=np.float32)
    us = rng.random((B, 2), dtype=np.float32)
    tokens = rng.integers(0, V, size=(B, N)).astype(np.int32)
    cases = {"p == q": (p, p[:, :1 + Nin].copy())}
    pe, qo = np.zeros_like(p), np.zeros((B, 1 + Nin, V), dtype=np.float32)
    pe[:, :, 0::2] = 1 / 32
    qo[:, :, 1::2] = 1 / 32
    cases["disjoint"] = (pe, qo)
    pz = p.copy()
    qz = p[:, :1 + Nin].copy()
    pz[:, :, 0] = 0.0                      # token 0 has p = 0 < q: rejected, then residual is identically zero
    cases["vanished"] = (pz, qz)
    for name, (pp, qq) in cases.items():
        tk = tokens.copy()
        if name == "disjoint":
            tk = (tk | 1).astype(np.int32)
        if name == "vanished":
            tk[:] = 0
        vi = dict(p_target=pp, q_draft=qq, tokens=tk, u_accept=ua, u_sample=us)
        for mode in (DRAFT_INIT, TARGET_INIT):
            got = H.run_verify(binding, v, mode, vi)
            want = oracle.verify_tree(mode, br, tk, pp, qq, ua, us)
            for a, b_ in zip(got, want):
                assert np.array_equal(a, b_), (name, mode, a, b_)


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_verify_fork_shaped_tree_width_16_depth_5(binding, oracle, H, mode):
    """The paper's dynamic setting: 16 candidates at the root (up to 16 rejection rounds there), chains below."""
    w = scaled(WORKLOADS["fork"], B=4)
    _check_verify(binding, oracle, H, w, mode)
    _check_verify(binding, oracle, H, w, mode, gamma=3, seed=5)


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
def test_verify_greedy_target_rows(binding, oracle, H, mode):
    """Temperature 0 (Sec. 4.1): one-hot target rows.  A candidate is accepted iff it is the target's arg-max, and
    the new token is the arg-max of the row the walk ends on; the general rule must reduce to that."""
    w = scaled(WORKLOADS["cfg2"], B=6, V=5000, cfg_id=63)
    vi = verify_inputs(w, seed=3, mode=mode)
    p = vi["p_target"]
    top = p.argmax(-1)
    hot = np.zeros_like(p)
    np.put_along_axis(hot, top[..., None], 1.0, axis=-1)
    tokens = vi["tokens"].copy()
    # make some candidates hit the arg-max of their context so that paths of several lengths occur
    parent, _ = oracle.tree_tables(w.branching)
    rng = np.random.default_rng(12)
    for b in range(w.B):
        for node in range(tokens.shape[1]):
            if rng.random() < 0.45:
                tokens[b, node] = top[b, 1 + parent[node]]
    vi = dict(vi, p_target=hot, tokens=tokens)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    path, alen, new = H.run_verify(binding, v, mode, vi)
    want = oracle.verify_tree(mode, w.branching, tokens, hot, vi["q_draft"], vi["u_accept"], vi["u_sample"])
    for a, b_ in zip((path, alen, new), want):
        assert np.array_equal(a, b_)
    assert len(set(alen.tolist())) > 1
    for b in range(w.B):
        start = 1 if mode == TARGET_INIT else 0           # level-1 nodes of a target-initialised tree are untested
        for j in range(start, alen[b]):
            ctx = -1 if j == 0 else path[b, j - 1]
            assert tokens[b, path[b, j]] == top[b, 1 + ctx]
        last = path[b, alen[b] - 1] if alen[b] else -1
        assert np.all(new[b] == top[b, 1 + last])


def test_verify_without_new_tokens(binding, oracle, H):
    w = scaled(WORKLOADS["cfg1"], B=3, cfg_id=62)
    _check_verify(binding, oracle, H, w, DRAFT_INIT, n_new=0)


# ------------------------------------------------------------------------------------------------
# the whole step under HIP graph capture
# ------------------------------------------------------------------------------------------------
def test_step_replayed_from_a_hip_graph_matches_eager_launches(binding, oracle, H):
    """Attention (split keys, so sweep + fold kernels) and verification captured once and replayed several times,
    with eager work and synchronisations between the replays; every replay must leave the eager results."""
    w = WORKLOADS["cfg2"]
    inp = attention_inputs(w, seed=2)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    ws = binding.new_workspace(binding.tree_attention_workspace(ad.B, ad.H, ad.d, v.n_nodes, ad.max_prefix))
    vi = verify_inputs(w, seed=2, gamma=w.gamma_max, mode=DRAFT_INIT)
    p, q = H.dev(vi["p_target"]), H.dev(vi["q_draft"])
    tokens, ua, us = H.dev(vi["tokens"]), H.dev(vi["u_accept"]), H.dev(vi["u_sample"])
    n_new = vi["u_sample"].shape[1]
    path = torch.zeros((w.B, v.gamma), dtype=torch.int32, device="cuda")
    alen = torch.zeros((w.B,), dtype=torch.int32, device="cuda")
    new = torch.zeros((w.B, n_new), dtype=torch.int32, device="cuda")

    def step():
        binding.tree_attention(v, ad.code, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp,
                               ad.base, ad.lens, ad.head_stride, ad.max_prefix, ad.scale, ad.out, ws)
        binding.verify_tree(v, DRAFT_INIT, w.B, w.V, tokens, p, q, vi["p_target"].shape[1] * w.V,
                            vi["q_draft"].shape[1] * w.V, ua, us, n_new, path, alen, new, None)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (ad.out, path, alen, new)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for r in range(4):
        for t in (ad.out, path, alen, new):
            t.fill_(-3)                                  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, (ad.out, path, alen, new)):
            assert torch.equal(a, b), f"replay {r} differs from the eager step"
    M = oracle.build_mask(w.branching)
    H.assert_close(ad.out[:, :, :v.n_nodes].float().cpu().numpy().astype(np.float64),
                   oracle.tree_attention(inp, M, v.n_nodes), "bf16", "graph replay")


# ------------------------------------------------------------------------------------------------
# update after acceptance: the accepted path joins the prefix cache (Fig. 1 step 6)
# ------------------------------------------------------------------------------------------------
def _commit_case(binding, oracle, H, w, mode, lens, n_layers, seed, gamma=None, explicit=None):
    gamma = w.gamma_max if gamma is None else gamma
    cap = int(max(lens)) + gamma + 5
    layers_host = [attention_inputs(w, seed=seed, lens=lens, kv_capacity=cap, variant=l) for l in range(n_layers)]
    layers = [H.AttnDevice(inp) for inp in layers_host]
    v = binding.slice_mask(binding.build_mask(w.branching), gamma)
    vi = verify_inputs(w, seed=seed, gamma=gamma, mode=mode)
    path, alen, new = H.run_verify(binding, v, mode, vi)                       # numpy results of the GPU walk
    want_v = oracle.verify_tree(mode, w.branching[:gamma], vi["tokens"], vi["p_target"], vi["q_draft"], vi["u_accept"],
                                vi["u_sample"])
    assert np.array_equal(path, want_v[0]) and np.array_equal(alen, want_v[1])
    if explicit is not None:                                                   # paths chosen by hand instead
        path, alen = explicit
    n_new = vi["u_sample"].shape[1]
    n_append = 1 if mode == DRAFT_INIT and n_new > 0 else 0
    d_path, d_alen, d_new = H.dev(path), H.dev(alen), H.dev(new.reshape(w.B, -1))
    d_tokens = H.dev(vi["tokens"])
    lens_dev = layers[0].lens.clone()
    ids = torch.full((w.B, gamma + n_append), -9, dtype=torch.int32, device="cuda")
    n_ids = torch.full((w.B,), -9, dtype=torch.int32, device="cuda")
    a0 = layers[0]
    binding.commit_path(v, a0.code, a0.B, a0.H, a0.d, [a.kt for a in layers], [a.vt for a in layers], a0.node_stride,
                        [a.kp for a in layers], [a.vp for a in layers], a0.base, a0.head_stride, int(max(lens)), cap,
                        d_path, d_alen, d_tokens, d_new, n_new, n_append, lens_dev, ids, n_ids)
    torch.cuda.synchronize()
    for l, (inp, ad) in enumerate(zip(layers_host, layers)):
        kp, vp, new_lens = oracle.commit_path(inp, gamma, v.n_nodes, path, alen)
        store = torch.int16 if inp["dtype"] == "bf16" else torch.float32
        assert np.array_equal(ad.kp.view(store).cpu().numpy().view(kp.dtype), kp), f"layer {l}: K cache differs"
        assert np.array_equal(ad.vp.view(store).cpu().numpy().view(vp.dtype), vp), f"layer {l}: V cache differs"
    assert np.array_equal(lens_dev.cpu().numpy(), new_lens)
    want_ids, want_n = oracle.commit_ids(gamma, vi["tokens"], path, alen, new.reshape(w.B, -1), n_append)
    assert np.array_equal(ids.cpu().numpy(), want_ids) and np.array_equal(n_ids.cpu().numpy(), want_n)
    return layers_host, layers, lens_dev, path, alen


@pytest.mark.parametrize("mode", [DRAFT_INIT, TARGET_INIT])
@pytest.mark.parametrize("name,B,Hh", [("cfg1", 1, 4), ("cfg2", 1, 32), ("cfg4", 16, 4), ("cfg5", 8, 4)])
def test_commit_path_bit_exact(binding, oracle, H, name, B, Hh, mode):
    w = scaled(WORKLOADS[name], B=B, H=Hh, cfg_id=70)
    lens = [37 + 61 * b for b in range(B)]
    _commit_case(binding, oracle, H, w, mode, lens, n_layers=3, seed=4)


def test_commit_path_nothing_accepted_and_full_depth(binding, oracle, H):
    w = scaled(WORKLOADS["cfg3"], B=4, H=2, cfg_id=71)
    parent, level = oracle.tree_tables(w.branching)
    path = np.full((4, 8), -1, dtype=np.int32)
    alen = np.array([0, 8, 3, 1], dtype=np.int32)
    for b, leaf in ((1, int(np.where(level == 8)[0][-1])), (2, int(np.where(level == 3)[0][4])), (3, 2)):
        chain = []
        while leaf >= 0:
            chain.append(leaf)
            leaf = int(parent[leaf])
        path[b, :len(chain)] = chain[::-1]
        assert len(chain) == alen[b]
    _commit_case(binding, oracle, H, w, DRAFT_INIT, [0, 5, 64, 9], n_layers=2, seed=1, explicit=(path, alen))


def test_commit_then_attend_over_the_grown_cache(binding, oracle, H):
    """The next iteration's tree attention reads the cache and the lengths exactly as the commit left them."""
    w = scaled(WORKLOADS["cfg2"], B=2, H=4, cfg_id=72)
    lens = [200, 77]
    layers_host, layers, lens_dev, path, alen = _commit_case(binding, oracle, H, w, TARGET_INIT, lens, n_layers=1, seed=6)
    inp, ad = layers_host[0], layers[0]
    kp, vp, new_lens = oracle.commit_path(inp, w.gamma_max, w.n_nodes(), path, alen)
    assert int(alen.min()) >= 1
    grown = dict(inp, k_prefix=kp, v_prefix=vp, lens=new_lens)
    ad.lens.copy_(lens_dev)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    got = H.run_attention(binding, v, ad, max_prefix=int(max(lens)) + w.gamma_max)
    want = oracle.tree_attention(grown, oracle.build_mask(w.branching), v.n_nodes)
    H.assert_close(got, want, "bf16", "attention after commit")


def test_commit_path_rejects_bad_arguments(binding, H):
    w = scaled(WORKLOADS["cfg2"], B=1, H=2, cfg_id=73)
    inp = attention_inputs(w, seed=0, lens=[10], kv_capacity=12)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), 4)
    z = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    args = lambda n_layers, cap, n_append: (v, ad.code, 1, 2, ad.d, [ad.kt] * n_layers, [ad.vt] * n_layers, ad.node_stride,
                                             [ad.kp] * n_layers, [ad.vp] * n_layers, ad.base, ad.head_stride, 10, cap,
                                             z, z, z, z, 1, n_append, ad.lens, z, z)
    with pytest.raises(RuntimeError):
        binding.commit_path(*args(1, 12, 1))          # capacity < max_prefix + gamma
    with pytest.raises(RuntimeError):
        binding.commit_path(*args(65, 14, 1))         # more layers than one call takes
    with pytest.raises(RuntimeError):
        binding.commit_path(*args(1, 14, 2))          # n_append > n_new
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------------
# draft side: attention for the newest tree level only, the mask sliced anew at every level (Fig. 1 step 3, Sec. 3.2)
# ------------------------------------------------------------------------------------------------
def _attend_rows(binding, H, v, ad, row_begin, max_prefix, fill):
    ws_bytes = binding.tree_attention_rows_workspace(ad.B, ad.H, ad.d, v.n_nodes, row_begin, max_prefix)
    assert ws_bytes <= binding.tree_attention_workspace(ad.B, ad.H, ad.d, v.n_nodes, max_prefix)
    ws = binding.new_workspace(ws_bytes)
    ad.out.fill_(fill)
    binding.tree_attention_rows(v, ad.code, ad.B, ad.H, ad.d, row_begin, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp,
                                ad.vp, ad.base, ad.lens, ad.head_stride, max_prefix, ad.scale, ad.out, ws)
    torch.cuda.synchronize()
    return ad.out.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("name,B,Hh,lens", [("cfg3", 1, 32, None), ("cfg5", 2, 4, (700, 33)), ("cfg1", 1, 4, None),
                                            ("cfg4", 16, 32, None)])
def test_level_by_level_attention_with_a_fresh_slice_per_level(binding, oracle, H, name, B, Hh, lens):
    w = scaled(WORKLOADS[name], B=B, H=Hh, cfg_id=80)
    if name == "cfg4":
        w = scaled(w, prefix_min=64, prefix_max=512)
    inp = attention_inputs(w, seed=8, lens=lens)
    ad = H.AttnDevice(inp)
    m = binding.build_mask(w.branching)                      # once, for the deepest tree
    M = oracle.build_mask(w.branching)
    for g in range(1, w.gamma_max + 1):
        v = binding.slice_mask(m, g)
        row_begin = int(v.level_off_host[g - 1])
        out = _attend_rows(binding, H, v, ad, row_begin, ad.max_prefix, fill=55.0)
        want = oracle.tree_attention(inp, M, v.n_nodes)
        H.assert_close(out[:, :, row_begin:v.n_nodes], want[:, :, row_begin:], w.dtype, f"{name} level {g}")
        assert np.all(out[:, :, :row_begin] == 55.0) and np.all(out[:, :, v.n_nodes:] == 55.0), "rows outside the level touched"


@pytest.mark.parametrize("row_begin", [0, 1, 31, 32, 33, 64, 100, 119])
def test_attention_rows_any_first_row(binding, oracle, H, row_begin):
    w = scaled(WORKLOADS["cfg5"], B=1, H=8, cfg_id=81)
    inp = attention_inputs(w, seed=row_begin, lens=(1500,))
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    out = _attend_rows(binding, H, v, ad, row_begin, 1500, fill=-4.0)
    want = oracle.tree_attention(inp, oracle.build_mask(w.branching), v.n_nodes)
    H.assert_close(out[:, :, row_begin:v.n_nodes], want[:, :, row_begin:], "bf16", f"rows from {row_begin}")
    assert np.all(out[:, :, :row_begin] == -4.0)
    with pytest.raises(binding.McsdError):
        binding.tree_attention_rows(v, ad.code, 1, 8, ad.d, v.n_nodes, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp,
                                    ad.base, ad.lens, ad.head_stride, 1500, ad.scale, ad.out, None)


# ------------------------------------------------------------------------------------------------
# grouped-query attention: several query heads share the K/V of one head
# ------------------------------------------------------------------------------------------------
def _gqa_case(binding, oracle, H, br, B, Hq, Hkv, d, dtype, lens, max_prefix=None, row_begin=0, seed=0):
    wq = scaled(WORKLOADS["cfg2"], B=B, H=Hq, d=d, dtype=dtype, branching=tuple(br), cfg_id=90)
    wk = scaled(wq, H=Hkv, cfg_id=91)
    qi = attention_inputs(wq, seed=seed, lens=lens)               # q of all query heads
    ki = attention_inputs(wk, seed=seed, lens=lens)               # K/V of the shared heads
    G = Hq // Hkv
    cap = ki["k_prefix"].shape[2]
    # what the oracle sees: plain multi-head attention with every K/V head repeated for its G query heads
    rep = dict(qi, k_tree=np.repeat(ki["k_tree"], G, axis=1), v_tree=np.repeat(ki["v_tree"], G, axis=1),
               k_prefix=np.repeat(ki["k_prefix"], G, axis=1), v_prefix=np.repeat(ki["v_prefix"], G, axis=1),
               head_stride=cap * d, seq_base=(np.arange(B, dtype=np.int64) * (Hq * cap * d)))
    aq, ak = H.AttnDevice(qi), H.AttnDevice(ki)
    m = binding.build_mask(br)
    v = binding.slice_mask(m, len(br))
    mp = ak.max_prefix if max_prefix is None else max_prefix
    ws_bytes = binding.tree_attention_gqa_workspace(B, Hq, Hkv, d, v.n_nodes, row_begin, mp)
    ws = binding.new_workspace(ws_bytes)
    aq.out.fill_(31.0)
    binding.tree_attention_gqa(v, aq.code, B, Hq, Hkv, d, row_begin, aq.q, ak.kt, ak.vt, ak.node_stride, ak.kp, ak.vp,
                               ak.base, ak.lens, ak.head_stride, mp, aq.scale, aq.out, ws)
    torch.cuda.synchronize()
    got = aq.out.float().cpu().numpy().astype(np.float64)
    want = oracle.tree_attention(rep, oracle.build_mask(br), v.n_nodes)
    H.assert_close(got[:, :, row_begin:v.n_nodes], want[:, :, row_begin:], dtype, f"gqa {Hq}/{Hkv} tree {br}")
    assert np.all(got[:, :, :row_begin] == 31.0) and np.all(got[:, :, v.n_nodes:] == 31.0)


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (8, 2), (8, 1), (12, 4), (6, 2)])
@pytest.mark.parametrize("br,dtype,d", [((4, 2, 2, 1), "bf16", 128), ((3, 2), "bf16", 128), ((8, 2, 2, 1, 1), "bf16", 128),
                                        ((3, 2, 2, 1, 1, 1, 1, 1), "bf16", 64), ((4, 2, 2, 2), "bf16", 64),
                                        ((2, 2, 2), "f32", 64)])
def test_grouped_query_attention(binding, oracle, H, br, dtype, d, Hq, Hkv):
    _gqa_case(binding, oracle, H, br, 2, Hq, Hkv, d, dtype, lens=(150, 37))


def test_grouped_query_attention_split_keys_and_levels(binding, oracle, H):
    # long prefix with few heads: the keys are split over workgroups and folded; then the newest level only
    _gqa_case(binding, oracle, H, (4, 2, 2, 1), 1, 8, 2, 128, "bf16", lens=(2000,))
    _gqa_case(binding, oracle, H, (4, 2, 2, 1), 1, 8, 2, 128, "bf16", lens=(2000,), row_begin=28)
    _gqa_case(binding, oracle, H, (8, 2, 2, 1, 1), 2, 16, 4, 128, "bf16", lens=(900, 1300), row_begin=88)
    _gqa_case(binding, oracle, H, (2, 2, 2), 1, 4, 2, 64, "f32", lens=(300,), row_begin=6)


def test_grouped_query_attention_llama3_like_batch(binding, oracle, H):
    """32 query heads on 8 key/value heads, 16 ragged sequences (the pairing mode's grid: 16 x 8 x 4 = 512 units)."""
    br = (4, 2, 2, 2)
    B, Hq, Hkv, d = 16, 32, 8, 128
    rng = np.random.default_rng(3)
    lens = tuple(int(x) for x in rng.integers(40, 700, size=B))
    wq = scaled(WORKLOADS["cfg4"], B=B, H=Hq, cfg_id=92)
    wk = scaled(wq, H=Hkv, cfg_id=93)
    qi, ki = attention_inputs(wq, seed=1, lens=lens), attention_inputs(wk, seed=1, lens=lens)
    G, cap = Hq // Hkv, ki["k_prefix"].shape[2]
    rep = dict(qi, k_tree=np.repeat(ki["k_tree"], G, axis=1), v_tree=np.repeat(ki["v_tree"], G, axis=1),
               k_prefix=np.repeat(ki["k_prefix"], G, axis=1), v_prefix=np.repeat(ki["v_prefix"], G, axis=1),
               head_stride=cap * d, seq_base=(np.arange(B, dtype=np.int64) * (Hq * cap * d)))
    aq, ak = H.AttnDevice(qi), H.AttnDevice(ki)
    v = binding.slice_mask(binding.build_mask(br), 4)
    ws = binding.new_workspace(binding.tree_attention_gqa_workspace(B, Hq, Hkv, d, v.n_nodes, 0, 700))
    binding.tree_attention_gqa(v, aq.code, B, Hq, Hkv, d, 0, aq.q, ak.kt, ak.vt, ak.node_stride, ak.kp, ak.vp, ak.base,
                               ak.lens, ak.head_stride, 700, aq.scale, aq.out, ws)
    torch.cuda.synchronize()
    got = aq.out[:, :, :v.n_nodes].float().cpu().numpy().astype(np.float64)
    H.assert_close(got, oracle.tree_attention(rep, oracle.build_mask(br), v.n_nodes), "bf16", "gqa ragged batch")
    with pytest.raises(binding.McsdError):
        binding.tree_attention_gqa(v, aq.code, B, Hq, 5, d, 0, aq.q, ak.kt, ak.vt, ak.node_stride, ak.kp, ak.vp, ak.base,
                                   ak.lens, ak.head_stride, 700, aq.scale, aq.out, ws)


@pytest.mark.parametrize("B,Hh", [(12, 32), (24, 32), (5, 64), (40, 16)])
def test_ragged_batches_with_more_workgroups_than_compute_units(binding, oracle, H, B, Hh):
    """Grids between one and two workgroups per compute unit (long/short pairs, some compute units with one
    workgroup) and beyond two (longest first): the order in which workgroups take (sequence, head) items is
    computed in the kernel from the lengths; every item must still be computed exactly once."""
    br = (4, 2, 2, 2)
    rng = np.random.default_rng(B * 100 + Hh)
    lens = tuple(int(x) for x in rng.integers(0, 600, size=B))
    w = scaled(WORKLOADS["cfg4"], B=B, H=Hh, cfg_id=96)
    inp = attention_inputs(w, seed=3, lens=lens, kv_capacity=640)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(br), 4)
    got = H.run_attention(binding, v, ad, max_prefix=640, fill=float("nan"))
    # the output started as NaN: every row of every (sequence, head) was written, and with the right values
    H.assert_close(got, oracle.tree_attention(inp, oracle.build_mask(br), v.n_nodes), "bf16", f"B{B} H{Hh}")


# ------------------------------------------------------------------------------------------------
# measurement aids
def test_issue_probe_runs_every_schedule_and_rejects_bad_arguments(binding):
    """The matrix / vector overlap probe (a measurement aid): every schedule runs to completion and writes finite
    values; arguments outside the documented ranges are refused before anything is launched."""
    out = torch.full((4 * 512,), float("nan"), dtype=torch.float32, device="cuda")
    for schedule in range(5):
        out.fill_(float("nan"))
        binding.issue_probe(schedule, 4, 16, out)
        torch.cuda.synchronize()
        lanes = out.view(4, 512)[:, :256] if schedule in (0, 3) else out.view(4, 512)    # one wavefront per SIMD: the upper half retires at once
        assert bool(torch.isfinite(lanes).all()), schedule
    for bad in ((5, 4, 16), (-1, 4, 16), (0, 0, 16), (0, 4, 15), (0, 4, 0), (0, 70000, 16)):
        with pytest.raises(binding.McsdError) as e:
            binding.issue_probe(*bad, out)
        assert e.value.status == binding.MCSD_EINVAL


def test_placement_probe_reports_dies_and_compute_units(binding):
    """The placement probe (a measurement aid): ids congruent modulo the number of dies share a die, which is what
    the fold inside the sweep relies on (the library checks it itself before planning that fold)."""
    n = 64
    out = torch.full((2 * n,), -1, dtype=torch.int32, device="cuda")
    binding.placement_probe(n, 1000, out)
    torch.cuda.synchronize()
    die = out.cpu().numpy().reshape(n, 2)[:, 0]
    n_die = int(die.max()) + 1
    assert n_die in (1, 2, 4, 8) and (die >= 0).all()
    assert all(die[i] == die[i % n_die] for i in range(n))
    with pytest.raises(binding.McsdError):
        binding.placement_probe(0, 0, out)

