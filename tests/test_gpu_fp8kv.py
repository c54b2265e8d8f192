"""GPU parity of mcsd_tree_attention_fp8kv (bf16 queries and tree keys/values over an fp8 E4M3 prefix cache) against
the CPU oracle on the same seeded inputs, to the bf16 path's tolerance (2e-2 relative + 1e-2 absolute): the kernel
converts fp8 to bf16 exactly, so its arithmetic is that of the bf16 sweep."""
import numpy as np
import pytest
import torch

from workloads import WORKLOADS, attention_inputs, e4m3_bits_to_f32, f32_to_e4m3_bits, scaled

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


class Dev:
    def __init__(self, H, inp):
        self.q, self.kt, self.vt = (H.dev(inp[k], "bf16") for k in ("q", "k_tree", "v_tree"))
        self.kp, self.vp = (torch.from_numpy(inp[k]).cuda() for k in ("k_prefix", "v_prefix"))
        assert self.kp.dtype == torch.uint8
        self.lens = H.dev(np.ascontiguousarray(inp["lens"], dtype=np.int32))
        self.base = H.dev(np.ascontiguousarray(inp["seq_base"], dtype=np.int64))
        self.B, self.H, self.node_stride, self.d = inp["q"].shape
        self.head_stride = int(inp["head_stride"])
        self.max_prefix = int(max(int(np.max(inp["lens"])), 0))
        self.scale = float(np.float32(inp["scale"]))
        self.ks, self.vs = inp["k_scale"], inp["v_scale"]
        self.out = torch.full(self.q.shape, 31.0, dtype=torch.bfloat16, device="cuda")


def run(binding, view, qd, kd, Hq, Hkv, row_begin=0, max_prefix=None, tuning=None):
    mp = kd.max_prefix if max_prefix is None else max_prefix
    if tuning is None:
        ws = binding.new_workspace(binding.tree_attention_fp8kv_workspace(qd.B, Hq, Hkv, view.n_nodes, row_begin, mp))
        binding.tree_attention_fp8kv(view, qd.B, Hq, Hkv, row_begin, qd.q, kd.kt, kd.vt, kd.node_stride, kd.kp, kd.vp,
                                     kd.ks, kd.vs, kd.base, kd.lens, kd.head_stride, mp, qd.scale, qd.out, ws)
    else:
        ws = binding.new_workspace(binding.tree_attention_tuned_workspace(tuning, 1, qd.B, Hq, Hkv, 128, view.n_nodes,
                                                                          row_begin, mp))
        binding.tree_attention_tuned(tuning, view, 1, 1, kd.ks, kd.vs, qd.B, Hq, Hkv, 128, row_begin, qd.q, kd.kt, kd.vt,
                                     kd.node_stride, kd.kp, kd.vp, kd.base, kd.lens, kd.head_stride, mp, qd.scale,
                                     qd.out, ws)
    torch.cuda.synchronize()
    return qd.out.float().cpu().numpy().astype(np.float64)


def case(binding, oracle, H, br, B, Hh, lens, scales=(0.5, 0.25), seed=0, cfg_id=80, cap=None, row_begin=0, tuning=None):
    w = scaled(WORKLOADS["cfg2"], B=B, H=Hh, branching=br, cfg_id=cfg_id)
    inp = attention_inputs(w, seed=seed, lens=lens, kv_fp8=scales, kv_capacity=cap)
    d = Dev(H, inp)
    v = binding.slice_mask(binding.build_mask(br), len(br))
    got = run(binding, v, d, d, Hh, Hh, row_begin, tuning=tuning)
    want = oracle.tree_attention_fp8kv(inp, oracle.build_mask(br), v.n_nodes)
    H.assert_close(got[:, :, row_begin:v.n_nodes], want[:, :, row_begin:], "bf16", f"fp8kv tree {br} lens {lens}")
    assert np.all(got[:, :, :row_begin] == 31.0)            # rows before row_begin are never written
    return got


def test_cfg2_shape_with_split_keys(binding, oracle, H):
    w = WORKLOADS["cfg2"]
    got = case(binding, oracle, H, w.branching, 1, 32, (1024,))
    again = case(binding, oracle, H, w.branching, 1, 32, (1024,))
    assert np.array_equal(got, again)                       # deterministic


TREES = [(4, 2, 2, 1), (3, 2), (8, 2, 2, 1, 1)]           # 44 nodes (two query blocks), 9 (one, run as two), 120 (four)


@pytest.mark.parametrize("br", TREES)
@pytest.mark.parametrize("L", [0, 1, 63, 64, 65, 128, 200, 273, 1000, 2049])
def test_prefix_lengths_around_tile_and_split_boundaries(binding, oracle, H, br, L):
    case(binding, oracle, H, br, 1, 2, (L,), cfg_id=81)


@pytest.mark.parametrize("br", [(4, 2, 2, 1), (8, 2, 2, 1, 1)])
@pytest.mark.parametrize("tiles", [1, 2, 3, 4, 5, 6, 7, 8, 9, 13])
def test_every_length_of_the_four_stage_ring(binding, oracle, H, br, tiles):
    """One workgroup walks all the tiles of a head (no key splits): every remainder of the unrolled step sequence."""
    one = binding.AttentionTuning(key_splits=1)
    case(binding, oracle, H, br, 1, 2, (64 * tiles,), cfg_id=82, tuning=one)
    case(binding, oracle, H, br, 2, 1, (64 * tiles + 17, 64 * tiles), cfg_id=83, tuning=one)


def test_ragged_batch_two_workgroups_per_compute_unit(binding, oracle, H):
    """16 sequences x 32 heads = 512 workgroups: the grid of the pairing mode."""
    br = (4, 2, 2, 2)
    rng = np.random.default_rng(7)
    lens = tuple(int(x) for x in rng.integers(0, 700, size=16))
    w = scaled(WORKLOADS["cfg4"], cfg_id=84)
    inp = attention_inputs(w, seed=2, lens=lens, kv_fp8=(0.5, 0.5), kv_capacity=704)
    d = Dev(H, inp)
    v = binding.slice_mask(binding.build_mask(br), 4)
    d.out.fill_(float("nan"))
    got = run(binding, v, d, d, 32, 32)
    want = oracle.tree_attention_fp8kv(inp, oracle.build_mask(br), v.n_nodes)
    H.assert_close(got[:, :, :v.n_nodes], want, "bf16", "fp8kv ragged batch, every element")


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (8, 2), (12, 4), (6, 2)])
@pytest.mark.parametrize("br,row_begin", [((4, 2, 2, 1), 0), ((3, 2), 3), ((8, 2, 2, 1, 1), 88)])
def test_grouped_query_heads_and_newest_level_only(binding, oracle, H, br, row_begin, Hq, Hkv):
    B, lens = 2, (150, 37)
    wq = scaled(WORKLOADS["cfg2"], B=B, H=Hq, branching=br, cfg_id=85)
    wk = scaled(wq, H=Hkv, cfg_id=86)
    qi = attention_inputs(wq, seed=1, lens=lens, kv_fp8=(0.37, 0.61))
    ki = attention_inputs(wk, seed=1, lens=lens, kv_fp8=(0.37, 0.61))
    G, cap, dd = Hq // Hkv, ki["k_prefix"].shape[2], 128
    rep = dict(qi, k_tree=np.repeat(ki["k_tree"], G, axis=1), v_tree=np.repeat(ki["v_tree"], G, axis=1),
               k_prefix=np.repeat(ki["k_prefix"], G, axis=1), v_prefix=np.repeat(ki["v_prefix"], G, axis=1),
               head_stride=cap * dd, seq_base=(np.arange(B, dtype=np.int64) * (Hq * cap * dd)))
    qd, kd = Dev(H, qi), Dev(H, ki)
    v = binding.slice_mask(binding.build_mask(br), len(br))
    got = run(binding, v, qd, kd, Hq, Hkv, row_begin)
    want = oracle.tree_attention_fp8kv(rep, oracle.build_mask(br), v.n_nodes)
    H.assert_close(got[:, :, row_begin:v.n_nodes], want[:, :, row_begin:], "bf16", f"fp8kv gqa {Hq}/{Hkv}")
    assert np.all(got[:, :, :row_begin] == 31.0)


def test_extreme_codes_in_the_cache(binding, oracle, H):
    """Largest finite values, subnormals, both zeros: conversion must be exact for every code that is a number."""
    br = (4, 2, 2, 1)
    w = scaled(WORKLOADS["cfg2"], B=1, H=2, branching=br, cfg_id=87)
    inp = attention_inputs(w, seed=3, lens=(300,), kv_fp8=(1.0 / 64, 1.0 / 256))
    rng = np.random.default_rng(11)
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    inp["k_prefix"][:, :, :300] = rng.choice(codes, size=(1, 2, 300, 128))
    inp["v_prefix"][:, :, :300] = rng.choice(codes, size=(1, 2, 300, 128))
    assert np.abs(e4m3_bits_to_f32(inp["k_prefix"])).max() == 448.0
    d = Dev(H, inp)
    v = binding.slice_mask(binding.build_mask(br), 4)
    got = run(binding, v, d, d, 2, 2)
    want = oracle.tree_attention_fp8kv(inp, oracle.build_mask(br), v.n_nodes)
    H.assert_close(got[:, :, :v.n_nodes], want, "bf16", "all fp8 codes")


def test_bad_arguments_are_status_codes(binding, H):
    br = (4, 2, 2, 1)
    w = scaled(WORKLOADS["cfg2"], B=1, H=2, branching=br, cfg_id=88)
    inp = attention_inputs(w, seed=0, lens=(2000,), kv_fp8=(0.5, 0.5))
    d = Dev(H, inp)
    v = binding.slice_mask(binding.build_mask(br), 4)
    ws = binding.new_workspace(binding.tree_attention_fp8kv_workspace(1, 2, 2, v.n_nodes, 0, 2000))

    def call(ks=0.5, vs=0.5, head_stride=d.head_stride, workspace=ws, Hkv=2):
        binding.tree_attention_fp8kv(v, 1, 2, Hkv, 0, d.q, d.kt, d.vt, d.node_stride, d.kp, d.vp, ks, vs, d.base, d.lens,
                                     head_stride, 2000, d.scale, d.out, workspace)

    call()
    torch.cuda.synchronize()
    for kw, status in ((dict(ks=0.0), binding.MCSD_EINVAL), (dict(ks=-1.0), binding.MCSD_EINVAL),
                       (dict(ks=float("inf")), binding.MCSD_EINVAL), (dict(vs=float("nan")), binding.MCSD_EINVAL),
                       (dict(head_stride=d.head_stride + 8), binding.MCSD_EINVAL),
                       (dict(workspace=ws[:256]), binding.MCSD_EWORKSPACE), (dict(workspace=None), binding.MCSD_EWORKSPACE),
                       (dict(Hkv=3), binding.MCSD_EINVAL)):
        with pytest.raises(binding.McsdError) as e:
            call(**kw)
        assert e.value.status == status, kw
    assert binding.tree_attention_fp8kv_workspace(1, 2, 2, 129, 0, 2000) == 0
