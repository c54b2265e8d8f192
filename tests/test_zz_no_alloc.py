"""mcsd_tree_attention_static (the entry point that allocates nothing: its workspace is a device array inside the
library) against mcsd_tree_attention on the same inputs, through the C ABI.  Both run the same kernels under the same
plan, so the outputs must agree bit for bit, also on a second call with a smaller input that finds the array as the
first call left it.  Collected last: a failure here must not hide the tests after it."""
import numpy as np
import pytest
import torch

from workloads import WORKLOADS, attention_inputs, scaled

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


def _both(binding, H, w, seed, lens=None, gamma=None):
    inp = attention_inputs(w, seed=seed, lens=lens)
    ad = H.AttnDevice(inp)
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max if gamma is None else gamma)
    want = H.run_attention(binding, v, ad, fill=float("nan"))              # the existing entry point, own workspace
    ad.out.fill_(float("nan"))
    binding.tree_attention_static(v, ad.code, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp, ad.base,
                                  ad.lens, ad.head_stride, ad.max_prefix, ad.scale, ad.out)
    torch.cuda.synchronize()
    got = ad.out[:, :, :v.n_nodes].float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got)), f"{w.name}: rows not written"
    assert np.array_equal(got, want), f"{w.name}: static-scratch entry point differs from mcsd_tree_attention"
    return inp, v, got


def test_two_calls_in_a_row_the_second_smaller(binding, oracle, H):
    # cfg3's shape (81 nodes, 2048 keys, 6 key splits + the tree's workgroup), then cfg2's (44 nodes, 1024 keys)
    inp3, v3, got3 = _both(binding, H, WORKLOADS["cfg3"], seed=3)
    inp2, v2, got2 = _both(binding, H, WORKLOADS["cfg2"], seed=4)
    H.assert_close(got3, oracle.tree_attention(inp3, oracle.build_mask(WORKLOADS["cfg3"].branching), v3.n_nodes), "bf16", "cfg3 static")
    H.assert_close(got2, oracle.tree_attention(inp2, oracle.build_mask(WORKLOADS["cfg2"].branching), v2.n_nodes), "bf16", "cfg2 static")
    # a third, smaller still and in fp32 (second kernel folds), and one that needs no workspace at all
    _both(binding, H, WORKLOADS["cfg1"], seed=0)
    _both(binding, H, scaled(WORKLOADS["cfg4"], B=16, H=32, cfg_id=97), seed=1, lens=tuple(range(40, 680, 40)))


def test_the_same_call_repeated_gives_the_same_bits(binding, H):
    _, _, a = _both(binding, H, WORKLOADS["cfg2"], seed=5)
    _, _, b = _both(binding, H, WORKLOADS["cfg2"], seed=5)
    assert np.array_equal(a, b)


def test_shapes_beyond_the_array_are_rejected_before_any_launch(binding, H):
    w = scaled(WORKLOADS["cfg5"], B=14, prefix_min=64, prefix_max=64, cfg_id=98)     # the plan is made from max_prefix
    ad = H.AttnDevice(attention_inputs(w, seed=0))
    v = binding.slice_mask(binding.build_mask(w.branching), w.gamma_max)
    assert binding.tree_attention_workspace(ad.B, ad.H, ad.d, v.n_nodes, 16384) > binding.STATIC_SCRATCH_BYTES
    ad.out.fill_(7.0)
    with pytest.raises(binding.McsdError) as e:
        binding.tree_attention_static(v, ad.code, ad.B, ad.H, ad.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp,
                                      ad.base, ad.lens, ad.head_stride, 16384, ad.scale, ad.out)
    assert e.value.status == binding.MCSD_EUNSUPPORTED
    torch.cuda.synchronize()
    assert bool((ad.out == 7.0).all())                     # nothing was enqueued
    with pytest.raises(binding.McsdError) as e:            # argument errors are reported as by mcsd_tree_attention
        binding.tree_attention_static(v, ad.code, ad.B, ad.H, 96, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp,
                                      ad.base, ad.lens, ad.head_stride, 64, ad.scale, ad.out)
    assert e.value.status in (binding.MCSD_EUNSUPPORTED, binding.MCSD_EINVAL)
