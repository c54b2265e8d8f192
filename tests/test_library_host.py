"""No-GPU checks of libmcsd.so: it loads, exports every symbol the header declares, its host-side mask
logic matches the oracle bit for bit, and argument validation answers with status codes."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

TREES = [(2, 2, 2), (4, 2, 2, 1), (3, 2, 2, 1, 1, 1, 1, 1), (4, 2, 2, 2), (8, 2, 2, 1, 1), (2, 4, 3, 1, 1),
         (3, 1, 1), (1, 1, 1), (1,), (16, 1, 1, 1, 1), (8, 3, 4), (5, 5, 5)]


@pytest.fixture(scope="module")
def binding():
    from paper_2409_10644_amd import binding as b
    return b


def test_every_declared_symbol_is_exported(binding):
    header = open(os.path.join(ROOT, "include", "mcsd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(mcsd_[a-z0-9_]+)\s*\(", header)))
    assert declared == sorted(binding.EXPORTS)
    lib = C.CDLL(binding.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("br", TREES)
def test_mask_and_every_slice_match_the_oracle(binding, oracle, br):
    m = binding.build_mask(br)
    full = oracle.build_mask(br)
    parent, level = oracle.tree_tables(br)
    sizes = oracle.level_sizes(br)
    for g in range(1, len(br) + 1):
        v = binding.slice_mask(m, g)
        n = int(sizes[:g].sum())
        assert (v.gamma, v.n_nodes, v.gamma_max, v.n_nodes_max) == (g, n, len(br), full.shape[0])
        assert v.words_per_row == (full.shape[0] + 63) // 64
        got = binding.mask_bits_host(v)
        assert np.array_equal(got, oracle.slice_mask(full, n))          # the slice of the big mask ...
        assert np.array_equal(got, oracle.build_mask(br[:g]))           # ... equals a freshly built mask
        assert [v.parent_host[i] for i in range(n)] == parent[:n].tolist()
        assert [v.level_host[i] for i in range(n)] == level[:n].tolist()
        assert [v.level_off_host[l] for l in range(g + 1)] == [0] + np.cumsum(sizes[:g]).tolist()
        # a slice is a view: same storage as the full mask, nothing rebuilt
        assert C.addressof(v.bits_host.contents) == C.addressof(binding.slice_mask(m, len(br)).bits_host.contents)
    binding.free_mask(m)


def test_slice_has_no_bits_outside_itself(binding):
    m = binding.build_mask((3, 2, 2, 1, 1, 1, 1, 1))
    v = binding.slice_mask(m, 8)
    W = v.words_per_row
    words = np.ctypeslib.as_array(v.bits_host, shape=(v.n_nodes_max * W,)).reshape(v.n_nodes_max, W)
    for g in range(1, 9):
        n = binding.slice_mask(m, g).n_nodes
        for i in range(n):
            row = int(words[i, 0]) | (int(words[i, 1]) << 64)
            assert row >> n == 0


def test_build_and_slice_validation(binding):
    with pytest.raises(binding.McsdError) as e:
        binding.build_mask((2, 0, 2))
    assert e.value.status == binding.MCSD_EINVAL
    with pytest.raises(binding.McsdError):
        binding.build_mask(())
    with pytest.raises(binding.McsdError):
        binding.build_mask((1,) * 33)
    with pytest.raises(binding.McsdError) as e:
        binding.build_mask((64, 64, 2))                 # 64 + 4096 + ... > MCSD_MAX_NODES
    assert e.value.status == binding.MCSD_EUNSUPPORTED
    with pytest.raises(binding.McsdError):
        binding.build_mask((65,))
    m = binding.build_mask((2, 2))
    for g in (0, 3, -1):
        with pytest.raises(binding.McsdError) as e:
            binding.slice_mask(m, g)
        assert e.value.status == binding.MCSD_EINVAL
    assert binding.strerror(0) == "ok" and "workspace" in binding.strerror(binding.MCSD_EWORKSPACE)
    binding.lib.mcsd_free_mask(None)                    # NULL is allowed


def test_device_entry_points_reject_bad_arguments_before_any_launch(binding):
    """Null tensors, unsupported sizes and host-only views are turned into status codes on the host."""
    m = binding.build_mask((4, 2, 2, 1))
    v = binding.slice_mask(m, 4)
    lib = binding.lib
    one = C.c_void_p(256)            # never dereferenced: validation fails first
    args = dict(dtype=1, B=1, H=32, d=128)
    st = lib.mcsd_tree_attention(C.byref(v), 1, 1, 32, 128, None, one, one, 44, one, one, one, one, 1024 * 128, 1024,
                                 0.1, one, None, 0, None)
    assert st == binding.MCSD_EINVAL
    if v.device < 0:                 # no GPU here: a host-only view must be refused
        st = lib.mcsd_tree_attention(C.byref(v), 1, 1, 32, 128, one, one, one, 44, one, one, one, one, 1024 * 128,
                                     1024, 0.1, one, None, 0, None)
        assert st == binding.MCSD_EINVAL
    assert lib.mcsd_tree_attention_workspace(1, 32, 96, 44, 1024) == 0           # d not in {64,128}
    assert lib.mcsd_tree_attention_workspace(1, 32, 128, 129, 1024) == 0         # too many nodes
    assert lib.mcsd_tree_attention_workspace(1, 32, 128, 44, 1024) > 0
    st = lib.mcsd_verify_tree(C.byref(v), 0, 1, 32000, None, one, one, 45 * 32000, 29 * 32000, one, one, 1, one, one,
                              one, None, 0, None)
    assert st == binding.MCSD_EINVAL
    st = lib.mcsd_verify_tree(C.byref(v), 0, 1, 300000, one, one, one, 45 * 300000, 29 * 300000, one, one, 1, one,
                              one, one, None, 0, None)
    assert st == binding.MCSD_EUNSUPPORTED
    st = lib.mcsd_verify_tree(C.byref(v), 0, 1, 32000, one, one, one, 44 * 32000, 29 * 32000, one, one, 1, one, one,
                              one, None, 0, None)
    assert st == binding.MCSD_EINVAL                                              # p stride shorter than 1+N rows
    st = lib.mcsd_verify_tree(C.byref(v), 1, 1, 32000, one, one, one, 45 * 32000, 29 * 32000, one, one, 4, one, one,
                              one, None, 0, None)
    assert st == binding.MCSD_EWORKSPACE                                          # target-init needs a workspace


def test_early_stop_entry_points_reject_bad_arguments_before_any_launch(binding):
    lib, one = binding.lib, C.c_void_p(256)

    def mlp(widths, null_layer=None):
        m = binding.Mlp()
        m.n_layers = len(widths) - 1
        for i, w in enumerate(widths):
            m.width[i] = w
        for l in range(m.n_layers):
            m.weight[l] = None if l == null_layer else 256
            m.bias[l] = 256
        return m

    def dist(m, B=1, W=16, V=32000, k=10, rows=one, prob=one, stop=one):
        return lib.mcsd_early_stop_distribution(C.byref(m) if m is not None else None, B, W, V, k, rows, 17 * V, V, 0.4,
                                                None, prob, stop, None)

    ok = mlp((11, 64, 1))
    assert dist(None) == binding.MCSD_EINVAL
    assert dist(mlp((12, 64, 1))) == binding.MCSD_EINVAL                  # inputs must be k + 1
    assert dist(mlp((11, 64, 2))) == binding.MCSD_EINVAL                  # one output
    assert dist(mlp((11, 64, 1), null_layer=1)) == binding.MCSD_EINVAL
    assert dist(mlp((11, 513, 1))) == binding.MCSD_EUNSUPPORTED           # hidden width limit
    assert dist(mlp((18, 64, 1)), k=17) == binding.MCSD_EUNSUPPORTED      # k limit
    assert dist(mlp((1, 64, 1)), k=0) == binding.MCSD_EINVAL
    assert dist(ok, V=300000) == binding.MCSD_EUNSUPPORTED
    assert dist(ok, W=0) == binding.MCSD_EINVAL
    assert dist(ok, rows=None) == binding.MCSD_EINVAL
    assert dist(ok, prob=None) == binding.MCSD_EINVAL
    assert dist(ok, stop=None) == binding.MCSD_EINVAL
    assert dist(ok, B=0, rows=None) == binding.MCSD_OK                    # nothing to do, nothing touched

    def hid(m, B=1, W=16, x=one):
        return lib.mcsd_early_stop_hidden(C.byref(m), B, W, x, 16 * 768, 768, 0.4, one, one, None)

    assert hid(mlp((768, 256, 64, 1)), x=None) == binding.MCSD_EINVAL
    assert hid(mlp((8193, 256, 64, 1))) == binding.MCSD_EUNSUPPORTED
    m4 = mlp((768, 256, 64, 1))
    m4.n_layers = 4
    assert hid(m4) == binding.MCSD_EINVAL
    assert hid(mlp((768, 256, 64, 1)), B=0, x=None) == binding.MCSD_OK
