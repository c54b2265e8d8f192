"""The entry points added beyond the verification step, captured into one HIP graph and replayed: a draft turn's
early-stop decision, the fp8-cache attention of the tree, verification for candidates drawn without replacement,
and the update after acceptance.  Every replay must leave exactly what the eager calls leave (the graph holds only
this library's kernels)."""
import numpy as np
import pytest
import torch

from workloads import DRAFT_INIT, WORKLOADS, attention_inputs, mlp_weights, scaled, verify_inputs

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


def test_added_entry_points_replayed_from_a_hip_graph(binding, oracle, H):
    w = scaled(WORKLOADS["fork"], B=2, H=4, branching=(16, 1, 1), prefix_min=700, prefix_max=700, cfg_id=95)
    br, g = w.branching, w.gamma_max
    v = binding.slice_mask(binding.build_mask(br), g)
    n = v.n_nodes
    gamma_cap = 700 + g
    inp = attention_inputs(w, seed=6, lens=(700, 333), kv_fp8=(0.5, 0.25), kv_capacity=gamma_cap)
    q, kt, vt = (H.dev(inp[k], "bf16") for k in ("q", "k_tree", "v_tree"))
    kp8, vp8 = torch.from_numpy(inp["k_prefix"]).cuda(), torch.from_numpy(inp["v_prefix"]).cuda()
    lens = H.dev(np.ascontiguousarray(inp["lens"], dtype=np.int32))
    base = H.dev(np.ascontiguousarray(inp["seq_base"], dtype=np.int64))
    out = torch.zeros_like(q)
    ws = binding.new_workspace(binding.tree_attention_fp8kv_workspace(w.B, w.H, w.H, n, 0, 700))
    vi = verify_inputs(w, seed=6, mode=DRAFT_INIT, replacement=False)
    p, qd = H.dev(vi["p_target"]), H.dev(vi["q_draft"])
    tokens, ua, us = H.dev(vi["tokens"]), H.dev(vi["u_accept"]), H.dev(vi["u_sample"])
    path = torch.zeros((w.B, g), dtype=torch.int32, device="cuda")
    alen = torch.zeros((w.B,), dtype=torch.int32, device="cuda")
    new = torch.zeros((w.B, 1), dtype=torch.int32, device="cuda")
    k = 10
    mws, mbs = mlp_weights((k + 1, 64, 1), seed=4, out_bias=-0.3)
    mlp = binding.make_mlp([torch.from_numpy(a).cuda() for a in mws], [torch.from_numpy(a).cuda() for a in mbs])
    prob = torch.zeros((w.B, 16), dtype=torch.float32, device="cuda")
    stop = torch.zeros((w.B,), dtype=torch.int32, device="cuda")
    # a bf16 cache of the same shape for the update after acceptance (its own tensors: the update writes into it)
    binp = attention_inputs(w, seed=7, lens=(700, 333), kv_capacity=gamma_cap)
    bkt, bvt = (H.dev(binp[x], "bf16") for x in ("k_tree", "v_tree"))
    kp0, vp0 = (H.dev(binp[x], "bf16") for x in ("k_prefix", "v_prefix"))
    kp, vp = kp0.clone(), vp0.clone()
    lens0 = H.dev(np.ascontiguousarray(binp["lens"], dtype=np.int32))
    lens_c = lens0.clone()
    ids = torch.zeros((w.B, g + 1), dtype=torch.int32, device="cuda")
    n_ids = torch.zeros((w.B,), dtype=torch.int32, device="cuda")
    V, rows_p, rows_q = w.V, vi["p_target"].shape[1], vi["q_draft"].shape[1]

    def turn():
        binding.early_stop_distribution(mlp, w.B, 16, V, k, qd[:, 1:17], rows_q * V, V, 0.4, None, prob, stop)
        binding.tree_attention_fp8kv(v, w.B, w.H, w.H, 0, q, kt, vt, inp["node_stride"], kp8, vp8, inp["k_scale"],
                                     inp["v_scale"], base, lens, inp["head_stride"], 700, float(np.float32(inp["scale"])),
                                     out, ws)
        binding.verify_tree_sampling(v, DRAFT_INIT, binding.MCSD_WITHOUT_REPLACEMENT, w.B, V, tokens, p, qd, rows_p * V,
                                     rows_q * V, ua, us, 1, path, alen, new, None)
        binding.commit_path(v, 1, w.B, w.H, w.d, [bkt], [bvt], binp["node_stride"], [kp], [vp], base, binp["head_stride"],
                            700, gamma_cap, path, alen, tokens, new, 1, 1, lens_c, ids, n_ids)

    def reset():
        kp.copy_(kp0)
        vp.copy_(vp0)
        lens_c.copy_(lens0)

    results = (prob, stop, out, path, alen, new, kp, vp, lens_c, ids, n_ids)
    turn()
    torch.cuda.synchronize()
    want = [t.clone() for t in results]
    # the eager results are the oracle's
    wp, wl, wn = oracle.verify_tree(DRAFT_INIT, br, vi["tokens"], vi["p_target"], vi["q_draft"], vi["u_accept"],
                                    vi["u_sample"], replacement=False)
    assert np.array_equal(path.cpu().numpy(), wp) and np.array_equal(alen.cpu().numpy(), wl)
    H.assert_close(out[:, :, :n].float().cpu().numpy().astype(np.float64),
                   oracle.tree_attention_fp8kv(inp, oracle.build_mask(br), n), "bf16", "fp8 attention before capture")
    reset()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        turn()
    torch.cuda.current_stream().wait_stream(side)
    reset()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        turn()
    for r in range(4):
        reset()
        for t in (prob, out, path, alen, new, ids, n_ids, stop):
            t.fill_(-3)                                  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(want, results):
            assert torch.equal(a, b), f"replay {r} differs from the eager calls"
