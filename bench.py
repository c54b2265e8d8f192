#!/usr/bin/env python3
"""Benchmark of the MCSD verification hot path on one MI355X.

One STEP is one pass of the whole hot path over one batch of seeded synthetic input:
    mcsd_slice_mask(gamma)  ->  one mcsd_tree_attention call per transformer layer (32 for Llama-2-7B, every
    layer with its own KV cache and q/k/v)  ->  one mcsd_verify_tree call.
All inputs are resident in HBM before the timed region.  The headline value is verified tree-tokens/s =
B * N(gamma) / step time.  The line also carries the roofline of the dominant kernel (the tree-attention
key sweep), measured with HIP events that bracket that kernel's launches, and the CPU oracle timed on the
host cores as a reported baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--extra cfg4,cfg5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
N_LAYERS = 32                   # Llama-2-7B

# HBM traffic per launch of the sweep kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (bytes, already
# scaled by the copy-kernel calibration); filled from the summaries under profiles/.  None = not measured.
MEASURED_TRAFFIC = {"cfg2": 21_810_000, "cfg4": 664_280_000, "cfg5": 2_213_340_000, "cfg4_b64": 2_742_320_000,
                    "cfg4_fp8kv": 348_030_000, "cfg5_fp8kv": 1_142_800_000}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def attention_algorithmic(w, lens, n):
    """Algorithmic bytes and flops of one mcsd_tree_attention call: prefix K and V read once, tree q/k/v read and
    the output written once, plus the mask slice; 4*N*(L+N)*d flops per (sequence, head)."""
    e = 2 if w.dtype == "bf16" else 4
    by = sum(w.H * e * w.d * (2 * int(L) + 4 * n) for L in lens) + n * ((w.n_nodes() + 63) // 64) * 8
    fl = sum(w.H * 4 * n * (int(L) + n) * w.d for L in lens)
    return by, fl


class Step:
    """Device-resident inputs of one step and the calls that make it."""

    def __init__(self, name, n_kv_sets, gamma=None, mode=None, seed=0, with_verify=True, tuning=None):
        import numpy as np
        import torch
        from paper_2409_10644_amd import binding
        from workloads import WORKLOADS, attention_inputs, prefix_lens, scaled, verify_inputs
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import gpu_helpers as H

        self.binding, self.H, self.torch, self.np = binding, H, torch, np
        self.w = w = WORKLOADS[name]
        self.gamma = w.gamma_max if gamma is None else gamma
        self.mode = w.mode if mode is None else mode
        self.lens = prefix_lens(w, seed)
        self.cap = int(w.prefix_max)
        t0 = time.time()
        self.layers_host = [attention_inputs(w, seed=seed, kv_capacity=self.cap, variant=l) for l in range(n_kv_sets)]
        self.layers = [H.AttnDevice(inp) for inp in self.layers_host]
        self.with_verify = with_verify
        self.vi = verify_inputs(w if with_verify else scaled(w, B=1), seed=seed, gamma=self.gamma, mode=self.mode)
        log(f"[bench] {name}: {n_kv_sets} KV set(s) generated and uploaded in {time.time() - t0:.1f}s")
        self.mask = binding.build_mask(w.branching)                   # once, at gamma_max
        self.view = binding.slice_mask(self.mask, self.gamma)
        self.n = self.view.n_nodes
        self.tuning = tuning                                          # None: the library's own plan
        ws_bytes = binding.tree_attention_tuned_workspace(tuning, 0, w.B, w.H, w.H, w.d, self.n, 0, self.cap)
        self.ws_bytes = ws_bytes
        self.ws = binding.new_workspace(ws_bytes)
        vi = self.vi
        self.p, self.q = H.dev(vi["p_target"]), H.dev(vi["q_draft"])
        self.tokens, self.ua, self.us = H.dev(vi["tokens"]), H.dev(vi["u_accept"]), H.dev(vi["u_sample"])
        self.n_new = vi["n_new"]
        self.path = torch.zeros((w.B, self.gamma), dtype=torch.int32, device="cuda")
        self.alen = torch.zeros((w.B,), dtype=torch.int32, device="cuda")
        self.new = torch.zeros((w.B, max(self.n_new, 1)), dtype=torch.int32, device="cuda")
        vws = binding.verify_tree_workspace(self.view, self.mode, w.B, self.n_new)
        self.vws = torch.empty(max(vws, 256), dtype=torch.uint8, device="cuda") if vws else None
        self.alg_bytes, self.alg_flops = attention_algorithmic(w, self.lens, self.n)

    def attention(self, layer):
        ad, w, b = self.layers[layer % len(self.layers)], self.w, self.binding
        if self.tuning is None:
            b.tree_attention(self.view, ad.code, w.B, w.H, w.d, ad.q, ad.kt, ad.vt, ad.node_stride, ad.kp, ad.vp, ad.base,
                             ad.lens, ad.head_stride, self.cap, ad.scale, ad.out, self.ws)
        else:
            b.tree_attention_tuned(self.tuning, self.view, ad.code, 0, 1.0, 1.0, w.B, w.H, w.H, w.d, 0, ad.q, ad.kt, ad.vt,
                                   ad.node_stride, ad.kp, ad.vp, ad.base, ad.lens, ad.head_stride, self.cap, ad.scale,
                                   ad.out, self.ws)

    def verify(self):
        w, b, vi = self.w, self.binding, self.vi
        b.verify_tree(self.view, self.mode, w.B, w.V, self.tokens, self.p, self.q, vi["p_target"].shape[1] * w.V,
                      vi["q_draft"].shape[1] * w.V, self.ua, self.us, self.n_new, self.path, self.alen, self.new,
                      self.vws)

    def commit(self, lens_dev, ids, n_ids):
        """Update after acceptance over all layers' caches (not part of the timed step: the row after it).  The
        benchmark's caches are exactly prefix_max rows long, so lengths are clamped gamma rows below that."""
        w, b = self.w, self.binding
        L = self.layers
        b.commit_path(self.view, L[0].code, w.B, w.H, w.d, [a.kt for a in L], [a.vt for a in L], L[0].node_stride,
                      [a.kp for a in L], [a.vp for a in L], L[0].base, L[0].head_stride, self.cap - self.gamma, self.cap,
                      self.path, self.alen, self.tokens, self.new, self.n_new, 1 if self.mode == 0 else 0, lens_dev,
                      ids, n_ids)

    def step(self):
        self.view = self.binding.slice_mask(self.mask, self.gamma)    # O(1): the per-step slice
        for l in range(N_LAYERS):
            self.attention(l)
        self.verify()

    def check_against_oracle(self, rows=24):
        """'Verified': the outputs of this very configuration match the oracle (sampled attention rows of layer
        0, full verification result)."""
        import oracle
        np_, torch = self.np, self.torch
        w = self.w
        self.attention(0)
        if self.with_verify:
            self.verify()
        torch.cuda.synchronize()
        M = oracle.build_mask(w.branching)
        got = self.layers[0].out[:, :, :self.n].float().cpu().numpy().astype(np_.float64)
        rng = np_.random.default_rng(1)
        for _ in range(rows):
            b, h, i = int(rng.integers(w.B)), int(rng.integers(w.H)), int(rng.integers(self.n))
            want = oracle.tree_attention_row(self.layers_host[0], M, self.n, b, h, i)
            self.H.assert_close(got[b, h, i], want, w.dtype, f"bench {w.name} row {(b, h, i)}")
        if not self.with_verify:
            return float("nan")
        vi = self.vi
        want = oracle.verify_tree(self.mode, w.branching[:self.gamma], vi["tokens"], vi["p_target"], vi["q_draft"],
                                  vi["u_accept"], vi["u_sample"])
        got_v = (self.path.cpu().numpy(), self.alen.cpu().numpy(), self.new.cpu().numpy()[:, :self.n_new])
        for a, b_ in zip(got_v, want):
            assert np_.array_equal(a, b_), "verification differs from the oracle"
        return float(want[1].mean())


class Ctx:
    """What time_kernel needs of a Step, for the sections that are not a Step."""

    def __init__(self, binding, torch):
        self.binding, self.torch = binding, torch


def time_kernel(st, hip, kernel_id, launch, reps, warm=0):
    """Average device execution time (ms) of one library kernel over `reps` back-to-back launches, from event
    pairs that the library places around that kernel's launch.  `warm` untimed launches go first in the same
    burst, so that the timed ones see the clocks of sustained work rather than the ramp out of idle."""
    b, torch = st.binding, st.torch
    pairs = [(hip.event(), hip.event()) for _ in range(reps)]
    for i in range(warm):
        launch(i)
    for i, (e0, e1) in enumerate(pairs):
        b.profile_next(kernel_id, e0, e1)
        launch(warm + i)
    torch.cuda.synchronize()
    ms = [hip.elapsed_ms(e0, e1) for e0, e1 in pairs]
    for e0, e1 in pairs:
        hip.destroy(e0)
        hip.destroy(e1)
    ms.sort()
    return sum(ms) / len(ms), ms[len(ms) // 2], ms[len(ms) // 10], ms[(len(ms) * 9) // 10]


def roofline_of(st, hip, reps, warm=0):
    b = st.binding
    avg, med, p10, p90 = time_kernel(st, hip, b.KERNEL_ATTN_SWEEP, lambda i: st.attention(i), reps, warm)
    ach = st.alg_bytes / (avg * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC.get(st.w.name)
    return {"bound": "hbm", "kernel": "tree_attn_bf16_kernel" if st.w.dtype == "bf16" else "tree_attn_f32_kernel",
            "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
            "traffic": traffic, "algorithmic_bytes_per_launch": int(st.alg_bytes),
            "flops_per_launch": int(st.alg_flops), "avg_launch_us": round(avg * 1e3, 2),
            "median_launch_us": round(med * 1e3, 2), "p10_us": round(p10 * 1e3, 2), "p90_us": round(p90 * 1e3, 2),
            "mfma_tflops": round(st.alg_flops / (avg * 1e-3) / 1e12, 1), "launches_timed": reps}


def verify_algorithmic_bytes(st):
    """Vocabulary rows the acceptance walk has to read, from its own result (draft-initialised mode: one walk per
    sequence): a context with at least one rejection needs its target and draft row (2 * V * 4 bytes, read once);
    a terminal context without rejections needs its target row for the new token (V * 4 bytes); every tested
    candidate needs p(x), q(x), its token id and its uniform (16 bytes).  None in target-initialised mode, where
    the walks of the losing level-1 subtrees are not part of the result."""
    if st.mode != 0:
        return None
    w = st.w
    path = st.path.cpu().numpy()
    alen = st.alen.cpu().numpy()
    br = list(w.branching[:st.gamma])
    off = [0]
    for l, b in enumerate(br):
        off.append(off[-1] + (b if l == 0 else (off[-1] - off[-2]) * b))
    total = 0
    for bi in range(w.B):
        cur = -1
        for level in range(st.gamma):
            cnt = br[level]
            first = 0 if cur < 0 else off[level] + (cur - off[level - 1]) * cnt
            if level < alen[bi]:
                rejected = int(path[bi, level]) - first
                total += 16 * (rejected + 1) + (2 * w.V * 4 if rejected else 0)
                cur = int(path[bi, level])
            else:
                total += 16 * cnt + 2 * w.V * 4          # every child rejected: terminal context
                break
        else:
            total += w.V * 4 if st.n_new else 0          # all levels accepted: bonus token from one target row
    return total


def cpu_baseline(st, budget_s=20.0):
    """The oracle as it stands on the host cores: attention of as many layers as fit the time budget (scaled to
    32 layers) plus one verification; tree-tokens/s of a whole step."""
    import oracle
    w = st.w
    M = oracle.build_mask(w.branching)
    inp = st.layers_host[0]
    B, Hh = w.B, w.H
    # bounded sample: whole layers if one fits in the budget, else a subset of (b,h) rows of one layer
    t0 = time.time()
    probe_rows = 8
    for k in range(probe_rows):
        oracle.tree_attention_row(inp, M, st.n, k % B, k % Hh, k % st.n)
    t_row = (time.time() - t0) / probe_rows
    threads = oracle.threads()
    est_layer = t_row * B * Hh * st.n / max(1, min(threads, B * Hh))
    vi = st.vi
    t0 = time.time()
    oracle.verify_tree(st.mode, w.branching[:st.gamma], vi["tokens"], vi["p_target"], vi["q_draft"], vi["u_accept"],
                       vi["u_sample"])
    t_verify = time.time() - t0
    if est_layer <= budget_s:
        n_layers = max(1, min(N_LAYERS, int(budget_s / max(est_layer, 1e-3))))
        t0 = time.time()
        for l in range(n_layers):
            oracle.tree_attention(st.layers_host[l % len(st.layers_host)], M, st.n)
        t_layer = (time.time() - t0) / n_layers
        sample = f"{n_layers} of {N_LAYERS} attention layers in full + 1 verification, attention time scaled to {N_LAYERS} layers"
    else:
        rows = max(threads, int(budget_s / t_row) // threads * threads)
        import concurrent.futures as cf
        picks = [(r % B, (r // B) % Hh, (r * 7) % st.n) for r in range(rows)]
        t0 = time.time()
        with cf.ThreadPoolExecutor(threads) as ex:       # ctypes releases the GIL: rows run on all cores
            list(ex.map(lambda a: oracle.tree_attention_row(inp, M, st.n, *a), picks))
        t_layer = (time.time() - t0) / rows * (B * Hh * st.n)
        sample = (f"{rows} of {B * Hh * st.n} output rows of one attention layer + 1 verification, scaled to "
                  f"{N_LAYERS} full layers")
    t_step = N_LAYERS * t_layer + t_verify
    return {"value": round(w.B * st.n / t_step, 3), "unit": "tree-tokens/s", "cores": threads, "kind": "oracle",
            "sample": sample, "attention_layer_s": round(t_layer, 4), "verify_s": round(t_verify, 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--extra", default="cfg4,cfg5,cfg4_b64", help="other workloads whose attention roofline is reported too")
    ap.add_argument("--kernel-reps", type=int, default=64)
    ap.add_argument("--extra-reps", type=int, default=200,
                    help="timed launches (after as many untimed ones) of each extra workload's attention")
    ap.add_argument("--gqa-kv-heads", type=int, default=8,
                    help="key/value heads of the grouped-query variant of cfg4 (0 skips that section)")
    ap.add_argument("--verify-batch", type=int, default=128,
                    help="sequences of the batched verification section (0 skips it)")
    ap.add_argument("--decision-batch", type=int, default=64,
                    help="trees per call in the early-stop decision-model section (0 = skip)")
    ap.add_argument("--no-fp8kv", action="store_true", help="skip the fp8 prefix-cache variants of cfg4 / cfg5")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="launch the step's kernels one by one instead of replaying a HIP graph")
    ap.add_argument("--key-splits", type=int, default=0,
                    help="measurement sweeps: key splits of the headline workload's attention (0 = the library's plan)")
    ap.add_argument("--stages", type=int, default=0, help="measurement sweeps: LDS stages of the bf16 K/V ring (0 = the library's plan)")
    ap.add_argument("--fold-kernel", action="store_true",
                    help="measurement sweeps: fold the key splits' partial results in a second kernel")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="only run a 1 GiB device-to-device copy a few times (the known-size kernel that the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (the path shards by sequence and head without any "
                 "exchange, so N GPUs are N independent copies of this run); run with --gpus 1")
    import torch
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    if args.traffic_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "3 device-to-device copies", "bytes_read_each": src.numel() * 4,
                          "bytes_written_each": src.numel() * 4}))
        return
    from paper_2409_10644_amd import binding
    hip = binding.HipRuntime()

    w_name = args.workload
    from workloads import WORKLOADS
    w = WORKLOADS[w_name]
    kv_bytes = w.B * w.H * w.prefix_max * w.d * (2 if w.dtype == "bf16" else 4) * 2
    n_sets = N_LAYERS if kv_bytes * N_LAYERS <= (8 << 30) else max(1, min(N_LAYERS, (2 << 30) // kv_bytes))
    tuning = None
    if args.key_splits or args.fold_kernel or args.stages:
        tuning = binding.AttentionTuning(key_splits=args.key_splits, fold=1 if args.fold_kernel else 0, stages=args.stages)
    st = Step(w_name, n_sets, tuning=tuning)
    alpha = st.check_against_oracle()
    log(f"[bench] {w_name}: outputs verified against the oracle (mean accepted length {alpha:.2f})")

    # The 65 launches of a step are captured once into a HIP graph and replayed (the library's calls neither
    # allocate nor synchronise, so they can be captured); --eager launches them one by one instead.
    run_step, launch = st.step, "eager"
    if not args.eager:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                st.step()
            torch.cuda.current_stream().wait_stream(side)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                st.step()
            run_step, launch = graph.replay, "hip-graph"
        except Exception as ex:
            log(f"[bench] graph capture failed ({ex!r}); timing eager launches")
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if launch == "hip-graph":                     # the replayed step must leave what the eager step leaves
        got_v = (st.path.clone(), st.alen.clone(), st.new.clone(), st.layers[N_LAYERS % len(st.layers) - 1].out.clone())
        st.step()
        torch.cuda.synchronize()
        now_v = (st.path, st.alen, st.new, st.layers[N_LAYERS % len(st.layers) - 1].out)
        assert all(torch.equal(a, b) for a, b in zip(got_v, now_v)), "graph replay differs from eager launches"
    ms_per_step = dt / args.steps * 1e3
    value = w.B * st.n / (ms_per_step * 1e-3)

    roof = roofline_of(st, hip, args.kernel_reps, warm=args.kernel_reps)
    # the same launch on ONE K/V set over and over: the 16 MiB of a small workload then come from the 256 MB
    # last-level cache, not from HBM.  Reported beside the cold figure (which rotates over n_sets sets), never as it.
    warm_avg = time_kernel(st, hip, binding.KERNEL_ATTN_SWEEP, lambda i: st.attention(0), args.kernel_reps, warm=10)[0]
    roof["warm_cache_launch_us"] = round(warm_avg * 1e3, 2)
    m_avg = time_kernel(st, hip, binding.KERNEL_ATTN_MERGE, lambda i: st.attention(i), args.kernel_reps)[0] \
        if st.ws_bytes > 0 and args.fold_kernel else 0.0
    v_avg = time_kernel(st, hip, binding.KERNEL_VERIFY_WALK, lambda i: st.verify(), args.kernel_reps)[0]
    out = {
        "metric": "verified tree-tokens/s, whole verification step (32 tree-attention layers + acceptance)",
        "value": round(value, 1), "unit": "tree-tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w_name}: B{w.B} H{w.H} d{w.d} {w.dtype} prefix {w.prefix_min}"
                               f"{'' if w.prefix_min == w.prefix_max else '-' + str(w.prefix_max)} tree {w.branching} "
                               f"N={st.n} gamma={st.gamma} V={w.V} mode={'target' if st.mode else 'draft'}-init",
                   "layers_per_step": N_LAYERS, "kv_sets": n_sets, "launch": launch, "verified_vs_oracle": True,
                   "mean_accept_len": round(alpha, 3)},
        "roofline": roof,
        "kernels_us": {"attn_sweep": roof["avg_launch_us"], "attn_merge": round(m_avg * 1e3, 2),
                       "verify_walk": round(v_avg * 1e3, 2)},
    }
    vb = verify_algorithmic_bytes(st)
    if vb is not None:          # the vocabulary pass: one workgroup per sequence, latency-bound at this batch size
        out["verify_roofline"] = {"bound": "hbm", "kernel": "verify_walk_kernel", "achieved": round(vb / (v_avg * 1e-3) / 1e9, 2),
                                  "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(vb / (v_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 6),
                                  "algorithmic_bytes_per_launch": int(vb), "avg_launch_us": round(v_avg * 1e3, 2)}
    # the same verification for candidates drawn without replacement (a scheme next to the paper's), same shapes
    try:
        import numpy as np
        import oracle
        from workloads import verify_inputs
        vi2 = verify_inputs(w, seed=0, gamma=st.gamma, mode=st.mode, replacement=False)
        d2 = [st.H.dev(vi2[k]) for k in ("tokens", "p_target", "q_draft", "u_accept", "u_sample")]
        o2 = [torch.zeros_like(st.path), torch.zeros_like(st.alen), torch.zeros_like(st.new)]

        def v2call(i):
            binding.verify_tree_sampling(st.view, st.mode, binding.MCSD_WITHOUT_REPLACEMENT, w.B, w.V, d2[0], d2[1], d2[2],
                                         vi2["p_target"].shape[1] * w.V, vi2["q_draft"].shape[1] * w.V, d2[3], d2[4],
                                         st.n_new, o2[0], o2[1], o2[2], st.vws)
        v2call(0)
        torch.cuda.synchronize()
        want2 = oracle.verify_tree(st.mode, w.branching[:st.gamma], vi2["tokens"], vi2["p_target"], vi2["q_draft"],
                                   vi2["u_accept"], vi2["u_sample"], replacement=False)
        got2 = (o2[0].cpu().numpy(), o2[1].cpu().numpy(), o2[2].cpu().numpy()[:, :st.n_new])
        assert all(np.array_equal(a, b) for a, b in zip(got2, want2)), "without-replacement verification differs from the oracle"
        v2_avg = time_kernel(st, hip, binding.KERNEL_VERIFY_WALK, v2call, args.kernel_reps)[0]
        out["kernels_us"]["verify_walk_without_replacement"] = round(v2_avg * 1e3, 2)
        out["verify_without_replacement"] = {"avg_launch_us": round(v2_avg * 1e3, 2), "verified_vs_oracle": True,
                                             "mean_accept_len": round(float(want2[1].mean()), 3)}
    except Exception as ex:
        out["verify_without_replacement"] = {"error": repr(ex)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(st)
    # the draft side of the loop: attention for the newest level only, a fresh slice of the mask per level
    lvl = {}
    for g in range(1, st.gamma + 1):
        vg = binding.slice_mask(st.mask, g)
        rb = int(vg.level_off_host[g - 1])
        ad = st.layers[0]

        def level_call(i, vg=vg, rb=rb):
            a = st.layers[i % len(st.layers)]
            binding.tree_attention_rows(vg, a.code, w.B, w.H, w.d, rb, a.q, a.kt, a.vt, a.node_stride, a.kp, a.vp, a.base,
                                        a.lens, a.head_stride, st.cap, a.scale, a.out, st.ws)
        for i in range(8):
            level_call(i)
        torch.cuda.synchronize()
        t0l = time.perf_counter()
        for i in range(64):
            level_call(i)
        torch.cuda.synchronize()
        lvl[f"gamma{g}_rows{vg.n_nodes - rb}"] = round((time.perf_counter() - t0l) / 64 * 1e6, 1)
    out["level_attention_call_us"] = lvl
    # the row after the step: accepted path appended to every layer's cache (last: it overwrites cache rows)
    ids = torch.zeros((w.B, st.gamma + 1), dtype=torch.int32, device="cuda")
    n_ids = torch.zeros((w.B,), dtype=torch.int32, device="cuda")
    lens_c = st.layers[0].lens.clone()

    def commit_once(i):
        lens_c.copy_(st.layers[0].lens)
        st.commit(lens_c, ids, n_ids)
    c_avg = time_kernel(st, hip, binding.KERNEL_COMMIT_COPY, commit_once, 20, warm=5)[0]
    torch.cuda.synchronize()
    t0c = time.perf_counter()
    for i in range(20):
        st.commit(lens_c, ids, n_ids)
    torch.cuda.synchronize()
    out["commit_path"] = {"layers_per_call": len(st.layers), "copy_kernel_us": round(c_avg * 1e3, 2),
                          "call_us": round((time.perf_counter() - t0c) / 20 * 1e6, 1),
                          "mean_accept_len": round(float(st.alen.float().mean().item()), 3)}
    del st
    torch.cuda.empty_cache()

    extra = {}
    for name in [x for x in args.extra.split(",") if x and x != w_name]:
        try:
            es = Step(name, 1, with_verify=name in ("cfg4", "cfg5"))
            es.check_against_oracle(rows=8)
            for i in range(3):
                es.attention(i)
            r = roofline_of(es, hip, args.extra_reps, warm=args.extra_reps)
            torch.cuda.synchronize()
            t0e = time.perf_counter()
            for i in range(args.extra_reps):
                es.attention(i)
            torch.cuda.synchronize()
            call_us = (time.perf_counter() - t0e) / args.extra_reps * 1e6
            r["attention_call_us"] = round(call_us, 1)
            r["attn_tree_tokens_per_s"] = round(es.w.B * es.n / (call_us * 1e-6), 1)
            r["workload"] = f"{name}: B{es.w.B} N={es.n} prefix {es.w.prefix_min}-{es.w.prefix_max}"
            extra[name] = r
            del es
            torch.cuda.empty_cache()
        except Exception as ex:      # an extra workload must not lose the headline line
            extra[name] = {"error": repr(ex)}
    # grouped-query variant of the ragged batch (beyond the paper's multi-head shape): 32 query heads on 8 kv heads
    if args.gqa_kv_heads > 0 and "cfg4" in args.extra:
        try:
            from workloads import scaled, attention_inputs, prefix_lens
            sys.path.insert(0, os.path.join(ROOT, "tests"))
            import gpu_helpers as H
            import oracle
            import numpy as np
            wq = WORKLOADS["cfg4"]
            Hkv = args.gqa_kv_heads
            wk = scaled(wq, H=Hkv, cfg_id=wq.cfg_id + 100)
            lens = prefix_lens(wq, 0)
            qi = attention_inputs(wq, seed=0, lens=lens, kv_capacity=int(wq.prefix_max))
            ki = attention_inputs(wk, seed=0, lens=lens, kv_capacity=int(wq.prefix_max))
            aq, ak = H.AttnDevice(qi), H.AttnDevice(ki)
            vg = binding.slice_mask(binding.build_mask(wq.branching), wq.gamma_max)
            n = vg.n_nodes
            wsb = binding.tree_attention_gqa_workspace(wq.B, wq.H, Hkv, wq.d, n, 0, int(wq.prefix_max))
            wsg = binding.new_workspace(wsb)

            def gcall(i):
                binding.tree_attention_gqa(vg, 1, wq.B, wq.H, Hkv, wq.d, 0, aq.q, ak.kt, ak.vt, ak.node_stride, ak.kp, ak.vp,
                                           ak.base, ak.lens, ak.head_stride, int(wq.prefix_max), aq.scale, aq.out, wsg)
            gcall(0)
            torch.cuda.synchronize()
            G = wq.H // Hkv
            cap = ki["k_prefix"].shape[2]
            rep_ = dict(qi, k_tree=np.repeat(ki["k_tree"], G, axis=1), v_tree=np.repeat(ki["v_tree"], G, axis=1),
                        k_prefix=np.repeat(ki["k_prefix"], G, axis=1), v_prefix=np.repeat(ki["v_prefix"], G, axis=1),
                        head_stride=cap * wq.d, seq_base=(np.arange(wq.B, dtype=np.int64) * (wq.H * cap * wq.d)))
            got = aq.out[:, :, :n].float().cpu().numpy().astype(np.float64)
            M = oracle.build_mask(wq.branching)
            rng = np.random.default_rng(2)
            for _ in range(8):
                b_, h_, i_ = int(rng.integers(wq.B)), int(rng.integers(wq.H)), int(rng.integers(n))
                H.assert_close(got[b_, h_, i_], oracle.tree_attention_row(rep_, M, n, b_, h_, i_), "bf16", "bench gqa")

            gs = Ctx(binding, torch)
            g_avg, g_med, g_p10, g_p90 = time_kernel(gs, hip, binding.KERNEL_ATTN_SWEEP, gcall, args.extra_reps, warm=args.extra_reps)
            gbytes = sum(2 * wq.d * (Hkv * (2 * int(L) + 2 * n) + wq.H * 2 * n) for L in lens)
            gflops = sum(wq.H * 4 * n * (int(L) + n) * wq.d for L in lens)
            extra["cfg4_gqa"] = {"bound": "mfma", "kernel": "tree_attn_bf16_kernel", "achieved": round(gflops / (g_avg * 1e-3) / 1e12, 1),
                                 "peak": 2500.0, "unit": "TFLOP/s", "frac": round(gflops / (g_avg * 1e-3) / 1e12 / 2500.0, 4),
                                 "traffic": None, "flops_per_launch": int(gflops), "algorithmic_bytes_per_launch": int(gbytes),
                                 "hbm_GBps": round(gbytes / (g_avg * 1e-3) / 1e9, 1), "avg_launch_us": round(g_avg * 1e3, 2),
                                 "p10_us": round(g_p10 * 1e3, 2), "p90_us": round(g_p90 * 1e3, 2), "launches_timed": args.extra_reps,
                                 "verified_vs_oracle": True,
                                 "workload": f"cfg4 with {wq.H} query heads on {Hkv} key/value heads (B{wq.B} N={n})"}
            del aq, ak
            torch.cuda.empty_cache()
        except Exception as ex:
            extra["cfg4_gqa"] = {"error": repr(ex)}
    # the same sweeps over an fp8 (E4M3) prefix cache (beyond the paper's bf16 setting): half the prefix bytes
    if not args.no_fp8kv:
        for name in [x for x in args.extra.split(",") if x in ("cfg4", "cfg5")]:
            try:
                import numpy as np
                from workloads import attention_inputs, prefix_lens
                import oracle
                sys.path.insert(0, os.path.join(ROOT, "tests"))
                import gpu_helpers as H
                w8 = WORKLOADS[name]
                lens = prefix_lens(w8, 0)
                cap = int(w8.prefix_max)
                inp8 = attention_inputs(w8, seed=0, kv_capacity=cap, kv_fp8=(0.5, 0.25))
                q8, kt8, vt8 = (H.dev(inp8[k], "bf16") for k in ("q", "k_tree", "v_tree"))
                kp8, vp8 = torch.from_numpy(inp8["k_prefix"]).cuda(), torch.from_numpy(inp8["v_prefix"]).cuda()
                lens8 = H.dev(np.ascontiguousarray(inp8["lens"], dtype=np.int32))
                base8 = H.dev(np.ascontiguousarray(inp8["seq_base"], dtype=np.int64))
                out8 = torch.zeros_like(q8)
                v8 = binding.slice_mask(binding.build_mask(w8.branching), w8.gamma_max)
                n8 = v8.n_nodes
                ws8 = binding.new_workspace(binding.tree_attention_fp8kv_workspace(w8.B, w8.H, w8.H, n8, 0, cap))

                def fcall(i):
                    binding.tree_attention_fp8kv(v8, w8.B, w8.H, w8.H, 0, q8, kt8, vt8, inp8["node_stride"],
                                                 kp8, vp8, inp8["k_scale"], inp8["v_scale"], base8, lens8, inp8["head_stride"],
                                                 cap, float(np.float32(inp8["scale"])), out8, ws8)
                fcall(0)
                torch.cuda.synchronize()
                got8 = out8[:, :, :n8].float().cpu().numpy().astype(np.float64)
                M8 = oracle.build_mask(w8.branching)
                rng8 = np.random.default_rng(3)
                for _ in range(8):
                    b_, h_, i_ = int(rng8.integers(w8.B)), int(rng8.integers(w8.H)), int(rng8.integers(n8))
                    H.assert_close(got8[b_, h_, i_], oracle.tree_attention_row_fp8kv(inp8, M8, n8, b_, h_, i_), "bf16", "bench fp8kv")

                fs = Ctx(binding, torch)
                f_avg, f_med, f_p10, f_p90 = time_kernel(fs, hip, binding.KERNEL_ATTN_SWEEP, fcall, args.extra_reps, warm=args.extra_reps)
                fbytes = sum(w8.H * w8.d * (2 * int(L) * 1 + 4 * n8 * 2) for L in lens)
                fflops = sum(w8.H * 4 * n8 * (int(L) + n8) * w8.d for L in lens)
                extra[name + "_fp8kv"] = {
                    "bound": "hbm", "kernel": "tree_attn_bf16_kernel<fp8 prefix>", "achieved": round(fbytes / (f_avg * 1e-3) / 1e9, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(fbytes / (f_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                    "traffic": MEASURED_TRAFFIC.get(name + "_fp8kv"), "algorithmic_bytes_per_launch": int(fbytes),
                    "flops_per_launch": int(fflops),
                    "avg_launch_us": round(f_avg * 1e3, 2), "p10_us": round(f_p10 * 1e3, 2), "p90_us": round(f_p90 * 1e3, 2),
                    "mfma_tflops": round(fflops / (f_avg * 1e-3) / 1e12, 1), "launches_timed": args.extra_reps,
                    "attn_tree_tokens_per_s": round(w8.B * n8 / (f_avg * 1e-3), 1), "verified_vs_oracle": True,
                    "workload": f"{name} with the prefix cache in fp8 E4M3 (B{w8.B} N={n8})"}
                del kp8, vp8
                torch.cuda.empty_cache()
            except Exception as ex:
                extra[name + "_fp8kv"] = {"error": repr(ex)}
    # the vocabulary pass at a batch that fills half the chip's compute units (one workgroup per sequence)
    if args.verify_batch > 0:
        try:
            from workloads import scaled, verify_inputs
            import oracle
            sys.path.insert(0, os.path.join(ROOT, "tests"))
            import gpu_helpers as H
            wb = scaled(WORKLOADS[w_name], B=args.verify_batch)
            vi = verify_inputs(wb, seed=1, mode=0)
            vv = binding.slice_mask(binding.build_mask(wb.branching), wb.gamma_max)
            got = H.run_verify(binding, vv, 0, vi)
            want = oracle.verify_tree(0, wb.branching, vi["tokens"], vi["p_target"], vi["q_draft"], vi["u_accept"], vi["u_sample"])
            assert all((a == b).all() for a, b in zip(got, want)), "batched verification differs from the oracle"
            dp, dq = H.dev(vi["p_target"]), H.dev(vi["q_draft"])
            dt_, dua, dus = H.dev(vi["tokens"]), H.dev(vi["u_accept"]), H.dev(vi["u_sample"])
            o_path = torch.zeros((wb.B, vv.gamma), dtype=torch.int32, device="cuda")
            o_len = torch.zeros((wb.B,), dtype=torch.int32, device="cuda")
            o_new = torch.zeros((wb.B, 1), dtype=torch.int32, device="cuda")

            vs = Ctx(binding, torch)
            vs.mode, vs.w, vs.gamma, vs.n_new, vs.path, vs.alen = 0, wb, vv.gamma, 1, o_path, o_len

            def vcall(i):
                binding.verify_tree(vv, 0, wb.B, wb.V, dt_, dp, dq, vi["p_target"].shape[1] * wb.V, vi["q_draft"].shape[1] * wb.V,
                                    dua, dus, 1, o_path, o_len, o_new, None)
            vb_avg = time_kernel(vs, hip, binding.KERNEL_VERIFY_WALK, vcall, 30, warm=10)[0]
            vbytes = verify_algorithmic_bytes(vs)
            extra["verify_batch%d" % wb.B] = {
                "bound": "hbm", "kernel": "verify_walk_kernel", "achieved": round(vbytes / (vb_avg * 1e-3) / 1e9, 1),
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(vbytes / (vb_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "algorithmic_bytes_per_launch": int(vbytes), "avg_launch_us": round(vb_avg * 1e3, 2),
                "sequences_per_s": round(wb.B / (vb_avg * 1e-3), 1), "mean_accept_len": round(float(got[1].mean()), 3),
                "verified_vs_oracle": True, "workload": f"{w_name} verification, B={wb.B}, V={wb.V}"}
            del dp, dq
        except Exception as ex:
            extra["verify_batch"] = {"error": repr(ex)}
    # early-stop decision models (Sec. 3.3) on the newest contexts of fork-shaped trees of width 16: one tree, and a
    # batch whose rows (4 distinct copies, > 512 MB) cannot stay in the last-level cache between launches
    if args.decision_batch > 0:
        try:
            import numpy as np
            from workloads import hidden_states, mlp_weights, scaled, verify_inputs
            import oracle
            k, Wd, beta = 10, 16, 0.4
            Bd = args.decision_batch
            wd = scaled(WORKLOADS["fork"], B=Bd, branching=(Wd, 1))
            q = verify_inputs(wd, seed=1, mode=0)["q_draft"]                  # [Bd][1 + 16][V]; rows 1.. are the new contexts
            V = wd.V
            ws, bs = mlp_weights((k + 1, 64, 1), seed=0, out_bias=-0.3)
            mlp2 = binding.make_mlp([torch.from_numpy(a).cuda() for a in ws], [torch.from_numpy(a).cuda() for a in bs])
            wbytes = sum(a.nbytes for a in ws + bs)
            copies = 4
            rows = torch.from_numpy(np.ascontiguousarray(q[:, 1:])).cuda().repeat(copies, 1, 1)   # [copies*Bd][16][V]
            prob = torch.zeros((copies * Bd, Wd), dtype=torch.float32, device="cuda")
            stop = torch.zeros((copies * Bd,), dtype=torch.int32, device="cuda")

            ds = Ctx(binding, torch)
            nb = min(Bd, 4)
            want = oracle.mlp(ws, bs, oracle.decision_features(q[:nb, 1:].reshape(nb * Wd, V), k)).reshape(nb, Wd)
            for trees, tag in ((1, "1"), (copies * Bd, str(copies * Bd))):
                def dcall(i, trees=trees):
                    binding.early_stop_distribution(mlp2, trees, Wd, V, k, rows, Wd * V, V, beta, None, prob, stop)
                dcall(0)
                torch.cuda.synchronize()
                nchk = min(nb, trees)
                gotp = prob[:nchk].cpu().numpy()
                assert np.abs(gotp - want[:nchk]).max() <= 1e-5, "decision model differs from the oracle"
                assert stop[:nchk].cpu().tolist() == [int((gotp[b] < np.float32(beta)).all()) for b in range(nchk)]
                d_avg = time_kernel(ds, hip, binding.KERNEL_DECISION, dcall, 30, warm=10)[0]
                t0 = time.perf_counter()
                for i in range(50):
                    dcall(i)
                torch.cuda.synchronize()
                call_us = (time.perf_counter() - t0) / 50 * 1e6
                dbytes = trees * Wd * V * 4 + wbytes
                extra["early_stop_distribution_trees" + tag] = {
                    "bound": "hbm", "kernel": "decision_distribution_kernel", "achieved": round(dbytes / (d_avg * 1e-3) / 1e9, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(dbytes / (d_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                    "algorithmic_bytes_per_launch": int(dbytes), "avg_launch_us": round(d_avg * 1e3, 2),
                    "call_us": round(call_us, 1), "verified_vs_oracle": True,
                    "workload": f"{trees} fork tree(s) of width {Wd}, V={V}, top-{k} + entropy, MLP {k + 1}-64-1, beta {beta}"}
            del rows
            hw = (768, 256, 64, 1)                                          # hidden width of the 68M draft model
            ws1, bs1 = mlp_weights(hw, seed=1, out_bias=-0.4)
            mlp1 = binding.make_mlp([torch.from_numpy(a).cuda() for a in ws1], [torch.from_numpy(a).cuda() for a in bs1])
            hx = hidden_states(Bd, Wd, hw[0], seed=1)
            hxd = torch.from_numpy(hx).cuda()

            def hcall(i):
                binding.early_stop_hidden(mlp1, Bd, Wd, hxd, Wd * hw[0], hw[0], beta, prob, stop)
            hcall(0)
            torch.cuda.synchronize()
            want1 = oracle.mlp(ws1, bs1, hx[:nb].reshape(nb * Wd, hw[0]).astype(np.float64)).reshape(nb, Wd)
            assert np.abs(prob[:nb].cpu().numpy() - want1).max() <= 1e-6, "hidden-state decision model differs from the oracle"
            h_avg = time_kernel(ds, hip, binding.KERNEL_DECISION, hcall, 30, warm=10)[0]
            extra["early_stop_hidden_trees%d" % Bd] = {
                "kernel": "decision_hidden_kernel", "avg_launch_us": round(h_avg * 1e3, 2), "verified_vs_oracle": True,
                "bytes_per_launch": int(hx.nbytes + sum(a.nbytes for a in ws1 + bs1)),
                "workload": f"{Bd} trees of width {Wd}, hidden width {hw[0]}, MLP {'-'.join(map(str, hw))} (latency-bound)"}
        except Exception as ex:
            extra["early_stop"] = {"error": repr(ex)}
    # yardstick: what the HBM of this machine delivers to a plain read-only streaming kernel (4 GiB buffer)
    try:
        buf = torch.empty(4 << 30, dtype=torch.uint8, device="cuda")
        buf.fill_(1)
        sink = torch.zeros(16, dtype=torch.uint8, device="cuda")

        ss = Ctx(binding, torch)
        per_grid = {}
        for wgs in (256, 512, 2048, 8192):      # the rate depends on how the grid's stride falls on the memory channels
            s_avg = time_kernel(ss, hip, binding.KERNEL_STREAM_READ, lambda i: binding.stream_read(buf, sink, wgs), 10, warm=10)[0]
            per_grid[wgs] = round(buf.numel() / (s_avg * 1e-3) / 1e9, 1)
        gbps = max(per_grid.values())
        out["stream_read_probe"] = {"GB/s": gbps, "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4), "bytes": buf.numel(),
                                    "GB/s_by_workgroups": per_grid}
        for r in [out["roofline"]] + [v for v in extra.values() if v.get("bound") == "hbm"]:
            r["frac_of_stream_read"] = round(r["achieved"] / gbps, 4)
        del buf
    except Exception as ex:
        out["stream_read_probe"] = {"error": repr(ex)}
    if extra:
        out["other_workloads"] = extra
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
