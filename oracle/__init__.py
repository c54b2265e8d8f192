"""Python access to the CPU oracle (oracle/mcsd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's CPU-baseline
leg.  The product package never imports this module, and this module never imports the product.
It only marshals numpy arrays into the plain-C oracle; all arithmetic lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mcsd_oracle.c")
_LIB = os.path.join(_HERE, "libmcsd_oracle.so")
_lib = None


_LIB_SAN = os.path.join(_HERE, "libmcsd_oracle_san.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc: -O2, contraction off (explicit fma only), OpenMP over sequences/heads.
    sanitize=True builds a second library, -O1 with AddressSanitizer and UndefinedBehaviorSanitizer (any finding
    aborts), which a process loads instead when MCSD_ORACLE_SANITIZED=1 is set and the sanitizer runtime is
    preloaded (see tests/test_sanitized_host_code.py)."""
    lib = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] \
            if sanitize else ["-O2"]
        cmd = ["gcc", *opt, "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", lib, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return lib


def sanitizer_runtime() -> str:
    """Path of gcc's AddressSanitizer runtime, to be preloaded by a process that loads the sanitized library."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


def _load():
    global _lib
    if _lib is None:
        sanitized = os.environ.get("MCSD_ORACLE_SANITIZED") == "1"
        L = C.CDLL(build(sanitize=sanitized))
        vp, i32, i64, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        L.mcsd_oracle_level_sizes.restype = i64
        L.mcsd_oracle_level_sizes.argtypes = [vp, i32, vp]
        L.mcsd_oracle_tree_tables.restype = C.c_int
        L.mcsd_oracle_tree_tables.argtypes = [vp, i32, vp, vp]
        L.mcsd_oracle_build_mask.restype = C.c_int
        L.mcsd_oracle_build_mask.argtypes = [vp, i32, vp]
        L.mcsd_oracle_slice_mask.restype = None
        L.mcsd_oracle_slice_mask.argtypes = [vp, i64, i64, vp]
        L.mcsd_oracle_tree_attention.restype = None
        L.mcsd_oracle_tree_attention.argtypes = [i32, i32, i32, i32, i32, i64, vp, vp, vp, vp, vp, vp, vp, i64,
                                                 f64, vp, i64, vp]
        L.mcsd_oracle_tree_attention_row.restype = None
        L.mcsd_oracle_tree_attention_row.argtypes = [i32, i32, i32, i32, i64, vp, vp, vp, vp, vp, vp, vp, i64,
                                                     f64, vp, i64, i32, i32, i32, vp]
        L.mcsd_oracle_fp8_e4m3_value.restype = f64
        L.mcsd_oracle_fp8_e4m3_value.argtypes = [C.c_uint8]
        L.mcsd_oracle_tree_attention_fp8kv.restype = None
        L.mcsd_oracle_tree_attention_fp8kv.argtypes = [i32, i32, i32, i32, i64, vp, vp, vp, vp, vp, f64, f64, vp, vp, i64,
                                                       f64, vp, i64, vp]
        L.mcsd_oracle_tree_attention_row_fp8kv.restype = None
        L.mcsd_oracle_tree_attention_row_fp8kv.argtypes = [i32, i32, i32, i64, vp, vp, vp, vp, vp, f64, f64, vp, vp, i64,
                                                           f64, vp, i64, i32, i32, i32, vp]
        L.mcsd_oracle_verify_tree.restype = C.c_int
        L.mcsd_oracle_verify_tree.argtypes = [i32, vp, i32, i32, i32, vp, vp, vp, i64, i64, vp, vp, i32, vp, vp, vp]
        L.mcsd_oracle_verify_tree_without_replacement.restype = C.c_int
        L.mcsd_oracle_verify_tree_without_replacement.argtypes = L.mcsd_oracle_verify_tree.argtypes
        L.mcsd_oracle_tree_sum.restype = f64
        L.mcsd_oracle_tree_sum.argtypes = [vp, i64]
        L.mcsd_oracle_tree_sample.restype = i32
        L.mcsd_oracle_tree_sample.argtypes = [vp, i64, C.c_float]
        L.mcsd_oracle_improvement_factor.restype = f64
        L.mcsd_oracle_improvement_factor.argtypes = [f64, f64, f64]
        L.mcsd_oracle_commit_path.restype = C.c_int
        L.mcsd_oracle_commit_path.argtypes = [i32, i32, i32, i32, i32, i32, i64, vp, vp, vp, vp, vp, i64, vp, vp, vp, vp]
        L.mcsd_oracle_commit_ids.restype = C.c_int
        L.mcsd_oracle_commit_ids.argtypes = [i32, i32, i32, vp, vp, vp, vp, i32, i32, vp, vp]
        L.mcsd_oracle_decision_features.restype = C.c_int
        L.mcsd_oracle_decision_features.argtypes = [i64, i32, vp, vp]
        L.mcsd_oracle_mlp.restype = f64
        L.mcsd_oracle_mlp.argtypes = [i32, vp, vp, vp, vp]
        L.mcsd_oracle_early_stop.restype = i32
        L.mcsd_oracle_early_stop.argtypes = [vp, i32, f64]
        L.mcsd_oracle_threads.restype = i32
        L.mcsd_oracle_threads.argtypes = []
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _branching(b: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(b, dtype=np.int32))


def level_sizes(branching: Sequence[int]) -> np.ndarray:
    b = _branching(branching)
    sizes = np.zeros(len(b), dtype=np.int64)
    n = _load().mcsd_oracle_level_sizes(_ptr(b), len(b), _ptr(sizes))
    if n < 0:
        raise ValueError("bad branching")
    return sizes


def n_nodes(branching: Sequence[int]) -> int:
    return int(level_sizes(branching).sum())


def tree_tables(branching: Sequence[int]):
    b = _branching(branching)
    n = n_nodes(b)
    parent = np.zeros(n, dtype=np.int32)
    level = np.zeros(n, dtype=np.int32)
    if _load().mcsd_oracle_tree_tables(_ptr(b), len(b), _ptr(parent), _ptr(level)) != 0:
        raise ValueError("bad branching")
    return parent, level


def build_mask(branching: Sequence[int]) -> np.ndarray:
    """Dense uint8 [N][N] topology-aware causal mask of the whole tree."""
    b = _branching(branching)
    n = n_nodes(b)
    M = np.zeros((n, n), dtype=np.uint8)
    if _load().mcsd_oracle_build_mask(_ptr(b), len(b), _ptr(M)) != 0:
        raise ValueError("bad branching")
    return M


def slice_mask(M: np.ndarray, n: int) -> np.ndarray:
    M = np.ascontiguousarray(M, dtype=np.uint8)
    out = np.zeros((n, n), dtype=np.uint8)
    _load().mcsd_oracle_slice_mask(_ptr(M), M.shape[0], n, _ptr(out))
    return out


def _dtype_code(dtype: str) -> int:
    return {"f32": 0, "bf16": 1}[dtype]


def _check_store(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    assert a.dtype == want, (a.dtype, want)
    return np.ascontiguousarray(a)


def tree_attention(inp: dict, M: np.ndarray, n: int) -> np.ndarray:
    """All outputs, binary64 [B][H][n][d], for an input dict as made by workloads.attention_inputs."""
    dt = inp["dtype"]
    q, kt, vt = (_check_store(inp[k], dt) for k in ("q", "k_tree", "v_tree"))
    kp, vp = (_check_store(inp[k], dt) for k in ("k_prefix", "v_prefix"))
    B, H, _, d = q.shape
    M = np.ascontiguousarray(M, dtype=np.uint8)
    lens = np.ascontiguousarray(inp["lens"], dtype=np.int32)
    base = np.ascontiguousarray(inp["seq_base"], dtype=np.int64)
    out = np.zeros((B, H, n, d), dtype=np.float64)
    _load().mcsd_oracle_tree_attention(_dtype_code(dt), B, H, d, n, int(inp["node_stride"]), _ptr(q), _ptr(kt),
                                       _ptr(vt), _ptr(kp), _ptr(vp), _ptr(base), _ptr(lens),
                                       int(inp["head_stride"]), float(np.float32(inp["scale"])), _ptr(M),
                                       M.shape[1], _ptr(out))
    return out


def tree_attention_row(inp: dict, M: np.ndarray, n: int, b: int, h: int, i: int) -> np.ndarray:
    """One output row (d values, binary64) for sequence b, head h, tree node i."""
    dt = inp["dtype"]
    q, kt, vt = (_check_store(inp[k], dt) for k in ("q", "k_tree", "v_tree"))
    kp, vp = (_check_store(inp[k], dt) for k in ("k_prefix", "v_prefix"))
    _, H, _, d = q.shape
    M = np.ascontiguousarray(M, dtype=np.uint8)
    lens = np.ascontiguousarray(inp["lens"], dtype=np.int32)
    base = np.ascontiguousarray(inp["seq_base"], dtype=np.int64)
    out = np.zeros(d, dtype=np.float64)
    _load().mcsd_oracle_tree_attention_row(_dtype_code(dt), H, d, n, int(inp["node_stride"]), _ptr(q), _ptr(kt),
                                           _ptr(vt), _ptr(kp), _ptr(vp), _ptr(base), _ptr(lens),
                                           int(inp["head_stride"]), float(np.float32(inp["scale"])), _ptr(M),
                                           M.shape[1], b, h, i, _ptr(out))
    return out


def fp8_e4m3_value(code: int) -> float:
    """The number an 8-bit E4M3 code stands for (NaN for S.1111.111)."""
    return float(_load().mcsd_oracle_fp8_e4m3_value(int(code) & 255))


def _fp8_args(inp: dict):
    q, kt, vt = (_check_store(inp[k], "bf16") for k in ("q", "k_tree", "v_tree"))
    kp, vp = (np.ascontiguousarray(inp[k]) for k in ("k_prefix", "v_prefix"))
    assert kp.dtype == np.uint8 and vp.dtype == np.uint8 and inp["dtype"] == "bf16"
    lens = np.ascontiguousarray(inp["lens"], dtype=np.int32)
    base = np.ascontiguousarray(inp["seq_base"], dtype=np.int64)
    return q, kt, vt, kp, vp, lens, base


def tree_attention_fp8kv(inp: dict, M: np.ndarray, n: int) -> np.ndarray:
    """All outputs, binary64 [B][H][n][d], for an input dict as made by workloads.attention_inputs(kv_fp8=True)."""
    q, kt, vt, kp, vp, lens, base = _fp8_args(inp)
    B, H, _, d = q.shape
    M = np.ascontiguousarray(M, dtype=np.uint8)
    out = np.zeros((B, H, n, d), dtype=np.float64)
    _load().mcsd_oracle_tree_attention_fp8kv(B, H, d, n, int(inp["node_stride"]), _ptr(q), _ptr(kt), _ptr(vt), _ptr(kp),
                                             _ptr(vp), float(np.float32(inp["k_scale"])), float(np.float32(inp["v_scale"])),
                                             _ptr(base), _ptr(lens), int(inp["head_stride"]),
                                             float(np.float32(inp["scale"])), _ptr(M), M.shape[1], _ptr(out))
    return out


def tree_attention_row_fp8kv(inp: dict, M: np.ndarray, n: int, b: int, h: int, i: int) -> np.ndarray:
    q, kt, vt, kp, vp, lens, base = _fp8_args(inp)
    _, H, _, d = q.shape
    M = np.ascontiguousarray(M, dtype=np.uint8)
    out = np.zeros(d, dtype=np.float64)
    _load().mcsd_oracle_tree_attention_row_fp8kv(H, d, n, int(inp["node_stride"]), _ptr(q), _ptr(kt), _ptr(vt), _ptr(kp),
                                                 _ptr(vp), float(np.float32(inp["k_scale"])),
                                                 float(np.float32(inp["v_scale"])), _ptr(base), _ptr(lens),
                                                 int(inp["head_stride"]), float(np.float32(inp["scale"])), _ptr(M),
                                                 M.shape[1], b, h, i, _ptr(out))
    return out


def verify_tree(mode: int, branching: Sequence[int], tokens: np.ndarray, p: np.ndarray, q: np.ndarray,
                u_accept: np.ndarray, u_sample: np.ndarray, replacement: bool = True):
    """Returns (path int32 [B][G] padded with -1, accept_len int32 [B], new_tokens int32 [B][n_new]).
    replacement=False: the siblings of a context were drawn without replacement."""
    b = _branching(branching)
    G = len(b)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    p = np.ascontiguousarray(p, dtype=np.float32)
    q = np.ascontiguousarray(q, dtype=np.float32)
    ua = np.ascontiguousarray(u_accept, dtype=np.float32)
    us = np.ascontiguousarray(u_sample, dtype=np.float32)
    B, N = tokens.shape
    V = p.shape[-1]
    sizes = level_sizes(b)
    assert N == int(sizes.sum()), (N, sizes)
    assert p.shape == (B, 1 + N, V), p.shape
    assert q.shape == (B, 1 + N - int(sizes[-1]), V), q.shape
    assert ua.shape == (B, N)
    n_new = us.shape[1]
    path = np.zeros((B, G), dtype=np.int32)
    alen = np.zeros(B, dtype=np.int32)
    new = np.zeros((B, n_new), dtype=np.int32)
    fn = _load().mcsd_oracle_verify_tree if replacement else _load().mcsd_oracle_verify_tree_without_replacement
    rc = fn(int(mode), _ptr(b), G, B, V, _ptr(tokens), _ptr(p), _ptr(q), p.shape[1] * V, q.shape[1] * V, _ptr(ua),
            _ptr(us), n_new, _ptr(path), _ptr(alen), _ptr(new))
    if rc != 0:
        raise ValueError(f"oracle verify_tree failed: {rc}")
    return path, alen, new


def commit_path(inp: dict, gamma: int, n: int, path: np.ndarray, accept_len: np.ndarray):
    """Appends the accepted path's tree K/V rows to a COPY of the prefix cache of `inp` (one layer, as made by
    workloads.attention_inputs).  Returns (k_prefix, v_prefix, lens) after the update."""
    dt = inp["dtype"]
    kt, vt = (_check_store(inp[k], dt) for k in ("k_tree", "v_tree"))
    kp, vp = (_check_store(inp[k], dt).copy() for k in ("k_prefix", "v_prefix"))
    B, H, _, d = kt.shape
    path = np.ascontiguousarray(path, dtype=np.int32)
    alen = np.ascontiguousarray(accept_len, dtype=np.int32)
    assert path.shape == (B, gamma) and alen.shape == (B,)
    lens = np.ascontiguousarray(inp["lens"], dtype=np.int32)
    base = np.ascontiguousarray(inp["seq_base"], dtype=np.int64)
    cap = kp.shape[2]
    assert int((lens + alen).max()) <= cap, "cache too small for the accepted path"
    lens_out = np.zeros(B, dtype=np.int32)
    rc = _load().mcsd_oracle_commit_path(kt.itemsize, B, H, d, gamma, n, int(inp["node_stride"]), _ptr(kt), _ptr(vt),
                                         _ptr(kp), _ptr(vp), _ptr(base), int(inp["head_stride"]), _ptr(path),
                                         _ptr(alen), _ptr(lens), _ptr(lens_out))
    if rc != 0:
        raise ValueError("oracle commit_path: bad path or length")
    return kp, vp, lens_out


def commit_ids(gamma: int, tokens: np.ndarray, path: np.ndarray, accept_len: np.ndarray, new_tokens: np.ndarray,
               n_append: int):
    """(ids int32 [B][gamma + n_append] padded with -1, n_ids int32 [B])."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    path = np.ascontiguousarray(path, dtype=np.int32)
    alen = np.ascontiguousarray(accept_len, dtype=np.int32)
    new = np.ascontiguousarray(new_tokens, dtype=np.int32).reshape(tokens.shape[0], -1)
    B, n = tokens.shape
    n_new = new.shape[1]
    if n_new == 0:
        new = np.zeros((B, 1), dtype=np.int32)
    ids = np.zeros((B, gamma + n_append), dtype=np.int32)
    n_ids = np.zeros(B, dtype=np.int32)
    rc = _load().mcsd_oracle_commit_ids(B, gamma, n, _ptr(tokens), _ptr(path), _ptr(alen), _ptr(new), n_new, n_append,
                                        _ptr(ids), _ptr(n_ids))
    if rc != 0:
        raise ValueError("oracle commit_ids: bad argument")
    return ids, n_ids


def decision_features(rows: np.ndarray, k: int) -> np.ndarray:
    """Concat(Topk(y), Ent(y)) of every distribution: rows fp32 [M][V] -> binary64 [M][k+1]."""
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    M, V = rows.shape
    out = np.zeros((M, k + 1), dtype=np.float64)
    for m in range(M):
        if _load().mcsd_oracle_decision_features(V, int(k), _ptr(rows[m]), _ptr(out[m])) != 0:
            raise ValueError("oracle decision_features: bad argument")
    return out


def mlp(weights: Sequence[np.ndarray], biases: Sequence[np.ndarray], X: np.ndarray) -> np.ndarray:
    """Decision-model output for every row of X (binary64 [M][width0]); weights[l] fp32 [out_l][in_l]."""
    n = len(weights)
    assert len(biases) == n and n >= 1
    ws = [np.ascontiguousarray(w, dtype=np.float32) for w in weights]
    bs = [np.ascontiguousarray(b, dtype=np.float32) for b in biases]
    width = [ws[0].shape[1]] + [w.shape[0] for w in ws]
    for l in range(n):
        assert ws[l].shape == (width[l + 1], width[l]) and bs[l].shape == (width[l + 1],), (l, ws[l].shape)
    assert width[-1] == 1
    X = np.ascontiguousarray(X, dtype=np.float64)
    assert X.ndim == 2 and X.shape[1] == width[0]
    warr = np.asarray(width, dtype=np.int32)
    wp = (C.c_void_p * n)(*[_ptr(w) for w in ws])
    bp = (C.c_void_p * n)(*[_ptr(b) for b in bs])
    return np.array([_load().mcsd_oracle_mlp(n, _ptr(warr), wp, bp, _ptr(X[m])) for m in range(X.shape[0])],
                    dtype=np.float64)


def early_stop(P: np.ndarray, beta: float) -> np.ndarray:
    """P binary64 [B][W] -> int32 [B]: 1 where every candidate sequence is predicted below beta."""
    P = np.ascontiguousarray(P, dtype=np.float64)
    B, W = P.shape
    return np.array([_load().mcsd_oracle_early_stop(_ptr(P[b]), W, float(beta)) for b in range(B)], dtype=np.int32)


def tree_sum(a: np.ndarray) -> float:
    a = np.ascontiguousarray(a, dtype=np.float64)
    return float(_load().mcsd_oracle_tree_sum(_ptr(a), a.size))


def tree_sample(a: np.ndarray, u: float) -> int:
    a = np.ascontiguousarray(a, dtype=np.float64)
    return int(_load().mcsd_oracle_tree_sample(_ptr(a), a.size, float(np.float32(u))))


def improvement_factor(alpha: float, gamma: float, c: float) -> float:
    return float(_load().mcsd_oracle_improvement_factor(alpha, gamma, c))


def threads() -> int:
    """Threads the oracle's outer loops use."""
    return int(_load().mcsd_oracle_threads())
