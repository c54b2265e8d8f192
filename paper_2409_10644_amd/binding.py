"""ctypes binding of libmcsd.so: same names and argument order as include/mcsd.h, marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmcsd.so")

MCSD_OK, MCSD_EINVAL, MCSD_ENOMEM, MCSD_EHIP, MCSD_EWORKSPACE, MCSD_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
MCSD_F32, MCSD_BF16 = 0, 1
MCSD_DRAFT_INIT, MCSD_TARGET_INIT = 0, 1
MCSD_WITH_REPLACEMENT, MCSD_WITHOUT_REPLACEMENT = 0, 1

EXPORTS = ["mcsd_strerror", "mcsd_build_mask", "mcsd_slice_mask", "mcsd_free_mask",
           "mcsd_tree_attention_workspace", "mcsd_tree_attention",
           "mcsd_tree_attention_rows_workspace", "mcsd_tree_attention_rows",
           "mcsd_tree_attention_gqa_workspace", "mcsd_tree_attention_gqa",
           "mcsd_tree_attention_fp8kv_workspace", "mcsd_tree_attention_fp8kv",
           "mcsd_verify_tree_workspace", "mcsd_verify_tree", "mcsd_verify_tree_sampling", "mcsd_commit_path", "mcsd_early_stop_distribution",
           "mcsd_early_stop_hidden", "mcsd_profile_next", "mcsd_stream_read", "mcsd_issue_probe", "mcsd_placement_probe", "mcsd_workspace_init",
           "mcsd_tree_attention_tuned_workspace", "mcsd_tree_attention_tuned", "mcsd_tree_attention_static",
           "mcsd_tree_attention_plan"]
STATIC_SCRATCH_BYTES = 24 * 1024 * 1024
DECISION_MAX_K, MLP_MAX_LAYERS, MLP_MAX_WIDTH, MLP_MAX_INPUTS = 16, 3, 512, 8192


class MaskView(C.Structure):
    """mcsd_mask_view_t"""
    _fields_ = [("gamma", C.c_int32), ("n_nodes", C.c_int32), ("gamma_max", C.c_int32),
                ("n_nodes_max", C.c_int32), ("words_per_row", C.c_int32), ("device", C.c_int32),
                ("bits_host", C.POINTER(C.c_uint64)), ("bits_dev", C.c_void_p),
                ("parent_host", C.POINTER(C.c_int32)), ("parent_dev", C.c_void_p),
                ("level_host", C.POINTER(C.c_int32)), ("level_off_host", C.POINTER(C.c_int32)),
                ("branching_host", C.POINTER(C.c_int32))]


class Mlp(C.Structure):
    """mcsd_mlp_t"""
    _fields_ = [("n_layers", C.c_int32), ("width", C.c_int32 * (MLP_MAX_LAYERS + 1)),
                ("weight", C.c_void_p * MLP_MAX_LAYERS), ("bias", C.c_void_p * MLP_MAX_LAYERS)]


class AttentionTuning(C.Structure):
    """mcsd_attention_tuning_t"""
    _fields_ = [("key_splits", C.c_int32), ("natural_order", C.c_int32), ("fold", C.c_int32), ("stages", C.c_int32),
                ("tree_keys", C.c_int32)]


class AttentionPlan(C.Structure):
    """mcsd_attention_plan_t"""
    _fields_ = [("mfma_path", C.c_int32), ("query_blocks", C.c_int32), ("key_splits", C.c_int32),
                ("workgroups", C.c_int32), ("stages", C.c_int32), ("fold_in_kernel", C.c_int32),
                ("ordered_by_length", C.c_int32)]


class McsdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2409_10644_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    # The library must share the HIP runtime that PyTorch loaded (streams and allocations cross the boundary).
    with open("/proc/self/maps") as f:
        runtimes = {line.split()[-1] for line in f if "libamdhip64" in line}
    if len(runtimes) > 1:
        raise ImportError(f"two HIP runtimes in one process: {sorted(runtimes)}")
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    lib.mcsd_strerror.restype = C.c_char_p
    lib.mcsd_strerror.argtypes = [C.c_int]
    lib.mcsd_build_mask.restype = C.c_int
    lib.mcsd_build_mask.argtypes = [C.POINTER(i32), i32, C.POINTER(vp)]
    lib.mcsd_slice_mask.restype = C.c_int
    lib.mcsd_slice_mask.argtypes = [vp, i32, C.POINTER(MaskView)]
    lib.mcsd_free_mask.restype = None
    lib.mcsd_free_mask.argtypes = [vp]
    lib.mcsd_tree_attention_workspace.restype = sz
    lib.mcsd_tree_attention_workspace.argtypes = [i32, i32, i32, i32, i32]
    lib.mcsd_tree_attention.restype = C.c_int
    lib.mcsd_tree_attention.argtypes = [C.POINTER(MaskView), C.c_int, i32, i32, i32, vp, vp, vp, i64, vp, vp, vp,
                                        vp, i64, i32, C.c_float, vp, vp, sz, vp]
    lib.mcsd_verify_tree_workspace.restype = sz
    lib.mcsd_verify_tree_workspace.argtypes = [C.POINTER(MaskView), C.c_int, i32, i32]
    lib.mcsd_verify_tree.restype = C.c_int
    lib.mcsd_verify_tree.argtypes = [C.POINTER(MaskView), C.c_int, i32, i32, vp, vp, vp, i64, i64, vp, vp, i32,
                                     vp, vp, vp, vp, sz, vp]
    lib.mcsd_verify_tree_sampling.restype = C.c_int
    lib.mcsd_verify_tree_sampling.argtypes = [C.POINTER(MaskView), C.c_int, C.c_int, i32, i32, vp, vp, vp, i64, i64, vp,
                                              vp, i32, vp, vp, vp, vp, sz, vp]
    lib.mcsd_profile_next.restype = C.c_int
    lib.mcsd_tree_attention_rows_workspace.restype = C.c_size_t
    lib.mcsd_tree_attention_rows_workspace.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.mcsd_tree_attention_rows.restype = C.c_int
    lib.mcsd_tree_attention_rows.argtypes = [C.POINTER(MaskView), C.c_int, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp,
                                             vp, vp, i64, i32, C.c_float, vp, vp, C.c_size_t, vp]
    lib.mcsd_tree_attention_gqa_workspace.restype = C.c_size_t
    lib.mcsd_tree_attention_gqa_workspace.argtypes = [i32, i32, i32, i32, i32, i32, i32]
    lib.mcsd_tree_attention_gqa.restype = C.c_int
    lib.mcsd_tree_attention_gqa.argtypes = [C.POINTER(MaskView), C.c_int, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp,
                                            vp, vp, vp, i64, i32, C.c_float, vp, vp, C.c_size_t, vp]
    lib.mcsd_tree_attention_fp8kv_workspace.restype = C.c_size_t
    lib.mcsd_tree_attention_fp8kv_workspace.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.mcsd_tree_attention_fp8kv.restype = C.c_int
    lib.mcsd_tree_attention_fp8kv.argtypes = [C.POINTER(MaskView), i32, i32, i32, i32, vp, vp, vp, i64, vp, vp,
                                              C.c_float, C.c_float, vp, vp, i64, i32, C.c_float, vp, vp, C.c_size_t, vp]
    lib.mcsd_commit_path.restype = C.c_int
    lib.mcsd_commit_path.argtypes = [C.POINTER(MaskView), C.c_int, i32, i32, i32, i32, C.POINTER(vp), C.POINTER(vp),
                                     i64, C.POINTER(vp), C.POINTER(vp), vp, i64, i32, i32, vp, vp, vp, vp, i32, i32,
                                     vp, vp, vp, vp]
    lib.mcsd_profile_next.argtypes = [C.c_int, vp, vp]
    lib.mcsd_early_stop_distribution.restype = C.c_int
    lib.mcsd_early_stop_distribution.argtypes = [C.POINTER(Mlp), i32, i32, i32, i32, vp, i64, i64, C.c_float, vp, vp,
                                                 vp, vp]
    lib.mcsd_early_stop_hidden.restype = C.c_int
    lib.mcsd_early_stop_hidden.argtypes = [C.POINTER(Mlp), i32, i32, vp, i64, i64, C.c_float, vp, vp, vp]
    lib.mcsd_stream_read.restype = C.c_int
    lib.mcsd_stream_read.argtypes = [vp, C.c_size_t, vp, i32, vp]
    lib.mcsd_issue_probe.restype = C.c_int
    lib.mcsd_issue_probe.argtypes = [i32, i32, i32, vp, vp]
    lib.mcsd_placement_probe.restype = C.c_int
    lib.mcsd_placement_probe.argtypes = [i32, i32, vp, vp]
    lib.mcsd_tree_attention_static.restype = C.c_int
    lib.mcsd_tree_attention_static.argtypes = [C.POINTER(MaskView), C.c_int, i32, i32, i32, vp, vp, vp, i64, vp, vp, vp,
                                               vp, i64, i32, C.c_float, vp, vp]
    lib.mcsd_tree_attention_plan.restype = C.c_int
    lib.mcsd_tree_attention_plan.argtypes = [C.POINTER(AttentionTuning), C.c_int, i32, i32, i32, i32, i32, i32, i32, i32,
                                             C.POINTER(AttentionPlan)]
    lib.mcsd_workspace_init.restype = C.c_int
    lib.mcsd_workspace_init.argtypes = [vp, sz, vp]
    lib.mcsd_tree_attention_tuned_workspace.restype = sz
    lib.mcsd_tree_attention_tuned_workspace.argtypes = [C.POINTER(AttentionTuning), i32, i32, i32, i32, i32, i32, i32, i32]
    lib.mcsd_tree_attention_tuned.restype = C.c_int
    lib.mcsd_tree_attention_tuned.argtypes = [C.POINTER(AttentionTuning), C.POINTER(MaskView), C.c_int, i32, C.c_float,
                                              C.c_float, i32, i32, i32, i32, i32, vp, vp, vp, i64, vp, vp, vp, vp, i64,
                                              i32, C.c_float, vp, vp, sz, vp]
    return lib


lib = _load()

KERNEL_ATTN_SWEEP, KERNEL_ATTN_MERGE, KERNEL_VERIFY_WALK, KERNEL_COMMIT_COPY, KERNEL_STREAM_READ = 0, 1, 2, 3, 4
KERNEL_DECISION = 5


def strerror(status: int) -> str:
    return lib.mcsd_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != MCSD_OK:
        raise McsdError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream=None) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


class Mask:
    """Owner of an mcsd_mask_t handle (built once at gamma_max)."""

    def __init__(self, handle: int, gamma_max: int):
        self.handle = handle
        self.gamma_max = gamma_max
        self._free = lib.mcsd_free_mask      # bound here: module globals may be gone at interpreter exit

    def close(self) -> None:
        if self.handle:
            self._free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def build_mask(branching: Sequence[int], gamma_max: Optional[int] = None) -> Mask:
    g = len(branching) if gamma_max is None else int(gamma_max)
    if g > len(branching):
        raise McsdError(MCSD_EINVAL, "mcsd_build_mask (gamma_max beyond the branching vector)")
    arr = (C.c_int32 * max(len(branching), 1))(*[int(x) for x in branching])
    handle = C.c_void_p()
    _check(lib.mcsd_build_mask(arr, g, C.byref(handle)), "mcsd_build_mask")
    return Mask(handle.value, g)


def slice_mask(mask: Mask, gamma: int) -> MaskView:
    view = MaskView()
    _check(lib.mcsd_slice_mask(mask.handle, int(gamma), C.byref(view)), "mcsd_slice_mask")
    view._owner = mask          # keep the handle alive as long as the view
    return view


def free_mask(mask: Mask) -> None:
    mask.close()


def workspace_init(workspace: Optional[torch.Tensor], stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.mcsd_workspace_init(_ptr(workspace), ws_bytes, _stream(stream)), "mcsd_workspace_init")


def new_workspace(nbytes: int, stream=None) -> torch.Tensor:
    """A device buffer of at least nbytes (and at least 256) bytes, prepared with mcsd_workspace_init."""
    ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")
    workspace_init(ws, stream)
    return ws


def _tuning_ref(tuning: Optional[AttentionTuning]):
    return None if tuning is None else C.byref(tuning)


def tree_attention_tuned_workspace(tuning: Optional[AttentionTuning], prefix_fp8: int, B: int, H_q: int, H_kv: int, d: int,
                                   n_nodes: int, row_begin: int, max_prefix: int) -> int:
    return int(lib.mcsd_tree_attention_tuned_workspace(_tuning_ref(tuning), prefix_fp8, B, H_q, H_kv, d, n_nodes,
                                                       row_begin, max_prefix))


def tree_attention_tuned(tuning: Optional[AttentionTuning], view: MaskView, dtype: int, prefix_fp8: int, k_scale: float,
                         v_scale: float, B: int, H_q: int, H_kv: int, d: int, row_begin: int, q: torch.Tensor,
                         k_tree: torch.Tensor, v_tree: torch.Tensor, node_stride: int, k_prefix: Optional[torch.Tensor],
                         v_prefix: Optional[torch.Tensor], seq_base_dev: torch.Tensor, prefix_lens_dev: torch.Tensor,
                         head_stride: int, max_prefix: int, softmax_scale: float, out: torch.Tensor,
                         workspace: Optional[torch.Tensor], stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mcsd_tree_attention_tuned(_tuning_ref(tuning), C.byref(view), dtype, prefix_fp8, k_scale, v_scale, B, H_q,
                                       H_kv, d, row_begin, _ptr(q), _ptr(k_tree), _ptr(v_tree), node_stride,
                                       _ptr(k_prefix), _ptr(v_prefix), _ptr(seq_base_dev), _ptr(prefix_lens_dev),
                                       head_stride, max_prefix, softmax_scale, _ptr(out), _ptr(workspace), ws_bytes,
                                       _stream(stream))
    _check(st, "mcsd_tree_attention_tuned")


def tree_attention_workspace(B: int, H: int, d: int, n_nodes: int, max_prefix: int) -> int:
    return int(lib.mcsd_tree_attention_workspace(B, H, d, n_nodes, max_prefix))


def tree_attention(view: MaskView, dtype: int, B: int, H: int, d: int, q: torch.Tensor, k_tree: torch.Tensor,
                   v_tree: torch.Tensor, node_stride: int, k_prefix: Optional[torch.Tensor],
                   v_prefix: Optional[torch.Tensor], seq_base_dev: torch.Tensor, prefix_lens_dev: torch.Tensor,
                   head_stride: int, max_prefix: int, softmax_scale: float, out: torch.Tensor,
                   workspace: Optional[torch.Tensor], stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mcsd_tree_attention(C.byref(view), dtype, B, H, d, _ptr(q), _ptr(k_tree), _ptr(v_tree), node_stride,
                                 _ptr(k_prefix), _ptr(v_prefix), _ptr(seq_base_dev), _ptr(prefix_lens_dev),
                                 head_stride, max_prefix, softmax_scale, _ptr(out), _ptr(workspace), ws_bytes,
                                 _stream(stream))
    _check(st, "mcsd_tree_attention")


def tree_attention_static(view: MaskView, dtype: int, B: int, H: int, d: int, q: torch.Tensor, k_tree: torch.Tensor,
                          v_tree: torch.Tensor, node_stride: int, k_prefix: Optional[torch.Tensor],
                          v_prefix: Optional[torch.Tensor], seq_base_dev: torch.Tensor, prefix_lens_dev: torch.Tensor,
                          head_stride: int, max_prefix: int, softmax_scale: float, out: torch.Tensor, stream=None) -> None:
    st = lib.mcsd_tree_attention_static(C.byref(view), dtype, B, H, d, _ptr(q), _ptr(k_tree), _ptr(v_tree), node_stride,
                                        _ptr(k_prefix), _ptr(v_prefix), _ptr(seq_base_dev), _ptr(prefix_lens_dev),
                                        head_stride, max_prefix, softmax_scale, _ptr(out), _stream(stream))
    _check(st, "mcsd_tree_attention_static")


def tree_attention_plan(tuning: Optional[AttentionTuning], dtype: int, prefix_fp8: int, B: int, H_q: int, H_kv: int,
                        d: int, n_nodes: int, row_begin: int, max_prefix: int) -> AttentionPlan:
    plan = AttentionPlan()
    _check(lib.mcsd_tree_attention_plan(_tuning_ref(tuning), dtype, prefix_fp8, B, H_q, H_kv, d, n_nodes, row_begin,
                                        max_prefix, C.byref(plan)), "mcsd_tree_attention_plan")
    return plan


def tree_attention_rows_workspace(B: int, H: int, d: int, n_nodes: int, row_begin: int, max_prefix: int) -> int:
    return int(lib.mcsd_tree_attention_rows_workspace(B, H, d, n_nodes, row_begin, max_prefix))


def tree_attention_rows(view: MaskView, dtype: int, B: int, H: int, d: int, row_begin: int, q: torch.Tensor,
                        k_tree: torch.Tensor, v_tree: torch.Tensor, node_stride: int,
                        k_prefix: Optional[torch.Tensor], v_prefix: Optional[torch.Tensor],
                        seq_base_dev: torch.Tensor, prefix_lens_dev: torch.Tensor, head_stride: int, max_prefix: int,
                        softmax_scale: float, out: torch.Tensor, workspace: Optional[torch.Tensor], stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mcsd_tree_attention_rows(C.byref(view), dtype, B, H, d, row_begin, _ptr(q), _ptr(k_tree), _ptr(v_tree),
                                      node_stride, _ptr(k_prefix), _ptr(v_prefix), _ptr(seq_base_dev),
                                      _ptr(prefix_lens_dev), head_stride, max_prefix, softmax_scale, _ptr(out),
                                      _ptr(workspace), ws_bytes, _stream(stream))
    _check(st, "mcsd_tree_attention_rows")


def tree_attention_gqa_workspace(B: int, H_q: int, H_kv: int, d: int, n_nodes: int, row_begin: int,
                                 max_prefix: int) -> int:
    return int(lib.mcsd_tree_attention_gqa_workspace(B, H_q, H_kv, d, n_nodes, row_begin, max_prefix))


def tree_attention_gqa(view: MaskView, dtype: int, B: int, H_q: int, H_kv: int, d: int, row_begin: int,
                       q: torch.Tensor, k_tree: torch.Tensor, v_tree: torch.Tensor, node_stride: int,
                       k_prefix: Optional[torch.Tensor], v_prefix: Optional[torch.Tensor], seq_base_dev: torch.Tensor,
                       prefix_lens_dev: torch.Tensor, head_stride: int, max_prefix: int, softmax_scale: float,
                       out: torch.Tensor, workspace: Optional[torch.Tensor], stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mcsd_tree_attention_gqa(C.byref(view), dtype, B, H_q, H_kv, d, row_begin, _ptr(q), _ptr(k_tree),
                                     _ptr(v_tree), node_stride, _ptr(k_prefix), _ptr(v_prefix), _ptr(seq_base_dev),
                                     _ptr(prefix_lens_dev), head_stride, max_prefix, softmax_scale, _ptr(out),
                                     _ptr(workspace), ws_bytes, _stream(stream))
    _check(st, "mcsd_tree_attention_gqa")


def tree_attention_fp8kv_workspace(B: int, H_q: int, H_kv: int, n_nodes: int, row_begin: int, max_prefix: int) -> int:
    return int(lib.mcsd_tree_attention_fp8kv_workspace(B, H_q, H_kv, n_nodes, row_begin, max_prefix))


def tree_attention_fp8kv(view: MaskView, B: int, H_q: int, H_kv: int, row_begin: int, q: torch.Tensor,
                         k_tree: torch.Tensor, v_tree: torch.Tensor, node_stride: int,
                         k_prefix_fp8: Optional[torch.Tensor], v_prefix_fp8: Optional[torch.Tensor], k_scale: float,
                         v_scale: float, seq_base_dev: torch.Tensor, prefix_lens_dev: torch.Tensor, head_stride: int,
                         max_prefix: int, softmax_scale: float, out: torch.Tensor, workspace: Optional[torch.Tensor],
                         stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mcsd_tree_attention_fp8kv(C.byref(view), B, H_q, H_kv, row_begin, _ptr(q), _ptr(k_tree), _ptr(v_tree),
                                       node_stride, _ptr(k_prefix_fp8), _ptr(v_prefix_fp8), k_scale, v_scale,
                                       _ptr(seq_base_dev), _ptr(prefix_lens_dev), head_stride, max_prefix,
                                       softmax_scale, _ptr(out), _ptr(workspace), ws_bytes, _stream(stream))
    _check(st, "mcsd_tree_attention_fp8kv")


def verify_tree_workspace(view: MaskView, mode: int, B: int, n_new: int) -> int:
    return int(lib.mcsd_verify_tree_workspace(C.byref(view), mode, B, n_new))


def verify_tree(view: MaskView, mode: int, B: int, V: int, tokens: torch.Tensor, p_target: torch.Tensor,
                q_draft: Optional[torch.Tensor], p_batch_stride: int, q_batch_stride: int, u_accept: torch.Tensor,
                u_sample: Optional[torch.Tensor], n_new: int, out_path: torch.Tensor, out_accept_len: torch.Tensor,
                out_new_tokens: Optional[torch.Tensor], workspace: Optional[torch.Tensor], stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mcsd_verify_tree(C.byref(view), mode, B, V, _ptr(tokens), _ptr(p_target), _ptr(q_draft), p_batch_stride,
                              q_batch_stride, _ptr(u_accept), _ptr(u_sample), n_new, _ptr(out_path),
                              _ptr(out_accept_len), _ptr(out_new_tokens), _ptr(workspace), ws_bytes, _stream(stream))
    _check(st, "mcsd_verify_tree")


def verify_tree_sampling(view: MaskView, mode: int, sampling: int, B: int, V: int, tokens: torch.Tensor,
                         p_target: torch.Tensor, q_draft: Optional[torch.Tensor], p_batch_stride: int,
                         q_batch_stride: int, u_accept: torch.Tensor, u_sample: Optional[torch.Tensor], n_new: int,
                         out_path: torch.Tensor, out_accept_len: torch.Tensor, out_new_tokens: Optional[torch.Tensor],
                         workspace: Optional[torch.Tensor], stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib.mcsd_verify_tree_sampling(C.byref(view), mode, sampling, B, V, _ptr(tokens), _ptr(p_target), _ptr(q_draft),
                                       p_batch_stride, q_batch_stride, _ptr(u_accept), _ptr(u_sample), n_new,
                                       _ptr(out_path), _ptr(out_accept_len), _ptr(out_new_tokens), _ptr(workspace),
                                       ws_bytes, _stream(stream))
    _check(st, "mcsd_verify_tree_sampling")


def _ptr_array(tensors: Sequence[torch.Tensor]):
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def commit_path(view: MaskView, dtype: int, B: int, H: int, d: int, k_tree: Sequence[torch.Tensor],
                v_tree: Sequence[torch.Tensor], node_stride: int, k_prefix: Sequence[torch.Tensor],
                v_prefix: Sequence[torch.Tensor], seq_base_dev: torch.Tensor, head_stride: int, max_prefix: int,
                capacity: int, out_path: torch.Tensor, accept_len: torch.Tensor, tokens: torch.Tensor,
                new_tokens: Optional[torch.Tensor], n_new: int, n_append: int, prefix_lens_dev: torch.Tensor,
                out_ids: torch.Tensor, out_n_ids: torch.Tensor, stream=None) -> None:
    """One call for all layers: k_tree / v_tree / k_prefix / v_prefix are per-layer lists of device tensors."""
    n_layers = len(k_tree)
    assert len(v_tree) == len(k_prefix) == len(v_prefix) == n_layers
    st = lib.mcsd_commit_path(C.byref(view), dtype, B, H, d, n_layers, _ptr_array(k_tree), _ptr_array(v_tree),
                              node_stride, _ptr_array(k_prefix), _ptr_array(v_prefix), _ptr(seq_base_dev), head_stride,
                              max_prefix, capacity, _ptr(out_path), _ptr(accept_len), _ptr(tokens), _ptr(new_tokens),
                              n_new, n_append, _ptr(prefix_lens_dev), _ptr(out_ids), _ptr(out_n_ids), _stream(stream))
    _check(st, "mcsd_commit_path")


def make_mlp(weights: Sequence[torch.Tensor], biases: Sequence[torch.Tensor]) -> Mlp:
    """mcsd_mlp_t for per-layer device tensors weight[l] fp32 [out_l][in_l], bias[l] fp32 [out_l]."""
    n = len(weights)
    if not (1 <= n <= MLP_MAX_LAYERS and len(biases) == n):
        raise McsdError(MCSD_EINVAL, "make_mlp")
    m = Mlp()
    m.n_layers = n
    m.width[0] = weights[0].shape[1]
    for l in range(n):
        m.width[l + 1] = weights[l].shape[0]
        m.weight[l] = weights[l].data_ptr()
        m.bias[l] = biases[l].data_ptr()
    m._keep = (list(weights), list(biases))       # the struct holds raw pointers
    return m


def early_stop_distribution(mlp: Mlp, B: int, W: int, V: int, k: int, draft_rows: torch.Tensor, batch_stride: int,
                            row_stride: int, beta: float, features: Optional[torch.Tensor], prob: torch.Tensor,
                            stop: torch.Tensor, stream=None) -> None:
    _check(lib.mcsd_early_stop_distribution(C.byref(mlp), B, W, V, k, _ptr(draft_rows), batch_stride, row_stride,
                                            beta, _ptr(features), _ptr(prob), _ptr(stop), _stream(stream)),
           "mcsd_early_stop_distribution")


def early_stop_hidden(mlp: Mlp, B: int, W: int, hidden: torch.Tensor, batch_stride: int, row_stride: int,
                      beta: float, prob: torch.Tensor, stop: torch.Tensor, stream=None) -> None:
    _check(lib.mcsd_early_stop_hidden(C.byref(mlp), B, W, _ptr(hidden), batch_stride, row_stride, beta, _ptr(prob),
                                      _ptr(stop), _stream(stream)), "mcsd_early_stop_hidden")


def stream_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int = 0, stream=None) -> None:
    _check(lib.mcsd_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), workgroups, _stream(stream)),
           "mcsd_stream_read")


def placement_probe(workgroups: int, spin: int, out: torch.Tensor, stream=None) -> None:
    _check(lib.mcsd_placement_probe(workgroups, spin, _ptr(out), _stream(stream)), "mcsd_placement_probe")


def issue_probe(schedule: int, workgroups: int, iterations: int, out: torch.Tensor, stream=None) -> None:
    _check(lib.mcsd_issue_probe(schedule, workgroups, iterations, _ptr(out), _stream(stream)), "mcsd_issue_probe")


def mask_bits_host(view: MaskView):
    """The slice as a dense uint8 [n][n] numpy array, unpacked from the handle's host copy (for checks)."""
    import numpy as np
    n, W = view.n_nodes, view.words_per_row
    words = np.ctypeslib.as_array(view.bits_host, shape=(view.n_nodes_max * W,)).reshape(view.n_nodes_max, W)
    out = np.zeros((n, n), dtype=np.uint8)
    for j in range(n):
        out[:, j] = (words[:n, j >> 6] >> np.uint64(j & 63)) & np.uint64(1)
    return out


def profile_next(kernel: int, start_event: Optional[int], stop_event: Optional[int]) -> None:
    _check(lib.mcsd_profile_next(kernel, start_event, stop_event), "mcsd_profile_next")


class HipRuntime:
    """The process's HIP runtime (the one PyTorch loaded), for raw events and copies in tests and benchmarks."""

    def __init__(self):
        path = None
        with open("/proc/self/maps") as f:
            for line in f:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        if path is None:
            raise RuntimeError("no HIP runtime is loaded in this process")
        self.lib = C.CDLL(path)
        self.lib.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.lib.hipEventDestroy.argtypes = [C.c_void_p]
        self.lib.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.lib.hipEventSynchronize.argtypes = [C.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.lib.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]

    def _ok(self, err: int, what: str) -> None:
        if err != 0:
            raise RuntimeError(f"{what} failed with HIP error {err}")

    def event(self) -> int:
        ev = C.c_void_p()
        self._ok(self.lib.hipEventCreate(C.byref(ev)), "hipEventCreate")
        return ev.value

    def destroy(self, ev: int) -> None:
        self.lib.hipEventDestroy(ev)

    def record(self, ev: int, stream=None) -> None:
        self._ok(self.lib.hipEventRecord(ev, _stream(stream)), "hipEventRecord")

    def elapsed_ms(self, start: int, stop: int) -> float:
        self._ok(self.lib.hipEventSynchronize(stop), "hipEventSynchronize")
        ms = C.c_float()
        self._ok(self.lib.hipEventElapsedTime(C.byref(ms), start, stop), "hipEventElapsedTime")
        return float(ms.value)

    def memcpy_dtoh(self, host_ptr: int, dev_ptr: int, nbytes: int) -> None:
        self._ok(self.lib.hipMemcpy(host_ptr, dev_ptr, nbytes, 2), "hipMemcpy")
