"""ctypes binding of libstructkv.so: same names as the C entry points, marshalling only.

Tensors are torch tensors (device memory + streams are PyTorch's job); every step of the path
runs inside the library's HIP kernels.  cu_seqlens / k_per_seq / rows_per_seq are host sequences.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstructkv.so")

STRUCTKV_OK = 0
STRUCTKV_ERR_INVALID_ARG = 1
STRUCTKV_ERR_UNSUPPORTED = 2
STRUCTKV_ERR_WORKSPACE = 3
STRUCTKV_ERR_HIP = 4
STRUCTKV_DTYPE_F32 = 0
STRUCTKV_DTYPE_BF16 = 1
STRUCTKV_MAX_BATCH = 64
STRUCTKV_STATIC_TOPK_MAX_TOKENS = 1048576

EXPORTS = (
    "structkv_last_error", "structkv_version", "structkv_workspace_bytes", "structkv_score_layer",
    "structkv_accumulate_centrality", "structkv_score_layer_accumulate", "structkv_score_layer_groups",
    "structkv_select_topk", "structkv_select_topk_static",
    "structkv_gather_kv", "structkv_layer_step", "structkv_layer_step_workspace_bytes", "structkv_layer_begin",
    "structkv_layer_finish",
    "structkv_truncate_hidden", "structkv_block_scores",
    "structkv_pivot_workspace_bytes", "structkv_pivot_metrics", "structkv_score_layer_pivot", "structkv_transition_scores",
    "structkv_debug_probs", "structkv_debug_score_steps",
)


class structkv_shape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("window", ctypes.c_int32), ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class StructKVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("structkv status %d: %s" % (status, message))
        self.status = status


if not os.path.exists(LIB_PATH):
    raise ImportError("libstructkv.so is not built: run `python -m paper_2604_06746_amd.build` "
                      "(hipcc, --offload-arch=gfx950).  There is no fallback path.")
_lib = ctypes.CDLL(LIB_PATH)

_vp, _i32, _i64, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
_sp = ctypes.POINTER(structkv_shape)
_lib.structkv_last_error.restype = ctypes.c_char_p
_lib.structkv_last_error.argtypes = []
_lib.structkv_version.restype = _i32
_lib.structkv_workspace_bytes.restype = _sz
_lib.structkv_workspace_bytes.argtypes = [_sp, _i32, _i64]
_lib.structkv_score_layer.restype = _i32
_lib.structkv_score_layer.argtypes = [_sp, _vp, _vp, _i64, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.structkv_debug_score_steps.restype = _i32
_lib.structkv_debug_score_steps.argtypes = _lib.structkv_score_layer.argtypes + [_i32, _i32]
_lib.structkv_accumulate_centrality.restype = _i32
_lib.structkv_accumulate_centrality.argtypes = [_vp, _vp, _i64, _f32, _f32, _vp]
_lib.structkv_score_layer_accumulate.restype = _i32
_lib.structkv_score_layer_accumulate.argtypes = [_sp, _vp, _vp, _i64, _i64, _i32, _vp, _vp, _vp, _f32, _f32, _vp,
                                                 _vp, _vp, _sz, _vp]
_lib.structkv_score_layer_groups.restype = _i32
_lib.structkv_score_layer_groups.argtypes = [_sp, _vp, _vp, _i64, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.structkv_select_topk.restype = _i32
_lib.structkv_select_topk.argtypes = [_vp, _i32, _vp, _vp, _i32, _vp, _vp, _sz, _vp]
_lib.structkv_select_topk_static.restype = _i32
_lib.structkv_select_topk_static.argtypes = [_vp, _i32, _vp, _vp, _i32, _vp, _vp]
_lib.structkv_gather_kv.restype = _i32
_lib.structkv_gather_kv.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp, _i64, _i64, _i32, _i32, _i32, _i32, _vp,
                                    _vp, _vp, _vp]
_lib.structkv_layer_step_workspace_bytes.restype = _sz
_lib.structkv_layer_step_workspace_bytes.argtypes = [_sp, _i32, _i64]
_lib.structkv_layer_step.restype = _i32
_lib.structkv_layer_step.argtypes = [_sp, _vp, _vp, _vp, _i64, _i64, _i32, _vp, _vp, _i32, _vp, _vp, _f32, _f32, _vp,
                                     _vp, _vp, _vp, _vp, _i64, _i64, _vp, _sz, _vp]
_lib.structkv_layer_begin.restype = _i32
_lib.structkv_layer_begin.argtypes = _lib.structkv_layer_step.argtypes
_lib.structkv_layer_finish.restype = _i32
_lib.structkv_layer_finish.argtypes = [_sp, _vp, _vp, _i64, _i64, _i32, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _i64, _i64,
                                       _vp, _sz, _vp]
_lib.structkv_truncate_hidden.restype = _i32
_lib.structkv_truncate_hidden.argtypes = [_vp, _i64, _vp, _i64, _i32, _i32, _vp, _vp, _i32, _vp, _vp, _vp, _vp]
_lib.structkv_block_scores.restype = _i32
_lib.structkv_block_scores.argtypes = [_vp, _i32, _vp, _i32, _vp, _vp]
_lib.structkv_pivot_workspace_bytes.restype = _sz
_lib.structkv_pivot_workspace_bytes.argtypes = [_sp, _i64]
_lib.structkv_score_layer_pivot.restype = _i32
_lib.structkv_score_layer_pivot.argtypes = [_sp, _vp, _vp, _i64, _i64, _i32, _vp, ctypes.c_double, _vp, _vp, _vp, _vp,
                                            _vp, _vp, _sz, _vp]
_lib.structkv_pivot_metrics.restype = _i32
_lib.structkv_pivot_metrics.argtypes = [_sp, _vp, _vp, _i64, _i64, _i32, _vp, ctypes.c_double, _vp, _vp, _vp, _sz,
                                        _vp]
_lib.structkv_transition_scores.restype = _i32
_lib.structkv_transition_scores.argtypes = [_vp, _vp, _vp, _i32, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                            _vp, _vp]
_lib.structkv_debug_probs.restype = _i32
_lib.structkv_debug_probs.argtypes = [_sp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _sz, _vp, _i32]


def make_shape(n_q_heads: int, n_kv_heads: int, head_dim: int, window: int, dtype: int,
               causal: bool = False, scale: float = 0.0) -> structkv_shape:
    return structkv_shape(n_q_heads, n_kv_heads, head_dim, window, dtype, int(bool(causal)), float(scale))


def _host_i64(values: Sequence[int]):
    return (ctypes.c_int64 * len(values))(*[int(v) for v in values])


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int) -> None:
    if status != STRUCTKV_OK:
        raise StructKVError(status, _lib.structkv_last_error().decode())


def structkv_last_error() -> str:
    return _lib.structkv_last_error().decode()


def structkv_version() -> int:
    return int(_lib.structkv_version())


def structkv_workspace_bytes(shape: Optional[structkv_shape], batch: int, total_tokens: int) -> int:
    return int(_lib.structkv_workspace_bytes(ctypes.byref(shape) if shape is not None else None, batch,
                                             total_tokens))


def structkv_score_layer(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor,
                         cu_seqlens: Sequence[int], indeg_out: torch.Tensor, entropy_out: torch.Tensor,
                         entropy_per_head_out: Optional[torch.Tensor], workspace: torch.Tensor,
                         stream=None) -> None:
    """k: [G, total, d] view with d contiguous (head/token strides are passed through)."""
    assert k.dim() == 3 and k.stride(2) == 1 and q_win.is_contiguous()
    cu = _host_i64(cu_seqlens)
    _check(_lib.structkv_score_layer(ctypes.byref(shape), _ptr(q_win), _ptr(k), k.stride(0), k.stride(1),
                                     len(cu_seqlens) - 1, cu, _ptr(indeg_out), _ptr(entropy_out),
                                     _ptr(entropy_per_head_out), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)))


def structkv_debug_score_steps(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor,
                               cu_seqlens: Sequence[int], indeg_out: torch.Tensor, entropy_out: torch.Tensor,
                               entropy_per_head_out: Optional[torch.Tensor], workspace: torch.Tensor,
                               step_mask: int, stream=None, force_simt: bool = False) -> None:
    cu = _host_i64(cu_seqlens)
    _check(_lib.structkv_debug_score_steps(ctypes.byref(shape), _ptr(q_win), _ptr(k), k.stride(0), k.stride(1),
                                           len(cu_seqlens) - 1, cu, _ptr(indeg_out), _ptr(entropy_out),
                                           _ptr(entropy_per_head_out), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream(stream),
                                           step_mask, int(bool(force_simt))))


def structkv_accumulate_centrality(centrality: torch.Tensor, indeg: torch.Tensor, lam: float, inv_w: float,
                                   stream=None) -> None:
    assert centrality.numel() == indeg.numel()
    _check(_lib.structkv_accumulate_centrality(_ptr(centrality), _ptr(indeg), centrality.numel(), lam, inv_w,
                                               _stream(stream)))


def structkv_score_layer_accumulate(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor,
                                    cu_seqlens: Sequence[int], indeg_out: torch.Tensor, centrality: torch.Tensor,
                                    lam: float, inv_w: float, entropy_out: torch.Tensor,
                                    entropy_per_head_out: Optional[torch.Tensor], workspace: torch.Tensor,
                                    stream=None) -> None:
    assert k.dim() == 3 and k.stride(2) == 1 and q_win.is_contiguous()
    assert centrality.numel() == indeg_out.numel()
    cu = _host_i64(cu_seqlens)
    _check(_lib.structkv_score_layer_accumulate(ctypes.byref(shape), _ptr(q_win), _ptr(k), k.stride(0), k.stride(1),
                                                len(cu_seqlens) - 1, cu, _ptr(indeg_out), _ptr(centrality), lam,
                                                inv_w, _ptr(entropy_out), _ptr(entropy_per_head_out),
                                                _ptr(workspace), workspace.numel() * workspace.element_size(),
                                                _stream(stream)))


def structkv_score_layer_groups(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor,
                                cu_seqlens: Sequence[int], indeg_out: torch.Tensor, indeg_groups_out: torch.Tensor,
                                entropy_out: torch.Tensor, entropy_per_head_out: Optional[torch.Tensor],
                                workspace: torch.Tensor, stream=None) -> None:
    """indeg_groups_out: [G, total] fp32, contiguous."""
    assert k.dim() == 3 and k.stride(2) == 1 and q_win.is_contiguous() and indeg_groups_out.is_contiguous()
    cu = _host_i64(cu_seqlens)
    _check(_lib.structkv_score_layer_groups(ctypes.byref(shape), _ptr(q_win), _ptr(k), k.stride(0), k.stride(1),
                                            len(cu_seqlens) - 1, cu, _ptr(indeg_out), _ptr(indeg_groups_out),
                                            _ptr(entropy_out), _ptr(entropy_per_head_out), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream)))


def structkv_select_topk(scores: torch.Tensor, cu_seqlens: Sequence[int], k_per_seq: Sequence[int],
                         keep_tail: int, idx_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    cu, ks = _host_i64(cu_seqlens), _host_i64(k_per_seq)
    _check(_lib.structkv_select_topk(_ptr(scores), len(k_per_seq), cu, ks, keep_tail, _ptr(idx_out),
                                     _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)))


def structkv_select_topk_static(scores: torch.Tensor, cu_seqlens: Sequence[int], k_per_seq: Sequence[int],
                                keep_tail: int, idx_out: torch.Tensor, stream=None) -> None:
    cu, ks = _host_i64(cu_seqlens), _host_i64(k_per_seq)
    _check(_lib.structkv_select_topk_static(_ptr(scores), len(k_per_seq), cu, ks, keep_tail, _ptr(idx_out),
                                            _stream(stream)))


def structkv_gather_kv(k_src: Optional[torch.Tensor], v_src: Optional[torch.Tensor],
                       k_dst: Optional[torch.Tensor], v_dst: Optional[torch.Tensor],
                       cu_seqlens: Sequence[int], rows_per_seq: Sequence[int], idx: torch.Tensor,
                       stream=None) -> None:
    """src/dst: [G, tokens, d] views with d contiguous; K and V must share strides."""
    src = k_src if k_src is not None else v_src
    dst = k_dst if k_dst is not None else v_dst
    if v_src is not None and k_src is not None:
        assert v_src.stride() == k_src.stride() and v_dst.stride() == k_dst.stride()
    cu, rows = _host_i64(cu_seqlens), _host_i64(rows_per_seq)
    _check(_lib.structkv_gather_kv(_ptr(k_src), _ptr(v_src), src.stride(0), src.stride(1), _ptr(k_dst),
                                   _ptr(v_dst), dst.stride(0), dst.stride(1), src.shape[0], src.shape[2],
                                   src.element_size(), len(rows_per_seq), cu, rows, _ptr(idx),
                                   _stream(stream)))


def structkv_layer_step_workspace_bytes(shape: structkv_shape, batch: int, total_tokens: int) -> int:
    return int(_lib.structkv_layer_step_workspace_bytes(ctypes.byref(shape), batch, total_tokens))


def structkv_layer_step(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor, v: Optional[torch.Tensor],
                        cu_seqlens: Sequence[int], k_per_seq: Sequence[int], keep_tail: int,
                        indeg_out: torch.Tensor, centrality: Optional[torch.Tensor], lam: float, inv_w: float,
                        entropy_out: torch.Tensor, entropy_per_head_out: Optional[torch.Tensor],
                        idx_out: torch.Tensor, k_dst: Optional[torch.Tensor], v_dst: Optional[torch.Tensor],
                        workspace: torch.Tensor, stream=None, _entry=None) -> None:
    """k, v: [G, total, d] views sharing strides; k_dst, v_dst: [G, rows, d] views sharing strides (or None)."""
    fn = _entry or _lib.structkv_layer_step
    assert k.dim() == 3 and k.stride(2) == 1 and q_win.is_contiguous()
    if v is not None:
        assert v.stride() == k.stride() and v.dtype == k.dtype
    dst = k_dst if k_dst is not None else v_dst
    if k_dst is not None and v_dst is not None:
        assert k_dst.stride() == v_dst.stride()
    cu, ks = _host_i64(cu_seqlens), _host_i64(k_per_seq)
    _check(fn(ctypes.byref(shape), _ptr(q_win), _ptr(k), _ptr(v), k.stride(0), k.stride(1),
              len(k_per_seq), cu, ks, keep_tail, _ptr(indeg_out), _ptr(centrality), lam, inv_w,
              _ptr(entropy_out), _ptr(entropy_per_head_out), _ptr(idx_out), _ptr(k_dst),
              _ptr(v_dst), dst.stride(0) if dst is not None else 0,
              dst.stride(1) if dst is not None else 0, _ptr(workspace),
              workspace.numel() * workspace.element_size(), _stream(stream)))


def structkv_layer_begin(*args, **kwargs) -> None:
    """Same arguments as structkv_layer_step; enqueues its first half."""
    structkv_layer_step(*args, _entry=_lib.structkv_layer_begin, **kwargs)


def structkv_layer_finish(shape: structkv_shape, k: torch.Tensor, v: Optional[torch.Tensor],
                          cu_seqlens: Sequence[int], k_per_seq: Sequence[int], keep_tail: int, indeg: torch.Tensor,
                          idx_out: torch.Tensor, k_dst: Optional[torch.Tensor], v_dst: Optional[torch.Tensor],
                          workspace: torch.Tensor, stream=None) -> None:
    dst = k_dst if k_dst is not None else v_dst
    cu, ks = _host_i64(cu_seqlens), _host_i64(k_per_seq)
    _check(_lib.structkv_layer_finish(ctypes.byref(shape), _ptr(k), _ptr(v), k.stride(0), k.stride(1), len(k_per_seq),
                                      cu, ks, keep_tail, _ptr(indeg), _ptr(idx_out), _ptr(k_dst), _ptr(v_dst),
                                      dst.stride(0) if dst is not None else 0,
                                      dst.stride(1) if dst is not None else 0, _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream(stream)))


def structkv_truncate_hidden(h_src: Optional[torch.Tensor], h_dst: Optional[torch.Tensor],
                             pos_src: Optional[torch.Tensor], pos_dst: Optional[torch.Tensor],
                             cu_seqlens: Sequence[int], rows_per_seq: Sequence[int], idx: torch.Tensor,
                             stream=None) -> None:
    """h_src [total, hidden], h_dst [rows, hidden] (last dim contiguous); pos_* int64 vectors or None."""
    hidden = elem = ss = ds = 0
    if h_src is not None:
        assert h_src.dim() == 2 and h_src.stride(1) == 1 and h_dst.stride(1) == 1 and h_dst.dtype == h_src.dtype
        hidden, elem, ss, ds = h_src.shape[1], h_src.element_size(), h_src.stride(0), h_dst.stride(0)
    for p in (pos_src, pos_dst):
        assert p is None or (p.dtype == torch.int64 and p.is_contiguous())
    cu, rows = _host_i64(cu_seqlens), _host_i64(rows_per_seq)
    _check(_lib.structkv_truncate_hidden(_ptr(h_src), ss, _ptr(h_dst), ds, hidden, elem, _ptr(pos_src),
                                         _ptr(pos_dst), len(rows_per_seq), cu, rows, _ptr(idx), _stream(stream)))


def structkv_block_scores(scores: torch.Tensor, cu_seqlens: Sequence[int], block_size: int,
                          block_scores_out: torch.Tensor, stream=None) -> None:
    cu = _host_i64(cu_seqlens)
    _check(_lib.structkv_block_scores(_ptr(scores), len(cu_seqlens) - 1, cu, block_size, _ptr(block_scores_out),
                                      _stream(stream)))


def structkv_pivot_workspace_bytes(shape: structkv_shape, max_seq_len: int) -> int:
    return int(_lib.structkv_pivot_workspace_bytes(ctypes.byref(shape), int(max_seq_len)))


def structkv_pivot_metrics(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor, cu_seqlens: Sequence[int],
                           top_frac: float, sparsity_out: torch.Tensor, variance_out: torch.Tensor,
                           workspace: torch.Tensor, stream=None) -> None:
    assert k.dim() == 3 and k.stride(2) == 1 and q_win.is_contiguous()
    cu = _host_i64(cu_seqlens)
    _check(_lib.structkv_pivot_metrics(ctypes.byref(shape), _ptr(q_win), _ptr(k), k.stride(0), k.stride(1),
                                       len(cu_seqlens) - 1, cu, top_frac, _ptr(sparsity_out), _ptr(variance_out),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       _stream(stream)))


def structkv_score_layer_pivot(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor,
                               cu_seqlens: Sequence[int], top_frac: float, indeg_out: torch.Tensor,
                               entropy_out: torch.Tensor, entropy_per_head_out: Optional[torch.Tensor],
                               sparsity_out: torch.Tensor, variance_out: torch.Tensor, workspace: torch.Tensor,
                               stream=None) -> None:
    assert k.dim() == 3 and k.stride(2) == 1 and q_win.is_contiguous()
    cu = _host_i64(cu_seqlens)
    _check(_lib.structkv_score_layer_pivot(ctypes.byref(shape), _ptr(q_win), _ptr(k), k.stride(0), k.stride(1),
                                           len(cu_seqlens) - 1, cu, top_frac, _ptr(indeg_out), _ptr(entropy_out),
                                           _ptr(entropy_per_head_out), _ptr(sparsity_out), _ptr(variance_out),
                                           _ptr(workspace), workspace.numel() * workspace.element_size(),
                                           _stream(stream)))


def structkv_transition_scores(entropy: Sequence[float], sparsity: Sequence[float], variance: Sequence[float],
                               weights: Sequence[float] = (0.2, 0.3, 0.5)):
    """Host arithmetic (Eq. 7-9): returns (list of T_l, pivot layer L*)."""
    n = len(entropy)
    assert len(sparsity) == n and len(variance) == n
    arr = ctypes.c_double * max(n, 1)
    H, R, V, T = arr(*entropy), arr(*sparsity), arr(*variance), arr()
    ls = ctypes.c_int32(0)
    _check(_lib.structkv_transition_scores(H, R, V, n, weights[0], weights[1], weights[2], T, ctypes.byref(ls)))
    return list(T)[:n], int(ls.value)


def structkv_debug_probs(shape: structkv_shape, q_win: torch.Tensor, k: torch.Tensor, n: int,
                         probs_out: torch.Tensor, workspace: torch.Tensor, stream=None,
                         force_simt: bool = False) -> None:
    _check(_lib.structkv_debug_probs(ctypes.byref(shape), _ptr(q_win), _ptr(k), k.stride(0), k.stride(1), n,
                                     _ptr(probs_out), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream),
                                     int(bool(force_simt))))
