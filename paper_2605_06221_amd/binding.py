"""ctypes binding of libuniprefill.so: argument marshalling only.

Every function has the name and argument order of its C entry point
(include/uniprefill.h).  Tensors are torch tensors on the GPU (device pointers)
or numpy arrays (host pointers); nothing is computed here and there is no
fallback: if the library is missing the import fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libuniprefill.so")

UP_OK, UP_ERR_NULL, UP_ERR_SHAPE, UP_ERR_RANGE, UP_ERR_UNSUPPORTED, UP_ERR_ALIGN, UP_ERR_WORKSPACE, UP_ERR_HIP, UP_ERR_SCRATCH = range(9)
STATIC_SCRATCH_BYTES = 32 << 20
UP_BF16, UP_F32 = 0, 1

EXPORTS = ["uniprefill_plan", "uniprefill_score", "uniprefill_select", "uniprefill_compact",
           "uniprefill_scatter", "uniprefill_fused", "uniprefill_fused_phases", "uniprefill_select_top_p",
           "uniprefill_compact_counted", "uniprefill_fused_top_p", "uniprefill_compose_index",
           "uniprefill_slot_mapping", "uniprefill_plan_chunked", "uniprefill_score_chunked",
           "uniprefill_select_chunked", "uniprefill_fused_chunked", "uniprefill_compact_column", "uniprefill_seqused",
           "uniprefill_score_paged", "uniprefill_fused_paged", "uniprefill_select_top_p_chunked",
           "uniprefill_fused_top_p_chunked", "uniprefill_keep_mask", "uniprefill_fused_lse",
           "uniprefill_score_lse", "uniprefill_fused_top_p_lse", "uniprefill_score_partial",
           "uniprefill_scores_from_partials", "uniprefill_fused_static",
           "uniprefill_status_string"]

UP_PHASE_PLAN, UP_PHASE_ROW_STATS, UP_PHASE_MERGE_STATS, UP_PHASE_SWEEP_SELECT, UP_PHASE_GATHER = 1, 2, 4, 8, 16
UP_PHASE_ALL = 31
UP_PHASE_GATHER_IN_SELECT = 32


class up_params(ctypes.Structure):
    _fields_ = [
        ("num_seqs", ctypes.c_int32), ("total_tokens", ctypes.c_int32),
        ("block_size", ctypes.c_int32), ("n_obs", ctypes.c_int32), ("n_sink", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("hidden_dim", ctypes.c_int32),
        ("q_row_stride", ctypes.c_int64), ("k_row_stride", ctypes.c_int64),
        ("hidden_row_stride", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float),
        ("qk_dtype", ctypes.c_int32), ("hidden_dtype", ctypes.c_int32),
    ]


class UniPrefillError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    P = ctypes.POINTER(up_params)
    i64, i32, sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    ws = [vp, sz]                                   # workspace, workspace_bytes
    keys = [i32p, i32p]                             # cu_seqlens_k_dev, cu_seqlens_k_host
    table = [i32p, i64, i32]                        # block_table, block_table_stride, kv_block_size
    outs = [vp, i32p, i32p, i32p, f32p]             # hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores
    lib.uniprefill_plan.argtypes = [P, i32p, f32p, i32p, ctypes.POINTER(i64), ctypes.POINTER(sz)]
    lib.uniprefill_plan_chunked.argtypes = [P, i32p, i32p, f32p, i32p, ctypes.POINTER(i64), ctypes.POINTER(sz)]
    lib.uniprefill_score.argtypes = [P, vp, vp, i32p, i32p, f32p] + ws + [vp]
    lib.uniprefill_score_chunked.argtypes = [P, vp, vp, i32p, i32p] + keys + [f32p] + ws + [vp]
    lib.uniprefill_score_paged.argtypes = [P, vp, vp, i32p, i32p] + keys + table + [f32p] + ws + [vp]
    lib.uniprefill_score_lse.argtypes = [P, vp, vp, f32p, i64, i32p, i32p] + keys + table + [f32p] + ws + [vp]
    lib.uniprefill_score_partial.argtypes = [P, vp, vp, i32p, i32p] + keys + [vp] + ws + [vp]
    lib.uniprefill_scores_from_partials.argtypes = [vp, i32, i64, i32p, i32, i32, i32, i32, f32p, vp]
    lib.uniprefill_select.argtypes = [P, f32p, i32p, i32p, f32p, f32p, i32p, i32p, vp]
    lib.uniprefill_select_chunked.argtypes = [P, f32p, i32p, i32p] + keys + [f32p, f32p, i32p, i32p, vp]
    lib.uniprefill_select_top_p.argtypes = [P, f32p, i32p, i32p, f32p, f32p, i32p, i32p] + ws + [vp]
    lib.uniprefill_select_top_p_chunked.argtypes = [P, f32p, i32p, i32p] + keys + [f32p, f32p, i32p, i32p] + ws + [vp]
    lib.uniprefill_compact.argtypes = [P, vp, i32p, i32p, i64, vp, i32p, vp]
    lib.uniprefill_compact_counted.argtypes = [P, vp, i32p, i32p, i32p, i64, vp, i32p, vp]
    lib.uniprefill_compact_column.argtypes = [vp, i32, i32p, i64, i32p, vp, vp]
    lib.uniprefill_scatter.argtypes = [P, vp, i32p, i64, vp, vp]
    fused_in = [P, vp, vp, vp, i32p, i32p, i32p]    # params, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host
    lib.uniprefill_fused.argtypes = fused_in + [f32p, f32p] + outs + ws + [vp]
    lib.uniprefill_fused_static.argtypes = fused_in + [f32p, f32p] + outs + [vp]
    lib.uniprefill_fused_phases.argtypes = fused_in + [f32p, f32p] + outs + ws + [ctypes.c_int, vp]
    lib.uniprefill_fused_chunked.argtypes = fused_in + keys + [f32p, f32p] + outs + ws + [vp]
    lib.uniprefill_fused_paged.argtypes = fused_in + keys + table + [f32p, f32p] + outs + ws + [vp]
    lib.uniprefill_fused_top_p.argtypes = fused_in + [f32p, f32p] + outs + ws + [vp]
    lib.uniprefill_fused_top_p_chunked.argtypes = fused_in + keys + table + [f32p, f32p] + outs + ws + [vp]
    lse_in = [P, vp, vp, f32p, i64, vp, i32p, i32p, i32p]   # params, q, k, lse, lse_row_stride, hidden, pos, cu dev/host
    lib.uniprefill_fused_lse.argtypes = lse_in + keys + table + [f32p, f32p] + outs + ws + [vp]
    lib.uniprefill_fused_top_p_lse.argtypes = lse_in + keys + table + [f32p, f32p] + outs + ws + [vp]
    lib.uniprefill_compose_index.argtypes = [i32p, i64, i32p, i32p, i64, i32p, vp]
    lib.uniprefill_slot_mapping.argtypes = [i32p, i32p, i32, i32p, i64, i32, i64, vp, vp]
    lib.uniprefill_keep_mask.argtypes = [i32p, i64, i32p, i64, vp, vp]
    lib.uniprefill_seqused.argtypes = [i32p, i32, i32p, i32p, i32p, i32, i32, i32p, vp]
    for name in EXPORTS[:-1]:
        getattr(lib, name).restype = ctypes.c_int
    lib.uniprefill_status_string.argtypes = [ctypes.c_int]
    lib.uniprefill_status_string.restype = ctypes.c_char_p
    return lib


_lib = _load()


def lib():
    """The loaded ctypes library (for tests that poke the raw C ABI)."""
    return _lib


def status_string(status: int) -> str:
    return _lib.uniprefill_status_string(int(status)).decode()


def ptr(x):
    """Address of a torch tensor / numpy array / int / None as a void*."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    if isinstance(x, np.ndarray):
        return ctypes.c_void_p(x.ctypes.data)
    return ctypes.c_void_p(x.data_ptr())      # torch tensor


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, where: str, check: bool):
    if check and status != UP_OK:
        raise UniPrefillError(status, where)
    return status


def make_params(*, num_seqs, total_tokens, block_size, n_obs=128, n_sink=128, num_q_heads=0,
                num_kv_heads=0, head_dim=128, hidden_dim=0, q_row_stride=None, k_row_stride=None,
                hidden_row_stride=None, softmax_scale=0.0, qk_dtype=UP_BF16, hidden_dtype=UP_BF16) -> up_params:
    return up_params(
        num_seqs, total_tokens, block_size, n_obs, n_sink, num_q_heads, num_kv_heads, head_dim, hidden_dim,
        num_q_heads * head_dim if q_row_stride is None else q_row_stride,
        num_kv_heads * head_dim if k_row_stride is None else k_row_stride,
        hidden_dim if hidden_row_stride is None else hidden_row_stride,
        softmax_scale, qk_dtype, hidden_dtype)


def uniprefill_plan(p: up_params, cu_seqlens_host: np.ndarray, keep_ratio_host: np.ndarray, *,
                    want_workspace: bool = True, check: bool = True):
    """Returns (status, new_cu_seqlens_host, total_kept, workspace_bytes)."""
    new_cu = np.zeros(p.num_seqs + 1, dtype=np.int32)
    total = ctypes.c_int64(0)
    ws = ctypes.c_size_t(0)
    st = _lib.uniprefill_plan(ctypes.byref(p), ptr(cu_seqlens_host), ptr(keep_ratio_host), ptr(new_cu),
                              ctypes.byref(total), ctypes.byref(ws) if want_workspace else None)
    _check(st, "uniprefill_plan", check)
    return st, new_cu, int(total.value), int(ws.value)


def uniprefill_score(p, q, k, cu_seqlens_dev, cu_seqlens_host, scores_out, workspace, workspace_bytes,
                     stream=None, check=True):
    st = _lib.uniprefill_score(ctypes.byref(p), ptr(q), ptr(k), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                               ptr(scores_out), ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_score", check)


def uniprefill_select(p, scores, cu_seqlens_dev, cu_seqlens_host, keep_ratio_dev, keep_ratio_host,
                      kept_idx, new_cu_seqlens_dev, stream=None, check=True):
    st = _lib.uniprefill_select(ctypes.byref(p), ptr(scores), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                                ptr(keep_ratio_dev), ptr(keep_ratio_host), ptr(kept_idx),
                                ptr(new_cu_seqlens_dev), _stream(stream))
    return _check(st, "uniprefill_select", check)


def uniprefill_compact(p, hidden, pos, kept_idx, total_kept, hidden_out, pos_out, stream=None, check=True):
    st = _lib.uniprefill_compact(ctypes.byref(p), ptr(hidden), ptr(pos), ptr(kept_idx), int(total_kept),
                                 ptr(hidden_out), ptr(pos_out), _stream(stream))
    return _check(st, "uniprefill_compact", check)


def uniprefill_scatter(p, hidden_compact, kept_idx, total_kept, hidden_full_inout, stream=None, check=True):
    st = _lib.uniprefill_scatter(ctypes.byref(p), ptr(hidden_compact), ptr(kept_idx), int(total_kept),
                                 ptr(hidden_full_inout), _stream(stream))
    return _check(st, "uniprefill_scatter", check)


def uniprefill_fused(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, keep_ratio_dev, keep_ratio_host,
                     hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, workspace,
                     workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_fused(ctypes.byref(p), ptr(q), ptr(k), ptr(hidden), ptr(pos), ptr(cu_seqlens_dev),
                               ptr(cu_seqlens_host), ptr(keep_ratio_dev), ptr(keep_ratio_host),
                               ptr(hidden_out), ptr(pos_out), ptr(kept_idx), ptr(new_cu_seqlens_dev),
                               ptr(scores_out), ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_fused", check)


def uniprefill_fused_static(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, keep_ratio_dev, keep_ratio_host,
                            hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, stream=None, check=True):
    st = _lib.uniprefill_fused_static(ctypes.byref(p), ptr(q), ptr(k), ptr(hidden), ptr(pos), ptr(cu_seqlens_dev),
                                      ptr(cu_seqlens_host), ptr(keep_ratio_dev), ptr(keep_ratio_host),
                                      ptr(hidden_out), ptr(pos_out), ptr(kept_idx), ptr(new_cu_seqlens_dev),
                                      ptr(scores_out), _stream(stream))
    return _check(st, "uniprefill_fused_static", check)


def uniprefill_compact_column(column, elem_bytes, kept_idx, capacity, total_kept_dev, column_out, stream=None,
                              check=True):
    st = _lib.uniprefill_compact_column(ptr(column), int(elem_bytes), ptr(kept_idx), ctypes.c_int64(capacity),
                                        ptr(total_kept_dev), ptr(column_out), _stream(stream))
    return _check(st, "uniprefill_compact_column", check)


def uniprefill_fused_lse(p, q, k, lse, lse_row_stride, hidden, pos, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev,
                         cu_seqlens_k_host, block_table, block_table_stride, kv_block_size, keep_ratio_dev,
                         keep_ratio_host, hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, workspace,
                         workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_fused_lse(ctypes.byref(p), ptr(q), ptr(k), ptr(lse), ctypes.c_int64(lse_row_stride), ptr(hidden),
                                   ptr(pos), ptr(cu_seqlens_dev), ptr(cu_seqlens_host), ptr(cu_seqlens_k_dev),
                                   ptr(cu_seqlens_k_host), ptr(block_table), ctypes.c_int64(block_table_stride),
                                   int(kv_block_size), ptr(keep_ratio_dev), ptr(keep_ratio_host), ptr(hidden_out),
                                   ptr(pos_out), ptr(kept_idx), ptr(new_cu_seqlens_dev), ptr(scores_out),
                                   ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_fused_lse", check)


def uniprefill_score_lse(p, q, k, lse, lse_row_stride, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev,
                         cu_seqlens_k_host, block_table, block_table_stride, kv_block_size, scores_out, workspace,
                         workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_score_lse(ctypes.byref(p), ptr(q), ptr(k), ptr(lse), ctypes.c_int64(lse_row_stride),
                                   ptr(cu_seqlens_dev), ptr(cu_seqlens_host), ptr(cu_seqlens_k_dev),
                                   ptr(cu_seqlens_k_host), ptr(block_table), ctypes.c_int64(block_table_stride),
                                   int(kv_block_size), ptr(scores_out), ptr(workspace), workspace_bytes,
                                   _stream(stream))
    return _check(st, "uniprefill_score_lse", check)


def uniprefill_fused_top_p_lse(p, q, k, lse, lse_row_stride, hidden, pos, cu_seqlens_dev, cu_seqlens_host,
                               cu_seqlens_k_dev, cu_seqlens_k_host, block_table, block_table_stride, kv_block_size,
                               top_p_dev, top_p_host, hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores,
                               workspace, workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_fused_top_p_lse(ctypes.byref(p), ptr(q), ptr(k), ptr(lse), ctypes.c_int64(lse_row_stride),
                                         ptr(hidden), ptr(pos), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                                         ptr(cu_seqlens_k_dev), ptr(cu_seqlens_k_host), ptr(block_table),
                                         ctypes.c_int64(block_table_stride), int(kv_block_size), ptr(top_p_dev),
                                         ptr(top_p_host), ptr(hidden_out), ptr(pos_out), ptr(kept_idx),
                                         ptr(new_cu_seqlens_dev), ptr(scores), ptr(workspace), workspace_bytes,
                                         _stream(stream))
    return _check(st, "uniprefill_fused_top_p_lse", check)


def uniprefill_score_partial(p, q, k, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev, cu_seqlens_k_host, colsum_out,
                             workspace, workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_score_partial(ctypes.byref(p), ptr(q), ptr(k), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                                       ptr(cu_seqlens_k_dev), ptr(cu_seqlens_k_host), ptr(colsum_out), ptr(workspace),
                                       workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_score_partial", check)


def uniprefill_scores_from_partials(partials, num_parts, part_stride, cu_seqlens_dev, num_seqs, total_tokens, n_obs,
                                    total_q_heads, scores_out, stream=None, check=True):
    st = _lib.uniprefill_scores_from_partials(ptr(partials), int(num_parts), ctypes.c_int64(part_stride),
                                              ptr(cu_seqlens_dev), int(num_seqs), int(total_tokens), int(n_obs),
                                              int(total_q_heads), ptr(scores_out), _stream(stream))
    return _check(st, "uniprefill_scores_from_partials", check)


def uniprefill_keep_mask(kept_idx, capacity, total_kept_dev, total_tokens, mask_out, stream=None, check=True):
    st = _lib.uniprefill_keep_mask(ptr(kept_idx), ctypes.c_int64(capacity), ptr(total_kept_dev),
                                   ctypes.c_int64(total_tokens), ptr(mask_out), _stream(stream))
    return _check(st, "uniprefill_keep_mask", check)


def uniprefill_seqused(drop_layers_host, retained_dev, kv_len_dev, orig_len_dev, num_seqs, num_layers, seqused_out,
                       stream=None, check=True):
    layers = np.ascontiguousarray(drop_layers_host, dtype=np.int32)
    st = _lib.uniprefill_seqused(ptr(layers), int(layers.shape[0]), ptr(retained_dev), ptr(kv_len_dev),
                                 ptr(orig_len_dev), int(num_seqs), int(num_layers), ptr(seqused_out),
                                 _stream(stream))
    return _check(st, "uniprefill_seqused", check)


def uniprefill_plan_chunked(p: up_params, cu_seqlens_host: np.ndarray, cu_seqlens_k_host: np.ndarray,
                            keep_ratio_host: np.ndarray, *, want_workspace: bool = True, check: bool = True):
    """Returns (status, new_cu_seqlens_host, total_kept, workspace_bytes)."""
    new_cu = np.zeros(p.num_seqs + 1, dtype=np.int32)
    total = ctypes.c_int64(0)
    ws = ctypes.c_size_t(0)
    st = _lib.uniprefill_plan_chunked(ctypes.byref(p), ptr(cu_seqlens_host), ptr(cu_seqlens_k_host),
                                      ptr(keep_ratio_host), ptr(new_cu), ctypes.byref(total),
                                      ctypes.byref(ws) if want_workspace else None)
    _check(st, "uniprefill_plan_chunked", check)
    return st, new_cu, int(total.value), int(ws.value)


def uniprefill_score_chunked(p, q, k, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev, cu_seqlens_k_host,
                             scores_out, workspace, workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_score_chunked(ctypes.byref(p), ptr(q), ptr(k), ptr(cu_seqlens_dev),
                                       ptr(cu_seqlens_host), ptr(cu_seqlens_k_dev), ptr(cu_seqlens_k_host),
                                       ptr(scores_out), ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_score_chunked", check)


def uniprefill_select_chunked(p, scores, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev, cu_seqlens_k_host,
                              keep_ratio_dev, keep_ratio_host, kept_idx, new_cu_seqlens_dev, stream=None,
                              check=True):
    st = _lib.uniprefill_select_chunked(ctypes.byref(p), ptr(scores), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                                        ptr(cu_seqlens_k_dev), ptr(cu_seqlens_k_host), ptr(keep_ratio_dev),
                                        ptr(keep_ratio_host), ptr(kept_idx), ptr(new_cu_seqlens_dev),
                                        _stream(stream))
    return _check(st, "uniprefill_select_chunked", check)


def uniprefill_fused_chunked(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev,
                             cu_seqlens_k_host, keep_ratio_dev, keep_ratio_host, hidden_out, pos_out, kept_idx,
                             new_cu_seqlens_dev, scores_out, workspace, workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_fused_chunked(ctypes.byref(p), ptr(q), ptr(k), ptr(hidden), ptr(pos),
                                       ptr(cu_seqlens_dev), ptr(cu_seqlens_host), ptr(cu_seqlens_k_dev),
                                       ptr(cu_seqlens_k_host), ptr(keep_ratio_dev), ptr(keep_ratio_host),
                                       ptr(hidden_out), ptr(pos_out), ptr(kept_idx), ptr(new_cu_seqlens_dev),
                                       ptr(scores_out), ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_fused_chunked", check)


def uniprefill_score_paged(p, q, k_cache, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev, cu_seqlens_k_host,
                           block_table, block_table_stride, kv_block_size, scores_out, workspace, workspace_bytes,
                           stream=None, check=True):
    st = _lib.uniprefill_score_paged(ctypes.byref(p), ptr(q), ptr(k_cache), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                                     ptr(cu_seqlens_k_dev), ptr(cu_seqlens_k_host), ptr(block_table),
                                     ctypes.c_int64(block_table_stride), int(kv_block_size), ptr(scores_out),
                                     ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_score_paged", check)


def uniprefill_fused_paged(p, q, k_cache, hidden, pos, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev,
                           cu_seqlens_k_host, block_table, block_table_stride, kv_block_size, keep_ratio_dev,
                           keep_ratio_host, hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out, workspace,
                           workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_fused_paged(ctypes.byref(p), ptr(q), ptr(k_cache), ptr(hidden), ptr(pos),
                                     ptr(cu_seqlens_dev), ptr(cu_seqlens_host), ptr(cu_seqlens_k_dev),
                                     ptr(cu_seqlens_k_host), ptr(block_table), ctypes.c_int64(block_table_stride),
                                     int(kv_block_size), ptr(keep_ratio_dev), ptr(keep_ratio_host), ptr(hidden_out),
                                     ptr(pos_out), ptr(kept_idx), ptr(new_cu_seqlens_dev), ptr(scores_out),
                                     ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_fused_paged", check)


def uniprefill_select_top_p_chunked(p, scores, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev, cu_seqlens_k_host,
                                    top_p_dev, top_p_host, kept_idx, new_cu_seqlens_dev, workspace, workspace_bytes,
                                    stream=None, check=True):
    st = _lib.uniprefill_select_top_p_chunked(ctypes.byref(p), ptr(scores), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                                              ptr(cu_seqlens_k_dev), ptr(cu_seqlens_k_host), ptr(top_p_dev),
                                              ptr(top_p_host), ptr(kept_idx), ptr(new_cu_seqlens_dev), ptr(workspace),
                                              workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_select_top_p_chunked", check)


def uniprefill_fused_top_p_chunked(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, cu_seqlens_k_dev,
                                   cu_seqlens_k_host, block_table, block_table_stride, kv_block_size, top_p_dev,
                                   top_p_host, hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores, workspace,
                                   workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_fused_top_p_chunked(ctypes.byref(p), ptr(q), ptr(k), ptr(hidden), ptr(pos),
                                             ptr(cu_seqlens_dev), ptr(cu_seqlens_host), ptr(cu_seqlens_k_dev),
                                             ptr(cu_seqlens_k_host), ptr(block_table),
                                             ctypes.c_int64(block_table_stride), int(kv_block_size), ptr(top_p_dev),
                                             ptr(top_p_host), ptr(hidden_out), ptr(pos_out), ptr(kept_idx),
                                             ptr(new_cu_seqlens_dev), ptr(scores), ptr(workspace), workspace_bytes,
                                             _stream(stream))
    return _check(st, "uniprefill_fused_top_p_chunked", check)


def uniprefill_fused_phases(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, keep_ratio_dev,
                            keep_ratio_host, hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores_out,
                            workspace, workspace_bytes, phase_mask, stream=None, check=True):
    st = _lib.uniprefill_fused_phases(ctypes.byref(p), ptr(q), ptr(k), ptr(hidden), ptr(pos),
                                      ptr(cu_seqlens_dev), ptr(cu_seqlens_host), ptr(keep_ratio_dev),
                                      ptr(keep_ratio_host), ptr(hidden_out), ptr(pos_out), ptr(kept_idx),
                                      ptr(new_cu_seqlens_dev), ptr(scores_out), ptr(workspace),
                                      workspace_bytes, int(phase_mask), _stream(stream))
    return _check(st, "uniprefill_fused_phases", check)


def uniprefill_select_top_p(p, scores, cu_seqlens_dev, cu_seqlens_host, top_p_dev, top_p_host, kept_idx,
                            new_cu_seqlens_dev, workspace, workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_select_top_p(ctypes.byref(p), ptr(scores), ptr(cu_seqlens_dev), ptr(cu_seqlens_host),
                                      ptr(top_p_dev), ptr(top_p_host), ptr(kept_idx), ptr(new_cu_seqlens_dev),
                                      ptr(workspace), workspace_bytes, _stream(stream))
    return _check(st, "uniprefill_select_top_p", check)


def uniprefill_compact_counted(p, hidden, pos, kept_idx, total_kept_dev, capacity, hidden_out, pos_out,
                               stream=None, check=True):
    st = _lib.uniprefill_compact_counted(ctypes.byref(p), ptr(hidden), ptr(pos), ptr(kept_idx),
                                         ptr(total_kept_dev), int(capacity), ptr(hidden_out), ptr(pos_out),
                                         _stream(stream))
    return _check(st, "uniprefill_compact_counted", check)


def uniprefill_fused_top_p(p, q, k, hidden, pos, cu_seqlens_dev, cu_seqlens_host, top_p_dev, top_p_host,
                           hidden_out, pos_out, kept_idx, new_cu_seqlens_dev, scores, workspace,
                           workspace_bytes, stream=None, check=True):
    st = _lib.uniprefill_fused_top_p(ctypes.byref(p), ptr(q), ptr(k), ptr(hidden), ptr(pos),
                                     ptr(cu_seqlens_dev), ptr(cu_seqlens_host), ptr(top_p_dev),
                                     ptr(top_p_host), ptr(hidden_out), ptr(pos_out), ptr(kept_idx),
                                     ptr(new_cu_seqlens_dev), ptr(scores), ptr(workspace), workspace_bytes,
                                     _stream(stream))
    return _check(st, "uniprefill_fused_top_p", check)


def uniprefill_compose_index(outer_idx, n_outer, inner_idx, n_inner_dev, n_inner, composed_idx, stream=None,
                             check=True):
    st = _lib.uniprefill_compose_index(ptr(outer_idx), int(n_outer), ptr(inner_idx), ptr(n_inner_dev),
                                       int(n_inner), ptr(composed_idx), _stream(stream))
    return _check(st, "uniprefill_compose_index", check)


def uniprefill_slot_mapping(pos_kept, new_cu_seqlens_dev, num_seqs, block_table, block_table_stride,
                            kv_block_size, capacity, slots, stream=None, check=True):
    st = _lib.uniprefill_slot_mapping(ptr(pos_kept), ptr(new_cu_seqlens_dev), int(num_seqs), ptr(block_table),
                                      int(block_table_stride), int(kv_block_size), int(capacity), ptr(slots),
                                      _stream(stream))
    return _check(st, "uniprefill_slot_mapping", check)
