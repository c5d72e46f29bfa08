"""ctypes binding of ``libmooncake_hip.so``: argument marshalling only.

Function names and argument order are those of ``include/mc.h``.  torch is used
for device memory and streams; every step of the path runs in the library's
kernels.  There is no fallback: if the library has not been built, loading
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libmooncake_hip.so")

MC_OK = 0
MC_ERR_NULL, MC_ERR_SHAPE, MC_ERR_UNSUPPORTED, MC_ERR_ALIGN, MC_ERR_RANGE, MC_ERR_WORKSPACE, MC_ERR_HIP = range(1, 8)
MC_DTYPE_BF16, MC_DTYPE_F32 = 0, 1

EXPORTS = ("mc_status_string", "mc_prefill_attn_workspace_bytes", "mc_prefill_attn_paged",
           "mc_kv_pack_layer", "mc_kv_unpack_layer", "mc_kv_append_workspace_bytes", "mc_kv_append_paged",
           "mc_prefill_attn_split_workspace_bytes", "mc_prefill_attn_paged_split", "mc_attn_merge_lse",
           "mc_kv_load_layer", "mc_kv_store_layer", "mc_prefix_hash_workspace_bytes", "mc_prefix_hash",
           "mc_prefix_match_workspace_bytes", "mc_prefix_match", "mc_kv_page_order", "mc_kv_pack_layer_ordered",
           "mc_kv_unpack_layer_ordered", "mc_prefill_attn_suggest_kv_splits", "mc_kv_check_page_ids",
           "mc_prefill_attn_plan", "mc_prefill_attn_prepare", "mc_prefill_attn_run", "mc_prefill_attn_run_split",
           "mc_kv_append_run", "mc_prefill_attn_auto_workspace_bytes", "mc_prefill_attn_auto",
           "mc_prefill_attn_paged_noalloc")
MC_MAX_KV_SPLITS = 256


class McAttnParams(ctypes.Structure):
    _fields_ = [("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_pages", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float)]


class McAttnPlan(ctypes.Structure):
    _fields_ = [("n_items", ctypes.c_int32), ("batch", ctypes.c_int32), ("kv_splits", ctypes.c_int32),
                ("need_pages", ctypes.c_int32), ("total_new_tokens", ctypes.c_int64), ("reqs_offset", ctypes.c_int64),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class McError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: mc_status {status} ({status_string(status)})")
        self.status = status


_lib = None


def lib():
    """The loaded library; raises if it was never built (run ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_00079_amd.build` "
                               "(there is no CPU fallback)")
        # torch first: its bundled HIP runtime must be the one in the process, so that the
        # streams and device pointers it hands out belong to the runtime this library calls
        import torch  # noqa: F401
        l = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        l.mc_status_string.restype = ctypes.c_char_p
        l.mc_status_string.argtypes = [ctypes.c_int]
        l.mc_prefill_attn_workspace_bytes.restype = ctypes.c_size_t
        l.mc_prefill_attn_workspace_bytes.argtypes = [ctypes.POINTER(McAttnParams), i32, i64]
        l.mc_prefill_attn_paged.restype = ctypes.c_int
        l.mc_prefill_attn_paged.argtypes = [ctypes.POINTER(McAttnParams), vp, vp, vp, vp, i32, vp, vp, i32,
                                            vp, vp, vp, ctypes.c_size_t, vp]
        for f in (l.mc_kv_pack_layer, l.mc_kv_unpack_layer):
            f.restype = ctypes.c_int
            f.argtypes = [vp, vp, i64, i64, vp, i64, vp, vp, vp]
        l.mc_kv_page_order.restype = ctypes.c_int
        l.mc_kv_page_order.argtypes = [vp, i64, vp, vp]
        l.mc_kv_check_page_ids.restype = ctypes.c_int
        l.mc_kv_check_page_ids.argtypes = [vp, i64, i64, vp, vp]
        for f in (l.mc_kv_pack_layer_ordered, l.mc_kv_unpack_layer_ordered):
            f.restype = ctypes.c_int
            f.argtypes = [vp, vp, i64, i64, vp, vp, i64, vp, vp, vp]
        l.mc_kv_append_workspace_bytes.restype = ctypes.c_size_t
        l.mc_kv_append_workspace_bytes.argtypes = [i32]
        l.mc_kv_append_paged.restype = ctypes.c_int
        l.mc_kv_append_paged.argtypes = [ctypes.POINTER(McAttnParams), vp, vp, vp, vp, vp, i32, vp, vp, i32, vp,
                                         ctypes.c_size_t, vp]
        l.mc_prefill_attn_split_workspace_bytes.restype = ctypes.c_size_t
        l.mc_prefill_attn_split_workspace_bytes.argtypes = [ctypes.POINTER(McAttnParams), i32, i64, i32]
        pp, pl_ = ctypes.POINTER(McAttnParams), ctypes.POINTER(McAttnPlan)
        l.mc_prefill_attn_auto_workspace_bytes.restype = ctypes.c_size_t
        l.mc_prefill_attn_auto_workspace_bytes.argtypes = [pp, vp, vp, i32]
        l.mc_prefill_attn_auto.restype = ctypes.c_int
        l.mc_prefill_attn_auto.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp, ctypes.c_size_t, vp]
        l.mc_prefill_attn_paged_noalloc.restype = ctypes.c_int
        l.mc_prefill_attn_paged_noalloc.argtypes = [pp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp]
        l.mc_prefill_attn_prepare.restype = ctypes.c_int
        l.mc_prefill_attn_prepare.argtypes = [pp, vp, vp, i32, i32, vp, ctypes.c_size_t, vp, pl_]
        l.mc_prefill_attn_run.restype = ctypes.c_int
        l.mc_prefill_attn_run.argtypes = [pp, pl_, vp, vp, vp, vp, i32, vp, vp, vp, vp]
        l.mc_prefill_attn_run_split.restype = ctypes.c_int
        l.mc_prefill_attn_run_split.argtypes = [pp, pl_, vp, vp, vp, vp, i32, vp, vp, vp, vp]
        l.mc_kv_append_run.restype = ctypes.c_int
        l.mc_kv_append_run.argtypes = [pp, pl_, vp, vp, vp, vp, vp, i32, vp, vp]
        l.mc_prefill_attn_plan.restype = ctypes.c_int
        l.mc_prefill_attn_plan.argtypes = [ctypes.POINTER(McAttnParams), vp, vp, i32, i32, vp, i64, vp]
        l.mc_prefill_attn_suggest_kv_splits.restype = ctypes.c_int32
        l.mc_prefill_attn_suggest_kv_splits.argtypes = [ctypes.POINTER(McAttnParams), vp, vp, i32]
        l.mc_prefill_attn_paged_split.restype = ctypes.c_int
        l.mc_prefill_attn_paged_split.argtypes = [ctypes.POINTER(McAttnParams), vp, vp, vp, vp, i32, vp, vp, i32, i32,
                                                  vp, vp, vp, ctypes.c_size_t, vp]
        l.mc_kv_load_layer.restype = ctypes.c_int
        l.mc_kv_load_layer.argtypes = [vp, vp, vp, vp, i64, i64, vp, i64, vp, vp, vp]
        l.mc_kv_store_layer.restype = ctypes.c_int
        l.mc_kv_store_layer.argtypes = [vp, vp, i64, i64, vp, i64, vp, vp, vp, vp, vp]
        l.mc_prefix_hash_workspace_bytes.restype = ctypes.c_size_t
        l.mc_prefix_hash_workspace_bytes.argtypes = [i32]
        l.mc_prefix_hash.restype = ctypes.c_int
        l.mc_prefix_hash.argtypes = [vp, vp, i32, i32, vp, vp, ctypes.c_size_t, vp]
        l.mc_prefix_match_workspace_bytes.restype = ctypes.c_size_t
        l.mc_prefix_match_workspace_bytes.argtypes = [i32, i32]
        l.mc_prefix_match.restype = ctypes.c_int
        l.mc_prefix_match.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        l.mc_attn_merge_lse.restype = ctypes.c_int
        l.mc_attn_merge_lse.argtypes = [vp, vp, i32, i64, i32, i32, vp, vp, vp]
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().mc_status_string(int(status)).decode()


def _dev_ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) or None


def mc_prefill_attn_workspace_bytes(params: McAttnParams, batch: int, total_new_tokens: int) -> int:
    return int(lib().mc_prefill_attn_workspace_bytes(ctypes.byref(params), batch, total_new_tokens))


def mc_prefill_attn_paged_raw(params, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens,
                              batch, out, lse, workspace, workspace_bytes, hip_stream) -> int:
    """Plain-pointer call: every argument is an int address / ctypes object; returns the status."""
    return int(lib().mc_prefill_attn_paged(ctypes.byref(params) if params is not None else None, q, k_pool, v_pool,
                                           block_tables, max_pages_per_req, prefix_lens, new_lens, batch, out, lse,
                                           workspace, workspace_bytes, hip_stream))


def mc_prefill_attn_paged(params: McAttnParams, q, k_pool, v_pool, block_tables, prefix_lens, new_lens,
                          out, lse=None, workspace=None, stream=None) -> None:
    """Enqueue attention on ``stream`` (torch stream; default: current).

    q, k_pool, v_pool, out: torch device tensors; block_tables: int32 device
    tensor [batch, max_pages]; prefix_lens / new_lens: host sequences of ints;
    workspace: uint8 device tensor of at least the size the library asks for.
    """
    batch = len(prefix_lens)
    pl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in prefix_lens])
    nl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in new_lens])
    max_pages = int(block_tables.shape[1]) if block_tables is not None and block_tables.dim() == 2 else 0
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    st = mc_prefill_attn_paged_raw(params, _dev_ptr(q), _dev_ptr(k_pool), _dev_ptr(v_pool), _dev_ptr(block_tables),
                                   max_pages, ctypes.cast(pl, ctypes.c_void_p), ctypes.cast(nl, ctypes.c_void_p),
                                   batch, _dev_ptr(out), _dev_ptr(lse), _dev_ptr(workspace), ws_bytes,
                                   _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_paged")


def mc_prefill_attn_split_workspace_bytes(params: McAttnParams, batch: int, total_new_tokens: int,
                                          kv_splits: int) -> int:
    return int(lib().mc_prefill_attn_split_workspace_bytes(ctypes.byref(params), batch, total_new_tokens, kv_splits))


def _lens(prefix_lens, new_lens):
    batch = len(prefix_lens)
    pl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in prefix_lens])
    nl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in new_lens])
    return batch, pl, nl


def mc_prefill_attn_auto_workspace_bytes(params: McAttnParams, prefix_lens, new_lens) -> int:
    batch, pl, nl = _lens(prefix_lens, new_lens)
    return int(lib().mc_prefill_attn_auto_workspace_bytes(ctypes.byref(params), pl, nl, batch))


def mc_prefill_attn_auto(params: McAttnParams, q, k_pool, v_pool, block_tables, prefix_lens, new_lens, out, lse,
                         workspace, stream=None) -> None:
    """mc_prefill_attn_paged with the whole-row / key-slices choice made by the library (larger workspace)."""
    batch, pl, nl = _lens(prefix_lens, new_lens)
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    max_pages = int(block_tables.shape[1]) if block_tables is not None and block_tables.dim() == 2 else 0
    st = int(lib().mc_prefill_attn_auto(ctypes.byref(params), _dev_ptr(q), _dev_ptr(k_pool), _dev_ptr(v_pool),
                                        _dev_ptr(block_tables), max_pages, pl, nl, batch, _dev_ptr(out), _dev_ptr(lse),
                                        _dev_ptr(workspace), ws_bytes, _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_auto")


def mc_prefill_attn_paged_noalloc_raw(params, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens,
                                      new_lens, batch, out, lse, hip_stream) -> int:
    return int(lib().mc_prefill_attn_paged_noalloc(ctypes.byref(params) if params is not None else None, q, k_pool,
                                                   v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens,
                                                   batch, out, lse, hip_stream))


def mc_prefill_attn_paged_noalloc(params: McAttnParams, q, k_pool, v_pool, block_tables, prefix_lens, new_lens, out,
                                  lse=None, stream=None) -> None:
    """mc_prefill_attn_paged without a workspace: the work list is built on the device in the library's own
    fixed array (no allocation, no upload)."""
    batch, pl, nl = _lens(prefix_lens, new_lens)
    st = mc_prefill_attn_paged_noalloc_raw(params, _dev_ptr(q), _dev_ptr(k_pool), _dev_ptr(v_pool),
                                           _dev_ptr(block_tables), _max_pages(block_tables), pl, nl, batch,
                                           _dev_ptr(out), _dev_ptr(lse), _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_paged_noalloc")


def _max_pages(block_tables) -> int:
    return int(block_tables.shape[1]) if block_tables is not None and block_tables.dim() == 2 else 0


def mc_prefill_attn_prepare(params: McAttnParams, prefix_lens, new_lens, kv_splits: int, workspace,
                            stream=None) -> McAttnPlan:
    """Build and upload the work list and request table of a batch ONCE; the returned plan drives any number of
    mc_prefill_attn_run / mc_prefill_attn_run_split / mc_kv_append_run calls (one per layer) on the same workspace."""
    batch = len(prefix_lens)
    pl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in prefix_lens])
    nl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in new_lens])
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    plan = McAttnPlan()
    st = int(lib().mc_prefill_attn_prepare(ctypes.byref(params), pl, nl, batch, kv_splits, _dev_ptr(workspace), ws_bytes,
                                           _stream_handle(stream), ctypes.byref(plan)))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_prepare")
    return plan


def mc_prefill_attn_run(params: McAttnParams, plan: McAttnPlan, q, k_pool, v_pool, block_tables, out, lse, workspace,
                        stream=None) -> None:
    st = int(lib().mc_prefill_attn_run(ctypes.byref(params), ctypes.byref(plan), _dev_ptr(q), _dev_ptr(k_pool),
                                       _dev_ptr(v_pool), _dev_ptr(block_tables), _max_pages(block_tables),
                                       _dev_ptr(out), _dev_ptr(lse), _dev_ptr(workspace), _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_run")


def mc_prefill_attn_run_split(params: McAttnParams, plan: McAttnPlan, q, k_pool, v_pool, block_tables, o_parts,
                              lse_parts, workspace, stream=None) -> None:
    st = int(lib().mc_prefill_attn_run_split(ctypes.byref(params), ctypes.byref(plan), _dev_ptr(q), _dev_ptr(k_pool),
                                             _dev_ptr(v_pool), _dev_ptr(block_tables), _max_pages(block_tables),
                                             _dev_ptr(o_parts), _dev_ptr(lse_parts), _dev_ptr(workspace),
                                             _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_run_split")


def mc_kv_append_run(params: McAttnParams, plan: McAttnPlan, k_new, v_new, k_pool, v_pool, block_tables, workspace,
                     stream=None) -> None:
    st = int(lib().mc_kv_append_run(ctypes.byref(params), ctypes.byref(plan), _dev_ptr(k_new), _dev_ptr(v_new),
                                    _dev_ptr(k_pool), _dev_ptr(v_pool), _dev_ptr(block_tables),
                                    _max_pages(block_tables), _dev_ptr(workspace), _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_kv_append_run")


def mc_prefill_attn_plan(params: McAttnParams, prefix_lens, new_lens, kv_splits: int = 0):
    """The work list of an attention launch, in launch order: a list of (request, kv_head, row0, slice) tuples.
    Host arithmetic only (no GPU)."""
    batch = len(prefix_lens)
    pl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in prefix_lens])
    nl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in new_lens])
    n = ctypes.c_int64(-1)
    st = int(lib().mc_prefill_attn_plan(ctypes.byref(params), pl, nl, batch, kv_splits, None, 0, ctypes.byref(n)))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_plan")
    buf = (ctypes.c_int32 * (4 * max(n.value, 1)))()
    st = int(lib().mc_prefill_attn_plan(ctypes.byref(params), pl, nl, batch, kv_splits, buf, n.value, ctypes.byref(n)))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_plan")
    return [tuple(buf[4 * i:4 * i + 4]) for i in range(n.value)]


def mc_prefill_attn_suggest_kv_splits(params: McAttnParams, prefix_lens, new_lens) -> int:
    """Key slices that fill the GPU for this batch (1: use the whole-row call); 0 for arguments the library rejects."""
    batch = len(prefix_lens)
    pl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in prefix_lens])
    nl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in new_lens])
    return int(lib().mc_prefill_attn_suggest_kv_splits(ctypes.byref(params), pl, nl, batch))


def mc_prefill_attn_paged_split_raw(params, q, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens,
                                    batch, kv_splits, o_parts, lse_parts, workspace, workspace_bytes, hip_stream) -> int:
    return int(lib().mc_prefill_attn_paged_split(ctypes.byref(params) if params is not None else None, q, k_pool,
                                                 v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens, batch,
                                                 kv_splits, o_parts, lse_parts, workspace, workspace_bytes, hip_stream))


def mc_prefill_attn_paged_split(params: McAttnParams, q, k_pool, v_pool, block_tables, prefix_lens, new_lens,
                                kv_splits: int, o_parts, lse_parts, workspace, stream=None) -> None:
    """Enqueue attention over ``kv_splits`` key slices; partial results go to the fp32 device tensors
    ``o_parts`` [kv_splits, total_new, Hq, D] and ``lse_parts`` [kv_splits, total_new, Hq]."""
    batch = len(prefix_lens)
    pl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in prefix_lens])
    nl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in new_lens])
    max_pages = int(block_tables.shape[1]) if block_tables is not None and block_tables.dim() == 2 else 0
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    st = mc_prefill_attn_paged_split_raw(params, _dev_ptr(q), _dev_ptr(k_pool), _dev_ptr(v_pool),
                                         _dev_ptr(block_tables), max_pages, ctypes.cast(pl, ctypes.c_void_p),
                                         ctypes.cast(nl, ctypes.c_void_p), batch, kv_splits, _dev_ptr(o_parts),
                                         _dev_ptr(lse_parts), _dev_ptr(workspace), ws_bytes, _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_prefill_attn_paged_split")


def mc_attn_merge_lse_raw(o_parts, lse_parts, kv_splits, rows, head_dim, dtype, out, lse, hip_stream) -> int:
    return int(lib().mc_attn_merge_lse(o_parts, lse_parts, kv_splits, rows, head_dim, dtype, out, lse, hip_stream))


def mc_attn_merge_lse(o_parts, lse_parts, kv_splits: int, rows: int, head_dim: int, dtype: int, out, lse=None,
                      stream=None) -> None:
    """Enqueue the merge of ``kv_splits`` partial results (fp32 device tensors) into ``out`` / ``lse``."""
    st = mc_attn_merge_lse_raw(_dev_ptr(o_parts), _dev_ptr(lse_parts), kv_splits, rows, head_dim, dtype,
                               _dev_ptr(out), _dev_ptr(lse), _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_attn_merge_lse")


def mc_kv_pack_layer_raw(k_pool, v_pool, num_pages, page_bytes, page_ids, n, k_out, v_out, hip_stream) -> int:
    return int(lib().mc_kv_pack_layer(k_pool, v_pool, num_pages, page_bytes, page_ids, n, k_out, v_out, hip_stream))


def mc_kv_unpack_layer_raw(k_in, v_in, num_pages, page_bytes, page_ids, n, k_pool, v_pool, hip_stream) -> int:
    return int(lib().mc_kv_unpack_layer(k_in, v_in, num_pages, page_bytes, page_ids, n, k_pool, v_pool, hip_stream))


def mc_kv_pack_layer(k_pool_layer, v_pool_layer, num_pages: int, page_bytes: int, page_ids, n: int,
                     k_out, v_out, stream=None) -> None:
    st = mc_kv_pack_layer_raw(_dev_ptr(k_pool_layer), _dev_ptr(v_pool_layer), num_pages, page_bytes,
                              _dev_ptr(page_ids), n, _dev_ptr(k_out), _dev_ptr(v_out), _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_kv_pack_layer")


def mc_kv_unpack_layer(k_in, v_in, num_pages: int, page_bytes: int, page_ids, n: int,
                       k_pool_layer, v_pool_layer, stream=None) -> None:
    st = mc_kv_unpack_layer_raw(_dev_ptr(k_in), _dev_ptr(v_in), num_pages, page_bytes, _dev_ptr(page_ids), n,
                                _dev_ptr(k_pool_layer), _dev_ptr(v_pool_layer), _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_kv_unpack_layer")


def mc_kv_page_order(page_ids, n: int, order, stream=None) -> None:
    """Enqueue order[r] = position of the r-th smallest page id (int32 device tensors)."""
    st = int(lib().mc_kv_page_order(_dev_ptr(page_ids), n, _dev_ptr(order), _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_kv_page_order")


def mc_kv_check_page_ids(page_ids, n: int, num_pages: int, report, stream=None) -> None:
    """Enqueue the range check of an int32 device id list: report[0] = ids outside [0, num_pages), report[1] =
    position of the first of them (n if none); ``report`` is an int32 device tensor of 2."""
    st = int(lib().mc_kv_check_page_ids(_dev_ptr(page_ids), n, num_pages, _dev_ptr(report), _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_kv_check_page_ids")


def mc_kv_pack_layer_ordered(k_pool_layer, v_pool_layer, num_pages: int, page_bytes: int, page_ids, order, n: int,
                             k_out, v_out, stream=None) -> None:
    st = int(lib().mc_kv_pack_layer_ordered(_dev_ptr(k_pool_layer), _dev_ptr(v_pool_layer), num_pages, page_bytes,
                                            _dev_ptr(page_ids), _dev_ptr(order), n, _dev_ptr(k_out), _dev_ptr(v_out),
                                            _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_kv_pack_layer_ordered")


def mc_kv_unpack_layer_ordered(k_in, v_in, num_pages: int, page_bytes: int, page_ids, order, n: int, k_pool_layer,
                               v_pool_layer, stream=None) -> None:
    st = int(lib().mc_kv_unpack_layer_ordered(_dev_ptr(k_in), _dev_ptr(v_in), num_pages, page_bytes,
                                              _dev_ptr(page_ids), _dev_ptr(order), n, _dev_ptr(k_pool_layer),
                                              _dev_ptr(v_pool_layer), _stream_handle(stream)))
    if st != MC_OK:
        raise McError(st, "mc_kv_unpack_layer_ordered")


def mc_kv_load_layer_raw(k_host, v_host, k_stage, v_stage, num_pages, page_bytes, page_ids, n, k_pool, v_pool,
                         hip_stream) -> int:
    return int(lib().mc_kv_load_layer(k_host, v_host, k_stage, v_stage, num_pages, page_bytes, page_ids, n, k_pool,
                                      v_pool, hip_stream))


def mc_kv_store_layer_raw(k_pool, v_pool, num_pages, page_bytes, page_ids, n, k_stage, v_stage, k_host, v_host,
                          hip_stream) -> int:
    return int(lib().mc_kv_store_layer(k_pool, v_pool, num_pages, page_bytes, page_ids, n, k_stage, v_stage, k_host,
                                       v_host, hip_stream))


def mc_kv_load_layer(k_host, v_host, k_stage, v_stage, num_pages: int, page_bytes: int, page_ids, n: int,
                     k_pool_layer, v_pool_layer, stream=None) -> None:
    """Host (pinned torch tensors) -> staging -> the listed pool pages, enqueued on ``stream``."""
    st = mc_kv_load_layer_raw(_dev_ptr(k_host), _dev_ptr(v_host), _dev_ptr(k_stage), _dev_ptr(v_stage), num_pages,
                              page_bytes, _dev_ptr(page_ids), n, _dev_ptr(k_pool_layer), _dev_ptr(v_pool_layer),
                              _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_kv_load_layer")


def mc_kv_store_layer(k_pool_layer, v_pool_layer, num_pages: int, page_bytes: int, page_ids, n: int, k_stage,
                      v_stage, k_host, v_host, stream=None) -> None:
    """The listed pool pages -> staging -> host (pinned torch tensors), enqueued on ``stream``."""
    st = mc_kv_store_layer_raw(_dev_ptr(k_pool_layer), _dev_ptr(v_pool_layer), num_pages, page_bytes,
                               _dev_ptr(page_ids), n, _dev_ptr(k_stage), _dev_ptr(v_stage), _dev_ptr(k_host),
                               _dev_ptr(v_host), _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_kv_store_layer")


def mc_prefix_hash_workspace_bytes(batch: int) -> int:
    return int(lib().mc_prefix_hash_workspace_bytes(batch))


def mc_prefix_match_workspace_bytes(batch: int, n_inst: int) -> int:
    return int(lib().mc_prefix_match_workspace_bytes(batch, n_inst))


def _i64_array(values):
    arr = (ctypes.c_int64 * max(len(values), 1))(*[int(x) for x in values])
    return arr, ctypes.cast(arr, ctypes.c_void_p)


def mc_prefix_hash_raw(tokens, tok_offsets, batch, block_tokens, keys, workspace, workspace_bytes, hip_stream) -> int:
    return int(lib().mc_prefix_hash(tokens, tok_offsets, batch, block_tokens, keys, workspace, workspace_bytes,
                                    hip_stream))


def mc_prefix_hash(tokens, tok_offsets, block_tokens: int, keys, workspace, stream=None) -> None:
    """Enqueue the block keys of every request: ``tokens`` int32 device tensor, ``tok_offsets`` host sequence of
    batch + 1 ints, ``keys`` int64 device tensor (the uint64 bit patterns) with one entry per block."""
    keep, off = _i64_array(tok_offsets)
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    st = mc_prefix_hash_raw(_dev_ptr(tokens), off, len(tok_offsets) - 1, block_tokens, _dev_ptr(keys),
                            _dev_ptr(workspace), ws_bytes, _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_prefix_hash")


def mc_prefix_match_raw(keys, key_offsets, batch, cache_keys, cache_offsets, n_inst, prefix_len, best_len, best_inst,
                        workspace, workspace_bytes, hip_stream) -> int:
    return int(lib().mc_prefix_match(keys, key_offsets, batch, cache_keys, cache_offsets, n_inst, prefix_len, best_len,
                                     best_inst, workspace, workspace_bytes, hip_stream))


def mc_prefix_match(keys, key_offsets, cache_keys, cache_offsets, prefix_len, best_len, best_inst, workspace,
                    stream=None) -> None:
    """Enqueue the longest-prefix match of every request against every instance (device tensors; offsets on the host)."""
    keep_k, koff = _i64_array(key_offsets)
    keep_c, coff = _i64_array(cache_offsets)
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    st = mc_prefix_match_raw(_dev_ptr(keys), koff, len(key_offsets) - 1, _dev_ptr(cache_keys), coff,
                             len(cache_offsets) - 1, _dev_ptr(prefix_len), _dev_ptr(best_len), _dev_ptr(best_inst),
                             _dev_ptr(workspace), ws_bytes, _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_prefix_match")


def mc_kv_append_workspace_bytes(batch: int) -> int:
    return int(lib().mc_kv_append_workspace_bytes(batch))


def mc_kv_append_paged_raw(params, k_new, v_new, k_pool, v_pool, block_tables, max_pages_per_req, prefix_lens,
                           new_lens, batch, workspace, workspace_bytes, hip_stream) -> int:
    return int(lib().mc_kv_append_paged(ctypes.byref(params) if params is not None else None, k_new, v_new, k_pool,
                                        v_pool, block_tables, max_pages_per_req, prefix_lens, new_lens, batch,
                                        workspace, workspace_bytes, hip_stream))


def mc_kv_append_paged(params: McAttnParams, k_new, v_new, k_pool, v_pool, block_tables, prefix_lens, new_lens,
                       workspace, stream=None) -> None:
    """Enqueue the scatter of the new tokens' K/V rows into their page slots (torch device tensors)."""
    batch = len(prefix_lens)
    pl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in prefix_lens])
    nl = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in new_lens])
    max_pages = int(block_tables.shape[1]) if block_tables is not None and block_tables.dim() == 2 else 0
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    st = mc_kv_append_paged_raw(params, _dev_ptr(k_new), _dev_ptr(v_new), _dev_ptr(k_pool), _dev_ptr(v_pool),
                                _dev_ptr(block_tables), max_pages, ctypes.cast(pl, ctypes.c_void_p),
                                ctypes.cast(nl, ctypes.c_void_p), batch, _dev_ptr(workspace), ws_bytes,
                                _stream_handle(stream))
    if st != MC_OK:
        raise McError(st, "mc_kv_append_paged")


def attn_params(num_q_heads: int, num_kv_heads: int, head_dim: int, page_size: int, num_pages: int,
                dtype: str, softmax_scale: float = 0.0) -> McAttnParams:
    return McAttnParams(num_q_heads, num_kv_heads, head_dim, page_size, num_pages,
                        MC_DTYPE_BF16 if dtype == "bf16" else MC_DTYPE_F32, softmax_scale)
