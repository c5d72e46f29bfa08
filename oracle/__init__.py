"""ctypes front end of the CPU oracle (``mc_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg import
this package.  It shares no code with the HIP library and never imports it.
Arguments are numpy arrays in the stored dtype (uint16 bf16 bit patterns or
float32); results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mc_oracle.c")
# MC_ORACLE_SANITIZE=1 (tests only): the same source built with AddressSanitizer and UBSan, for a
# process that was started with the sanitizer runtime preloaded
_SANITIZE = os.environ.get("MC_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libmc_oracle_san.so" if _SANITIZE else "libmc_oracle.so")

BF16, F32 = 0, 1
_DTYPES = {"bf16": BF16, "f32": F32}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 arithmetic, no fast-math, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", *opt, "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        lib.mco_num_threads.restype = ctypes.c_int
        lib.mco_attn_rows.restype = ctypes.c_int
        lib.mco_attn_rows.argtypes = [i32, vp, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, f64,
                                      i64, vp, vp, vp, vp, vp, vp]
        lib.mco_prefill_attn_paged.restype = ctypes.c_int
        lib.mco_prefill_attn_paged.argtypes = [i32, vp, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32,
                                               f64, vp, vp, vp]
        for f in (lib.mco_kv_pack_layer, lib.mco_kv_unpack_layer):
            f.restype = ctypes.c_int
            f.argtypes = [vp, vp, i64, i64, vp, i64, vp, vp, i32]
        lib.mco_kv_append_paged.restype = ctypes.c_int
        lib.mco_kv_append_paged.argtypes = [vp, vp, vp, vp, i64, vp, i32, vp, vp, i32, i32, i32, i64]
        lib.mco_mix64.restype = ctypes.c_uint64
        lib.mco_mix64.argtypes = [ctypes.c_uint64]
        lib.mco_prefix_hash.restype = ctypes.c_int64
        lib.mco_prefix_hash.argtypes = [vp, vp, i32, i32, vp]
        lib.mco_prefix_match.restype = ctypes.c_int
        lib.mco_prefix_match.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp]
        lib.mco_attn_merge_lse.restype = ctypes.c_int
        lib.mco_attn_merge_lse.argtypes = [vp, vp, i32, i64, i32, vp, vp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().mco_num_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_stored(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.uint16 if dtype == "bf16" else np.float32
    assert a.dtype == want, f"{dtype} tensors are passed as {want}, got {a.dtype}"
    return np.ascontiguousarray(a)


def _scale(scale: Optional[float], head_dim: int) -> float:
    return float(scale) if scale else 1.0 / float(np.sqrt(np.float64(head_dim)))


def attn_rows(dtype: str, q, k_pool, v_pool, block_tables, prefix_lens, new_lens, num_q_heads: int,
              num_kv_heads: int, rows, scale: Optional[float] = None, key_lo=None, key_hi=None):
    """Rows (request, head, chunk row) of prefix-reused causal attention.

    Returns (out [n, D] f64, lse [n] f64, psum [n] f64).  ``key_lo`` /
    ``key_hi`` restrict each row's keys to [lo, hi) within its visible range.
    """
    lib = _load()
    q, k_pool, v_pool = (_check_stored(x, dtype) for x in (q, k_pool, v_pool))
    N, Hkv, S, D = k_pool.shape
    assert Hkv == num_kv_heads and v_pool.shape == k_pool.shape
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    pl = np.ascontiguousarray(prefix_lens, dtype=np.int32)
    nl = np.ascontiguousarray(new_lens, dtype=np.int32)
    B = pl.shape[0]
    assert bt.ndim == 2 and bt.shape[0] == B
    assert q.shape == (int(nl.sum()), num_q_heads, D)
    used = np.concatenate([bt[r, :(int(pl[r]) + int(nl[r]) + S - 1) // S] for r in range(B)]) if B else bt[:0, 0]
    assert used.size == 0 or (used.min() >= 0 and used.max() < N), "block table id outside the pool"
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    n = rows.shape[0]
    out = np.zeros((n, D), dtype=np.float64)
    lse = np.zeros(n, dtype=np.float64)
    psum = np.zeros(n, dtype=np.float64)
    klo = None if key_lo is None else np.ascontiguousarray(key_lo, dtype=np.int64)
    khi = None if key_hi is None else np.ascontiguousarray(key_hi, dtype=np.int64)
    rc = lib.mco_attn_rows(_DTYPES[dtype], _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(bt), bt.shape[1],
                           _ptr(pl), _ptr(nl), B, num_q_heads, num_kv_heads, D, S, _scale(scale, D),
                           n, _ptr(rows), _ptr(klo), _ptr(khi), _ptr(out), _ptr(lse), _ptr(psum))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return out, lse, psum


def prefill_attn_paged(dtype: str, q, k_pool, v_pool, block_tables, prefix_lens, new_lens,
                       num_q_heads: int, num_kv_heads: int, scale: Optional[float] = None):
    """All rows: (out [total_new, Hq, D] f64, lse [total_new, Hq] f64, psum like lse)."""
    nl = np.asarray(new_lens, dtype=np.int32)
    D = k_pool.shape[3]
    total = int(nl.sum())
    rows = np.empty((total * num_q_heads, 3), dtype=np.int32)
    t = 0
    for r in range(nl.shape[0]):
        c = int(nl[r])
        blk = rows[t:t + c * num_q_heads].reshape(c, num_q_heads, 3)
        blk[:, :, 0] = r
        blk[:, :, 1] = np.arange(num_q_heads)[None, :]
        blk[:, :, 2] = np.arange(c)[:, None]
        t += c * num_q_heads
    out, lse, psum = attn_rows(dtype, q, k_pool, v_pool, block_tables, prefix_lens, new_lens,
                               num_q_heads, num_kv_heads, rows, scale)
    return (out.reshape(total, num_q_heads, D), lse.reshape(total, num_q_heads),
            psum.reshape(total, num_q_heads))


def case_rows(case, rows, scale=None, key_lo=None, key_hi=None):
    """``attn_rows`` on a workloads.AttnCase-shaped object (duck-typed; nothing imported)."""
    return attn_rows(case.dtype, case.q, case.k_pool, case.v_pool, case.block_tables, case.prefix_lens,
                     case.new_lens, case.num_q_heads, case.num_kv_heads, rows, scale, key_lo, key_hi)


def case_full(case, scale=None):
    return prefill_attn_paged(case.dtype, case.q, case.k_pool, case.v_pool, case.block_tables,
                              case.prefix_lens, case.new_lens, case.num_q_heads, case.num_kv_heads, scale)


def kv_pack_layer(k_pool: np.ndarray, v_pool: np.ndarray, page_ids, threads: int = 1):
    """Gather pages [N, page_bytes] uint8 -> contiguous (k_out, v_out) [n, page_bytes] in list order."""
    lib = _load()
    k_pool = np.ascontiguousarray(k_pool).view(np.uint8).reshape(k_pool.shape[0], -1)
    v_pool = np.ascontiguousarray(v_pool).view(np.uint8).reshape(v_pool.shape[0], -1)
    ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    N, pb = k_pool.shape
    n = ids.shape[0]
    k_out = np.zeros((n, pb), dtype=np.uint8)
    v_out = np.zeros((n, pb), dtype=np.uint8)
    rc = lib.mco_kv_pack_layer(_ptr(k_pool), _ptr(v_pool), N, pb, _ptr(ids), n, _ptr(k_out), _ptr(v_out), threads)
    if rc != 0:
        raise ValueError("page id outside the pool")
    return k_out, v_out


def kv_unpack_layer(k_in: np.ndarray, v_in: np.ndarray, page_ids, k_pool: np.ndarray, v_pool: np.ndarray,
                    threads: int = 1) -> None:
    """Scatter contiguous pages into the listed pages of (k_pool, v_pool) [N, page_bytes] uint8, in place."""
    lib = _load()
    assert k_pool.dtype == np.uint8 and v_pool.dtype == np.uint8 and k_pool.flags.c_contiguous and v_pool.flags.c_contiguous
    k_in = np.ascontiguousarray(k_in).view(np.uint8).reshape(k_in.shape[0], -1)
    v_in = np.ascontiguousarray(v_in).view(np.uint8).reshape(v_in.shape[0], -1)
    ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    assert len(np.unique(ids)) == len(ids), "unpack needs unique destination pages"
    N, pb = k_pool.shape
    n = ids.shape[0]
    assert k_in.shape == (n, pb) and v_in.shape == (n, pb)
    rc = lib.mco_kv_unpack_layer(_ptr(k_in), _ptr(v_in), N, pb, _ptr(ids), n, _ptr(k_pool), _ptr(v_pool), threads)
    if rc != 0:
        raise ValueError("page id outside the pool")


def kv_append_paged(k_new: np.ndarray, v_new: np.ndarray, k_pool: np.ndarray, v_pool: np.ndarray,
                    block_tables, prefix_lens, new_lens) -> None:
    """Write new tokens' K/V rows [total_new, Hkv, D] into their page slots of pools [N, Hkv, S, D], in place."""
    lib = _load()
    assert k_pool.flags.c_contiguous and v_pool.flags.c_contiguous and k_pool.shape == v_pool.shape
    N, Hkv, S, D = k_pool.shape
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    assert k_new.dtype == k_pool.dtype and v_new.dtype == v_pool.dtype
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    pl = np.ascontiguousarray(prefix_lens, dtype=np.int32)
    nl = np.ascontiguousarray(new_lens, dtype=np.int32)
    assert k_new.shape == (int(nl.sum()), Hkv, D) and v_new.shape == k_new.shape
    rc = lib.mco_kv_append_paged(_ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool), N, _ptr(bt), bt.shape[1],
                                 _ptr(pl), _ptr(nl), pl.shape[0], Hkv, S, D * k_pool.itemsize)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")


def attn_merge_lse(o_parts: np.ndarray, lse_parts: np.ndarray):
    """Merge partial attention results over disjoint key subsets.

    ``o_parts`` [n_parts, rows, D] and ``lse_parts`` [n_parts, rows] are float32 (the form the
    partials are stored in); returns (out [rows, D] f64, lse [rows] f64).
    """
    lib = _load()
    assert o_parts.dtype == np.float32 and lse_parts.dtype == np.float32
    o_parts = np.ascontiguousarray(o_parts)
    lse_parts = np.ascontiguousarray(lse_parts)
    n_parts, rows, D = o_parts.shape
    assert lse_parts.shape == (n_parts, rows)
    out = np.zeros((rows, D), dtype=np.float64)
    lse = np.zeros(rows, dtype=np.float64)
    rc = lib.mco_attn_merge_lse(_ptr(o_parts), _ptr(lse_parts), n_parts, rows, D, _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return out, lse


def mix64(x: int) -> int:
    """The 64-bit mixing function the prefix keys are built from (the splitmix64 output function)."""
    return int(_load().mco_mix64(ctypes.c_uint64(x & 0xFFFFFFFFFFFFFFFF)))


def prefix_hash(tokens, tok_offsets, block_tokens: int = 512):
    """Chained block keys of every request: (keys uint64 [total_blocks], key_offsets int64 [batch + 1])."""
    lib = _load()
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    off = np.ascontiguousarray(tok_offsets, dtype=np.int64)
    batch = off.shape[0] - 1
    blocks = (-(-np.diff(off) // block_tokens)) if batch > 0 else np.zeros(0, dtype=np.int64)
    key_off = np.zeros(batch + 1, dtype=np.int64)
    np.cumsum(blocks, out=key_off[1:])
    keys = np.zeros(int(key_off[-1]), dtype=np.uint64)
    n = lib.mco_prefix_hash(_ptr(tokens), _ptr(off), batch, block_tokens, _ptr(keys))
    if n != keys.shape[0]:
        raise ValueError("oracle rejected its arguments")
    return keys, key_off


def prefix_match(keys, key_offsets, cache_keys, cache_offsets):
    """(prefix_len int32 [batch, n_inst], best_len int32 [batch], best_inst int32 [batch])."""
    lib = _load()
    keys = np.ascontiguousarray(keys, dtype=np.uint64)
    koff = np.ascontiguousarray(key_offsets, dtype=np.int64)
    ck = np.ascontiguousarray(cache_keys, dtype=np.uint64)
    coff = np.ascontiguousarray(cache_offsets, dtype=np.int64)
    batch, n_inst = koff.shape[0] - 1, coff.shape[0] - 1
    plen = np.zeros((batch, n_inst), dtype=np.int32)
    best_len = np.zeros(batch, dtype=np.int32)
    best_inst = np.zeros(batch, dtype=np.int32)
    rc = lib.mco_prefix_match(_ptr(keys), _ptr(koff), batch, _ptr(ck), _ptr(coff), n_inst, _ptr(plen), _ptr(best_len),
                              _ptr(best_inst))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return plen, best_len, best_inst


def kv_check_page_ids(page_ids, num_pages: int):
    """(how many ids lie outside [0, num_pages), position of the first of them or len(page_ids) if none): one pass
    over the list, by its definition."""
    count, first = 0, len(page_ids)
    for i, v in enumerate(page_ids):
        if int(v) < 0 or int(v) >= num_pages:
            count += 1
            if first == len(page_ids):
                first = i
    return count, first


def kv_page_order(page_ids) -> np.ndarray:
    """order[r] = position in ``page_ids`` of the r-th smallest id, equal ids in list order: the stable
    ascending sort of the positions, by the library's stable argsort."""
    ids = np.ascontiguousarray(page_ids, dtype=np.int32)
    return np.argsort(ids, kind="stable").astype(np.int32)
