"""Seeded synthetic inputs for the KVCache-reuse hot path.

This module only draws random numbers and lays bytes out in memory: Q for the
new tokens of each request, K/V scattered into a paged pool through a random
block table, page-id lists for layer-wise pack/unpack.  It holds none of the
method's arithmetic (no scores, no softmax, no page copies), so both the CPU
oracle's tests and the HIP path's tests may use it without sharing code.

Shapes follow the paper's workloads: a dummy LLaMA2-70B architecture
(Section 8, testbed: 64 query heads / 8 KV heads / head_dim 128 / 80 layers),
simulated long-context prompts of 16k..128k tokens with half of them cached
(Table "datasets"), and incremental prefill of the uncached tokens in chunks
(Section 3, step 2).  All values are synthetic N(0,1) draws.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np

BF16 = "bf16"
F32 = "f32"

#: bf16 quiet-NaN bit pattern used to poison memory that must never be read as a value
BF16_NAN_BITS = 0x7FC1
F32_NAN_BITS = 0x7FC00001

BASE_SEED = 20240700


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if nan.any():
        out[nan] = BF16_NAN_BITS
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly to float32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored tensor (bf16 bits or float32) to float64."""
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    return f32_to_bf16_bits(x32) if dtype == BF16 else np.ascontiguousarray(x32, dtype=np.float32)


def _storage_np(dtype: str):
    return np.uint16 if dtype == BF16 else np.float32


def _poison_value(dtype: str):
    if dtype == BF16:
        return np.uint16(BF16_NAN_BITS)
    return np.array([F32_NAN_BITS], dtype=np.uint32).view(np.float32)[0]


@dataclasses.dataclass
class AttnCase:
    """One batch for ``mc_prefill_attn_paged``.

    q            [total_new, Hq, D]       stored dtype (uint16 bf16 bits or float32)
    k_pool       [N, Hkv, S, D]           stored dtype, one layer
    v_pool       [N, Hkv, S, D]
    block_tables [B, max_pages] int32     logical page -> physical page id
    prefix_lens  [B] int32                P_r, tokens whose KV was reused
    new_lens     [B] int32                C_r, tokens computed by this call
    """
    dtype: str
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    num_pages: int
    q: np.ndarray
    k_pool: np.ndarray
    v_pool: np.ndarray
    block_tables: np.ndarray
    prefix_lens: np.ndarray
    new_lens: np.ndarray
    seed: int
    #: un-paged copies [L_r, Hkv, D] per request (only kept when keep_logical=True)
    k_logical: Optional[List[np.ndarray]] = None
    v_logical: Optional[List[np.ndarray]] = None

    @property
    def batch(self) -> int:
        return int(self.prefix_lens.shape[0])

    @property
    def total_new(self) -> int:
        return int(self.new_lens.sum())

    @property
    def max_pages(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def q_offsets(self) -> np.ndarray:
        off = np.zeros(self.batch + 1, dtype=np.int64)
        np.cumsum(self.new_lens, out=off[1:])
        return off

    def visible_pairs(self) -> int:
        """Sum over requests of C*P + C*(C+1)/2: query-key pairs the causal rule lets through."""
        p = self.prefix_lens.astype(np.int64)
        c = self.new_lens.astype(np.int64)
        return int((c * p + c * (c + 1) // 2).sum())

    def flops(self) -> int:
        """Algorithmic flops: both contractions over visible pairs only, softmax not counted."""
        return 4 * self.head_dim * self.num_q_heads * self.visible_pairs()


def make_attn_case(seed: int, dtype: str, num_q_heads: int, num_kv_heads: int, head_dim: int,
                   page_size: int, prefix_lens, new_lens, num_pages: int,
                   poison: bool = True, keep_logical: bool = False,
                   q_scale: float = 1.0, shared_prefix_pages: int = 0,
                   logical=None) -> AttnCase:
    """Draw Q, K, V ~ N(0,1) and scatter K/V into a paged pool.

    Each request takes a disjoint slice of one seeded permutation of the
    ``num_pages`` physical page ids.  With ``shared_prefix_pages`` > 0 every
    request's first that-many logical pages alias the SAME physical pages
    (true prefix reuse, read-only) and hold identical values.  Pages nobody
    references and token slots past a request's length in its last page are
    filled with a NaN pattern when ``poison`` is set, so that a stray read
    shows up in the result.  ``logical`` = (q, [k_r], [v_r]) in the stored
    dtype re-uses given tensors instead of drawing new ones (same values under
    another paging).
    """
    rng = np.random.default_rng(seed)
    prefix_lens = np.asarray(prefix_lens, dtype=np.int32).reshape(-1)
    new_lens = np.asarray(new_lens, dtype=np.int32).reshape(-1)
    assert prefix_lens.shape == new_lens.shape
    B = prefix_lens.shape[0]
    S, D, Hkv, Hq = page_size, head_dim, num_kv_heads, num_q_heads
    tot_lens = prefix_lens.astype(np.int64) + new_lens.astype(np.int64)
    pages_per_req = (tot_lens + S - 1) // S
    max_pages = int(max(1, pages_per_req.max() if B else 1))
    own_pages = np.maximum(pages_per_req - shared_prefix_pages, 0)
    need = int(own_pages.sum()) + shared_prefix_pages
    assert need <= num_pages, f"pool of {num_pages} pages cannot hold {need}"
    perm = rng.permutation(num_pages).astype(np.int32)

    st = _storage_np(dtype)
    if poison:
        k_pool = np.full((num_pages, Hkv, S, D), _poison_value(dtype), dtype=st)
        v_pool = np.full((num_pages, Hkv, S, D), _poison_value(dtype), dtype=st)
    else:
        k_pool = np.zeros((num_pages, Hkv, S, D), dtype=st)
        v_pool = np.zeros((num_pages, Hkv, S, D), dtype=st)
    block_tables = np.zeros((B, max_pages), dtype=np.int32)

    total_new = int(new_lens.sum())
    if logical is None:
        q32 = rng.standard_normal((total_new, Hq, D), dtype=np.float32)
        if q_scale != 1.0:
            q32 *= np.float32(q_scale)
        q = _store(q32, dtype)
        del q32
    else:
        q = np.ascontiguousarray(logical[0], dtype=st)
        assert q.shape == (total_new, Hq, D)

    shared_ids = perm[:shared_prefix_pages]
    shared_k = shared_v = None
    if shared_prefix_pages:
        shared_k = _store(rng.standard_normal((shared_prefix_pages * S, Hkv, D), dtype=np.float32), dtype)
        shared_v = _store(rng.standard_normal((shared_prefix_pages * S, Hkv, D), dtype=np.float32), dtype)

    k_logical = [] if keep_logical else None
    v_logical = [] if keep_logical else None
    cursor = shared_prefix_pages
    for r in range(B):
        L = int(tot_lens[r])
        npg = int(pages_per_req[r])
        nshared = min(shared_prefix_pages, npg)
        ids = np.concatenate([shared_ids[:nshared], perm[cursor:cursor + int(own_pages[r])]])
        cursor += int(own_pages[r])
        block_tables[r, :npg] = ids
        if logical is None:
            kr = _store(rng.standard_normal((L, Hkv, D), dtype=np.float32), dtype)
            vr = _store(rng.standard_normal((L, Hkv, D), dtype=np.float32), dtype)
        else:
            kr = np.ascontiguousarray(logical[1][r], dtype=st)
            vr = np.ascontiguousarray(logical[2][r], dtype=st)
            assert kr.shape == (L, Hkv, D) and vr.shape == (L, Hkv, D)
        if nshared:
            n_tok = min(nshared * S, L)
            kr[:n_tok] = shared_k[:n_tok]
            vr[:n_tok] = shared_v[:n_tok]
        if L:
            full = L // S
            if full:
                k_pool[ids[:full]] = kr[:full * S].reshape(full, S, Hkv, D).transpose(0, 2, 1, 3)
                v_pool[ids[:full]] = vr[:full * S].reshape(full, S, Hkv, D).transpose(0, 2, 1, 3)
            tail = L - full * S
            if tail:
                k_pool[ids[full], :, :tail, :] = kr[full * S:].transpose(1, 0, 2)
                v_pool[ids[full], :, :tail, :] = vr[full * S:].transpose(1, 0, 2)
        if keep_logical:
            k_logical.append(kr)
            v_logical.append(vr)
    return AttnCase(dtype, Hq, Hkv, D, S, num_pages, q, k_pool, v_pool, block_tables,
                    prefix_lens, new_lens, seed, k_logical, v_logical)


@dataclasses.dataclass
class PackCase:
    """Inputs for ``mc_kv_pack_layer`` / ``mc_kv_unpack_layer`` over ``layers`` layers.

    k_pools, v_pools [layers, N, page_bytes] uint8   scattered source pools
    src_ids          [n] int32                       pages to pack, logical order
    dst_ids          [n] int32                       unique destination pages in a pool of N2
    """
    layers: int
    num_pages: int
    num_pages_dst: int
    page_bytes: int
    k_pools: np.ndarray
    v_pools: np.ndarray
    src_ids: np.ndarray
    dst_ids: np.ndarray
    seed: int


def make_pack_case(seed: int, layers: int, num_pages: int, num_pages_dst: int, page_bytes: int,
                   n: int, unique_src: bool = True) -> PackCase:
    """Random bytes in every page of every layer's pools, and two independent page-id lists."""
    rng = np.random.default_rng(seed)
    k_pools = rng.integers(0, 256, size=(layers, num_pages, page_bytes), dtype=np.uint8)
    v_pools = rng.integers(0, 256, size=(layers, num_pages, page_bytes), dtype=np.uint8)
    if unique_src:
        assert n <= num_pages
        src = rng.permutation(num_pages)[:n].astype(np.int32)
    else:
        src = rng.integers(0, num_pages, size=n).astype(np.int32)
    assert n <= num_pages_dst
    dst = rng.permutation(num_pages_dst)[:n].astype(np.int32)
    return PackCase(layers, num_pages, num_pages_dst, page_bytes, k_pools, v_pools, src, dst, seed)


# ---------------------------------------------------------------------------
# The five named configurations
# ---------------------------------------------------------------------------

def config_shapes(idx: int, seed: Optional[int] = None) -> dict:
    """Shape recipe of configuration ``idx`` (1..5); lengths for 4 are drawn from the seed."""
    seed = BASE_SEED + idx if seed is None else seed
    if idx == 1:
        return dict(seed=seed, dtype=F32, num_q_heads=4, num_kv_heads=1, head_dim=64, page_size=16,
                    prefix_lens=[256], new_lens=[128], num_pages=64)
    if idx == 2:
        return dict(seed=seed, dtype=BF16, num_q_heads=64, num_kv_heads=8, head_dim=128, page_size=16,
                    prefix_lens=[8192], new_lens=[8192], num_pages=4096)
    if idx == 3:
        return dict(seed=seed, dtype=BF16, num_q_heads=8, num_kv_heads=1, head_dim=128, page_size=16,
                    prefix_lens=[122880], new_lens=[8192], num_pages=16384)
    if idx == 4:
        rng = np.random.default_rng(seed)
        B = 16
        prefix = (rng.integers(0, 32768, size=B, endpoint=True) // 16) * 16
        # median 2048 (mu = ln 2048), sigma 1 of the underlying normal
        new = np.clip(np.rint(rng.lognormal(mean=np.log(2048.0), sigma=1.0, size=B)), 1, 8192)
        return dict(seed=seed, dtype=BF16, num_q_heads=64, num_kv_heads=8, head_dim=128, page_size=16,
                    prefix_lens=prefix.astype(np.int32).tolist(), new_lens=new.astype(np.int32).tolist(),
                    num_pages=65536)
    if idx == 5:
        return dict(seed=seed, layers=80, num_kv_heads=8, head_dim=128, page_size=16, dtype=BF16,
                    tokens=32768, n=2048, page_bytes=16 * 8 * 128 * 2, num_pages=4096, num_pages_dst=4096)
    raise ValueError(f"no configuration {idx}")


def make_config_attn(idx: int, poison: bool = True, keep_logical: bool = False,
                     seed: Optional[int] = None) -> AttnCase:
    sh = config_shapes(idx, seed)
    assert idx in (1, 2, 3, 4)
    return make_attn_case(poison=poison, keep_logical=keep_logical, **sh)


def sample_rows(case: AttnCase, n_random: int, seed: int, tile_rows=(32, 64, 128, 256)) -> np.ndarray:
    """Pick (request, head, row) triples for spot checks at sizes the oracle cannot sweep.

    Always holds each request's first and last rows, rows around page and
    query-tile boundaries, and every head for a few rows; the rest is uniform.
    Returns int32 [n, 3].
    """
    rng = np.random.default_rng(seed)
    Hq, S = case.num_q_heads, case.page_size
    G = Hq // case.num_kv_heads
    picks = set()
    for r in range(case.batch):
        C = int(case.new_lens[r])
        P = int(case.prefix_lens[r])
        if C == 0:
            continue
        rows = {0, C - 1, C // 2}
        for t in tile_rows:
            step = max(1, t // G)
            for b in (step, 2 * step, (C // step) * step):
                rows.update({b - 1, b, b + 1})
        first_page_edge = (S - P % S) % S
        rows.update({first_page_edge - 1, first_page_edge, first_page_edge + S - 1, first_page_edge + S})
        rows = sorted(i for i in rows if 0 <= i < C)
        for i in rows:
            for h in {0, Hq - 1, int(rng.integers(0, Hq))}:
                picks.add((r, h, i))
        for h in range(Hq):
            picks.add((r, h, C - 1))
            picks.add((r, h, 0))
    nz = np.nonzero(case.new_lens)[0]
    while len(picks) < n_random and len(nz):
        r = int(rng.choice(nz))
        picks.add((r, int(rng.integers(0, Hq)), int(rng.integers(0, int(case.new_lens[r])))))
    return np.array(sorted(picks), dtype=np.int32).reshape(-1, 3)
