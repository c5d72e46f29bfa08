"""Key slices of split attention as the interface defines them, and the oracle's partial results over them."""
import numpy as np


def slice_bounds(L, kv_splits, tile=64):
    """Key range of every slice: whole 64-key tiles, ceil(tiles / kv_splits) per slice, the tail slices may be empty."""
    tiles = -(-L // tile)
    per = -(-tiles // kv_splits)
    return [(min(s * per * tile, L), min((s + 1) * per * tile, L)) for s in range(kv_splits)]


def all_rows(case):
    return np.array([(r, h, i) for r in range(case.batch) for i in range(int(case.new_lens[r]))
                     for h in range(case.num_q_heads)], dtype=np.int32)


def oracle_partials(oracle, case, kv_splits):
    """Partials over the key slices of every request, from the oracle's own range-restricted rows (fp64 -> fp32)."""
    rows = all_rows(case)
    n = rows.shape[0]
    o = np.zeros((kv_splits, n, case.head_dim), dtype=np.float32)
    l = np.zeros((kv_splits, n), dtype=np.float32)
    for s in range(kv_splits):
        lo = np.empty(n, dtype=np.int64)
        hi = np.empty(n, dtype=np.int64)
        for r in range(case.batch):
            b = slice_bounds(int(case.prefix_lens[r] + case.new_lens[r]), kv_splits)[s]
            sel = rows[:, 0] == r
            lo[sel], hi[sel] = b
        oo, ll, _ = oracle.case_rows(case, rows, key_lo=lo, key_hi=hi)
        o[s], l[s] = oo, ll
    return rows, o, l
