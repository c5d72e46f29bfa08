"""Input shaping shared by the append tests: pools as they stand before a chunk is stored, and the chunk's rows."""
import numpy as np

from paper_2407_00079_amd import workloads as W


def empty_chunk_pools(case):
    """Pools as they are BEFORE the chunk is appended: the chunk's slots hold a marker, everything else as built."""
    k, v = case.k_pool.copy(), case.v_pool.copy()
    marker = np.array(0x1234 if case.dtype == W.BF16 else 7.25).astype(k.dtype)
    for r in range(case.batch):
        P, C = int(case.prefix_lens[r]), int(case.new_lens[r])
        for pos in range(P, P + C):
            pg = case.block_tables[r, pos // case.page_size]
            k[pg, :, pos % case.page_size, :] = marker
            v[pg, :, pos % case.page_size, :] = marker
    return k, v


def new_rows(case):
    k_new = np.concatenate([case.k_logical[r][int(case.prefix_lens[r]):] for r in range(case.batch)])
    v_new = np.concatenate([case.v_logical[r][int(case.prefix_lens[r]):] for r in range(case.batch)])
    return k_new, v_new
