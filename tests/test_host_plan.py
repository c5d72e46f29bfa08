"""The attention work list the host builds (mc_prefill_attn_plan: no GPU call): coverage, order, bounds."""
import os

import pytest

from paper_2407_00079_amd import binding as B
from paper_2407_00079_amd import workloads as W

ROWS = 256          # stacked query rows per work item


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2407_00079_amd import build
        build.build()
    return B.lib()


def expected(Hq, Hkv, prefix, new, kv_splits):
    """Every (request, head, tile, slice) with its cost, by enumeration."""
    G = Hq // Hkv
    out = {}
    for r, (P, C) in enumerate(zip(prefix, new)):
        tiles_of_request = -(-(P + C) // 64)
        per = -(-tiles_of_request // max(kv_splits, 1)) * 64
        for g in range(Hkv):
            for row0 in range(0, C * G, ROWS):
                tok_last = min(C - 1, (row0 + ROWS - 1) // G)
                keys = P + tok_last + 1
                if kv_splits == 0:
                    out[(r, g, row0, 0)] = keys
                else:
                    for s in range(kv_splits):
                        out[(r, g, row0, s)] = max(0, min(keys, (s + 1) * per) - s * per)
    return out


CASES = [
    (64, 8, [8192], [8192], 0),                       # configuration 2
    (8, 1, [122880], [8192], 0),                      # configuration 3
    (64, 8, [100, 0, 7, 3000], [0, 33, 1, 700], 0),   # empty request, ragged tiles, one token
    (16, 16, [5], [40], 0),                           # 16 KV heads: two heads per list
    (12, 3, [999, 1], [130, 257], 0),                 # 3 KV heads: five of the eight lists stay empty
    (64, 8, [131056], [16], 32),                      # small chunk, 32 slices
    (8, 2, [700, 30], [40, 150], 3),                  # split with ragged lengths
    (8, 2, [100, 5], [1, 60], 16),                    # more slices than tiles: empty slices still get an item
]


@pytest.mark.parametrize("Hq,Hkv,prefix,new,kv_splits", CASES)
def test_plan_covers_every_tile_once_in_dealing_order(Hq, Hkv, prefix, new, kv_splits):
    p = B.attn_params(Hq, Hkv, 128, 16, 1 << 20, "bf16")
    plan = B.mc_prefill_attn_plan(p, prefix, new, kv_splits)
    want = expected(Hq, Hkv, prefix, new, kv_splits)
    assert len(plan) == len(set(plan)) == len(want)
    assert set(plan) == set(want)
    # eight lists by (request * Hkv + head + slice) mod 8, each longest first
    lists = {x: [] for x in range(8)}
    for it in plan:
        lists[(it[0] * Hkv + it[1] + it[3]) % 8].append(it)
    for x, l in lists.items():
        costs = [want[it] for it in l]
        assert costs == sorted(costs, reverse=True), f"list {x} is not longest first"
    # dealt round-robin: dealing the eight lists again, skipping empty ones, gives the plan back
    cur, x, redeal = {k: 0 for k in lists}, 0, []
    while len(redeal) < len(plan):
        while cur[x] >= len(lists[x]):
            x = (x + 1) % 8
        redeal.append(lists[x][cur[x]])
        cur[x] += 1
        x = (x + 1) % 8
    assert redeal == plan
    # the workspace the size call asks for holds this list and the request table
    total_new = sum(new)
    need = (B.mc_prefill_attn_split_workspace_bytes(p, len(prefix), total_new, kv_splits) if kv_splits
            else B.mc_prefill_attn_workspace_bytes(p, len(prefix), total_new))
    assert need >= 16 * len(plan) + 16 * len(prefix)


def test_plan_of_the_mixed_configuration():
    sh = W.config_shapes(4)
    p = B.attn_params(64, 8, 128, 16, sh["num_pages"], "bf16")
    plan = B.mc_prefill_attn_plan(p, sh["prefix_lens"], sh["new_lens"], 0)
    want = expected(64, 8, sh["prefix_lens"], sh["new_lens"], 0)
    assert set(plan) == set(want) and len(plan) == len(want)
    # with 8 KV heads every list holds one head of every request: the first 8 items are the 8 heads of the
    # longest tile, one per XCD
    first = plan[:8]
    assert sorted(it[1] for it in first) == list(range(8))
    assert len({want[it] for it in first}) == 1 and want[first[0]] == max(want.values())


def test_plan_rejections_and_count_only():
    import ctypes
    p = B.attn_params(64, 8, 128, 16, 4096, "bf16")
    n = ctypes.c_int64(-1)
    pl, nl = (ctypes.c_int32 * 1)(8192), (ctypes.c_int32 * 1)(8192)
    call = B.lib().mc_prefill_attn_plan
    assert call(ctypes.byref(p), pl, nl, 1, 0, None, 0, ctypes.byref(n)) == B.MC_OK and n.value == 2048
    small = (ctypes.c_int32 * 40)(*([-5] * 40))
    assert call(ctypes.byref(p), pl, nl, 1, 0, small, 10, ctypes.byref(n)) == B.MC_ERR_WORKSPACE
    assert list(small) == [-5] * 40 and n.value == 2048
    assert call(ctypes.byref(p), pl, nl, 1, 0, None, 0, None) == B.MC_ERR_NULL
    assert call(ctypes.byref(p), pl, nl, 1, B.MC_MAX_KV_SPLITS + 1, None, 0, ctypes.byref(n)) == B.MC_ERR_SHAPE
    neg = (ctypes.c_int32 * 1)(-3)
    assert call(ctypes.byref(p), neg, nl, 1, 0, None, 0, ctypes.byref(n)) == B.MC_ERR_SHAPE
    bad = B.attn_params(64, 8, 96, 16, 4096, "bf16")
    assert call(ctypes.byref(bad), pl, nl, 1, 0, None, 0, ctypes.byref(n)) == B.MC_ERR_UNSUPPORTED
    assert B.mc_prefill_attn_plan(p, [], [], 0) == []
    assert B.mc_prefill_attn_plan(p, [10, 20], [0, 0], 4) == []
