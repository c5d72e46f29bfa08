"""GPU parity on seeded random small shapes: whole-row attention and split + merge against the CPU oracle,
every output row.  The shapes mix head groupings, unaligned prefixes, empty and one-token chunks and batches.

24 seeds by default; MC_RANDOM_SEEDS=lo:hi runs another range (seeds from 24 on draw larger shapes, groups of
up to 16 heads and Q scaled by up to 8 for peaked rows), e.g. MC_RANDOM_SEEDS=24:2000 for a long sweep."""
import os

import numpy as np
import pytest
import torch

from paper_2407_00079_amd import binding as B
from paper_2407_00079_amd import workloads as W

from gpu_util import TOL, DeviceCase, check_close

pytestmark = pytest.mark.gpu


def random_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    big = seed >= 24
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8, 16] if big else [1, 2, 4, 8]))
    batch = int(rng.integers(1, 6 if big else 5))
    prefix = [int(rng.choice([0, rng.integers(0, 3000 if big else 700)])) for _ in range(batch)]
    new = [int(rng.choice([0, 1, rng.integers(1, 600 if big else 330)])) for _ in range(batch)]
    if sum(new) == 0:
        new[0] = 17
    while sum(c * (p + c) for p, c in zip(prefix, new)) * Hkv * G > 6e8:    # keep the oracle within seconds
        new = [max(c // 2, 1) if c else 0 for c in new]
    dtype, D = (W.F32, 64) if seed % 6 == 5 else (W.BF16, 64) if seed % 6 == 2 else (W.BF16, 128)
    pages = sum(-(-(p + c) // 16) for p, c in zip(prefix, new)) + 8
    q_scale = float(rng.choice([1.0, 1.0, 3.0, 8.0])) if big else 1.0
    return dtype, Hkv * G, Hkv, D, prefix, new, pages, q_scale


def _seeds():
    spec = os.environ.get("MC_RANDOM_SEEDS")
    if not spec:
        return range(24)
    lo, hi = spec.split(":")
    return range(int(lo), int(hi))


@pytest.mark.parametrize("seed", _seeds())
def test_random_shapes_match_oracle(oracle, seed):
    dtype, Hq, Hkv, D, prefix, new, pages, q_scale = random_shape(seed)
    print(f"random case {seed}: {dtype} Hq={Hq} Hkv={Hkv} prefix={prefix} new={new} q_scale={q_scale}", flush=True)
    case = W.make_attn_case(2000 + seed, dtype, Hq, Hkv, D, 16, prefix, new, pages, q_scale=q_scale)
    ref_out, ref_lse, _ = oracle.case_full(case)
    dc = DeviceCase(case)
    dc.run()
    out, lse = dc.result()
    check_close(out, ref_out, dtype, "whole rows")
    assert np.abs(lse - ref_lse).max() <= TOL[dtype]["lse_abs"]
    # the same through key slices and the merge
    kv_splits = 1 + seed % 5
    n = case.total_new * Hq
    o_parts = torch.full((kv_splits, case.total_new, Hq, D), float("nan"), dtype=torch.float32, device="cuda:0")
    l_parts = torch.full((kv_splits, case.total_new, Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(B.mc_prefill_attn_split_workspace_bytes(dc.params, case.batch, case.total_new, kv_splits),
                     dtype=torch.uint8, device="cuda:0")
    B.mc_prefill_attn_paged_split(dc.params, dc.q, dc.k_pool, dc.v_pool, dc.block_tables, prefix, new, kv_splits,
                                  o_parts, l_parts, ws)
    out2 = torch.full_like(dc.out, float("nan"))
    lse2 = torch.full_like(dc.lse, float("nan"))
    B.mc_attn_merge_lse(o_parts, l_parts, kv_splits, n, D, dc.params.dtype, out2, lse2)
    torch.cuda.synchronize()
    check_close(out2.float().cpu().numpy().astype(np.float64), ref_out, dtype, "split + merge")
    assert np.abs(lse2.cpu().numpy().astype(np.float64) - ref_lse).max() <= TOL[dtype]["lse_abs"]
