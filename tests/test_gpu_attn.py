"""GPU parity: mc_prefill_attn_paged against the fp64 CPU oracle.

Tolerances (vs the fp64 oracle on the same stored inputs): bf16 max-abs 2e-2 and
relative L2 1e-2; f32 max-abs 1e-4 and relative L2 1e-5.
"""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2407_00079_amd import binding as B
from paper_2407_00079_amd import workloads as W
from gpu_util import DeviceCase, check_close, gather_rows, TOL

pytestmark = pytest.mark.gpu


def run_full(oracle, case, scale=0.0, what=""):
    print(f"attn case {what} dtype={case.dtype} Hq={case.num_q_heads} Hkv={case.num_kv_heads} "
          f"P={case.prefix_lens.tolist()} C={case.new_lens.tolist()} seed={case.seed}", flush=True)
    dc = DeviceCase(case)
    dc.run(scale)
    out, lse = dc.result()
    ref, lse_ref, _ = oracle.case_full(case, scale or None)
    check_close(out, ref, case.dtype, what)
    lse_err, lse_tol = np.abs(lse - lse_ref).max(), TOL[case.dtype]["lse_abs"]
    print(f"attn case {what}: max |lse - oracle| {lse_err:.3e} of {lse_tol:.1e} allowed", flush=True)
    assert lse_err <= lse_tol, f"{what}: lse off by {lse_err}"
    return out, lse


def test_config1_tiny_fp32(oracle):
    case = W.make_config_attn(1)
    run_full(oracle, case, what="config 1")


@pytest.mark.parametrize("Hq,Hkv,P,C", [
    (8, 1, [256], [128]),              # several Q tiles, prefix + diagonal tiles
    (8, 1, [0], [200]),                # no prefix: ordinary causal prefill, ragged tail
    (16, 2, [100], [37]),              # prefix not page aligned, partial last page
    (8, 8, [64], [130]),               # MHA (G = 1): long diagonal
    (4, 2, [33, 0, 512, 16], [5, 17, 1, 70]),   # varlen batch incl. a single-row request
    (24, 8, [48], [9]),                # G = 3: stacked rows need a real division
    (8, 1, [1000, 7], [0, 40]),        # a request with no rows
])
def test_bf16_small_shapes(oracle, Hq, Hkv, P, C):
    case = W.make_attn_case(100 + Hq + sum(C), W.BF16, Hq, Hkv, 128, 16, P, C, 256)
    run_full(oracle, case, what=f"bf16 {Hq}/{Hkv}")


@pytest.mark.parametrize("Hq,Hkv,P,C", [
    (8, 1, [256], [128]),              # several Q tiles, prefix + diagonal tiles
    (8, 2, [0], [200]),                # no prefix, ragged tail
    (16, 2, [100], [37]),              # prefix not page aligned, partial last page
    (4, 4, [64], [130]),               # MHA
    (4, 2, [33, 0, 512, 16], [5, 17, 1, 70]),   # varlen batch incl. a single-row request
    (8, 1, [2000], [300]),             # many pipelined tiles
])
def test_bf16_head_dim_64_small_shapes(oracle, Hq, Hkv, P, C):
    case = W.make_attn_case(300 + Hq + sum(C), W.BF16, Hq, Hkv, 64, 16, P, C, 256)
    run_full(oracle, case, what=f"bf16 D=64 {Hq}/{Hkv}")


@pytest.mark.parametrize("Hq,Hkv,P,C", [
    (4, 1, [0], [70]),
    (6, 2, [45, 16], [33, 1]),
    (2, 2, [130], [66]),
])
def test_fp32_small_shapes(oracle, Hq, Hkv, P, C):
    case = W.make_attn_case(200 + Hq + sum(C), W.F32, Hq, Hkv, 64, 16, P, C, 64)
    run_full(oracle, case, what=f"f32 {Hq}/{Hkv}")


def test_custom_scale_and_no_lse(oracle):
    case = W.make_attn_case(5, W.BF16, 8, 2, 128, 16, [80], [50], 64)
    run_full(oracle, case, scale=0.05, what="scale 0.05")
    dc = DeviceCase(case)
    dc.run(want_lse=False)
    out, lse = dc.result()
    assert np.isnan(lse).all()                      # untouched
    ref, _, _ = oracle.case_full(case)
    check_close(out, ref, case.dtype, "no lse")


def test_needle_through_block_table(oracle):
    """A key aligned with q dominates: the output must be that key's V row (pins page indirection, |O| ~ 1)."""
    Hq, Hkv, D, S, P, C = 8, 1, 128, 16, 720, 57
    L = P + C
    rng = np.random.default_rng(3)
    for needle in (0, 15, 16, 700, 719, 720, 775, L - 1):
        q = rng.standard_normal((C, Hq, D)).astype(np.float32)
        k = (0.01 * rng.standard_normal((L, Hkv, D))).astype(np.float32)
        v = rng.standard_normal((L, Hkv, D)).astype(np.float32)
        i = C - 1
        k[needle, 0] = 60.0 * q[i, 3] / np.linalg.norm(q[i, 3])
        case = W.make_attn_case(needle, W.BF16, Hq, Hkv, D, S, [P], [C], 128,
                                logical=(W.f32_to_bf16_bits(q), [W.f32_to_bf16_bits(k)], [W.f32_to_bf16_bits(v)]))
        out, _ = run_full(oracle, case, what=f"needle {needle}")
        v_row = W.bf16_bits_to_f32(W.f32_to_bf16_bits(v[needle, 0])).astype(np.float64)
        assert np.abs(out[i, 3] - v_row).max() <= 2e-2


def test_page_permutation_is_bitwise_invisible(oracle):
    base = W.make_attn_case(31, W.BF16, 8, 2, 128, 16, [300, 40], [90, 120], 128, keep_logical=True)
    other = W.make_attn_case(977, W.BF16, 8, 2, 128, 16, [300, 40], [90, 120], 512,
                             logical=(base.q, base.k_logical, base.v_logical))
    a = DeviceCase(base); a.run()
    b = DeviceCase(other); b.run()
    oa, la = a.result()
    ob, lb = b.result()
    np.testing.assert_array_equal(oa, ob)
    np.testing.assert_array_equal(la, lb)


def test_chunked_calls_match_one_call(oracle):
    """Section 3 step 2: chunks of the uncached tokens run one after another against a growing prefix."""
    case = W.make_attn_case(41, W.BF16, 8, 1, 128, 16, [128], [300], 64)
    whole, _ = run_full(oracle, case, what="one call")
    c1 = 112
    first = dataclasses.replace(case, q=case.q[:c1], new_lens=np.array([c1], np.int32))
    second = dataclasses.replace(case, q=case.q[c1:], prefix_lens=np.array([128 + c1], np.int32),
                                 new_lens=np.array([300 - c1], np.int32))
    o1, _ = run_full(oracle, first, what="chunk 1")
    o2, _ = run_full(oracle, second, what="chunk 2")
    ref, _, _ = oracle.case_full(case)
    check_close(np.concatenate([o1, o2]), ref, W.BF16, "chunks vs oracle")
    assert np.abs(np.concatenate([o1, o2]) - whole).max() <= 2e-2


def test_shared_prefix_pages(oracle):
    """Two requests alias the same physical prefix pages (true reuse), shaped like the paper's trace samples / 8."""
    case = W.make_attn_case(5, W.BF16, 8, 1, 128, 16, [768, 768], [101, 41], 256, shared_prefix_pages=48)
    run_full(oracle, case, what="shared prefix")


def test_large_scores(oracle):
    case = W.make_attn_case(81, W.BF16, 8, 1, 128, 16, [200], [40], 64, q_scale=30.0)
    run_full(oracle, case, what="q x30")


def test_bf16_head_dim_64_at_full_size_on_sampled_rows(oracle):
    """Configuration 2's lengths and heads with 128-byte rows: 2048 work items, every XCD list, many pipelined tiles."""
    case = W.make_attn_case(77, W.BF16, 64, 8, 64, 16, [8192], [8192], 1200)
    dc = DeviceCase(case)
    dc.run()
    out, lse = dc.result()
    assert np.isfinite(out).all() and np.isfinite(lse).all()     # every row written
    rows = W.sample_rows(case, 1100, seed=77)
    got, got_lse = gather_rows(out, lse, case, rows)
    ref, lse_ref, _ = oracle.case_rows(case, rows)
    max_abs, rel_l2 = check_close(got, ref, W.BF16, "bf16 head_dim 64, full size")
    lse_err = np.abs(got_lse - lse_ref).max()
    print(f"bf16 head_dim 64 full size: max_abs {max_abs:.3e} rel_l2 {rel_l2:.3e} lse {lse_err:.3e}", flush=True)
    assert lse_err <= TOL[W.BF16]["lse_abs"]


def test_scores_that_keep_outgrowing_the_reference(oracle):
    """Scores that rise along the keys at eight different rates, one per head (from 0.3 to 20 log2 units per 32-key
    block): the lazy softmax reference is outgrown by just under and just over its margin again and again, in the
    pipelined tiles (long prefix) and in the diagonal ones."""
    Hq, Hkv, D, S, P, C = 8, 1, 128, 16, 2000, 150
    L = P + C
    rng = np.random.default_rng(11)
    u = rng.standard_normal(D)
    u /= np.linalg.norm(u)
    rates = np.array([0.3, 3.0, 6.9, 7.4, 7.9, 8.1, 12.0, 20.0])               # log2 units per 32 keys
    ramp = (np.arange(L) / 32.0)[:, None, None]                                # blocks from key 0
    k = (ramp * u[None, None, :] + 0.05 * rng.standard_normal((L, Hkv, D))).astype(np.float32)
    v = rng.standard_normal((L, Hkv, D)).astype(np.float32)
    scale_log2e = np.log2(np.e) / np.sqrt(D)
    q = np.empty((C, Hq, D), np.float32)
    for h in range(Hq):
        q[:, h] = (rates[h] / scale_log2e) * u[None, :] + 0.05 * rng.standard_normal((C, D))
    case = W.make_attn_case(12, W.BF16, Hq, Hkv, D, S, [P], [C], 256,
                            logical=(W.f32_to_bf16_bits(q), [W.f32_to_bf16_bits(k)], [W.f32_to_bf16_bits(v)]))
    run_full(oracle, case, what="rising scores")


def test_outputs_do_not_depend_on_poison(oracle):
    case = W.make_attn_case(61, W.BF16, 8, 1, 128, 16, [37], [30], 32, keep_logical=True)
    clean = W.make_attn_case(61, W.BF16, 8, 1, 128, 16, [37], [30], 32, poison=False,
                             logical=(case.q, case.k_logical, case.v_logical))
    a = DeviceCase(case); a.run()
    b = DeviceCase(clean); b.run()
    np.testing.assert_array_equal(a.result()[0], b.result()[0])


@pytest.mark.parametrize("idx,n_rows", [(2, 1536), (3, 1100), (4, 1536)])
def test_full_size_configs_on_sampled_rows(oracle, idx, n_rows):
    """The benchmark configurations at full size; the oracle checks a seeded sample of rows."""
    case = W.make_config_attn(idx)
    print(f"config {idx}: flops {case.flops():.4e} P={case.prefix_lens.tolist()} C={case.new_lens.tolist()}", flush=True)
    dc = DeviceCase(case)
    dc.run()
    out, lse = dc.result()
    assert np.isfinite(out).all() and np.isfinite(lse).all()     # every row written
    rows = W.sample_rows(case, n_rows, seed=idx)
    got, got_lse = gather_rows(out, lse, case, rows)
    print(f"config {idx}: oracle on {rows.shape[0]} rows", flush=True)
    ref, lse_ref, _ = oracle.case_rows(case, rows)
    max_abs, rel_l2 = check_close(got, ref, W.BF16, f"config {idx}")
    # per-row relative error: the binding check at long context where |O| is small
    row_rel = np.linalg.norm(got - ref, axis=1) / np.linalg.norm(ref, axis=1)
    print(f"config {idx}: max_abs {max_abs:.3e} rel_l2 {rel_l2:.3e} worst row rel {row_rel.max():.3e}", flush=True)
    assert row_rel.max() <= 3e-2
    lse_err, lse_tol = np.abs(got_lse - lse_ref).max(), TOL[W.BF16]["lse_abs"]
    print(f"config {idx}: max |lse - oracle| {lse_err:.3e} of {lse_tol:.1e} allowed", flush=True)
    assert lse_err <= lse_tol
