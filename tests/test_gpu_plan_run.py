"""GPU: prepare once, run per layer (mc_prefill_attn_prepare / _run / _run_split, mc_kv_append_run) gives bit for bit
what the one-shot calls give, also when the runs are replayed from a HIP graph."""
import numpy as np
import pytest
import torch

from paper_2407_00079_amd import binding as B
from paper_2407_00079_amd import workloads as W

from append_util import empty_chunk_pools, new_rows
from gpu_util import TOL, DeviceCase, check_close, dev

pytestmark = pytest.mark.gpu

PREFIX, NEW = [700, 0, 33], [300, 129, 1]


def _layers(n):
    """n layers of one batch: same lengths and block tables (same seed for the paging), different values."""
    base = W.make_attn_case(900, W.BF16, 8, 2, 128, 16, PREFIX, NEW, 128, keep_logical=True)
    cases = [base]
    rng = np.random.default_rng(901)
    for _ in range(n - 1):
        q = W._store(rng.standard_normal(base.q.shape, dtype=np.float32), W.BF16)
        ks = [W._store(rng.standard_normal(k.shape, dtype=np.float32), W.BF16) for k in base.k_logical]
        vs = [W._store(rng.standard_normal(k.shape, dtype=np.float32), W.BF16) for k in base.k_logical]
        c = W.make_attn_case(900, W.BF16, 8, 2, 128, 16, PREFIX, NEW, 128, keep_logical=True, logical=(q, ks, vs))
        assert (c.block_tables == base.block_tables).all()
        cases.append(c)
    return cases


def test_one_plan_many_layers_matches_one_shot_and_oracle(oracle):
    cases = _layers(3)
    first = DeviceCase(cases[0])
    plan_ws = torch.empty_like(first.workspace)
    plan = B.mc_prefill_attn_prepare(first.params, PREFIX, NEW, 0, plan_ws)
    assert plan.n_items > 0 and plan.kv_splits == 0 and plan.total_new_tokens == sum(NEW)
    assert plan.n_items == len(B.mc_prefill_attn_plan(first.params, PREFIX, NEW, 0))
    for l, case in enumerate(cases):
        dc = DeviceCase(case)
        dc.run()                                                   # one-shot call
        out1, lse1 = dc.out.clone(), dc.lse.clone()
        dc.out.fill_(float("nan"))
        dc.lse.fill_(float("nan"))
        B.mc_prefill_attn_run(dc.params, plan, dc.q, dc.k_pool, dc.v_pool, dc.block_tables, dc.out, dc.lse, plan_ws)
        torch.cuda.synchronize()
        assert torch.equal(dc.out.view(torch.int16), out1.view(torch.int16)), f"layer {l}"
        assert torch.equal(dc.lse, lse1)
        out, lse = dc.result()
        ref_out, ref_lse, _ = oracle.case_full(case)
        check_close(out, ref_out, W.BF16, f"layer {l}")
        assert np.abs(lse - ref_lse).max() <= TOL[W.BF16]["lse_abs"]


def test_split_plan_and_append_run_match_one_shot(oracle):
    case = _layers(1)[0]
    dc = DeviceCase(case)
    splits, n = 3, case.total_new * case.num_q_heads
    ws = torch.empty(B.mc_prefill_attn_split_workspace_bytes(dc.params, case.batch, case.total_new, splits),
                     dtype=torch.uint8, device="cuda:0")
    shape_o, shape_l = (splits, case.total_new, 8, 128), (splits, case.total_new, 8)
    o1 = torch.full(shape_o, float("nan"), dtype=torch.float32, device="cuda:0")
    l1 = torch.full(shape_l, float("nan"), dtype=torch.float32, device="cuda:0")
    B.mc_prefill_attn_paged_split(dc.params, dc.q, dc.k_pool, dc.v_pool, dc.block_tables, PREFIX, NEW, splits, o1, l1, ws)
    ws2 = torch.empty_like(ws)
    plan = B.mc_prefill_attn_prepare(dc.params, PREFIX, NEW, splits, ws2)
    o2, l2 = torch.full_like(o1, float("nan")), torch.full_like(l1, float("nan"))
    B.mc_prefill_attn_run_split(dc.params, plan, dc.q, dc.k_pool, dc.v_pool, dc.block_tables, o2, l2, ws2)
    torch.cuda.synchronize()
    # slices without keys are written as zeros / -inf by both; compare bit patterns
    assert torch.equal(o1.view(torch.int32), o2.view(torch.int32)) and torch.equal(l1.view(torch.int32), l2.view(torch.int32))
    # append through the same plan = append_paged
    k0, v0 = empty_chunk_pools(case)
    k_new, v_new = new_rows(case)
    ka, va, kb, vb = dev(k0), dev(v0), dev(k0), dev(v0)
    aws = torch.empty(B.mc_kv_append_workspace_bytes(case.batch), dtype=torch.uint8, device="cuda:0")
    B.mc_kv_append_paged(dc.params, dev(k_new), dev(v_new), ka, va, dc.block_tables, PREFIX, NEW, aws)
    B.mc_kv_append_run(dc.params, plan, dev(k_new), dev(v_new), kb, vb, dc.block_tables, ws2)
    torch.cuda.synchronize()
    assert torch.equal(ka, kb) and torch.equal(va, vb)
    np.testing.assert_array_equal(kb.cpu().numpy().view(np.uint16), case.k_pool)
    # wrong form / foreign params / too few block-table columns are refused before anything is launched
    with pytest.raises(B.McError):
        B.mc_prefill_attn_run(dc.params, plan, dc.q, dc.k_pool, dc.v_pool, dc.block_tables, dc.out, dc.lse, ws2)
    other = B.attn_params(16, 2, 128, 16, case.num_pages, "bf16")
    with pytest.raises(B.McError):
        B.mc_prefill_attn_run_split(other, plan, dc.q, dc.k_pool, dc.v_pool, dc.block_tables, o2, l2, ws2)
    with pytest.raises(B.McError):
        B.mc_prefill_attn_run_split(dc.params, plan, dc.q, dc.k_pool, dc.v_pool, dc.block_tables[:, :10].contiguous(),
                                    o2, l2, ws2)


def test_layer_step_replays_from_a_hip_graph(oracle):
    """append_run + attn_run captured once; every replay, with new inputs copied in eagerly in between, matches the
    one-shot calls on the same inputs."""
    cases = _layers(3)
    c0 = cases[0]
    dc = DeviceCase(c0)                                            # the buffers the graph is bound to
    k0, v0 = empty_chunk_pools(c0)
    dc.k_pool, dc.v_pool = dev(k0), dev(v0)
    k_new_np, v_new_np = new_rows(c0)
    k_new, v_new = dev(k_new_np), dev(v_new_np)
    plan_ws = torch.empty_like(dc.workspace)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        plan = B.mc_prefill_attn_prepare(dc.params, PREFIX, NEW, 0, plan_ws, side)        # outside the graph

        def step():
            B.mc_kv_append_run(dc.params, plan, k_new, v_new, dc.k_pool, dc.v_pool, dc.block_tables, plan_ws, side)
            B.mc_prefill_attn_run(dc.params, plan, dc.q, dc.k_pool, dc.v_pool, dc.block_tables, dc.out, dc.lse,
                                  plan_ws, side)
        step()                                                     # once eagerly before the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for l, case in enumerate(cases):
        kk, vv = empty_chunk_pools(case)
        kn, vn = new_rows(case)
        dc.q.copy_(dev(case.q))                                    # eager work between the replays
        dc.k_pool.copy_(dev(kk))
        dc.v_pool.copy_(dev(vv))
        k_new.copy_(dev(kn))
        v_new.copy_(dev(vn))
        dc.out.fill_(float("nan"))
        dc.lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_out, got_lse = dc.out.clone(), dc.lse.clone()
        np.testing.assert_array_equal(dc.k_pool.cpu().numpy().view(np.uint16), case.k_pool, err_msg=f"replay {l}")
        ref = DeviceCase(case)
        ref.run()
        assert torch.equal(got_out.view(torch.int16), ref.out.view(torch.int16)), f"replay {l}"
        assert torch.equal(got_lse, ref.lse)
        ref_out, ref_lse, _ = oracle.case_full(case)
        check_close(got_out.float().cpu().numpy().astype(np.float64), ref_out, W.BF16, f"replay {l}")
