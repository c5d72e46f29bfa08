"""The reuse workflow of a prefill instance, end to end through every entry point (Section 3, steps 1-3;
Algorithm 1's prefix match; Section 5.2 store / load): request A is prefilled and its KVCache stored in the
host pool under its block keys; request B shares A's first two 512-token blocks; the match finds them, their
pages are loaded into B's own pages, B's remaining tokens are appended and attended to with the prefix reused.
The result must be what B gets when everything is recomputed, and what the oracle says."""
import numpy as np
import pytest
import torch

from paper_2407_00079_amd import binding as B
from paper_2407_00079_amd import workloads as W

from gpu_util import TOL, DeviceCase, check_close, dev

pytestmark = pytest.mark.gpu

Hq, Hkv, D, S, BLOCK = 8, 2, 128, 16, 512
PAGE_BYTES = Hkv * S * D * 2


def _keys(tokens):
    off = [0, len(tokens)]
    n = -(-len(tokens) // BLOCK)
    keys = torch.zeros((n,), dtype=torch.int64, device="cuda:0")
    ws = torch.empty(B.mc_prefix_hash_workspace_bytes(1), dtype=torch.uint8, device="cuda:0")
    B.mc_prefix_hash(dev(np.asarray(tokens, dtype=np.int32)), off, BLOCK, keys, ws)
    return keys


def test_prefix_reuse_equals_recompute(oracle):
    rng = np.random.default_rng(20240779)
    LA, SHARED, LB = 1536, 1024, 1324
    tok_a = rng.integers(0, 32000, size=LA, dtype=np.int32)
    tok_b = np.concatenate([tok_a[:SHARED], rng.integers(0, 32000, size=LB - SHARED, dtype=np.int32)])
    tok_b[SHARED] = (tok_a[SHARED] + 1) % 32000            # the third block certainly differs

    # ---- request A: its K/V rows are appended into its pages on "instance 0" and stored to the host pool
    N1 = 160
    case_a = W.make_attn_case(801, W.BF16, Hq, Hkv, D, S, [0], [LA], N1, keep_logical=True)
    prm1 = B.attn_params(Hq, Hkv, D, S, N1, "bf16")
    k1 = dev(np.full_like(case_a.k_pool, 0x7FC0))          # pools start as NaN patterns: only the calls fill them
    v1 = dev(np.full_like(case_a.v_pool, 0x7FC0))
    bt_a = dev(case_a.block_tables)
    ws = torch.empty(B.mc_kv_append_workspace_bytes(1), dtype=torch.uint8, device="cuda:0")
    B.mc_kv_append_paged(prm1, dev(case_a.k_logical[0]), dev(case_a.v_logical[0]), k1, v1, bt_a, [0], [LA], ws)
    n_a = LA // S
    ids_a = dev(case_a.block_tables[0, :n_a].copy())
    stage_k = torch.zeros((n_a, PAGE_BYTES), dtype=torch.uint8, device="cuda:0")
    stage_v = torch.zeros_like(stage_k)
    host_k = torch.zeros((n_a, PAGE_BYTES), dtype=torch.uint8, pin_memory=True)     # the CPU DRAM pool's copy
    host_v = torch.zeros_like(host_k).pin_memory()
    B.mc_kv_store_layer(k1, v1, N1, PAGE_BYTES, ids_a, n_a, stage_k, stage_v, host_k, host_v)
    cache_keys = _keys(tok_a)                               # 3 keys, what the scheduler knows of instance 0
    torch.cuda.synchronize()
    cache_sorted = torch.from_numpy(np.sort(cache_keys.cpu().numpy().view(np.uint64)).view(np.int64)).to("cuda:0")
    # ---- request B arrives: block keys, longest prefix match against two instances (the second holds nothing)
    keys_b = _keys(tok_b)
    n_inst = 2
    plen = torch.full((1, n_inst), -1, dtype=torch.int32, device="cuda:0")
    best_len = torch.full((1,), -1, dtype=torch.int32, device="cuda:0")
    best_inst = torch.full((1,), -1, dtype=torch.int32, device="cuda:0")
    ws_m = torch.empty(B.mc_prefix_match_workspace_bytes(1, n_inst), dtype=torch.uint8, device="cuda:0")
    B.mc_prefix_match(keys_b, [0, keys_b.numel()], cache_sorted, [0, 3, 3], plen, best_len, best_inst, ws_m)
    torch.cuda.synchronize()
    assert plen.cpu().tolist() == [[2, 0]] and best_len.item() == 2 and best_inst.item() == 0
    P = best_len.item() * BLOCK                             # 1024 tokens are reused, 300 are new
    C = LB - P

    # ---- B's tensors: K/V of the shared positions are A's (same tokens, same prefix), the rest and Q are B's own
    kb = np.concatenate([case_a.k_logical[0][:SHARED],
                         W._store(rng.standard_normal((LB - SHARED, Hkv, D), dtype=np.float32), W.BF16)])
    vb = np.concatenate([case_a.v_logical[0][:SHARED],
                         W._store(rng.standard_normal((LB - SHARED, Hkv, D), dtype=np.float32), W.BF16)])
    qb = W._store(rng.standard_normal((LB, Hq, D), dtype=np.float32), W.BF16)
    N2 = 200
    case_reuse = W.make_attn_case(802, W.BF16, Hq, Hkv, D, S, [P], [C], N2, logical=(qb[P:], [kb], [vb]))
    case_full = W.make_attn_case(803, W.BF16, Hq, Hkv, D, S, [0], [LB], N2, logical=(qb, [kb], [vb]))

    # ---- on "instance 1": load the reused pages from the host pool into B's pages, append the new rows, attend
    prm2 = B.attn_params(Hq, Hkv, D, S, N2, "bf16")
    dc = DeviceCase(case_reuse)
    dc.k_pool = dev(np.full_like(case_reuse.k_pool, 0x7FC0))
    dc.v_pool = dev(np.full_like(case_reuse.v_pool, 0x7FC0))
    n_pre = P // S
    ids_b = dev(case_reuse.block_tables[0, :n_pre].copy())
    report = torch.zeros((2,), dtype=torch.int32, device="cuda:0")
    B.mc_kv_check_page_ids(ids_b, n_pre, N2, report)
    B.mc_kv_load_layer(host_k[:n_pre], host_v[:n_pre], stage_k[:n_pre], stage_v[:n_pre], N2, PAGE_BYTES, ids_b, n_pre,
                       dc.k_pool, dc.v_pool)
    ws2 = torch.empty(B.mc_kv_append_workspace_bytes(1), dtype=torch.uint8, device="cuda:0")
    B.mc_kv_append_paged(prm2, dev(kb[P:]), dev(vb[P:]), dc.k_pool, dc.v_pool, dc.block_tables, [P], [C], ws2)
    dc.run()
    out_reuse, lse_reuse = dc.result()
    assert report.cpu().tolist() == [0, n_pre]
    # the pools now hold exactly what a from-scratch build of the same case holds
    np.testing.assert_array_equal(dc.k_pool.cpu().numpy().view(np.uint16)[case_reuse.block_tables[0, :n_pre]],
                                  case_reuse.k_pool[case_reuse.block_tables[0, :n_pre]])

    # ---- the same request with nothing reused: all 1324 tokens computed in one call
    dcf = DeviceCase(case_full)
    dcf.run()
    out_full, lse_full = dcf.result()

    ref_out, ref_lse, _ = oracle.case_full(case_reuse)
    ref_out_full, ref_lse_full, _ = oracle.case_full(case_full)
    # oracle: reuse is invisible (its own pin); GPU: both ways within tolerance of it, and of each other
    np.testing.assert_allclose(ref_out, ref_out_full[P:], rtol=0, atol=1e-12)
    check_close(out_reuse, ref_out, W.BF16, "prefix reused")
    check_close(out_full[P:], ref_out, W.BF16, "recomputed")
    assert np.abs(lse_reuse - ref_lse).max() <= TOL[W.BF16]["lse_abs"]
    assert np.abs(lse_full[P:] - ref_lse).max() <= TOL[W.BF16]["lse_abs"]
    assert np.abs(out_reuse - out_full[P:]).max() <= 2e-2
