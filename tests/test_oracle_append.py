"""Pins for the CPU oracle's KV append (Section 3 step 2: the new chunk's KVCache is stored into the request's pages)."""
import numpy as np
import pytest

from paper_2407_00079_amd import workloads as W

from append_util import empty_chunk_pools, new_rows


@pytest.mark.parametrize("dtype,D", [(W.BF16, 128), (W.F32, 64)])
def test_append_rebuilds_the_pools(oracle, dtype, D):
    # prefixes not page aligned, a chunk that ends mid page, a single token, an empty request
    case = W.make_attn_case(11, dtype, 4, 2, D, 16, [37, 0, 16, 5], [50, 33, 1, 0], 64, keep_logical=True)
    k, v = empty_chunk_pools(case)
    assert not np.array_equal(k.view(np.uint8), case.k_pool.view(np.uint8))
    k_new, v_new = new_rows(case)
    oracle.kv_append_paged(k_new, v_new, k, v, case.block_tables, case.prefix_lens, case.new_lens)
    # the generator wrote the same tokens through its own (numpy slicing) path: bytes must agree everywhere,
    # which also shows that prefix slots, tail slots and unreferenced pages were left alone
    np.testing.assert_array_equal(k.view(np.uint8), case.k_pool.view(np.uint8))
    np.testing.assert_array_equal(v.view(np.uint8), case.v_pool.view(np.uint8))


def test_append_in_two_chunks_equals_one(oracle):
    case = W.make_attn_case(12, W.BF16, 2, 1, 128, 16, [20], [45], 16, keep_logical=True)
    k, v = empty_chunk_pools(case)
    k_new, v_new = new_rows(case)
    oracle.kv_append_paged(k_new[:17], v_new[:17], k, v, case.block_tables, [20], [17])
    oracle.kv_append_paged(k_new[17:], v_new[17:], k, v, case.block_tables, [37], [28])
    np.testing.assert_array_equal(k, case.k_pool)
    np.testing.assert_array_equal(v, case.v_pool)


def test_append_then_attention_equals_prebuilt(oracle):
    case = W.make_attn_case(13, W.BF16, 4, 2, 128, 16, [33], [21], 16, keep_logical=True)
    k, v = empty_chunk_pools(case)
    k_new, v_new = new_rows(case)
    oracle.kv_append_paged(k_new, v_new, k, v, case.block_tables, case.prefix_lens, case.new_lens)
    a = oracle.prefill_attn_paged(W.BF16, case.q, k, v, case.block_tables, case.prefix_lens, case.new_lens, 4, 2)
    b = oracle.case_full(case)
    np.testing.assert_array_equal(a[0], b[0])


def test_append_rejects_bad_arguments(oracle):
    case = W.make_attn_case(14, W.BF16, 2, 1, 128, 16, [8], [8], 4, keep_logical=True)
    k, v = case.k_pool.copy(), case.v_pool.copy()
    k_new, v_new = new_rows(case)
    bad_bt = case.block_tables.copy()
    bad_bt[0, 0] = 4
    with pytest.raises(ValueError):
        oracle.kv_append_paged(k_new, v_new, k, v, bad_bt, [8], [8])
    with pytest.raises(ValueError):
        oracle.kv_append_paged(k_new, v_new, k, v, case.block_tables[:, :0].reshape(1, 0), [8], [8])
    np.testing.assert_array_equal(k, case.k_pool)
