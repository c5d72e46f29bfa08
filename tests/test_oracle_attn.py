"""Pins for the CPU oracle's attention (CPU only).

The paper prints no formula and no numbers for attention, so the oracle is
pinned by what the mathematics fixes: a literally different dense, un-paged
formulation; closed forms; invariances that prefix reuse, chunking and paging
must not break (Section 3 steps 1-2, Section 5.1's remark that attention is
associative over key subsets); and NaN poison behind everything the causal
rule hides.
"""
import dataclasses
import os

import numpy as np
import pytest

from paper_2407_00079_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------
# second formulation: full L x L score matrix, -inf mask, dense matmuls
# ---------------------------------------------------------------------------
def dense_causal_attention(q_full, k_log, v_log, num_q_heads, num_kv_heads, scale):
    """q_full [L, Hq, D], k_log/v_log [L, Hkv, D] float64 -> (O [L, Hq, D], LSE [L, Hq], P [Hq, L, L])."""
    L, Hq, D = q_full.shape
    G = num_q_heads // num_kv_heads
    k_rep = np.repeat(k_log, G, axis=1)          # [L, Hq, D], head h <- kv head h // G
    v_rep = np.repeat(v_log, G, axis=1)
    s = np.einsum("ihd,jhd->hij", q_full, k_rep) * scale
    hidden = np.triu(np.ones((L, L), dtype=bool), k=1)
    s = np.where(hidden[None], -np.inf, s)
    m = s.max(axis=2, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=2, keepdims=True)
    p = e / z
    o = np.einsum("hij,jhd->ihd", p, v_rep)
    lse = (m + np.log(z))[:, :, 0].T
    return o, lse, p


def small_case(seed=7, dtype=W.F32, Hq=4, Hkv=2, D=16, S=4, prefix=(10,), new=(7,), pages=32, **kw):
    return W.make_attn_case(seed, dtype, Hq, Hkv, D, S, list(prefix), list(new), pages,
                            poison=True, keep_logical=True, **kw)


def full_q(case, r, rng):
    """Q for all L positions of request r: random rows for the prefix, the case's rows for the chunk."""
    P, C = int(case.prefix_lens[r]), int(case.new_lens[r])
    off = case.q_offsets
    qc = W.to_f64(case.q[off[r]:off[r + 1]], case.dtype)
    qp = rng.standard_normal((P, case.num_q_heads, case.head_dim))
    return np.concatenate([qp, qc], axis=0)


# (i) reuse == recompute, (iii) brute force, (ii) rows sum to one
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("shape", [
    dict(Hq=4, Hkv=1, D=8, S=4, prefix=(0,), new=(9,)),
    dict(Hq=4, Hkv=2, D=16, S=4, prefix=(10,), new=(7,)),
    dict(Hq=6, Hkv=3, D=8, S=16, prefix=(33, 0, 16), new=(5, 17, 1)),
    dict(Hq=2, Hkv=2, D=32, S=8, prefix=(24,), new=(40,)),
])
def test_reuse_equals_dense_recompute(oracle, dtype, shape):
    case = small_case(seed=11, dtype=dtype, **shape)
    out, lse, psum = oracle.case_full(case)
    rng = np.random.default_rng(3)
    scale = 1.0 / np.sqrt(case.head_dim)
    off = case.q_offsets
    for r in range(case.batch):
        P = int(case.prefix_lens[r])
        o_ref, lse_ref, _ = dense_causal_attention(
            full_q(case, r, rng), W.to_f64(case.k_logical[r], dtype), W.to_f64(case.v_logical[r], dtype),
            case.num_q_heads, case.num_kv_heads, scale)
        np.testing.assert_allclose(out[off[r]:off[r + 1]], o_ref[P:], rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[off[r]:off[r + 1]], lse_ref[P:], rtol=0, atol=1e-12)
    assert np.all(np.abs(psum - 1.0) <= 1e-12)
    assert np.isfinite(out).all() and np.isfinite(lse).all()


def test_config1_against_dense(oracle):
    case = W.make_config_attn(1, keep_logical=True)
    assert case.block_tables.shape == (1, 24) and case.num_pages == 64
    assert case.flops() == 42008576 and case.visible_pairs() == 41024
    out, lse, psum = oracle.case_full(case)
    o_ref, lse_ref, _ = dense_causal_attention(
        full_q(case, 0, np.random.default_rng(0)), W.to_f64(case.k_logical[0], W.F32),
        W.to_f64(case.v_logical[0], W.F32), 4, 1, 1.0 / 8.0)
    np.testing.assert_allclose(out, o_ref[256:], rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, lse_ref[256:], rtol=0, atol=1e-12)
    assert np.all(np.abs(psum - 1.0) <= 1e-12)


# (v) uniform softmax: Q = 0 -> running mean of V; all K equal -> same
def test_uniform_scores_give_running_mean(oracle):
    case = small_case(seed=5, Hq=4, Hkv=2, D=8, S=4, prefix=(6,), new=(11,))
    v = W.to_f64(case.v_logical[0], case.dtype)
    G = 2
    zero_q = dataclasses.replace(case, q=np.zeros_like(case.q))
    out, lse, _ = oracle.case_full(zero_q)
    for i in range(11):
        n = 6 + i + 1
        for h in range(4):
            np.testing.assert_allclose(out[i, h], v[:n, h // G].mean(axis=0), atol=1e-13)
            assert abs(lse[i, h] - np.log(n)) < 1e-13
    # equal keys, arbitrary Q
    k_const = [np.broadcast_to(case.k_logical[0][:1], case.k_logical[0].shape).copy()]
    same_k = W.make_attn_case(5, case.dtype, 4, 2, 8, 4, [6], [11], 32, keep_logical=True,
                              logical=(case.q, k_const, case.v_logical))
    out2, _, _ = oracle.case_full(same_k)
    np.testing.assert_allclose(out2, out, atol=1e-13)


# (vi) constant V
def test_constant_v(oracle):
    case = small_case(seed=9, prefix=(13,), new=(6,))
    c = np.linspace(-2, 3, case.head_dim).astype(np.float32)
    v_const = [np.broadcast_to(c, case.v_logical[0].shape).copy()]
    cv = W.make_attn_case(9, case.dtype, 4, 2, 16, 4, [13], [6], 32, logical=(case.q, case.k_logical, v_const))
    out, _, _ = oracle.case_full(cv)
    np.testing.assert_allclose(out, np.broadcast_to(c.astype(np.float64), out.shape), atol=1e-14)


# (vii) first row without a prefix
def test_first_row_without_prefix(oracle):
    case = small_case(seed=21, Hq=4, Hkv=2, D=16, S=4, prefix=(0,), new=(5,))
    out, lse, _ = oracle.case_full(case)
    q = W.to_f64(case.q, case.dtype)
    k = W.to_f64(case.k_logical[0], case.dtype)
    v = W.to_f64(case.v_logical[0], case.dtype)
    for h in range(4):
        np.testing.assert_array_equal(out[0, h], v[0, h // 2])
        assert abs(lse[0, h] - (q[0, h] @ k[0, h // 2]) / 4.0) < 1e-14


# (viii) needle: one key aligned with q dominates; V rows encode their token index
@pytest.mark.parametrize("needle", [0, 15, 16, 37, 47, 48, 63, 64, 70])
def test_needle_through_block_table(oracle, needle):
    Hq, Hkv, D, S, P, C = 2, 1, 16, 16, 48, 23          # L = 71: last page holds 7 tokens
    L = P + C
    rng = np.random.default_rng(needle)
    q = rng.standard_normal((C, Hq, D)).astype(np.float32)
    k = (0.01 * rng.standard_normal((L, Hkv, D))).astype(np.float32)
    v = np.zeros((L, Hkv, D), dtype=np.float32)
    v[:, 0, 0] = np.arange(L)
    v[:, 0, 1] = 1.0
    i = C - 1                                            # last row sees every key
    beta = 400.0
    k[needle, 0] = beta * q[i, 0] / np.linalg.norm(q[i, 0])
    case = W.make_attn_case(1, W.F32, Hq, Hkv, D, S, [P], [C], 16, logical=(q, [k], [v]))
    out, _, _ = oracle.case_rows(case, [[0, 0, i]])
    assert abs(out[0, 0] - needle) < 1e-9
    assert abs(out[0, 1] - 1.0) < 1e-12


# (ix) page-permutation invariance
def test_page_permutation_invariance(oracle):
    case = small_case(seed=31, prefix=(19, 4), new=(9, 12), pages=40)
    other = W.make_attn_case(977, case.dtype, 4, 2, 16, 4, [19, 4], [9, 12], 64,
                             logical=(case.q, case.k_logical, case.v_logical))
    assert not np.array_equal(case.block_tables, other.block_tables[:, :case.max_pages])
    a = oracle.case_full(case)
    b = oracle.case_full(other)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


# (x) chunk-split invariance (Section 3 step 2: chunks run one after another on a growing prefix)
def test_chunk_split_invariance(oracle):
    case = small_case(seed=41, prefix=(8,), new=(21,), S=4)
    whole, lse_w, _ = oracle.case_full(case)
    c1 = 9
    first = dataclasses.replace(case, q=case.q[:c1], new_lens=np.array([c1], np.int32))
    second = dataclasses.replace(case, q=case.q[c1:], prefix_lens=np.array([8 + c1], np.int32),
                                 new_lens=np.array([21 - c1], np.int32))
    o1, l1, _ = oracle.case_full(first)
    o2, l2, _ = oracle.case_full(second)
    np.testing.assert_array_equal(np.concatenate([o1, o2]), whole)
    np.testing.assert_array_equal(np.concatenate([l1, l2]), lse_w)


# (xi) log-sum-exp merge of two key subsets (associativity remark in Section 5.1)
def test_lse_merge_of_key_subsets(oracle):
    case = small_case(seed=51, dtype=W.BF16, prefix=(30,), new=(10,), S=4, pages=16)
    rows = np.array([[0, h, i] for i in (0, 4, 9) for h in range(4)], dtype=np.int32)
    whole, lse_w, _ = oracle.case_rows(case, rows)
    for cut in (1, 17, 30, 33):
        n = rows.shape[0]
        oa, la, _ = oracle.case_rows(case, rows, key_lo=np.zeros(n), key_hi=np.full(n, cut))
        ob, lb, _ = oracle.case_rows(case, rows, key_lo=np.full(n, cut), key_hi=np.full(n, 1 << 40))
        m = np.maximum(la, lb)
        wa, wb = np.exp(la - m), np.exp(lb - m)
        merged = (oa * wa[:, None] + ob * wb[:, None]) / (wa + wb)[:, None]
        np.testing.assert_allclose(merged, whole, atol=1e-13)
        np.testing.assert_allclose(m + np.log(wa + wb), lse_w, atol=1e-13)
    # an empty subset contributes nothing
    oe, le, pe = oracle.case_rows(case, rows[:1], key_lo=[50], key_hi=[60])
    assert np.all(oe == 0) and np.isneginf(le[0]) and pe[0] == 0


# (xii) GQA expansion: replicate KV heads to MHA
def test_gqa_equals_replicated_mha(oracle):
    case = small_case(seed=61, Hq=6, Hkv=2, D=8, S=4, prefix=(7,), new=(9,))
    k_rep = [np.repeat(case.k_logical[0], 3, axis=1)]
    v_rep = [np.repeat(case.v_logical[0], 3, axis=1)]
    mha = W.make_attn_case(61, case.dtype, 6, 6, 8, 4, [7], [9], 32, logical=(case.q, k_rep, v_rep))
    a = oracle.case_full(case)
    b = oracle.case_full(mha)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])


# (xiii) mask tightness: NaN in every future key, page tail and unreferenced page
def test_hidden_slots_are_never_read(oracle):
    case = small_case(seed=71, dtype=W.BF16, prefix=(5,), new=(6,), S=4, pages=8)   # L = 11, tail of 1 slot
    bits = W.BF16_NAN_BITS
    assert (case.k_pool == bits).any()          # poison is there (tail slot, unused pages)
    i = 2                                        # row sees keys 0..7; poison keys 8..10 as well
    k_log = [case.k_logical[0].copy()]
    v_log = [case.v_logical[0].copy()]
    ref, lse_ref, _ = oracle.case_rows(case, [[0, 1, i]])
    k_log[0][5 + i + 1:] = bits
    v_log[0][5 + i + 1:] = bits
    poisoned = W.make_attn_case(71, W.BF16, 4, 2, 16, 4, [5], [6], 8, logical=(case.q, k_log, v_log))
    np.testing.assert_array_equal(poisoned.block_tables, case.block_tables)
    got, lse_got, _ = oracle.case_rows(poisoned, [[0, 1, i]])
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_array_equal(lse_got, lse_ref)
    assert np.isfinite(got).all()


# (xiv) overflow safety and shift invariance
def test_large_scores_stay_finite(oracle):
    case = small_case(seed=81, prefix=(40,), new=(8,), D=64, S=16, pages=8, q_scale=400.0)
    out, lse, psum = oracle.case_full(case)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert np.all(np.abs(psum - 1.0) <= 1e-12)
    assert lse.max() > 710.0                     # exp() of the raw scores would overflow fp64 without the max shift
    o_ref, lse_ref, _ = dense_causal_attention(
        full_q(case, 0, np.random.default_rng(0)), W.to_f64(case.k_logical[0], case.dtype),
        W.to_f64(case.v_logical[0], case.dtype), 4, 2, 1.0 / 8.0)
    np.testing.assert_allclose(out, o_ref[40:], atol=1e-10)


def test_custom_scale_and_gqa_head_mapping(oracle):
    """A swapped or strided head mapping, or a dropped scale, must fail here."""
    Hq, Hkv, D, S = 4, 2, 8, 4
    case = small_case(seed=91, Hq=Hq, Hkv=Hkv, D=D, S=S, prefix=(3,), new=(4,))
    q = W.to_f64(case.q, case.dtype)
    k = W.to_f64(case.k_logical[0], case.dtype)
    v = W.to_f64(case.v_logical[0], case.dtype)
    out, lse, _ = oracle.case_full(case, scale=0.37)
    for i in range(4):
        for h in range(Hq):
            g = h // (Hq // Hkv)                 # contiguous groups: heads 0,1 -> kv 0; 2,3 -> kv 1
            s = 0.37 * (k[:3 + i + 1, g] @ q[i, h])
            p = np.exp(s - s.max())
            p /= p.sum()
            np.testing.assert_allclose(out[i, h], p @ v[:3 + i + 1, g], atol=1e-13)


def test_empty_requests_and_single_rows(oracle):
    case = small_case(seed=101, prefix=(5, 0, 9), new=(0, 3, 1), Hq=2, Hkv=1, D=8, S=4)
    out, lse, _ = oracle.case_full(case)
    assert out.shape == (4, 2, 8)
    rng = np.random.default_rng(1)
    for r in (1, 2):
        P = int(case.prefix_lens[r])
        o_ref, _, _ = dense_causal_attention(full_q(case, r, rng), W.to_f64(case.k_logical[r], case.dtype),
                                             W.to_f64(case.v_logical[r], case.dtype), 2, 1, 1 / np.sqrt(8))
        off = case.q_offsets
        np.testing.assert_allclose(out[off[r]:off[r + 1]], o_ref[P:], atol=1e-13)
    with pytest.raises(ValueError):
        oracle.case_rows(case, [[0, 0, 0]])      # request 0 has no rows


def test_paper_trace_sample_shapes(oracle):
    """Two requests shaped like the paper's printed trace samples share 6144 prefix tokens (Section 4)."""
    vals = {}
    samples = []
    with open(os.path.join(GOLDEN, "trace_sample_shapes.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            tok = line.split()
            if tok[0] == "sample":
                samples.append(tuple(int(x) for x in tok[1:]))
            else:
                vals[tok[0]] = int(tok[1])
    B = vals["block_tokens"]
    assert vals["shared_prefix_tokens"] == samples[0][2] * B == 6144
    for length, blocks, _ in samples:
        assert blocks == -(-length // B)
    S, Hq, Hkv, D = 16, 2, 1, 16
    shared_pages = vals["shared_prefix_tokens"] // S
    prefix = [6144, 6144]
    new = [s[0] - 6144 for s in samples]
    assert new == [811, 328]
    case = W.make_attn_case(5, W.BF16, Hq, Hkv, D, S, prefix, new, 1024, keep_logical=True,
                            shared_prefix_pages=shared_pages)
    np.testing.assert_array_equal(case.block_tables[0, :shared_pages], case.block_tables[1, :shared_pages])
    rows = np.array([[0, 0, 0], [0, 1, 810], [1, 0, 0], [1, 1, 327], [1, 0, 100]], dtype=np.int32)
    out, lse, psum = oracle.case_rows(case, rows)
    scale = 1.0 / 4.0
    off = case.q_offsets
    for t, (r, h, i) in enumerate(rows):
        k = W.to_f64(case.k_logical[r], W.BF16)[:6144 + i + 1, 0]
        v = W.to_f64(case.v_logical[r], W.BF16)[:6144 + i + 1, 0]
        q = W.to_f64(case.q[off[r] + i, h], W.BF16)
        s = scale * (k @ q)
        p = np.exp(s - s.max())
        p /= p.sum()
        np.testing.assert_allclose(out[t], p @ v, atol=1e-12)
    assert np.all(np.abs(psum - 1) < 1e-12)
