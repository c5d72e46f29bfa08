"""Pins for the CPU oracle's prefix block keys and longest prefix match (Algorithm 1: PrefixHash,
FindBestPrefixMatch; Section 4: the hash_ids of the request trace)."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M64 = (1 << 64) - 1


def read_shapes():
    out = {"samples": []}
    for line in open(os.path.join(GOLDEN, "trace_sample_shapes.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "sample":
            out["samples"].append(tuple(int(x) for x in f[1:]))
        else:
            out[f[0]] = int(f[1])
    return out


def test_mixing_function_reproduces_published_splitmix64_outputs(oracle):
    want = [int(l, 16) for l in open(os.path.join(GOLDEN, "splitmix64_seed0.txt")) if l.startswith("0x")]
    gamma = 0x9E3779B97F4A7C15
    # the generator's k-th output is the output function applied to state k * gamma; mix64 adds one gamma itself
    got = [oracle.mix64((k * gamma) & M64) for k in range(3)]
    assert got == want


def test_paper_trace_samples_share_their_first_twelve_keys(oracle):
    # the two request samples of Section 4: 6955 and 6472 input tokens, 14 and 13 hash ids, the first 12 equal
    sh = read_shapes()
    B = sh["block_tokens"]
    (len_a, ids_a, shared), (len_b, ids_b, _) = sh["samples"]
    rng = np.random.default_rng(0)
    common = rng.integers(0, 32000, size=sh["shared_prefix_tokens"], dtype=np.int32)
    a = np.concatenate([common, rng.integers(0, 32000, size=len_a - common.size, dtype=np.int32)])
    b = np.concatenate([common, rng.integers(0, 32000, size=len_b - common.size, dtype=np.int32)])
    keys, off = oracle.prefix_hash(np.concatenate([a, b]), [0, len_a, len_a + len_b], B)
    ka, kb = keys[off[0]:off[1]], keys[off[1]:off[2]]
    assert (ka.size, kb.size) == (ids_a, ids_b)
    assert (ka[:shared] == kb[:shared]).all() and ka[shared] != kb[shared]
    assert shared * B == sh["shared_prefix_tokens"]


def test_keys_chain_over_the_whole_prefix(oracle):
    rng = np.random.default_rng(1)
    B, nb = 16, 10
    t = rng.integers(0, 1000, size=B * nb, dtype=np.int32)
    keys, _ = oracle.prefix_hash(t, [0, t.size], B)
    assert len(set(keys.tolist())) == nb
    for k in range(nb):
        u = t.copy()
        u[k * B + 3] += 1                              # one token of block k changes
        ku, _ = oracle.prefix_hash(u, [0, u.size], B)
        assert (ku[:k] == keys[:k]).all()              # blocks before it keep their keys
        assert (ku[k:] != keys[k:]).all()              # it and EVERY later block change, though later tokens are equal
    # a key depends only on the tokens up to the end of its block: the keys of a truncated prompt are a prefix
    kt, _ = oracle.prefix_hash(t[:B * 4], [0, B * 4], B)
    np.testing.assert_array_equal(kt, keys[:4])
    # identical blocks at different depths get different keys (the prefix enters), also in first place vs later
    rep = np.tile(t[:B], 5)
    kr, _ = oracle.prefix_hash(rep, [0, rep.size], B)
    assert len(set(kr.tolist())) == 5


def test_order_inside_a_block_and_partial_blocks_matter(oracle):
    B = 8
    t = np.arange(100, 100 + 2 * B, dtype=np.int32)
    k0, _ = oracle.prefix_hash(t, [0, t.size], B)
    u = t.copy()
    u[[1, 2]] = u[[2, 1]]                               # same multiset of tokens in block 0, other order
    k1, _ = oracle.prefix_hash(u, [0, u.size], B)
    assert k1[0] != k0[0]
    # a partial last block gets a key of its own; extending it changes that key and only that key
    k5, o5 = oracle.prefix_hash(t[:B + 5], [0, B + 5], B)
    k6, _ = oracle.prefix_hash(t[:B + 6], [0, B + 6], B)
    assert k5.size == 2 and o5.tolist() == [0, 2]
    assert k5[0] == k6[0] == k0[0] and k5[1] != k6[1] and k6[1] != k0[1]
    # a block of zeros is not the same as a shorter block of zeros
    z = np.zeros(B, dtype=np.int32)
    assert oracle.prefix_hash(z, [0, B], B)[0][0] != oracle.prefix_hash(z[:5], [0, 5], B)[0][0]
    # empty requests have no keys; requests do not see each other
    kk, off = oracle.prefix_hash(np.concatenate([t, t[:3], t]), [0, t.size, t.size, t.size + 3, 2 * t.size + 3], B)
    assert off.tolist() == [0, 2, 2, 3, 5]
    np.testing.assert_array_equal(kk[0:2], k0)
    np.testing.assert_array_equal(kk[3:5], k0)


def test_no_collisions_among_many_random_blocks(oracle):
    rng = np.random.default_rng(2)
    B, n = 32, 50000
    t = rng.integers(0, 8, size=(n, B), dtype=np.int32)            # tiny vocabulary: many near-equal blocks
    t = np.unique(t, axis=0)
    off = np.arange(t.shape[0] + 1, dtype=np.int64) * B
    keys, _ = oracle.prefix_hash(t.reshape(-1), off, B)
    assert np.unique(keys).size == t.shape[0]


def brute_match(req_keys, inst_sets):
    out = []
    for s in inst_sets:
        n = 0
        for k in req_keys:
            if k not in s:
                break
            n += 1
        out.append(n)
    return out


def test_prefix_match_against_python_sets(oracle):
    rng = np.random.default_rng(3)
    B = 4
    prompts = [rng.integers(0, 50, size=rng.integers(0, 60), dtype=np.int32) for _ in range(9)]
    prompts.append(prompts[0][:17].copy())                          # a prompt that is a prefix of another
    off = np.zeros(len(prompts) + 1, dtype=np.int64)
    np.cumsum([p.size for p in prompts], out=off[1:])
    keys, koff = oracle.prefix_hash(np.concatenate(prompts), off, B)
    per_req = [keys[koff[r]:koff[r + 1]] for r in range(len(prompts))]
    # instances hold: everything of request 0; the first 3 blocks of request 1 plus block 5 (a hole at 3, 4);
    # nothing; all keys of all requests
    inst = [set(per_req[0].tolist()), set(per_req[1][:3].tolist()) | set(per_req[1][5:6].tolist()), set(),
            set(keys.tolist())]
    cache = [np.array(sorted(s), dtype=np.uint64) for s in inst]
    coff = np.zeros(len(inst) + 1, dtype=np.int64)
    np.cumsum([c.size for c in cache], out=coff[1:])
    plen, best_len, best_inst = oracle.prefix_match(keys, koff, np.concatenate(cache), coff)
    for r, rk in enumerate(per_req):
        want = brute_match(rk.tolist(), inst)
        assert plen[r].tolist() == want
        assert best_len[r] == max(want) and best_inst[r] == want.index(max(want))
    assert plen[1, 1] == min(3, per_req[1].size)                    # the hole ends the match even though block 5 is there
    # no instances at all
    plen0, bl0, bi0 = oracle.prefix_match(keys, koff, np.zeros(0, dtype=np.uint64), [0])
    assert plen0.shape == (len(prompts), 0) and (bl0 == 0).all() and (bi0 == -1).all()
