"""GPU parity: prefix block keys and longest prefix match against the CPU oracle, bit for bit (Algorithm 1)."""
import numpy as np
import pytest
import torch

from paper_2407_00079_amd import binding as B

pytestmark = pytest.mark.gpu


def gpu_keys(tokens, off, block_tokens):
    total = int(sum(-(-(off[r + 1] - off[r]) // block_tokens) for r in range(len(off) - 1)))
    keys = torch.full((max(total, 1),), -1, dtype=torch.int64, device="cuda:0")
    ws = torch.empty(B.mc_prefix_hash_workspace_bytes(len(off) - 1), dtype=torch.uint8, device="cuda:0")
    t = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to("cuda:0")
    B.mc_prefix_hash(t, [int(x) for x in off], block_tokens, keys, ws)
    torch.cuda.synchronize()
    return keys.cpu().numpy().view(np.uint64)[:total]


@pytest.mark.parametrize("lens,block_tokens", [
    ([6955, 6472], 512),                          # the lengths of the paper's two trace samples
    ([0, 1, 511, 512, 513, 0, 1024, 70], 512),    # empty requests, one token, around a block boundary
    ([131072], 512),                              # one 128k prompt: 256 blocks
    ([37, 5, 64, 63, 129], 16),                   # small blocks: more than one pass of the lanes does not arise
    ([1000] * 40, 100),                           # blocks that are no multiple of the wave width
    ([3, 0, 9, 1] * 17500 + [5000], 4),           # 70001 requests: more than one request per grid row; one long
])
def test_keys_match_oracle(oracle, lens, block_tokens):
    print(f"prefix hash case lens={lens[:6]} block={block_tokens}", flush=True)
    rng = np.random.default_rng(len(lens) + block_tokens)
    tokens = rng.integers(-5, 128000, size=sum(lens), dtype=np.int32)      # negative ids too: they are hashed as uint32
    off = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=off[1:])
    ref, _ = oracle.prefix_hash(tokens, off, block_tokens)
    got = gpu_keys(tokens, off, block_tokens)
    np.testing.assert_array_equal(got, ref)


def test_match_matches_oracle(oracle):
    rng = np.random.default_rng(9)
    Bt = 32
    base = rng.integers(0, 32000, size=Bt * 300, dtype=np.int32)
    prompts = []
    for r in range(12):                                         # prompts sharing prefixes of the base of varying depth
        keep = int(rng.integers(0, 300)) * Bt
        tail = rng.integers(0, 32000, size=int(rng.integers(0, 5000)), dtype=np.int32)
        prompts.append(np.concatenate([base[:keep], tail]))
    prompts.append(np.zeros(0, dtype=np.int32))                 # a request without tokens
    prompts.append(base.copy())                                 # 300 keys: more than one pass of the 256 threads
    off = np.zeros(len(prompts) + 1, dtype=np.int64)
    np.cumsum([p.size for p in prompts], out=off[1:])
    tokens = np.concatenate(prompts)
    keys, koff = oracle.prefix_hash(tokens, off, Bt)
    per_req = [keys[koff[r]:koff[r + 1]] for r in range(len(prompts))]
    # instances: prefixes of the base of different depths, one with a hole, an empty one, one holding everything
    bk = per_req[-1]
    inst = [bk[:50], bk[:299], np.concatenate([bk[:120], bk[121:]]), np.zeros(0, dtype=np.uint64), keys,
            np.concatenate([per_req[3], bk[:10]])]
    cache = [np.unique(c) for c in inst]
    coff = np.zeros(len(cache) + 1, dtype=np.int64)
    np.cumsum([c.size for c in cache], out=coff[1:])
    ck = np.concatenate(cache).astype(np.uint64)
    ref_len, ref_best, ref_inst = oracle.prefix_match(keys, koff, ck, coff)

    dkeys = torch.from_numpy(gpu_keys(tokens, off, Bt).view(np.int64)).to("cuda:0")
    dcache = torch.from_numpy(ck.view(np.int64)).to("cuda:0")
    n_req, n_inst = len(prompts), len(cache)
    plen = torch.full((n_req, n_inst), -7, dtype=torch.int32, device="cuda:0")
    best_len = torch.full((n_req,), -7, dtype=torch.int32, device="cuda:0")
    best_inst = torch.full((n_req,), -7, dtype=torch.int32, device="cuda:0")
    ws = torch.empty(B.mc_prefix_match_workspace_bytes(n_req, n_inst), dtype=torch.uint8, device="cuda:0")
    B.mc_prefix_match(dkeys, koff.tolist(), dcache, coff.tolist(), plen, best_len, best_inst, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(plen.cpu().numpy(), ref_len)
    np.testing.assert_array_equal(best_len.cpu().numpy(), ref_best)
    np.testing.assert_array_equal(best_inst.cpu().numpy(), ref_inst)
    assert ref_len[-1].tolist()[:5] == [50, 299, 120, 0, 300]   # the base prompt itself: the hole at 120 ends the match


def test_match_without_instances_and_rejections(oracle):
    keys = torch.zeros(4, dtype=torch.int64, device="cuda:0")
    best_len = torch.full((2,), -7, dtype=torch.int32, device="cuda:0")
    best_inst = torch.full((2,), -7, dtype=torch.int32, device="cuda:0")
    ws = torch.empty(B.mc_prefix_match_workspace_bytes(2, 0), dtype=torch.uint8, device="cuda:0")
    B.mc_prefix_match(keys, [0, 2, 4], None, [0], None, best_len, best_inst, ws)
    torch.cuda.synchronize()
    assert best_len.tolist() == [0, 0] and best_inst.tolist() == [-1, -1]
    with pytest.raises(B.McError) as e:
        B.mc_prefix_match(keys, [0, 4, 2], None, [0], None, best_len, best_inst, ws)
    assert e.value.status == B.MC_ERR_SHAPE
    t = torch.zeros(10, dtype=torch.int32, device="cuda:0")
    with pytest.raises(B.McError) as e:
        B.mc_prefix_hash(t, [0, 10], 0, keys, ws)
    assert e.value.status == B.MC_ERR_SHAPE
    with pytest.raises(B.McError) as e:
        B.mc_prefix_hash(t, [0, 10], 4, keys, None)
    assert e.value.status == B.MC_ERR_WORKSPACE
    B.mc_prefix_hash(t, [0, 0], 4, keys, None)            # no tokens: nothing to do
