"""The C-ABI library loads, exports what include/mc.h declares, and rejects bad arguments on the host.

No kernel runs here: every case below fails validation before the first HIP call.
"""
import ctypes
import os
import re

import pytest

from paper_2407_00079_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000      # a non-null, 16-byte aligned address that is never dereferenced


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2407_00079_amd import build
        build.build()
    return B.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = {B.status_string(s) for s in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert B.status_string(99) == "unknown status"


def good_params():
    return B.attn_params(64, 8, 128, 16, 4096, "bf16")


def call(params, q=FAKE, k=FAKE, v=FAKE, bt=FAKE, max_pages=1024, prefix=(8192,), new=(8192,), out=FAKE, lse=None,
         ws=FAKE, ws_bytes=1 << 30, batch=None):
    n = len(prefix)
    pl = (ctypes.c_int32 * max(n, 1))(*prefix)
    nl = (ctypes.c_int32 * max(n, 1))(*new)
    return B.mc_prefill_attn_paged_raw(params, q, k, v, bt, max_pages, ctypes.cast(pl, ctypes.c_void_p),
                                       ctypes.cast(nl, ctypes.c_void_p), n if batch is None else batch, out, lse,
                                       ws, ws_bytes, None)


def test_attention_argument_errors(lib):
    assert call(None) == B.MC_ERR_NULL
    p = good_params(); p.num_kv_heads = 7
    assert call(p) == B.MC_ERR_SHAPE
    p = good_params(); p.head_dim = 96
    assert call(p) == B.MC_ERR_UNSUPPORTED
    p = good_params(); p.page_size = 32
    assert call(p) == B.MC_ERR_UNSUPPORTED
    p = good_params(); p.dtype = 5
    assert call(p) == B.MC_ERR_UNSUPPORTED
    p = B.attn_params(4, 1, 128, 16, 64, "f32")
    assert call(p) == B.MC_ERR_UNSUPPORTED
    p = good_params(); p.softmax_scale = -1.0
    assert call(p) == B.MC_ERR_SHAPE
    p = good_params()
    assert call(p, q=None) == B.MC_ERR_NULL
    assert call(p, out=None) == B.MC_ERR_NULL
    assert call(p, bt=None) == B.MC_ERR_NULL
    assert call(p, q=FAKE + 8) == B.MC_ERR_ALIGN
    assert call(p, k=FAKE + 2) == B.MC_ERR_ALIGN
    assert call(p, prefix=(-1,)) == B.MC_ERR_SHAPE
    assert call(p, new=(-5,)) == B.MC_ERR_SHAPE
    assert call(p, max_pages=1023) == B.MC_ERR_SHAPE            # 1023 * 16 < 16384
    assert call(p, ws=None) == B.MC_ERR_WORKSPACE
    assert call(p, ws_bytes=64) == B.MC_ERR_WORKSPACE
    assert call(p, batch=-1) == B.MC_ERR_SHAPE
    assert call(p, prefix=(2**31 - 8,), new=(16,), max_pages=2**27) == B.MC_ERR_RANGE


def test_attention_noops_need_no_buffers(lib):
    p = good_params()
    assert call(p, q=None, k=None, v=None, bt=None, out=None, ws=None, ws_bytes=0, prefix=(), new=()) == B.MC_OK
    assert call(p, q=None, k=None, v=None, bt=None, out=None, ws=None, ws_bytes=0, prefix=(100, 7), new=(0, 0)) == B.MC_OK


def test_workspace_size(lib):
    p = good_params()
    need = B.mc_prefill_attn_workspace_bytes(p, 1, 8192)
    assert 0 < need < (1 << 22)
    assert B.mc_prefill_attn_workspace_bytes(p, 16, 45000) > need
    p.head_dim = 77
    assert B.mc_prefill_attn_workspace_bytes(p, 1, 8192) == 0
    assert B.mc_prefill_attn_workspace_bytes(good_params(), -1, 10) == 0


@pytest.mark.parametrize("fn", [B.mc_kv_pack_layer_raw, B.mc_kv_unpack_layer_raw])
def test_copy_argument_errors(lib, fn):
    ok = dict(a=FAKE, b=FAKE, num_pages=64, page_bytes=4096, ids=FAKE, n=24, c=FAKE, d=FAKE)

    def run(**kw):
        x = dict(ok, **kw)
        return fn(x["a"], x["b"], x["num_pages"], x["page_bytes"], x["ids"], x["n"], x["c"], x["d"], None)

    assert run(a=None) == B.MC_ERR_NULL
    assert run(d=None) == B.MC_ERR_NULL
    assert run(ids=None) == B.MC_ERR_NULL
    assert run(page_bytes=4100) == B.MC_ERR_ALIGN
    assert run(b=FAKE + 4) == B.MC_ERR_ALIGN
    assert run(n=-1) == B.MC_ERR_SHAPE
    assert run(page_bytes=-16) == B.MC_ERR_SHAPE
    assert run(num_pages=0) == B.MC_ERR_SHAPE
    assert run(n=2**31) == B.MC_ERR_RANGE
    assert run(n=0, a=None, b=None, c=None, d=None, ids=None) == B.MC_OK


def test_suggested_key_slices(lib):
    """Host arithmetic only: the slice count with the fewest rounds of 256 work items (1 % per extra slice),
    capped by MC_MAX_KV_SPLITS and by 8 tiles of 64 keys per slice of the longest request."""
    p = good_params()                                            # 64 / 8 heads: 8 stacked rows per token
    s = B.mc_prefill_attn_suggest_kv_splits
    assert s(p, [8192], [8192]) == 1                             # 8 heads x 256 row tiles = 2048 items
    assert s(p, [131056], [16]) == 32                            # 8 items -> 256 / 8
    assert s(p, [131071], [1]) == 32                             # one token is still one item per KV head
    assert s(p, [944], [16]) == 1                                # 960 keys = 15 tiles: two slices of 8 do not fit
    assert s(p, [945], [16]) == 2                                # 961 keys = 16 tiles
    assert s(p, [32768, 40], [16, 0]) == 32                      # requests without new tokens add no items
    assert s(p, [32768] * 4, [16] * 4) == 8                      # 32 items -> 8
    assert s(p, [], []) == 1
    one = good_params()
    one.num_q_heads, one.num_kv_heads = 8, 1                     # config-3 heads: one item per 32 tokens
    assert s(one, [1 << 20], [8]) == B.MC_MAX_KV_SPLITS          # 256 / 1, within the cap
    assert s(one, [200000], [8192]) == 1                         # 256 items: one full round
    assert s(one, [120832], [10240]) == 4                        # 320 items: 2 rounds whole, 5 rounds of quarters
    assert s(one, [110592], [20480]) == 2                        # 640 items: 3 rounds whole, 5 rounds of halves
    assert s(one, [114688], [16384]) == 1                        # 512 items: two full rounds
    assert s(one, [1 << 20], [40000]) == 1                       # 1250 items: the launch order balances the tail
    assert s(p, [-1], [16]) == 0 and s(p, [5], [-2]) == 0
    bad = good_params()
    bad.head_dim = 77
    assert s(bad, [100], [16]) == 0


def test_prepare_and_run_host_side(lib):
    """What prepare / run decide without touching the GPU: empty plans, plans that do not fit the call."""
    p = good_params()

    def prepare(prefix, new, kv_splits, ws=None, ws_bytes=0):
        pl, nl = (ctypes.c_int32 * len(prefix))(*prefix), (ctypes.c_int32 * len(new))(*new)
        out = B.McAttnPlan()
        st = lib.mc_prefill_attn_prepare(ctypes.byref(p), pl, nl, len(prefix), kv_splits, ws, ws_bytes, None,
                                         ctypes.byref(out))
        return st, out

    st, plan = prepare([100, 7], [0, 0], 0)                      # no new tokens: empty plan, no workspace needed
    assert st == B.MC_OK
    assert (plan.n_items, plan.batch, plan.total_new_tokens, plan.kv_splits) == (0, 2, 0, 0)
    run = lib.mc_prefill_attn_run
    assert run(ctypes.byref(p), ctypes.byref(plan), None, None, None, None, 0, None, None, None, None) == B.MC_OK
    assert lib.mc_kv_append_run(ctypes.byref(p), ctypes.byref(plan), None, None, None, None, None, 0, None, None) == B.MC_OK
    # a plan is tied to the head counts and dtype it was prepared with, and to its form
    other = B.attn_params(32, 8, 128, 16, 4096, "bf16")
    assert run(ctypes.byref(other), ctypes.byref(plan), None, None, None, None, 0, None, None, None, None) == B.MC_ERR_SHAPE
    assert lib.mc_prefill_attn_run_split(ctypes.byref(p), ctypes.byref(plan), None, None, None, None, 0, None, None, None,
                                         None) == B.MC_ERR_SHAPE
    assert run(ctypes.byref(p), None, None, None, None, None, 0, None, None, None, None) == B.MC_ERR_NULL
    # a plan with work in it (filled in by hand here: no upload happens in this test) is checked against the buffers
    full = B.McAttnPlan(2048, 1, 0, 1024, 8192, 32768, 64, 8, B.MC_DTYPE_BF16, 0)
    assert run(ctypes.byref(p), ctypes.byref(full), FAKE, FAKE, FAKE, FAKE, 1000, FAKE, None, FAKE, None) == B.MC_ERR_SHAPE
    assert run(ctypes.byref(p), ctypes.byref(full), None, FAKE, FAKE, FAKE, 1024, FAKE, None, FAKE, None) == B.MC_ERR_NULL
    assert run(ctypes.byref(p), ctypes.byref(full), FAKE + 4, FAKE, FAKE, FAKE, 1024, FAKE, None, FAKE, None) == B.MC_ERR_ALIGN
    assert run(ctypes.byref(p), ctypes.byref(full), FAKE, FAKE, FAKE, FAKE, 1024, FAKE, None, None, None) == B.MC_ERR_WORKSPACE
    # prepare: bad lengths and a missing workspace are refused before any GPU call
    assert prepare([-1], [5], 0)[0] == B.MC_ERR_SHAPE
    assert prepare([8192], [8192], 0)[0] == B.MC_ERR_WORKSPACE
    assert prepare([8192], [8192], 0, FAKE, 64)[0] == B.MC_ERR_WORKSPACE
    assert prepare([8192], [8192], B.MC_MAX_KV_SPLITS + 1)[0] == B.MC_ERR_SHAPE


def test_auto_workspace_size(lib):
    p = good_params()
    w = B.mc_prefill_attn_auto_workspace_bytes
    assert w(p, [8192], [8192]) == B.mc_prefill_attn_workspace_bytes(p, 1, 8192)        # whole-row: nothing extra
    rows, s = 16 * 64, B.mc_prefill_attn_suggest_kv_splits(p, [131056], [16])
    need = w(p, [131056], [16])
    lower = B.mc_prefill_attn_split_workspace_bytes(p, 1, 16, s) + s * rows * 129 * 4
    assert s == 32 and lower <= need <= lower + 1024                                      # list + partials (+ alignment)
    assert w(p, [-1], [16]) == 0
    assert w(p, [], []) > 0
