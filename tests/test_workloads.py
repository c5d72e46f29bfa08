"""Host logic of the input generators: bf16 rounding, paging layout, configuration recipes."""
import numpy as np
import torch

from paper_2407_00079_amd import workloads as W


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 37.0,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.3895314e38], np.float32)])
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    back = W.bf16_bits_to_f32(bits)
    np.testing.assert_array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    assert np.isnan(W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.array([np.nan], np.float32)))).all()


def test_paging_layout_matches_logical():
    case = W.make_attn_case(3, W.BF16, 4, 2, 8, 4, [5, 0], [6, 3], 16, keep_logical=True)
    for r in range(2):
        L = int(case.prefix_lens[r] + case.new_lens[r])
        for j in range(L):
            pg = case.block_tables[r, j // 4]
            np.testing.assert_array_equal(case.k_pool[pg, :, j % 4, :], case.k_logical[r][j])
            np.testing.assert_array_equal(case.v_pool[pg, :, j % 4, :], case.v_logical[r][j])
    used = np.concatenate([case.block_tables[0, :3], case.block_tables[1, :1]])
    assert len(np.unique(used)) == 4
    # tail slots and unreferenced pages are poisoned
    assert (case.k_pool[case.block_tables[0, 2], :, 3, :] == W.BF16_NAN_BITS).all()
    unused = np.setdiff1d(np.arange(16), used)
    assert (case.v_pool[unused] == W.BF16_NAN_BITS).all()


def test_configuration_recipes():
    assert W.make_config_attn(1).flops() == 42008576
    sh2 = W.config_shapes(2)
    p, c = sh2["prefix_lens"][0], sh2["new_lens"][0]
    assert 4 * 128 * 64 * (c * p + c * (c + 1) // 2) == 3298669101056
    sh3 = W.config_shapes(3)
    p, c = sh3["prefix_lens"][0], sh3["new_lens"][0]
    assert c * p + c * (c + 1) // 2 == 1040191488
    sh4 = W.config_shapes(4)
    assert len(sh4["prefix_lens"]) == 16 and all(x % 16 == 0 and 0 <= x <= 32768 for x in sh4["prefix_lens"])
    assert all(1 <= x <= 8192 for x in sh4["new_lens"])
    assert sh4 == W.config_shapes(4)
    sh5 = W.config_shapes(5)
    assert sh5["page_bytes"] == 32768 and sh5["n"] * 16 == sh5["tokens"]


def test_sample_rows_cover_edges():
    case = W.make_attn_case(3, W.BF16, 8, 2, 8, 16, [40, 0], [100, 7], 64)
    rows = W.sample_rows(case, 200, seed=1)
    assert rows.shape[1] == 3 and rows.shape[0] >= 200
    s = {tuple(r) for r in rows.tolist()}
    for r, c in ((0, 100), (1, 7)):
        for h in range(8):
            assert (r, h, 0) in s and (r, h, c - 1) in s
    assert all(0 <= i < case.new_lens[r] for r, _, i in rows)
