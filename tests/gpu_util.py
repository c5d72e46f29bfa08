"""Helpers for the GPU parity tests: move a workloads case to the device, call the C ABI, compare."""
import numpy as np
import torch

from paper_2407_00079_amd import binding as B
from paper_2407_00079_amd import workloads as W


def dev(a: np.ndarray) -> torch.Tensor:
    """Raw bytes of a numpy array on cuda:0 (uint16 bit patterns travel as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to("cuda:0")


class DeviceCase:
    def __init__(self, case: W.AttnCase):
        self.case = case
        self.q = dev(case.q)
        self.k_pool = dev(case.k_pool)
        self.v_pool = dev(case.v_pool)
        self.block_tables = dev(case.block_tables)
        self.params = B.attn_params(case.num_q_heads, case.num_kv_heads, case.head_dim, case.page_size,
                                    case.num_pages, case.dtype)
        ws = B.mc_prefill_attn_workspace_bytes(self.params, case.batch, case.total_new)
        self.workspace = torch.empty(max(ws, 16), dtype=torch.uint8, device="cuda:0")
        # outputs start as NaN so that a row the kernel skips is caught
        if case.dtype == W.BF16:
            self.out = torch.full(case.q.shape, float("nan"), dtype=torch.bfloat16, device="cuda:0")
        else:
            self.out = torch.full(case.q.shape, float("nan"), dtype=torch.float32, device="cuda:0")
        self.lse = torch.full((case.total_new, case.num_q_heads), float("nan"), dtype=torch.float32, device="cuda:0")

    def run(self, scale: float = 0.0, stream=None, want_lse: bool = True):
        self.params.softmax_scale = scale
        B.mc_prefill_attn_paged(self.params, self.q, self.k_pool, self.v_pool, self.block_tables,
                                self.case.prefix_lens.tolist(), self.case.new_lens.tolist(), self.out,
                                self.lse if want_lse else None, self.workspace, stream)

    def result(self):
        torch.cuda.synchronize()
        return self.out.float().cpu().numpy().astype(np.float64), self.lse.cpu().numpy().astype(np.float64)


# lse (bf16): the row sum is taken over the probabilities as rounded to bf16 for P V.  Each rounded value is
# off by at most 2^-8 relative (8 significant bits), so is their sum, so |delta lse| <= 2^-8 = 3.9e-3 nats; the
# bound is met when one key dominates a row with a probability that bf16 does not represent.
TOL = {W.BF16: dict(max_abs=2e-2, rel_l2=1e-2, lse_abs=4e-3),
       W.F32: dict(max_abs=1e-4, rel_l2=1e-5, lse_abs=1e-4)}


def check_close(got: np.ndarray, ref: np.ndarray, dtype: str, what: str = ""):
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    tol = TOL[dtype]
    max_abs = float(np.abs(got - ref).max()) if got.size else 0.0
    rel_l2 = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)) if got.size else 0.0
    assert max_abs <= tol["max_abs"], f"{what}: max-abs {max_abs:.3e} > {tol['max_abs']}"
    assert rel_l2 <= tol["rel_l2"], f"{what}: rel-L2 {rel_l2:.3e} > {tol['rel_l2']}"
    return max_abs, rel_l2


def gather_rows(out: np.ndarray, lse: np.ndarray, case: W.AttnCase, rows: np.ndarray):
    off = case.q_offsets
    idx = off[rows[:, 0]] + rows[:, 2]
    return out[idx, rows[:, 1]], lse[idx, rows[:, 1]]
