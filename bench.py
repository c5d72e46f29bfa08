#!/usr/bin/env python3
"""Benchmark of the KVCache-reuse hot path on one MI355X.

One step = one layer of layer-wise prefill (paper Section 5.2) on two HIP streams:
  copy stream:    mc_kv_unpack_layer(l)  (load the layer's KV pages into the paged pool)
  compute stream: wait load(l) -> mc_kv_append_paged (the chunk's new K/V rows into their pages)
                  -> mc_prefill_attn_paged (the attention workload)
  copy stream:    wait attention(l) -> mc_kv_pack_layer(l)  (store the layer's pages)
The attention workload is configuration 2 (64/8 heads, head_dim 128, bf16, 8192 reused
prefix tokens + 8192 new tokens); the page traffic is one layer of configuration 5
(2048 pages of 32 KiB for K and for V, each direction).  Inputs are seeded synthetic
tensors, resident in HBM before the timed region.

Prints ONE JSON line.  `value` is attention TFLOP/s over the whole timed region
(visible query-key pairs only, both contractions), with the page traffic overlapped.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2516.6   # 256 CU x 4 SIMD x 1024 flop/cycle x 2.4 GHz
HBM_PEAK_GBS = 8000.0


def measured_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary (None if it is absent)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_bench_step.txt")
    out = {}
    try:
        for line in open(path):
            if "=" in line and not line.startswith("#"):
                k, v = line.split("=")
                out[k.strip()] = int(v)
    except OSError:
        pass
    return out


def mfma_ceiling():
    """Rate of back-to-back bf16 MFMAs alone on this board (zeros / ones / random operands), measured by the
    stand-alone program bench_probes.hip; None when it is missing or fails."""
    import subprocess
    exe = os.path.join(ROOT, "bench_probes")
    try:
        if not os.path.exists(exe):
            import __graft_entry__
            __graft_entry__.build_bench_probes()
        out = subprocess.run([exe], capture_output=True, text=True, timeout=60, check=True).stdout.split()
        return {out[i]: {"tflops": float(out[i + 1]), "shader_mhz": float(out[i + 2])} for i in (0, 3, 6)}
    except Exception as e:      # measurement aid only: the benchmark goes on without it
        sys.stderr.write(f"mfma_ceiling unavailable: {e}\n")
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--attn-config", type=int, default=2, choices=(2, 3, 4),
                    help="attention workload of the step (default: configuration 2)")
    ap.add_argument("--layers", type=int, default=8, help="distinct per-layer pools the steps cycle through")
    ap.add_argument("--cpu-rows", type=int, default=65536, help="rows the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-extra", action="store_true", help="skip the isolated / configuration-3 measurements")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="DIAGNOSTIC, not a measurement of the workload: Q, K and V all zero (same kernels, same "
                         "instruction stream, no operand bit activity) to show what the board's power limit costs")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch
    from paper_2407_00079_amd import binding as B
    from paper_2407_00079_amd import workloads as W

    B.lib()   # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    K, Wm = args.steps, args.warmup

    def to_dev(a):
        a = np.ascontiguousarray(a)
        return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(dev)

    class Attn:
        def __init__(self, idx):
            self.idx = idx
            self.case = W.make_config_attn(idx, poison=False)
            c = self.case
            self.q, self.k, self.v, self.bt = to_dev(c.q), to_dev(c.k_pool), to_dev(c.v_pool), to_dev(c.block_tables)
            self.params = B.attn_params(c.num_q_heads, c.num_kv_heads, c.head_dim, c.page_size, c.num_pages, c.dtype)
            self.ws = torch.empty(B.mc_prefill_attn_workspace_bytes(self.params, c.batch, c.total_new),
                                  dtype=torch.uint8, device=dev)
            self.out = torch.empty(c.q.shape, dtype=torch.bfloat16, device=dev)
            self.lse = torch.empty((c.total_new, c.num_q_heads), dtype=torch.float32, device=dev)
            self.pl, self.nl = c.prefix_lens.tolist(), c.new_lens.tolist()
            self.flops = c.flops()
            # the chunk's K/V rows as the projection would hand them over: [total_new, Hkv, D], gathered from the
            # pages they belong in, so that appending them leaves the pools as they are
            pos = torch.cat([torch.arange(p, p + n, device=dev) for p, n in zip(self.pl, self.nl)])
            req = torch.cat([torch.full((n,), r, device=dev, dtype=torch.long) for r, n in enumerate(self.nl)])
            page = self.bt.long()[req, pos // c.page_size]
            self.k_new = self.k[page, :, pos % c.page_size, :].contiguous()
            self.v_new = self.v[page, :, pos % c.page_size, :].contiguous()
            if args.zero_inputs:
                for t in (self.q, self.k, self.v, self.k_new, self.v_new):
                    t.zero_()

            # work list and request table: prepared and uploaded once per batch, as a prefill pass would for all of
            # its layers; append and attention of every step then only launch their kernels
            self.plan = B.mc_prefill_attn_prepare(self.params, self.pl, self.nl, 0, self.ws)
            self.ws_one_shot = torch.empty_like(self.ws)
            torch.cuda.synchronize()          # the upload has landed before any stream runs from the plan

        def append(self, stream):
            B.mc_kv_append_run(self.params, self.plan, self.k_new, self.v_new, self.k, self.v, self.bt, self.ws, stream)

        def launch(self, stream):
            B.mc_prefill_attn_run(self.params, self.plan, self.q, self.k, self.v, self.bt, self.out, self.lse, self.ws,
                                  stream)

        def launch_one_shot(self, stream):
            # the same attention through the call that builds and uploads its work list itself
            B.mc_prefill_attn_paged(self.params, self.q, self.k, self.v, self.bt, self.pl, self.nl, self.out,
                                    self.lse, self.ws_one_shot, stream)

        def time_isolated(self, iters=20, warm=5):
            s = torch.cuda.current_stream()
            for _ in range(warm):
                self.launch(s)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
            for a, b in ev:
                a.record(s)
                self.launch(s)
                b.record(s)
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in ev)
            return ms[len(ms) // 2], ms[0]

    attn = Attn(args.attn_config)

    # ---- one layer's page traffic (configuration 5), `layers` distinct pool sets so steps do not hit in cache
    sh = W.config_shapes(5)
    n, pb, N1, N2 = sh["n"], sh["page_bytes"], sh["num_pages"], sh["num_pages_dst"]
    rng = np.random.default_rng(sh["seed"])
    src_ids = to_dev(rng.permutation(N1)[:n].astype(np.int32))
    dst_ids = to_dev(rng.permutation(N2)[:n].astype(np.int32))
    gen = torch.Generator(device=dev)
    gen.manual_seed(sh["seed"])
    LAY = args.layers
    # remote (contiguous) copies to load from, pools to load into / store from, contiguous buffers to store to
    k_remote = torch.randint(0, 256, (LAY, n, pb), dtype=torch.uint8, device=dev, generator=gen)
    v_remote = torch.randint(0, 256, (LAY, n, pb), dtype=torch.uint8, device=dev, generator=gen)
    k_pool = torch.randint(0, 256, (LAY, N2, pb), dtype=torch.uint8, device=dev, generator=gen)
    v_pool = torch.randint(0, 256, (LAY, N2, pb), dtype=torch.uint8, device=dev, generator=gen)
    k_store = torch.empty((LAY, n, pb), dtype=torch.uint8, device=dev)
    v_store = torch.empty((LAY, n, pb), dtype=torch.uint8, device=dev)
    copy_bytes = 2 * 2 * n * pb          # read + write, K and V, one direction

    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()

    # the order in which unpack takes the pages (ascending pool address): computed once per page list, as a caller
    # would per request, and reused by every layer
    order = torch.empty(n, dtype=torch.int32, device=dev)
    B.mc_kv_page_order(dst_ids, n, order)

    def unpack(l, stream):
        B.mc_kv_unpack_layer_ordered(k_remote[l], v_remote[l], N2, pb, dst_ids, order, n, k_pool[l], v_pool[l], stream)

    def unpack_list_order(l, stream):
        B.mc_kv_unpack_layer(k_remote[l], v_remote[l], N2, pb, dst_ids, n, k_pool[l], v_pool[l], stream)

    def pack(l, stream):
        B.mc_kv_pack_layer(k_pool[l], v_pool[l], N2, pb, dst_ids, n, k_store[l], v_store[l], stream)

    def run_steps(count, timed):
        """Layer-wise schedule: load(l+1) is in flight while attention(l) runs; store(l) follows attention(l)."""
        marks, copy_marks = [], {"unpack": [], "pack": []}

        def timed_copy(name, fn, l):
            # events on the copy stream itself, around the one launch
            if not timed:
                return fn(l, copy)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(copy)
            fn(l, copy)
            b.record(copy)
            copy_marks[name].append((a, b))

        loaded = [torch.cuda.Event() for _ in range(count + 1)]
        attended = [torch.cuda.Event() for _ in range(count)]
        with torch.cuda.stream(copy):
            unpack(0, copy)
            loaded[0].record(copy)
        for i in range(count):
            l = i % LAY
            with torch.cuda.stream(copy):
                if i + 1 < count:
                    timed_copy("unpack", unpack, (i + 1) % LAY)
                    loaded[i + 1].record(copy)
            with torch.cuda.stream(compute):
                compute.wait_event(loaded[i])
                attn.append(compute)
                if timed:
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record(compute)
                attn.launch(compute)
                if timed:
                    b.record(compute)
                    marks.append((a, b))
                attended[i].record(compute)
            with torch.cuda.stream(copy):
                copy.wait_event(attended[i])
                timed_copy("pack", pack, l)
        return marks, copy_marks

    run_steps(Wm, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks, copy_marks = run_steps(K, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    attn_ms = sorted(a.elapsed_time(b) for a, b in marks)
    attn_ms_avg = sum(attn_ms) / len(attn_ms)
    value = attn.flops / (ms_per_step * 1e-3) / 1e12
    traffic = measured_traffic()

    def hbm(prefix):
        r, w = traffic.get(prefix + "_read_bytes"), traffic.get(prefix + "_write_bytes")
        return None if r is None or w is None else {"bytes": r + w, "read_bytes": r, "write_bytes": w, "unit": "B per launch",
                                                    "source": "profiles/hbm_traffic_bench_step.txt"}

    result = {
        "metric": "prefill attn TFLOP/s (% MFMA peak); KV pack/unpack GB/s (% HBM peak)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic" if not args.zero_inputs else "ALL-ZERO tensors: power diagnostic, not the workload",
        "config": {"workload": f"config {args.attn_config} attention "
                               f"(P={attn.pl if len(attn.pl) < 3 else 'varlen'}, C={attn.nl if len(attn.nl) < 3 else 'varlen'}, "
                               f"{attn.case.num_q_heads}/{attn.case.num_kv_heads} heads, D=128, 16-token pages) "
                               f"preceded by the append of its chunk's K/V rows (work list prepared once per batch: "
                               f"mc_prefill_attn_prepare, then mc_kv_append_run + mc_prefill_attn_run per step), "
                               f"+ one config-5 layer of KV unpack and pack (2048 pages x 32 KiB, K and V) on a second stream",
                   "attn_flops_per_step": attn.flops, "copy_bytes_per_step": 2 * copy_bytes},
        "pct_mfma_peak": round(100 * value / MFMA_BF16_PEAK_TFLOPS, 2),
        "roofline": {"kernel": "attn_prefill_kernel<Bf16>", "bound": "mfma",
                     "achieved": round(attn.flops / (attn_ms_avg * 1e-3) / 1e12, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s",
                     "frac": round(attn.flops / (attn_ms_avg * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "avg_launch_ms": round(attn_ms_avg, 4), "min_launch_ms": round(attn_ms[0], 4),
                     "launch_ms": [round(a.elapsed_time(b), 3) for a, b in marks],
                     "traffic": hbm("attn_config2") if args.attn_config == 2 else None},
    }

    # the copies as they ran inside the step, beside the attention of the neighbouring layer
    in_step = {}
    for name, ms in copy_marks.items():
        us = sorted(a.elapsed_time(b) * 1e3 for a, b in ms)
        if us:
            in_step[name] = {"us_median": round(us[len(us) // 2], 2), "us_min": round(us[0], 2), "us_max": round(us[-1], 2)}
    result["copies_in_step"] = in_step

    if not args.no_extra:
        # isolated kernels, same inputs, nothing else running
        med, mn = attn.time_isolated()
        result["attn_isolated"] = {"config": args.attn_config, "ms_median": round(med, 4), "ms_min": round(mn, 4),
                                   "tflops": round(attn.flops / (med * 1e-3) / 1e12, 2),
                                   "pct_mfma_peak": round(100 * attn.flops / (med * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2)}
        s = torch.cuda.current_stream()
        # the one-shot call (list built and uploaded inside every call), back to back like the isolated runs
        for _ in range(3):
            attn.launch_one_shot(s)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(s)
        for _ in range(10):
            attn.launch_one_shot(s)
        b.record(s)
        torch.cuda.synchronize()
        result["attn_one_shot_call"] = {"ms_per_call_back_to_back": round(a.elapsed_time(b) / 10, 4),
                                        "what": "mc_prefill_attn_paged: prepare + run in one call"}

        def pack_ordered(l, stream):
            B.mc_kv_pack_layer_ordered(k_pool[l], v_pool[l], N2, pb, dst_ids, order, n, k_store[l], v_store[l], stream)

        # pack writes its output in list order, unpack (with the order) its pool pages in address order; the other
        # two combinations are measured for comparison: the write side is the one that wants to be sequential
        for name, fn in (("pack", pack), ("unpack", unpack), ("pack_pool_order", pack_ordered),
                         ("unpack_list_order", unpack_list_order)):
            for l in range(LAY):
                fn(l, s)
            reps = 80
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(s)
            for i in range(reps):           # 80 layers back to back, launch gaps included
                fn(i % LAY, s)
            b.record(s)
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / reps
            gbs = copy_bytes / (us * 1e-6) / 1e9
            result[f"roofline_{name}"] = {"kernel": f"kv_copy_kernel<{name.split('_')[0]}>", "bound": "hbm", "achieved": round(gbs, 1),
                                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                                          "us_per_layer": round(us, 2), "bytes_per_launch": copy_bytes,
                                          "traffic": hbm(name.split("_")[0])}
        # what a copy of the same bytes reaches on this board with nothing scattered: the same kernel with the pages
        # in pool order (ids 0 .. n-1), and the runtime's device-to-device copy
        seq_ids = torch.arange(n, dtype=torch.int32, device=dev)

        def pack_contiguous(l, stream):
            B.mc_kv_pack_layer(k_pool[l], v_pool[l], N2, pb, seq_ids, n, k_store[l], v_store[l], stream)

        def runtime_copy(l, stream):
            k_store[l].copy_(k_pool[l, :n])
            v_store[l].copy_(v_pool[l, :n])

        ceiling = {}
        for name, fn in (("same_kernel_contiguous", pack_contiguous), ("runtime_d2d_copy", runtime_copy)):
            for l in range(LAY):
                fn(l, s)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(s)
            for i in range(80):
                fn(i % LAY, s)
            b.record(s)
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / 80
            ceiling[name] = {"GBs": round(copy_bytes / (us * 1e-6) / 1e9, 1), "us_per_layer": round(us, 2),
                             "frac_hbm_peak": round(copy_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
        result["copy_ceiling"] = {"what": "the same 2 x 64 MiB read and written with no scatter at all", **ceiling}
        # append of the step's chunk alone, launched back to back
        c = attn.case
        for _ in range(5):
            attn.append(s)
        reps = 80
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(s)
        for i in range(reps):
            attn.append(s)
        b.record(s)
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / reps
        ab = 2 * 2 * c.total_new * c.num_kv_heads * c.head_dim * 2
        result["roofline_append"] = {"kernel": "kv_append_kernel", "bound": "hbm",
                                     "achieved": round(ab / (us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                     "frac": round(ab / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "us_per_launch": round(us, 2),
                                     "bytes_per_launch": ab, "traffic": None,
                                     "note": "same buffers every launch: the working set fits the 256 MiB last-level cache"}
        # the same layer-wise step against the HOST pool: a layer's pages come from pinned host memory before its
        # attention and go back after it (load on one side stream, store on another, attention on the compute stream)
        HL = min(4, LAY)
        kh_in = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        vh_in = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        kh_out = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        vh_out = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        for t in kh_in + vh_in:
            t.random_(0, 256)
        st_load, st_store = torch.cuda.Stream(), torch.cuda.Stream()

        def host_steps(count):
            loaded = [torch.cuda.Event() for _ in range(count + 1)]
            attended = [torch.cuda.Event() for _ in range(count)]
            B.mc_kv_load_layer(kh_in[0], vh_in[0], k_remote[0], v_remote[0], N2, pb, dst_ids, n, k_pool[0], v_pool[0],
                               st_load)
            loaded[0].record(st_load)
            for i in range(count):
                l, ln = i % HL, (i + 1) % HL
                if i + 1 < count:
                    B.mc_kv_load_layer(kh_in[ln], vh_in[ln], k_remote[ln], v_remote[ln], N2, pb, dst_ids, n, k_pool[ln],
                                       v_pool[ln], st_load)
                    loaded[i + 1].record(st_load)
                compute.wait_event(loaded[i])
                attn.append(compute)
                attn.launch(compute)
                attended[i].record(compute)
                st_store.wait_event(attended[i])
                B.mc_kv_store_layer(k_pool[l], v_pool[l], N2, pb, dst_ids, n, k_store[l], v_store[l], kh_out[l],
                                    vh_out[l], st_store)

        host_steps(4)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        host_steps(12)
        torch.cuda.synchronize()
        ms_host = (time.perf_counter() - t0) * 1e3 / 12
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        ev[0].record(st_load)
        for l in range(HL):
            B.mc_kv_load_layer(kh_in[l], vh_in[l], k_remote[l], v_remote[l], N2, pb, dst_ids, n, k_pool[l], v_pool[l], st_load)
        ev[1].record(st_load)
        torch.cuda.synchronize()
        ev[2].record(st_store)
        for l in range(HL):
            B.mc_kv_store_layer(k_pool[l], v_pool[l], N2, pb, dst_ids, n, k_store[l], v_store[l], kh_out[l], vh_out[l], st_store)
        ev[3].record(st_store)
        torch.cuda.synchronize()
        layer_bytes = 2 * n * pb
        result["host_streaming"] = {
            "what": "the step with each layer's 2048 pages (K and V, 32 KiB each) loaded from and stored to pinned host "
                    "memory: load and store on two side streams, append + attention on the compute stream",
            "ms_per_step": round(ms_host, 4), "attn_tflops": round(attn.flops / (ms_host * 1e-3) / 1e12, 1),
            "load_layer_ms_alone": round(ev[0].elapsed_time(ev[1]) / HL, 3),
            "load_GBs_alone": round(layer_bytes / (ev[0].elapsed_time(ev[1]) / HL * 1e-3) / 1e9, 1),
            "store_layer_ms_alone": round(ev[2].elapsed_time(ev[3]) / HL, 3),
            "store_GBs_alone": round(layer_bytes / (ev[2].elapsed_time(ev[3]) / HL * 1e-3) / 1e9, 1),
            "bytes_per_layer_per_direction": layer_bytes}
        del kh_in, vh_in, kh_out, vh_out
        # prefix keys of a batch of long prompts and their match against 16 instances' cache keys
        NP, LP, BT, NI, NC = 64, 131072, 512, 16, 200000
        g3 = torch.Generator(device=dev)
        g3.manual_seed(20240707)
        toks = torch.randint(0, 128000, (NP * LP,), dtype=torch.int32, device=dev, generator=g3)
        toff = [i * LP for i in range(NP + 1)]
        nkeys = NP * (LP // BT)
        pkeys = torch.empty(nkeys, dtype=torch.int64, device=dev)
        koff = [i * (LP // BT) for i in range(NP + 1)]
        ws_h = torch.empty(B.mc_prefix_hash_workspace_bytes(NP), dtype=torch.uint8, device=dev)
        ws_m = torch.empty(B.mc_prefix_match_workspace_bytes(NP, NI), dtype=torch.uint8, device=dev)
        B.mc_prefix_hash(toks, toff, BT, pkeys, ws_h, s)
        torch.cuda.synchronize()
        # instance i holds NC random keys plus the first 16 (i + 1) keys of every request, ascending (uint64 order)
        pk = pkeys.view(NP, LP // BT)
        caches = []
        for i in range(NI):
            mine = torch.cat([torch.randint(-2 ** 62, 2 ** 62, (NC,), dtype=torch.int64, device=dev, generator=g3),
                              pk[:, :16 * (i + 1)].reshape(-1)])
            u = torch.unique(mine)
            caches.append(torch.cat([u[u >= 0], u[u < 0]]))       # int64 bit patterns in unsigned ascending order
        coff = [0]
        for cch in caches:
            coff.append(coff[-1] + cch.numel())
        ckeys = torch.cat(caches)
        plen = torch.empty((NP, NI), dtype=torch.int32, device=dev)
        bl = torch.empty(NP, dtype=torch.int32, device=dev)
        bi = torch.empty(NP, dtype=torch.int32, device=dev)
        prefix = {"workload": f"{NP} prompts x {LP} tokens, {BT}-token blocks; {NI} instances of ~{NC + NP * 136} keys"}
        for name, fn in (("hash", lambda: B.mc_prefix_hash(toks, toff, BT, pkeys, ws_h, s)),
                         ("match", lambda: B.mc_prefix_match(pkeys, koff, ckeys, coff, plen, bl, bi, ws_m, s))):
            for _ in range(3):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(s)
            for _ in range(20):
                fn()
            b.record(s)
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / 20
            prefix[name] = {"us": round(us, 1)}
        prefix["hash"]["GBs"] = round(4 * NP * LP / (prefix["hash"]["us"] * 1e-6) / 1e9, 1)
        prefix["hash"]["frac_hbm_peak"] = round(prefix["hash"]["GBs"] / HBM_PEAK_GBS, 4)
        prefix["match"]["lookups_per_s"] = round(nkeys * NI / (prefix["match"]["us"] * 1e-6), 0)
        prefix["match"]["best_len_of_request_0"] = int(bl[0].item())
        result["prefix_keys"] = prefix
        del toks, pkeys, ckeys, caches
        labels = {3: "config 3: 8/1 heads, P=122880, C=8192 (128k context)",
                  4: "config 4: 16 requests, 64/8 heads, prefixes U[0,32768] (page multiples), chunks lognormal(median 2048)"}
        del attn.q, attn.k, attn.v, attn.out, attn.k_new, attn.v_new
        for idx in (3, 4):
            if idx == args.attn_config:
                continue
            other = Attn(idx)
            med, mn = other.time_isolated()
            result[f"attn_config{idx}"] = {"workload": labels[idx], "flops": other.flops, "ms_median": round(med, 4),
                                          "ms_min": round(mn, 4), "tflops": round(other.flops / (med * 1e-3) / 1e12, 2),
                                          "pct_mfma_peak": round(100 * other.flops / (med * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2)}
            del other
            torch.cuda.empty_cache()

    if not args.no_extra:
        def whole_vs_split(P2, C2, Hq2, Hkv2, iters):
            """Whole-row kernel against the slice count the library suggests + merge, one request."""
            npg = (P2 + C2) // 16
            g2 = torch.Generator(device=dev)
            g2.manual_seed(20240706)
            q2 = torch.randn(C2, Hq2, 128, device=dev, dtype=torch.bfloat16, generator=g2)
            k2 = torch.randn(npg, Hkv2, 16, 128, device=dev, dtype=torch.bfloat16, generator=g2)
            v2 = torch.randn(npg, Hkv2, 16, 128, device=dev, dtype=torch.bfloat16, generator=g2)
            bt2 = torch.randperm(npg, device=dev, generator=g2).to(torch.int32).reshape(1, npg).contiguous()
            prm = B.attn_params(Hq2, Hkv2, 128, 16, npg, "bf16")
            SP = B.mc_prefill_attn_suggest_kv_splits(prm, [P2], [C2])
            out2 = torch.empty_like(q2)
            ws_a = torch.empty(B.mc_prefill_attn_workspace_bytes(prm, 1, C2), dtype=torch.uint8, device=dev)
            ws_b = torch.empty(B.mc_prefill_attn_split_workspace_bytes(prm, 1, C2, SP), dtype=torch.uint8, device=dev)
            o_parts = torch.empty(SP, C2, Hq2, 128, device=dev, dtype=torch.float32)
            l_parts = torch.empty(SP, C2, Hq2, device=dev, dtype=torch.float32)
            s = torch.cuda.current_stream()

            def whole():
                B.mc_prefill_attn_paged(prm, q2, k2, v2, bt2, [P2], [C2], out2, None, ws_a, s)

            def split():
                B.mc_prefill_attn_paged_split(prm, q2, k2, v2, bt2, [P2], [C2], SP, o_parts, l_parts, ws_b, s)
                B.mc_attn_merge_lse(o_parts, l_parts, SP, C2 * Hq2, 128, B.MC_DTYPE_BF16, out2, None, s)

            fl2 = 4 * 128 * Hq2 * (C2 * P2 + C2 * (C2 + 1) // 2)
            rec = {"workload": f"{Hq2}/{Hkv2} heads, P={P2}, C={C2}", "flops": fl2}
            for name, fn in (("whole_row", whole), (f"split{SP}_plus_merge", split)):
                for _ in range(3):
                    fn()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(s)
                for _ in range(iters):
                    fn()
                b.record(s)
                torch.cuda.synchronize()
                us = a.elapsed_time(b) * 1e3 / iters
                rec[name] = {"us": round(us, 1), "tflops": round(fl2 / (us * 1e-6) / 1e12, 1)}
            return rec

        # the fp32 instantiation (configuration 1's arithmetic) at configuration 2's lengths, against the fp32 MFMA peak
        def fp32_attention():
            P2, C2, Hq2, Hkv2 = 8192, 8192, 64, 8
            npg = (P2 + C2) // 16
            g2 = torch.Generator(device=dev)
            g2.manual_seed(20240701)
            q2 = torch.randn(C2, Hq2, 64, device=dev, dtype=torch.float32, generator=g2)
            k2 = torch.randn(npg, Hkv2, 16, 64, device=dev, dtype=torch.float32, generator=g2)
            v2 = torch.randn(npg, Hkv2, 16, 64, device=dev, dtype=torch.float32, generator=g2)
            bt2 = torch.randperm(npg, device=dev, generator=g2).to(torch.int32).reshape(1, npg).contiguous()
            prm = B.attn_params(Hq2, Hkv2, 64, 16, npg, "f32")
            out2 = torch.empty_like(q2)
            ws2 = torch.empty(B.mc_prefill_attn_workspace_bytes(prm, 1, C2), dtype=torch.uint8, device=dev)
            s2 = torch.cuda.current_stream()
            for _ in range(2):
                B.mc_prefill_attn_paged(prm, q2, k2, v2, bt2, [P2], [C2], out2, None, ws2, s2)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(s2)
            for _ in range(5):
                B.mc_prefill_attn_paged(prm, q2, k2, v2, bt2, [P2], [C2], out2, None, ws2, s2)
            b.record(s2)
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / 5
            fl = 4 * 64 * Hq2 * (C2 * P2 + C2 * (C2 + 1) // 2)
            return {"workload": "fp32, 64/8 heads, head_dim 64, P=8192, C=8192", "flops": fl, "ms": round(ms, 3),
                    "tflops": round(fl / (ms * 1e-3) / 1e12, 1), "peak": 157.3,
                    "frac_fp32_mfma_peak": round(fl / (ms * 1e-3) / 1e12 / 157.3, 4)}

        result["attn_fp32"] = fp32_attention()
        torch.cuda.empty_cache()
        # a small chunk against a long prefix (16 new tokens behind 131056 cached ones, 64/8 heads): 8 work
        # items for 256 CUs unless the keys are split
        result["attn_small_chunk"] = whole_vs_split(131056, 16, 64, 8, 20)
        # just above one work item per compute unit (10240 new tokens, 8/1 heads: 320 items): the whole-row form
        # runs a second, mostly empty round
        result["attn_uneven_rounds"] = whole_vs_split(120832, 10240, 8, 1, 6)
        torch.cuda.empty_cache()
        torch.cuda.synchronize()
        ceil = mfma_ceiling()
        if ceil is not None:
            result["mfma_alone"] = {
                "what": "back-to-back bf16 32x32x16 MFMAs, nothing else running, 2 waves per SIMD, ~15 ms per case: "
                        "the board lowers its clock to hold its power limit, and MFMA power follows operand bit activity",
                **ceil,
                "attn_vs_random_data_rate": round(result["roofline"]["achieved"] / ceil["random"]["tflops"], 4)}
    if args.cpu_rows > 0:
        # the CPU oracle, as it stands, on a bounded sample of the same attention workload
        import oracle
        case = W.make_config_attn(args.attn_config, poison=False) if args.attn_config != attn.idx else attn.case
        rng = np.random.default_rng(1)
        rq = rng.integers(0, case.batch, size=args.cpu_rows)
        rows = np.stack([rq, rng.integers(0, case.num_q_heads, size=args.cpu_rows),
                         (rng.random(args.cpu_rows) * case.new_lens[rq]).astype(np.int64)], axis=1).astype(np.int32)
        rows = rows[case.new_lens[rows[:, 0]] > 0]
        row_flops = int((4 * case.head_dim * (case.prefix_lens[rows[:, 0]].astype(np.int64) + rows[:, 2] + 1)).sum())
        t0 = time.perf_counter()
        oracle.case_rows(case, rows)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": round(row_flops / dt / 1e12, 6), "unit": "TFLOP/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": f"{rows.shape[0]} uniformly drawn (head, row) outputs of the same config-"
                                            f"{args.attn_config} tensors, fp64, {dt:.1f} s; "
                                            f"full tensor would take ~{case.flops() / (row_flops / dt):.0f} s"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
