#!/usr/bin/env python3
"""Benchmark of the KVCache-reuse hot path on one MI355X.

One step = one layer of layer-wise prefill (paper Section 5.2) on two HIP streams:
  copy stream:    mc_kv_unpack_layer(l + 1)  (load the next layer's KV pages into its paged pool)
  compute stream: wait load(l) -> mc_kv_append_run (the chunk's new K/V rows into their pages)
                  -> mc_prefill_attn_run (the attention workload)
  copy stream:    wait attention(l) -> mc_kv_pack_layer(l)  (store the layer's pages)
The attention workload of the headline is configuration 3, the long-context shape the target is stated on
(one GPU's tensor-parallel share of a 128k-token prompt: 8 query heads / 1 KV head, head_dim 128, bf16,
122880 reused prefix tokens + 8192 new tokens); the page traffic is one layer of configuration 5 (2048 pages
of 32 KiB for K and for V, each direction).  Inputs are seeded synthetic tensors, resident in HBM before the
timed region.

Prints ONE JSON line.  `value` is attention TFLOP/s over the whole timed region (visible query-key pairs
only, both contractions), with the page traffic overlapped.  Further fields: the roofline of every kernel,
the same step with configuration 2's attention, isolated kernels, what the board sustains for MFMAs alone
and for plain copies (bench_probes.hip), the step against a host-memory pool, and the CPU oracle timed on a
bounded sample.
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2516.6   # 256 CU x 4 SIMD x 1024 flop/cycle x 2.4 GHz
HBM_PEAK_GBS = 8000.0


def committed_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary ({} if it is absent).  Counters cannot be
    read inside a timed run: the figures are those of the profile named in the output."""
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


def probe(mode):
    """One mode of the stand-alone measurement program bench_probes.hip (None when it is missing or fails)."""
    exe = os.path.join(ROOT, "bench_probes")
    try:
        if not os.path.exists(exe):
            import __graft_entry__
            __graft_entry__.build_bench_probes()
        return json.loads(subprocess.run([exe, mode], capture_output=True, text=True, timeout=120, check=True).stdout)
    except Exception as e:      # measurement aid only: the benchmark goes on without it
        sys.stderr.write(f"bench_probes {mode} unavailable: {e}\n")
        return None


LABELS = {2: "config 2: 64/8 heads, P=8192, C=8192 (16k prompt, half cached)",
          3: "config 3: 8/1 heads, P=122880, C=8192 (last chunk of a 128k prompt, one GPU's tensor-parallel share)",
          4: "config 4: 16 requests, 64/8 heads, prefixes U[0,32768] (page multiples), chunks lognormal(median 2048)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--attn-config", type=int, default=3, choices=(2, 3, 4),
                    help="attention workload of the headline step (default: configuration 3, the 128k-context shape)")
    ap.add_argument("--layers", type=int, default=8, help="distinct per-layer pools the steps cycle through")
    ap.add_argument("--cpu-rows", type=int, default=8192, help="rows the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-extra", action="store_true", help="only the headline step")
    ap.add_argument("--copies-only", action="store_true",
                    help="only the isolated pack / unpack loops (80 launches back to back each), for profiling them alone")
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

    def timed_loop(fn, reps, warm, stream):
        """microseconds per call of fn, `reps` calls back to back on `stream` (launch gaps included)"""
        for _ in range(warm):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

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

        def label(self):
            c = self.case
            return (f"config {self.idx} attention (P={self.pl if len(self.pl) < 3 else 'varlen'}, "
                    f"C={self.nl if len(self.nl) < 3 else 'varlen'}, {c.num_q_heads}/{c.num_kv_heads} heads, D=128, "
                    f"16-token pages scattered over {c.num_pages} pool pages)")

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

        def free(self):
            for name in ("q", "k", "v", "out", "k_new", "v_new", "lse"):
                delattr(self, name)
            torch.cuda.empty_cache()

    # ---- one layer's page traffic (configuration 5), `layers` distinct pool sets so steps do not hit in cache
    sh = W.config_shapes(5)
    n, pb, N2 = sh["n"], sh["page_bytes"], sh["num_pages_dst"]
    rng = np.random.default_rng(sh["seed"])
    rng.permutation(sh["num_pages"])          # the source permutation of the recipe (drawn, unused here)
    dst_ids_host = rng.permutation(N2)[:n].astype(np.int32)
    dst_ids = to_dev(dst_ids_host)
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

    def run_steps(attn, count, timed):
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

    def time_steps(attn):
        run_steps(attn, Wm, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks, copy_marks = run_steps(attn, K, True)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / K
        attn_ms = [a.elapsed_time(b) for a, b in marks]
        in_step = {}
        for name, ms in copy_marks.items():
            us = sorted(a.elapsed_time(b) * 1e3 for a, b in ms)
            if us:
                in_step[name] = {"us_median": round(us[len(us) // 2], 2), "us_min": round(us[0], 2), "us_max": round(us[-1], 2)}
        return ms_per_step, attn_ms, in_step

    traffic = committed_traffic()

    def hbm(prefix):
        r, w = traffic.get(prefix + "_read_bytes"), traffic.get(prefix + "_write_bytes")
        return None if r is None or w is None else {
            "bytes": r + w, "read_bytes": r, "write_bytes": w, "unit": "B per launch",
            "source": "committed rocprofv3 counter summary profiles/hbm_traffic_bench_step.txt (FETCH_SIZE / WRITE_SIZE "
                      "calibrated on a plain copy), not counted in this run"}

    def isolated_copies(result, s):
        def pack_ordered(l, stream):
            B.mc_kv_pack_layer_ordered(k_pool[l], v_pool[l], N2, pb, dst_ids, order, n, k_store[l], v_store[l], stream)

        # pack writes its output in list order, unpack (with the order) its pool pages in address order; the other
        # two combinations are measured for comparison: the write side is the one that wants to be sequential
        for name, fn in (("pack", pack), ("unpack", unpack), ("pack_pool_order", pack_ordered),
                         ("unpack_list_order", unpack_list_order)):
            it = iter(range(10 ** 9))
            us = timed_loop(lambda: fn(next(it) % LAY, s), 80, LAY, s)      # 80 layers back to back, launch gaps included
            gbs = copy_bytes / (us * 1e-6) / 1e9
            result[f"roofline_{name}"] = {"kernel": f"kv_copy_kernel<{name.split('_')[0]}>", "bound": "hbm", "achieved": round(gbs, 1),
                                          "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                                          "us_per_layer": round(us, 2), "bytes_per_launch": copy_bytes,
                                          "traffic": hbm(name.split("_")[0])}
        # the same 80 layers with the launches alternating between two streams, so that the tail of one launch
        # overlaps the start of the next (layers are independent of each other): what is left of the gap to the
        # steady-state rate once the fixed cost per launch is hidden
        s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()
        for name, fn in (("pack", pack), ("unpack", unpack)):
            for l in range(LAY):
                fn(l, s_a if l % 2 == 0 else s_b)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            joined = torch.cuda.Event()
            e0.record(s_a)
            s_b.wait_event(e0)
            for i in range(80):
                fn(i % LAY, s_a if i % 2 == 0 else s_b)
            joined.record(s_b)
            s_a.wait_event(joined)
            e1.record(s_a)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 80
            gbs = copy_bytes / (us * 1e-6) / 1e9
            result[f"roofline_{name}_two_streams"] = {
                "kernel": f"kv_copy_kernel<{name}>", "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "us_per_layer": round(us, 2),
                "what": "80 layers, launches alternating between two streams (consecutive launches overlap)"}
        # what a copy of the same bytes reaches on this board with nothing scattered: the same kernel with the pages
        # in pool order (ids 0 .. n-1), the runtime's device-to-device copy, and the stand-alone probes: the read-only
        # and write-only halves of the access pattern, fixed cost per launch and steady-state rate
        seq_ids = torch.arange(n, dtype=torch.int32, device=dev)

        def pack_contiguous(l, stream):
            B.mc_kv_pack_layer(k_pool[l], v_pool[l], N2, pb, seq_ids, n, k_store[l], v_store[l], stream)

        def runtime_copy(l, stream):
            k_store[l].copy_(k_pool[l, :n])
            v_store[l].copy_(v_pool[l, :n])

        ceiling = {}
        for name, fn in (("same_kernel_contiguous", pack_contiguous), ("runtime_d2d_copy", runtime_copy)):
            it = iter(range(10 ** 9))
            us = timed_loop(lambda: fn(next(it) % LAY, s), 80, LAY, s)
            ceiling[name] = {"GBs": round(copy_bytes / (us * 1e-6) / 1e9, 1), "us_per_layer": round(us, 2),
                             "frac_hbm_peak": round(copy_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
        result["copy_ceiling"] = {"what": "the same 2 x 64 MiB read and written with no scatter at all", **ceiling}

    if args.copies_only:
        result = {"what": "isolated pack / unpack loops only (bench.py --copies-only)"}
        isolated_copies(result, torch.cuda.current_stream())
        print(json.dumps(result))
        return

    def attn_roofline(attn, attn_ms):
        avg = sum(attn_ms) / len(attn_ms)
        tf = attn.flops / (avg * 1e-3) / 1e12
        return {"kernel": "attn_prefill_bf16_kernel", "bound": "mfma", "achieved": round(tf, 2),
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                "avg_launch_ms": round(avg, 4), "min_launch_ms": round(min(attn_ms), 4),
                "launch_ms": [round(x, 3) for x in attn_ms], "flops_per_launch": attn.flops,
                "traffic": hbm(f"attn_config{attn.idx}")}

    # ---- the headline step
    attn = Attn(args.attn_config)
    ms_per_step, attn_ms, in_step = time_steps(attn)
    value = attn.flops / (ms_per_step * 1e-3) / 1e12
    step_what = ("preceded by the append of its chunk's K/V rows (work list prepared once per batch: "
                 "mc_prefill_attn_prepare, then mc_kv_append_run + mc_prefill_attn_run per step), + one config-5 layer of "
                 "KV unpack and pack (2048 pages x 32 KiB, K and V) on a second stream")
    result = {
        "metric": "prefill attn TFLOP/s (% MFMA peak); KV pack/unpack GB/s (% HBM peak)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic" if not args.zero_inputs else "ALL-ZERO tensors: power diagnostic, not the workload",
        "config": {"workload": f"{attn.label()} {step_what}",
                   "attn_flops_per_step": attn.flops, "copy_bytes_per_step": 2 * copy_bytes},
        "pct_mfma_peak": round(100 * value / MFMA_BF16_PEAK_TFLOPS, 2),
        "roofline": attn_roofline(attn, attn_ms),
        "copies_in_step": in_step,
    }

    if not args.no_extra:
        s = torch.cuda.current_stream()
        # isolated kernels, same inputs, nothing else running
        med, mn = attn.time_isolated()
        result["attn_isolated"] = {"config": args.attn_config, "ms_median": round(med, 4), "ms_min": round(mn, 4),
                                   "tflops": round(attn.flops / (med * 1e-3) / 1e12, 2),
                                   "pct_mfma_peak": round(100 * attn.flops / (med * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2)}
        # the one-shot call (list built and uploaded inside every call), back to back like the isolated runs
        us = timed_loop(lambda: attn.launch_one_shot(s), 10, 3, s)
        result["attn_one_shot_call"] = {"ms_per_call_back_to_back": round(us / 1e3, 4),
                                        "what": "mc_prefill_attn_paged: prepare + run in one call"}

        isolated_copies(result, s)
        # append of the step's chunk alone, launched back to back
        c = attn.case
        us = timed_loop(lambda: attn.append(s), 80, 5, s)
        ab = 2 * 2 * c.total_new * c.num_kv_heads * c.head_dim * 2
        result["roofline_append"] = {"kernel": "kv_append_kernel", "bound": "hbm",
                                     "achieved": round(ab / (us * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                     "frac": round(ab / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4), "us_per_launch": round(us, 2),
                                     "bytes_per_launch": ab, "traffic": None,
                                     "note": "same buffers every launch: the working set fits the 256 MiB last-level cache"}

        # ---- the same layer-wise step against the HOST pool (Section 3 steps 1 and 3): a layer's pages come from pinned
        # host memory before its attention and go back after it (load on one side stream, store on another, append +
        # attention on the compute stream).  Two traffic models: `prefix_and_chunk` is the paper's flow for a request
        # of configuration 5's size with half of it cached, as its simulated prompts are (the 1024 reused prefix
        # pages are loaded, the 1024 pages the new tokens filled are stored); `all_pages` moves all 2048 pages in
        # both directions.
        HL = min(4, LAY)
        kh_in = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        vh_in = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        kh_out = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        vh_out = [torch.empty((n, pb), dtype=torch.uint8, pin_memory=True) for _ in range(HL)]
        for t in kh_in + vh_in:
            t.random_(0, 256)
        st_load, st_store = torch.cuda.Stream(), torch.cuda.Stream()
        half = n // 2
        ids_prefix, ids_chunk = dst_ids[:half].contiguous(), dst_ids[half:].contiguous()

        def host_steps(count, load_ids, n_load, store_ids, n_store):
            loaded = [torch.cuda.Event() for _ in range(count + 1)]
            attended = [torch.cuda.Event() for _ in range(count)]
            stored = {}

            def load(i):
                ln = i % HL
                if ln in stored:                     # the pools of this layer are still being stored from
                    st_load.wait_event(stored[ln])
                B.mc_kv_load_layer(kh_in[ln], vh_in[ln], k_remote[ln], v_remote[ln], N2, pb, load_ids, n_load, k_pool[ln],
                                   v_pool[ln], st_load)
                loaded[i].record(st_load)

            load(0)
            for i in range(count):
                l = i % HL
                if i + 1 < count:
                    load(i + 1)
                compute.wait_event(loaded[i])
                attn.append(compute)
                attn.launch(compute)
                attended[i].record(compute)
                st_store.wait_event(attended[i])
                B.mc_kv_store_layer(k_pool[l], v_pool[l], N2, pb, store_ids, n_store, k_store[l], v_store[l], kh_out[l],
                                    vh_out[l], st_store)
                stored[l] = torch.cuda.Event()
                stored[l].record(st_store)

        host = {"what": "the step with each layer's pages loaded from and stored to pinned host memory: load and store on "
                        "two side streams, append + attention on the compute stream; a load waits for the last store "
                        "that read the same pools"}
        for name, (li, nl_, si, ns_) in (("prefix_and_chunk", (ids_prefix, half, ids_chunk, n - half)),
                                         ("all_pages", (dst_ids, n, dst_ids, n))):
            host_steps(4, li, nl_, si, ns_)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            host_steps(12, li, nl_, si, ns_)
            torch.cuda.synchronize()
            ms_host = (time.perf_counter() - t0) * 1e3 / 12
            host[name] = {"ms_per_step": round(ms_host, 4), "attn_tflops": round(attn.flops / (ms_host * 1e-3) / 1e12, 1),
                          "load_bytes_per_layer": 2 * nl_ * pb, "store_bytes_per_layer": 2 * ns_ * pb,
                          "vs_step_in_hbm": round(ms_host / ms_per_step, 3)}
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
        host["link_alone"] = {"load_GBs": round(layer_bytes / (ev[0].elapsed_time(ev[1]) / HL * 1e-3) / 1e9, 1),
                              "store_GBs": round(layer_bytes / (ev[2].elapsed_time(ev[3]) / HL * 1e-3) / 1e9, 1),
                              "bytes_per_layer_per_direction": layer_bytes}
        result["host_streaming"] = host
        del kh_in, vh_in, kh_out, vh_out

        # ---- prefix keys of a batch of long prompts and their match against 16 instances' cache keys
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
            prefix[name] = {"us": round(timed_loop(fn, 20, 3, s), 1)}
        prefix["hash"]["GBs"] = round(4 * NP * LP / (prefix["hash"]["us"] * 1e-6) / 1e9, 1)
        prefix["hash"]["frac_hbm_peak"] = round(prefix["hash"]["GBs"] / HBM_PEAK_GBS, 4)
        prefix["match"]["lookups_per_s"] = round(nkeys * NI / (prefix["match"]["us"] * 1e-6), 0)
        prefix["match"]["best_len_of_request_0"] = int(bl[0].item())
        result["prefix_keys"] = prefix
        del toks, pkeys, ckeys, caches

        # ---- the other attention configurations: configuration 2 inside the same step (configuration 5 of the
        # recipe names this pairing), the rest isolated
        attn.free()
        for idx in (2, 3, 4):
            if idx == args.attn_config:
                continue
            other = Attn(idx)
            med, mn = other.time_isolated()
            result[f"attn_config{idx}"] = {"workload": LABELS[idx], "flops": other.flops, "ms_median": round(med, 4),
                                          "ms_min": round(mn, 4), "tflops": round(other.flops / (med * 1e-3) / 1e12, 2),
                                          "pct_mfma_peak": round(100 * other.flops / (med * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2)}
            if idx == 2:
                ms2, attn_ms2, in_step2 = time_steps(other)
                result["step_config2"] = {
                    "workload": f"{other.label()} {step_what}", "ms_per_step": round(ms2, 4),
                    "value_tflops": round(other.flops / (ms2 * 1e-3) / 1e12, 2),
                    "pct_mfma_peak": round(100 * other.flops / (ms2 * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2),
                    "roofline": attn_roofline(other, attn_ms2), "copies_in_step": in_step2}
            other.free()
            del other

        def default_entry_forms(P2, C2, Hq2, Hkv2, iters):
            """mc_prefill_attn_paged with the minimal workspace (whole rows), with a workspace that has room for
            partial results (the call takes key slices by itself), and the explicit split + merge calls."""
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
            ws_c = torch.empty(B.mc_prefill_attn_auto_workspace_bytes(prm, [P2], [C2]), dtype=torch.uint8, device=dev)
            o_parts = torch.empty(SP, C2, Hq2, 128, device=dev, dtype=torch.float32)
            l_parts = torch.empty(SP, C2, Hq2, device=dev, dtype=torch.float32)
            s = torch.cuda.current_stream()

            def whole():
                B.mc_prefill_attn_paged(prm, q2, k2, v2, bt2, [P2], [C2], out2, None, ws_a, s)

            def default_roomy():
                B.mc_prefill_attn_paged(prm, q2, k2, v2, bt2, [P2], [C2], out2, None, ws_c, s)

            def split():
                B.mc_prefill_attn_paged_split(prm, q2, k2, v2, bt2, [P2], [C2], SP, o_parts, l_parts, ws_b, s)
                B.mc_attn_merge_lse(o_parts, l_parts, SP, C2 * Hq2, 128, B.MC_DTYPE_BF16, out2, None, s)

            fl2 = 4 * 128 * Hq2 * (C2 * P2 + C2 * (C2 + 1) // 2)
            rec = {"workload": f"{Hq2}/{Hkv2} heads, P={P2}, C={C2}", "flops": fl2, "suggested_key_slices": SP,
                   "workspace_bytes": {"minimal": ws_a.numel(), "with_room_for_partials": ws_c.numel()}}
            for name, fn in (("mc_prefill_attn_paged_minimal_workspace", whole),
                             ("mc_prefill_attn_paged_roomy_workspace", default_roomy),
                             (f"explicit_split{SP}_plus_merge", split)):
                us = timed_loop(fn, iters, 3, s)
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
            us = timed_loop(lambda: B.mc_prefill_attn_paged(prm, q2, k2, v2, bt2, [P2], [C2], out2, None, ws2, s2), 5, 2, s2)
            fl = 4 * 64 * Hq2 * (C2 * P2 + C2 * (C2 + 1) // 2)
            return {"workload": "fp32, 64/8 heads, head_dim 64, P=8192, C=8192", "flops": fl, "ms": round(us / 1e3, 3),
                    "tflops": round(fl / (us * 1e-6) / 1e12, 1), "peak": 157.3,
                    "frac_fp32_mfma_peak": round(fl / (us * 1e-6) / 1e12 / 157.3, 4)}

        result["attn_fp32"] = fp32_attention()

        # the bf16 instantiation for head_dim 64 (128-byte rows) at configuration 2's lengths; no workload uses it
        def bf16_head_dim_64():
            P2, C2, Hq2, Hkv2 = 8192, 8192, 64, 8
            npg = (P2 + C2) // 16
            g2 = torch.Generator(device=dev)
            g2.manual_seed(20240702)
            q2 = torch.randn(C2, Hq2, 64, device=dev, dtype=torch.bfloat16, generator=g2)
            k2 = torch.randn(npg, Hkv2, 16, 64, device=dev, dtype=torch.bfloat16, generator=g2)
            v2 = torch.randn(npg, Hkv2, 16, 64, device=dev, dtype=torch.bfloat16, generator=g2)
            bt2 = torch.randperm(npg, device=dev, generator=g2).to(torch.int32).reshape(1, npg).contiguous()
            prm = B.attn_params(Hq2, Hkv2, 64, 16, npg, "bf16")
            out2 = torch.empty_like(q2)
            ws2 = torch.empty(B.mc_prefill_attn_workspace_bytes(prm, 1, C2), dtype=torch.uint8, device=dev)
            s2 = torch.cuda.current_stream()
            us = timed_loop(lambda: B.mc_prefill_attn_paged(prm, q2, k2, v2, bt2, [P2], [C2], out2, None, ws2, s2), 10, 3, s2)
            fl = 4 * 64 * Hq2 * (C2 * P2 + C2 * (C2 + 1) // 2)
            return {"workload": "bf16, 64/8 heads, head_dim 64, P=8192, C=8192", "flops": fl, "ms": round(us / 1e3, 3),
                    "tflops": round(fl / (us * 1e-6) / 1e12, 1),
                    "pct_mfma_peak": round(100 * fl / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2)}

        result["attn_bf16_head_dim_64"] = bf16_head_dim_64()
        torch.cuda.empty_cache()
        # a small chunk against a long prefix (16 new tokens behind 131056 cached ones, 64/8 heads): 8 work
        # items for 256 CUs unless the keys are split
        result["attn_small_chunk"] = default_entry_forms(131056, 16, 64, 8, 20)
        # just above one work item per compute unit (10240 new tokens, 8/1 heads: 320 items): whole rows run a
        # second, mostly empty round
        result["attn_uneven_rounds"] = default_entry_forms(120832, 10240, 8, 1, 6)
        torch.cuda.empty_cache()
        torch.cuda.synchronize()
        mf = probe("mfma")
        if mf is not None:
            result["mfma_alone"] = {
                "what": "back-to-back bf16 MFMAs, nothing else running, 2 waves per SIMD: the board lowers its clock to hold "
                        "its power limit, and MFMA power follows operand bit activity and tile shape (the attention "
                        "kernel uses 16x16x32 tiles)", **mf,
                "attn_vs_random_data_rate": round(result["roofline"]["achieved"] / mf["16x16x32"]["random"]["tflops"], 4)}
        cp = probe("copy")
        if cp is not None:
            result["copy_ceiling"]["probes"] = {
                "what": "bench_probes.hip: the pack's access pattern (2048 scattered 32 KiB pages for K and for V -> "
                        "contiguous) as a copy, read only and write only; the copy at other sizes fitted to fixed cost "
                        "per launch + bytes / steady-state rate", **cp,
                "read_only_frac_hbm_peak": round(cp["read_only"]["GBs"] / HBM_PEAK_GBS, 4),
                "write_only_frac_hbm_peak": round(cp["write_only"]["GBs"] / HBM_PEAK_GBS, 4),
                "steady_state_frac_hbm_peak": round(cp["steady_state_GBs"] / HBM_PEAK_GBS, 4)}

    if args.cpu_rows > 0:
        # the CPU oracle, as it stands, on a bounded sample of the same workloads
        import oracle
        case = W.make_config_attn(args.attn_config, poison=False)
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
        del case
        # the copy leg: the oracle's per-page memcpy on a host copy of one configuration-5 layer
        hrng = np.random.default_rng(sh["seed"])
        kp = hrng.integers(0, 256, size=(N2, pb), dtype=np.uint8)
        vp = hrng.integers(0, 256, size=(N2, pb), dtype=np.uint8)
        cores = oracle.num_threads()
        cpu_copy = {"unit": "GB/s", "kind": "oracle", "bytes_per_layer": copy_bytes,
                    "sample": "one configuration-5 layer (2048 pages of 32 KiB, K and V) on host memory, best of 3 "
                              "passes per leg; pack as the oracle's wrapper does it, output buffers allocated per call"}
        for threads in sorted({1, cores}):
            best_p, best_u = 1e30, 1e30
            for _ in range(3):
                t0 = time.perf_counter()
                ko, vo = oracle.kv_pack_layer(kp, vp, dst_ids_host, threads=threads)
                best_p = min(best_p, time.perf_counter() - t0)
                t0 = time.perf_counter()
                oracle.kv_unpack_layer(ko, vo, dst_ids_host, kp, vp, threads=threads)
                best_u = min(best_u, time.perf_counter() - t0)
            cpu_copy[f"threads_{threads}"] = {"pack_GBs": round(copy_bytes / best_p / 1e9, 2),
                                              "unpack_GBs": round(copy_bytes / best_u / 1e9, 2)}
        cpu_copy["cores"] = cores
        result["cpu_baseline_copy"] = cpu_copy
    print(json.dumps(result))


if __name__ == "__main__":
    main()
