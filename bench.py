#!/usr/bin/env python3
"""Throughput of the list Gumbel-max coupling hot path on one MI355X.

One step = one llc_couple call (scan + finalize) over one synthetic batch that
is already resident in HBM.  Default workload: the large-vocabulary
configuration (B=1024, V=128256, K=8 i.i.d. drafts, fp32 logits, T=0.7) that
the headline metric is quoted on.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
                    [--materialised] [--keys] [--no-cpu-baseline]
    python bench.py --workload verify     (Algorithm 2's verification loop, llc_verify)
    python bench.py --workload topm       (Algorithm 1 on top-50 candidate lists, llc_couple_topm)
    python bench.py --workload lml        (Theorem 1's bound on config 3's rows)
    python bench.py --workload peaks      (machine probes: issue rates, streaming read, sustained clock)
"""
import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published figures used as denominators.
HBM_PEAK_GBS = 8000.0
# 256 CUs x 64 lanes x 2.4 GHz: 32-bit integer / fp32 lane-operations issued per second.
ALU_PEAK_TLANEOPS = 256 * 64 * 2.4e9 / 1e12


def algorithmic_lane_ops(K, min_first=False):
    """Vector-ALU lane operations per element that the method cannot avoid given how the shared
    uniforms are defined: one Philox4x32-10 block serves 8 elements
    (4 indices x 2 drafts, 16 upper bits each); per block 14 32x32->64 products and 16
    three-input xors depend on both the index and the draft pair (rounds 4-10, and round 3's
    xors), 2 + 2 more are shared by the draft pairs of a pass (both instructions issue at full rate
    on gfx950: measured), plus one packed compare per two elements.  The lower 16 bits are drawn
    for about one element in 10^4 and are not counted; nor are threshold construction and
    everything else the kernel executes.  With the race times drawn min-first one block serves four
    indices whatever K is (a 32-bit word each, none of its rounds shared), plus one compare per index."""
    if min_first:
        return (40.0 / 4.0 + 1.0) / K
    pairs = max(1, min(4, (K + 1) // 2))
    return (30.0 + 4.0 / pairs) / 8.0 + 0.5

# HBM bytes per scan launch (fetch + write) measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# each scaled by what the counter reads for a plain 1 GiB copy (x2.0 and x1.0); the summaries are
# under profiles/.  None for workloads that have not been measured.
MEASURED_TRAFFIC_BYTES = {
    "largevocab_v128256_k8_f32": 1052.3e6 + 0.3e6,
    "largevocab_v128256_k8_f32_minfirst": 1052.4e6 + 0.3e6,
    "largevocab_v128256_k8_f32_keys": 1053.6e6 + 3.4e6,
    "largevocab_v128256_k8_f32_minfirst_keys": 1056.2e6 + 6.6e6,
    "largevocab_v128256_k8_f32_materialised": 4948.7e6 + 2.0e6,
    "distinct_v152064_k16_bf16": 2726.6e6 + 2.1e6,
    "distinct_v152064_k16_bf16_minfirst": 2763.9e6 + 2.1e6,
    "is_n65536_l4_f32": 5379.9e6 + 0.6e6,
    "is_n65536_l4_f32_bins16": 2825.0e6 + 0.5e6,
    "specdec_v32000_k4_bf16": 33.4e6 + 0.5e6,
    "verify_largevocab_s128_l7_k8_v128256": 4207.1e6 + 1.6e6,
    "lml_largevocab_v128256_k8_f32": 11557.8e6 + 9397.3e6,
}


class HipEvents:
    """hipEvent pairs created through the HIP runtime that torch has already loaded."""

    def __init__(self, n):
        path = "libamdhip64.so"
        with open("/proc/self/maps") as fh:  # the copy of the runtime this process already uses
            for line in fh:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        self.hip = ctypes.CDLL(path)
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                 ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            assert self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.pairs[i][0], self.pairs[i][1])
        assert rc == 0, rc
        return ms.value

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def algorithmic_bytes(w, materialised):
    """Input bytes one call must read, every input row once (outputs are negligible)."""
    es = 4 if str(w.dtype).endswith("float32") else 2
    draft_rows = w.B * (w.K if (materialised or not w.shared_draft) else 1)
    return (draft_rows + w.B) * w.V * es


def _to_host(t):
    import numpy as np
    import torch
    import oracle
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).numpy().view(np.uint16), oracle.BF16
    return t.contiguous().numpy(), oracle.F32


def run_cpu_baseline_verify(w, budget_s=12.0):
    import oracle
    cores = oracle.threads()

    def run(n):
        t, dt = _to_host(w.target[:n])
        tok = w.tokens[:n].cpu().numpy()
        t0 = time.perf_counter()
        oracle.verify(t, tok, dtype=dt, temp_target=w.temp_target, seed=w.seed)
        return time.perf_counter() - t0

    probe = min(w.S, cores)
    per_seq = run(probe) / probe
    n = int(max(probe, min(w.S, budget_s / max(per_seq, 1e-9))))
    n = min(w.S, max(cores, n - n % cores) if n >= cores else n)
    dt = run(n)
    elems = n * (w.L + 1) * w.K * w.V
    return {"value": elems / dt / 1e9, "unit": "Gelem/s", "cores": cores, "kind": "oracle",
            "sample": f"first {n} of {w.S} sequences of the same workload, {elems} elements, "
                      f"{dt:.2f} s wall, OpenMP over sequences (the oracle stops a sequence at its "
                      f"first rejection, the GPU path evaluates every position)"}


def measure_verify(args, *, strong=False, steps=None, warmup=None, want_workload=False, min_first=None):
    import torch
    import paper_2506_05632_amd as llc
    from paper_2506_05632_amd import workloads

    steps = steps or args.steps
    warmup = args.warmup if warmup is None else warmup
    dev = "cuda:0"
    min_first = args.min_first if min_first is None else min_first
    flags = llc.FLAG_MIN_FIRST if min_first else 0
    every = max(1, args.event_every)
    w = workloads.make_verify("largevocab", dev)
    ws = torch.empty(llc.llc_verify_workspace_size(w.S, w.L, w.K, w.V), dtype=torch.uint8, device=dev)
    out = {"Y": torch.empty(w.S, w.L + 1, dtype=torch.int32, device=dev),
           "n_out": torch.empty(w.S, dtype=torch.int32, device=dev),
           "active": torch.empty(w.S, w.K, dtype=torch.uint8, device=dev)}
    ev = HipEvents(steps)

    def step(i=None, stats=None):
        llc.llc_verify(w.target, w.tokens, temp_target=w.temp_target, seed=w.seed + (0 if i is None else i),
                       workspace=ws, out=out, v_chunks=args.v_chunks, k_tile=args.k_tile, flags=flags,
                       scan_events=None if (i is None or i % every) else ev.pairs[i], strong=strong, stats=stats)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    scan_ms = [ev.elapsed_ms(i) for i in range(0, steps, every)]
    ev.close()
    stats = llc.new_stats(dev)
    step(None, stats)
    torch.cuda.synchronize()
    counters = dict(zip(llc.binding.STATS_FIELDS, (int(v) for v in stats.cpu().numpy())))
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    scan_avg_s = sum(scan_ms) / len(scan_ms) / 1e3
    elems = w.elems
    es = 4 if w.dtype == torch.float32 else 2
    alg_bytes = elems * es                      # every target row read once
    alg_ops = algorithmic_lane_ops(w.K)
    hbm_achieved = alg_bytes / scan_avg_s / 1e9
    alu_achieved = alg_ops * elems / scan_avg_s / 1e12
    hbm_frac, alu_frac = hbm_achieved / HBM_PEAK_GBS, alu_achieved / ALU_PEAK_TLANEOPS
    roofline = {"bound": "hbm", "achieved": hbm_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": hbm_frac, "kernel": "scan_kernel", "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                "traffic_source": "recorded from profiles/ (rocprofv3 --pmc of this command, scaled by a plain "
                                  "copy); not measured in this run",
                "kernel_ms": scan_avg_s * 1e3, "kernel_ms_min": min(scan_ms),
                "algorithmic_bytes": alg_bytes, "algorithmic_lane_ops_per_elem": alg_ops,
                "hbm_frac": hbm_frac, "alu_frac": alu_frac,
                "step_hbm_frac": alg_bytes / (wall / steps) / 1e9 / HBM_PEAK_GBS}
    res = {"value": elems / (wall / steps) / 1e9, "ms_per_step": wall / steps * 1e3, "steps": steps, "warmup": warmup,
           "config": {"workload": w.name + ("_strong" if strong else "") + ("_minfirst" if min_first else ""),
                      "S": w.S, "L": w.L, "K": w.K, "V": w.V,
                      "input_dtype": str(w.dtype), "temperature": w.temp_target,
                      "outputs": "Y,n_out,active",
                      "mean_tokens_per_block": float(out["n_out"].float().mean()),
                      "near_ties": counters["near_ties"], "slow_blocks": counters["slow_blocks"]},
           "roofline": roofline}
    if want_workload:
        res["_workload"] = w
    return res


def bench_verify(args):
    r = measure_verify(args, strong=args.strong, want_workload=True)
    w = r.pop("_workload")
    result = {
        "metric": "Gelem/s (S*(L+1)*K*V) of Algorithm 2's verification loop",
        "value": r["value"], "unit": "Gelem/s", "n_gpus": 1,
        "steps": r["steps"], "warmup": r["warmup"], "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32/u16+f32 (Philox words, packed 16-bit compares, fp32 thresholds, fp64 tie resolution and normalisers)",
        "data": "synthetic",
        "config": r["config"],
        "roofline": r["roofline"],
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = run_cpu_baseline_verify(w)
    print(json.dumps(result))


def bench_topm(args):
    import torch
    import oracle
    import paper_2506_05632_amd as llc
    from paper_2506_05632_amd import workloads

    dev = "cuda:0"
    w = workloads.make_topm("top50", dev)
    out = {"X": torch.empty(w.B, w.K, dtype=torch.int32, device=dev),
           "Y": torch.empty(w.B, dtype=torch.int32, device=dev),
           "accept": torch.empty(w.B, dtype=torch.uint8, device=dev),
           "match_k": torch.empty(w.B, dtype=torch.int32, device=dev)}
    ev = HipEvents(args.steps)

    def step(i=None):
        llc.llc_couple_topm(w.draft_ids, w.draft_val, w.target_ids, w.target_val, w.K,
                            seed=w.seed + (0 if i is None else i), out=out,
                            events=None if i is None else ev.pairs[i])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [ev.elapsed_ms(i) for i in range(args.steps)]
    ev.close()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    kern_s = sum(kern_ms) / len(kern_ms) / 1e3
    elems = w.elems
    # every key is evaluated exactly: per (k, entry) and side two Philox blocks (40 multiplies,
    # 40 three-input xors) and two fp64 logarithms; the lists (id + value) are read once
    alg_bytes = (w.draft_ids.numel() + w.target_ids.numel()) * (4 + w.draft_val.element_size())
    alg_ops = 2 * 80.0
    alu = alg_ops * elems / kern_s / 1e12
    hbm = alg_bytes / kern_s / 1e9
    roofline = {"bound": "alu", "achieved": alu, "peak": ALU_PEAK_TLANEOPS, "unit": "Tlane-op/s",
                "frac": alu / ALU_PEAK_TLANEOPS, "kernel": "topm_kernel", "traffic": None,
                "kernel_ms": kern_s * 1e3, "kernel_ms_min": min(kern_ms), "algorithmic_bytes": alg_bytes,
                "algorithmic_lane_ops_per_elem": alg_ops, "hbm_frac": hbm / HBM_PEAK_GBS,
                "alu_frac": alu / ALU_PEAK_TLANEOPS,
                "note": "a few hundred candidates per row: the call is bound by launch latency, not by a roofline"}
    result = {
        "metric": "Gelem/s (B*K*M) of list Gumbel-max coupling on top-M candidate lists",
        "value": elems / (wall / args.steps) / 1e9, "unit": "Gelem/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32+f64 (Philox words, every key in fp64)", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "K": w.K, "M": w.M, "V": w.V,
                   "input_dtype": str(w.dtype), "outputs": "X,Y,accept,match_k",
                   "accept_rate": float(out["accept"].float().mean())},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        cores = oracle.threads()
        args_cpu = [t.cpu().numpy() for t in (w.draft_ids, w.draft_val, w.target_ids, w.target_val)]
        reps, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < 5.0:
            oracle.couple_topm(*args_cpu, w.K, seed=w.seed + reps)
            reps += 1
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": reps * elems / dt / 1e9, "unit": "Gelem/s", "cores": cores,
                                  "kind": "oracle", "sample": f"{reps} passes over the whole workload, {dt:.2f} s wall, OpenMP over rows"}
    print(json.dumps(result))


def bench_peaks(args):
    """What this GPU sustains on the instruction kinds the scan kernel is made of and on a plain
    streaming read, and the clock it holds meanwhile (libllc_probe.so, csrc/probe.hip)."""
    import torch
    torch.cuda.init()
    path = os.path.join(ROOT, "paper_2506_05632_amd", "libllc_probe.so")
    lib = ctypes.CDLL(path)
    lib.llc_probe_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.llc_probe_run.restype = ctypes.c_int
    probes = [("fma_f32", 0, 1e12, "Tflop-pairs/s (fused multiply-adds)", 1.0), ("mad_u64_u32_plus_xor", 1, 1e12, "Tpair/s", 2.0),
              ("xor3", 2, 1e12, "Top/s", 1.0), ("philox4x32_10_words", 3, 1e9, "Gword/s", 10.0),
              ("stream_read_4GiB", 4, 1e9, "GB/s", None), ("copy_4GiB", 5, 1e9, "GB/s (read + written)", None),
              ("philox_block_per_8_bytes_read_4GiB", 6, 1e9, "GB/s", 5.0)]
    out = {}
    for name, which, scale, unit, slots in probes:
        res, clk = ctypes.c_double(), ctypes.c_double()
        reps = args.steps if which >= 4 else max(args.steps, 200)   # the ALU probes run long enough for the clock to settle
        rc = lib.llc_probe_run(which, reps, ctypes.byref(res), ctypes.byref(clk))
        assert rc == 0, (name, rc)
        entry = {"value": res.value / scale, "unit": unit, "launches": reps}
        if clk.value:
            entry["clock_ghz"] = clk.value
        if slots is not None:
            # issue slots per lane and second that the rate stands for, against 256 CUs x 64 lanes x 2.4 GHz
            entry["issue_slot_fraction_of_2p4ghz_peak"] = res.value * slots / (ALU_PEAK_TLANEOPS * 1e12)
        out[name] = entry
    print(json.dumps({"metric": "machine probes (not the sampler)", "n_gpus": 1, "peaks": out,
                      "reference": {"hbm_peak_gbs": HBM_PEAK_GBS, "alu_peak_tlaneops_at_2p4ghz": ALU_PEAK_TLANEOPS}}))


def bench_lml(args):
    """Theorem 1's bound for K = 1, 2, 4, 8 on config 3's rows (a diagnostic, not the hot path)."""
    import numpy as np
    import torch
    import paper_2506_05632_amd as llc
    from oracle import lml
    from paper_2506_05632_amd import workloads

    dev = "cuda:0"
    w = workloads.make(3, dev, rows=args.rows or None)
    draft = w.draft if w.draft.dim() == 2 else w.draft[:, 0]
    ks = [1, 2, 4, 8]
    ws = torch.empty(llc.llc_lml_workspace_size(w.B, w.V), dtype=torch.uint8, device=dev)
    out = {"bound": torch.empty(w.B, len(ks), dtype=torch.float64, device=dev),
           "relaxed": torch.empty(w.B, len(ks), dtype=torch.float64, device=dev),
           "tv": torch.empty(w.B, dtype=torch.float64, device=dev)}
    ev = HipEvents(args.steps)

    def step(i=None):
        llc.llc_lml_bound(draft, w.target, ks, temp_draft=w.temp_draft, temp_target=w.temp_target,
                          workspace=ws, out=out, events=None if i is None else ev.pairs[i])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [ev.elapsed_ms(i) for i in range(args.steps)]
    ev.close()
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    kern_s = sum(kern_ms) / len(kern_ms) / 1e3
    elems = w.B * w.V
    # what the kernel's own design moves per element: both inputs three times (normalisers twice,
    # then the keys), the key and its two masses written once (12 bytes), four radix passes that
    # read and write those 12 bytes, and the sorted masses read once more for the running sums
    esize = draft.element_size()
    alg_bytes = elems * (2 * esize + 8)          # inputs once, the sorted order written once
    design_bytes = elems * (6 * esize + 12 + 4 * 24 + 8)
    hbm = alg_bytes / kern_s / 1e9
    launches = -(-w.B // max(1, min(w.B, (ws.numel() - 256) // (24 * w.V))))
    roofline = {"bound": "hbm", "achieved": hbm, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm / HBM_PEAK_GBS,
                "kernel": "lml_kernel", "traffic": MEASURED_TRAFFIC_BYTES.get("lml_" + w.name), "kernel_ms": kern_s * 1e3, "kernel_ms_min": min(kern_ms),
                "kernel_launches_per_call": launches,
                "algorithmic_bytes": alg_bytes, "design_bytes": design_bytes,
                "note": "one workgroup sorts one row through memory (four stable 8-bit radix passes over 12-byte "
                        "entries, tiles laid out in LDS so that stores are contiguous): a diagnostic, bound by the "
                        "traffic of its own design (about 10x the algorithmic bytes), not by the streaming roofline; "
                        "kernel_ms, traffic and the byte counts are per call (kernel_launches_per_call launches of "
                        "at most 512 rows each, which is what the workspace holds)"}
    result = {
        "metric": "Melem/s (B*V) of Theorem 1's bound for four list sizes", "value": elems / (wall / args.steps) / 1e6,
        "unit": "Melem/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 sort keys + f64 sums", "data": "synthetic",
        "config": {"workload": "lml_" + w.name, "B": w.B, "V": w.V, "list_sizes": ks, "input_dtype": str(draft.dtype),
                   "mean_bound": [float(v) for v in out["bound"].mean(0)], "mean_tv": float(out["tv"].mean())},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        n = min(w.B, 64)
        d = draft[:n].float().cpu().numpy()
        t = w.target[:n].float().cpu().numpy()
        t0 = time.perf_counter()
        lml.lml_rows(d, t, ks, temp_draft=w.temp_draft, temp_target=w.temp_target)
        dt = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": n * w.V / dt / 1e6, "unit": "Melem/s", "cores": 1, "kind": "oracle",
                                  "sample": f"the first {n} rows, {dt:.2f} s wall, numpy on one thread"}
    print(json.dumps(result))


def run_cpu_baseline(w, budget_s=12.0, bins=None, min_first=False):
    import oracle
    kinds = {"logits": oracle.LOGITS, "probs": oracle.PROBS, "logw": oracle.LOGW}
    cores = oracle.threads()

    def run(rows):
        d, dt = _to_host(w.draft[:rows])
        t, _ = _to_host(w.target[:rows])
        if bins is not None:
            bb = bins[:rows].cpu().numpy()
            t0 = time.perf_counter()
            oracle.compress_select(t, d, bb, seed=w.seed, row_offset=w.row_offset)
            return time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.couple(d, t, w.K, dtype=dt, kind=kinds[w.kind], temp_target=w.temp_target,
                      temp_draft_all=w.temp_draft, seed=w.seed, row_offset=w.row_offset, min_first=min_first)
        return time.perf_counter() - t0

    probe_rows = min(w.B, cores)
    t_probe = run(probe_rows)
    per_row = t_probe / probe_rows
    rows = int(max(probe_rows, min(w.B, budget_s / max(per_row, 1e-9))))
    rows = max(cores, rows - rows % cores) if rows >= cores else rows
    rows = min(rows, w.B)
    dt = run(rows)
    elems = rows * w.K * w.V
    return {"value": elems / dt / 1e9, "unit": "Gelem/s", "cores": cores, "kind": "oracle",
            "sample": f"first {rows} of {w.B} rows of the same workload, {elems} elements, "
                      f"{dt:.2f} s wall, OpenMP over rows"}


def measure_couple(args, config, *, materialised=False, keys=False, bins=0, rows=0, steps=None, warmup=None,
                   want_workload=False, min_first=None, draft_only=None):
    """Time llc_couple (or, with bins, llc_compress_select) on one configuration; returns the
    fields of a bench line (without cpu_baseline)."""
    import torch
    import paper_2506_05632_amd as llc
    from paper_2506_05632_amd import workloads

    steps = steps or args.steps
    warmup = args.warmup if warmup is None else warmup
    min_first = args.min_first if min_first is None else min_first
    draft_only = args.draft_only if draft_only is None else draft_only
    flags = (llc.FLAG_MIN_FIRST if min_first else 0) | (llc.FLAG_DRAFT_ONLY if draft_only else 0)
    every = max(1, args.event_every)   # the scan kernel is timed on every `every`-th step of the timed region
    dev = "cuda:0"
    w = workloads.make(config, dev, rows=rows or None)
    draft = w.draft
    if materialised and w.shared_draft:
        draft = w.draft[:, None, :].expand(w.B, w.K, w.V).contiguous()
    ws = llc.new_workspace(w.B, w.K, w.V, dev, v_chunks=args.v_chunks)
    out = {"X": torch.empty(w.B, w.K, dtype=torch.int32, device=dev),
           "Y": torch.empty(w.B, dtype=torch.int32, device=dev),
           "accept": torch.empty(w.B, dtype=torch.uint8, device=dev),
           "match_k": torch.empty(w.B, dtype=torch.int32, device=dev)}
    if keys:
        out["keyX"] = torch.empty(w.B, w.K, dtype=torch.float32, device=dev)
        out["keyY"] = torch.empty(w.B, dtype=torch.float32, device=dev)
    if draft_only:   # the drafters' step of Algorithm 2: no target, no Y, no accept test
        assert not bins, "--draft-only goes with llc_couple"
        out = {k: v for k, v in out.items() if k in ("X", "keyX")}
    ev = HipEvents(steps)

    bin_t, decode = None, {}
    if bins:
        assert config == 5 and 1 <= bins <= 256, "--bins goes with --config 5"
        gb = torch.Generator(device=dev)
        gb.manual_seed(4242)
        bin_t = torch.randint(0, bins, (w.B, w.V), generator=gb, device=dev, dtype=torch.uint8)
        out["message"] = torch.empty(w.B, dtype=torch.int32, device=dev)
        # the decoders' outputs and the trial's distortion (Appendix C, Appendix D.2): candidates in
        # the paper's parametrisation W = A + eta, i.e. the standardised candidates divided by rho
        out["W"] = torch.empty(w.B, w.K, dtype=torch.float32, device=dev)
        out["A_hat"] = torch.empty(w.B, w.K, dtype=torch.float32, device=dev)
        out["sq_err"] = torch.empty(w.B, dtype=torch.float32, device=dev)
        decode = dict(cand=(w.extra["u"] / w.extra["rho"]).contiguous(), side=w.extra["y"], source=w.extra["x"],
                      var_w_given_a=w.extra["var_w_given_a"], var_t_given_a=w.extra["var_t_given_a"])

    def step(i=None, stats=None):
        if bin_t is not None:
            llc.llc_compress_select(w.target, w.draft, bin_t, seed=w.seed + (0 if i is None else i),
                                    row_offset=w.row_offset, workspace=ws, out=out, v_chunks=args.v_chunks,
                                    k_tile=args.k_tile, scan_events=None if (i is None or i % every) else ev.pairs[i],
                                    stats=stats, **decode)
            return
        llc.llc_couple(draft, None if draft_only else w.target, w.K, kind=w.kind, temp_target=w.temp_target,
                       temp_draft=w.temp_draft, seed=w.seed + (0 if i is None else i),
                       row_offset=w.row_offset, workspace=ws, out=out,
                       v_chunks=args.v_chunks, k_tile=args.k_tile, flags=flags,
                       scan_events=None if (i is None or i % every) else ev.pairs[i], stats=stats)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    scan_ms = [ev.elapsed_ms(i) for i in range(0, steps, every)]
    ev.close()
    # outside the timed region: one more call that counts near-ties and prefilter survivors
    stats = llc.new_stats(dev)
    step(None, stats)
    torch.cuda.synchronize()
    counters = dict(zip(llc.binding.STATS_FIELDS, (int(v) for v in stats.cpu().numpy())))
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    scan_avg_s = sum(scan_ms) / len(scan_ms) / 1e3
    ms_per_step = wall / steps * 1e3
    elems = w.elems
    value = elems / (wall / steps) / 1e9
    alg_bytes = algorithmic_bytes(w, materialised)
    if draft_only:
        alg_bytes -= w.B * w.V * (4 if str(w.dtype).endswith("float32") else 2)   # the target row is not read
    alg_ops = algorithmic_lane_ops(w.K, min_first)
    alu_achieved = alg_ops * elems / scan_avg_s / 1e12
    name = w.name + ("_materialised" if materialised and w.shared_draft else "")
    if bin_t is not None:
        name += f"_bins{bins}"
        # the timed kernel is the decoders' scan: their rows and one byte per candidate (the
        # encoder's pass before it reads its row once more and is part of the step, not of this figure)
        alg_bytes = w.B * w.K * w.V * 4 + w.B * w.V
    if rows:
        name += f"_rows{w.B}"
    if min_first:
        name += "_minfirst"
    if keys:
        name += "_keys"
    if draft_only:
        name += "_draftonly"
    hbm_achieved = alg_bytes / scan_avg_s / 1e9
    alu_frac, hbm_frac = alu_achieved / ALU_PEAK_TLANEOPS, hbm_achieved / HBM_PEAK_GBS
    # The figure of merit is the fraction of the HBM roofline on the algorithmic bytes; the
    # instruction-issue fraction is reported beside it (its per-element count describes this
    # kernel's design, it is not an independent floor).
    roofline = {"bound": "hbm", "achieved": hbm_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac,
                "kernel": "scan_kernel", "traffic": MEASURED_TRAFFIC_BYTES.get(name),
                "traffic_source": "recorded from profiles/ (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this "
                                  "command, scaled by a plain copy); not measured in this run",
                "kernel_ms": scan_avg_s * 1e3, "kernel_ms_min": min(scan_ms), "kernel_launches_timed": len(scan_ms),
                "algorithmic_bytes": alg_bytes, "algorithmic_lane_ops_per_elem": alg_ops,
                "hbm_frac": hbm_frac, "alu_frac": alu_frac,
                "step_hbm_frac": alg_bytes / (wall / steps) / 1e9 / HBM_PEAK_GBS}
    config_d = {"workload": name, "B": w.B, "K": w.K, "V": w.V, "input_dtype": str(w.dtype),
                "temperature": w.temp_target,
                "draft_layout": "[B,K,V]" if (materialised or not w.shared_draft) else "[B,V] shared by the K drafts",
                "race_times": "min-first (LLC_FLAG_MIN_FIRST)" if min_first else "one word per (k, i)",
                "outputs": ("X" + (",keyX" if keys else "")) if draft_only else "X,Y,accept,match_k" + (",keyX,keyY" if keys else ""),
                "accept_rate": None if draft_only else float(out["accept"].float().mean()),
                "near_ties": counters["near_ties"], "prefilter_survivors": counters["survivors"],
                "exact_evaluations": counters["exact_evals"], "slow_blocks": counters["slow_blocks"]}
    if bin_t is not None:
        db = 10.0 * torch.log10(out["sq_err"].double())
        config_d.update({"outputs": config_d["outputs"] + ",message,W,A_hat,sq_err",
                         "match_rate": config_d.pop("accept_rate"),
                         "distortion_db_mean_over_trials": float(db.mean()),
                         "distortion_db_of_mean": float(10.0 * torch.log10(out["sq_err"].double().mean())),
                         "rate_bits": math.log2(bins)})
    res = {"value": value, "ms_per_step": ms_per_step, "steps": steps, "warmup": warmup,
           "config": config_d, "roofline": roofline}
    if want_workload:
        res["_workload"], res["_bins"] = w, bin_t
    return res


def secondary_lines(args):
    """The other large workloads under the same clock, fewer steps each: kernel time, achieved
    fraction of the HBM roofline on the algorithmic bytes, whole-call throughput."""
    import gc
    import torch
    out = []
    todo = [("couple", dict(config=3, materialised=True)), ("couple", dict(config=3, keys=True)),
            ("couple", dict(config=4)), ("couple", dict(config=5)), ("couple", dict(config=5, bins=16)),
            ("couple", dict(config=2)), ("verify", dict(strong=False)), ("verify", dict(strong=True)),
            # the same workloads with the race times drawn min-first (LLC_FLAG_MIN_FIRST)
            ("couple", dict(config=3, min_first=True)), ("couple", dict(config=3, keys=True, min_first=True)),
            ("couple", dict(config=4, min_first=True)), ("couple", dict(config=5, min_first=True)),
            ("couple", dict(config=2, min_first=True)),
            # the drafters' step of Algorithm 2 (LLC_FLAG_DRAFT_ONLY: the draft side alone)
            ("couple", dict(config=3, draft_only=True)), ("couple", dict(config=3, draft_only=True, min_first=True)),
            ("couple", dict(config=4, draft_only=True))]
    for kind, kw in todo:
        if kind == "couple":
            r = measure_couple(args, steps=30, warmup=10, **kw)
        else:
            r = measure_verify(args, steps=30, warmup=10, **kw)
        rl = r["roofline"]
        out.append({"workload": r["config"]["workload"],
                    "value": r["value"], "unit": "Gelem/s", "ms_per_step": r["ms_per_step"], "steps": r["steps"],
                    "kernel_ms": rl["kernel_ms"], "frac": rl["frac"], "bound": rl["bound"],
                    "algorithmic_bytes": rl["algorithmic_bytes"], "traffic": rl["traffic"],
                    "near_ties": r["config"].get("near_ties")})
        gc.collect()
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--strong", action="store_true",
                    help="--workload verify: the strongly drafter-invariant loop (Appendix B)")
    ap.add_argument("--workload", choices=["couple", "verify", "topm", "lml", "peaks"], default="couple")
    ap.add_argument("--bins", type=int, default=0,
                    help="with --config 5: give every candidate one of BINS bins and run the compression "
                         "scheme's binned selection (llc_compress_select) instead of llc_couple_is")
    ap.add_argument("--rows", type=int, default=0, help="use only the first ROWS rows of the configuration")
    ap.add_argument("--materialised", action="store_true",
                    help="give the K i.i.d. drafts as a [B,K,V] tensor instead of one shared [B,V] row")
    ap.add_argument("--keys", action="store_true", help="also produce the winning keys (adds the normaliser pass)")
    ap.add_argument("--min-first", action="store_true",
                    help="draw the race times min-first (LLC_FLAG_MIN_FIRST) instead of one word per (k, i)")
    ap.add_argument("--draft-only", action="store_true",
                    help="the draft side alone (LLC_FLAG_DRAFT_ONLY): the drafters' step of Algorithm 2")
    ap.add_argument("--event-every", type=int, default=4,
                    help="record the event pair around the scan kernel on every N-th timed step only (an event "
                         "pair costs about 1.5 us of the step it brackets: 2 %% of the headline step, 13 %% of config 2's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="only the headline line: skip the other workloads that the default run also times")
    ap.add_argument("--v-chunks", type=int, default=0)
    ap.add_argument("--k-tile", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region run three plain 1 GiB device copies (a known-size "
                         "reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (rows shard across GPUs with no "
              "communication, through row_offset); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.workload == "verify":
        bench_verify(args)
        return
    if args.workload == "lml":
        return bench_lml(args)
    if args.workload == "peaks":
        return bench_peaks(args)
    if args.workload == "topm":
        bench_topm(args)
        return

    r = measure_couple(args, args.config, materialised=args.materialised, keys=args.keys, bins=args.bins,
                       rows=args.rows, want_workload=True)
    w, bins = r.pop("_workload"), r.pop("_bins")
    result = {
        "metric": "Gelem/s (B*K*V) of list Gumbel-max coupling",
        "value": r["value"], "unit": "Gelem/s", "n_gpus": 1, "steps": r["steps"], "warmup": r["warmup"],
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u32/u16+f32 (Philox words, packed 16-bit compares, fp32 thresholds, fp64 tie resolution)",
        "data": "synthetic",
        "config": r["config"],
        "roofline": r["roofline"],
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = run_cpu_baseline(w, bins=bins, min_first=args.min_first)
    headline = (args.config == 3 and not (args.materialised or args.keys or args.bins or args.rows or args.min_first or args.draft_only
                                          or args.v_chunks or args.k_tile or args.calibrate_copy))
    if headline and not args.no_secondary:
        del w, bins
        import gc
        import torch
        gc.collect()
        torch.cuda.empty_cache()
        result["secondary"] = secondary_lines(args)
        # the headline workload with the race times drawn min-first, lifted out of the list: the same
        # sampler in law (LLC_FLAG_MIN_FIRST; not the default, whose samples it does not reproduce)
        for line in result["secondary"]:
            if line["workload"] == result["config"]["workload"] + "_minfirst":
                result["min_first"] = {k: line[k] for k in ("value", "unit", "ms_per_step", "kernel_ms", "frac", "bound")}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
