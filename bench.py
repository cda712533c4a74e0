#!/usr/bin/env python3
"""Benchmark of the GraVAC compression hot path on one MI355X.

A "step" is one pass of the whole hot path over one gradient:
  gravac_compress   error feedback + Top-k at CF 1000 + residual update + compression gain
  gravac_decompress_accumulate   the worker's fresh message plus seven other workers' messages
                                 (W = 8) scatter-added into one dense buffer
Workload of the headline: the VGG16-shaped gradient (138,357,544 fp32 elements, conv part Normal(0,1e-3), fc part
Normal(0,1e-5)), residual carried from step to step, every step samples its thresholds anew, all inputs resident
in HBM before the timed region.  The same run then times one compress call of every other configuration (the
`configs` list of the line).  Prints ONE JSON line; everything else goes to stderr.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--no-configs] [--small] [--graph]
  python bench.py --configs      only the table of all configurations, with more columns (warm and cold)
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
ALGO_BYTES_PER_ELEMENT = 12.0  # read grad, read residual, write residual
N_GRADS = 3                    # distinct gradients cycled through the steps
N_WORKERS = 8


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(grad_host, cf):
    """The oracle, as it stands, timed on the workload's first gradient (single thread)."""
    from oracle import oracle
    r = np.zeros(grad_host.size, np.float32)
    t0 = time.perf_counter()
    oracle.compress(grad_host, r, [cf])
    dt = time.perf_counter() - t0
    return {"value": 4.0 * grad_host.size / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"one compress call (CF {cf:g}) on the full VGG16-shaped gradient of the timed workload, "
                      f"{grad_host.size} elements, {dt:.1f} s on one host core of {os.cpu_count()}"}


def cpu_select_baseline(grad_host, k):
    """A reasonable multi-core CPU implementation (nth_element on a key copy + OpenMP sweeps), full-size workload.
    Reported as a baseline only; returns None if it cannot be built."""
    import ctypes
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    src, lib = os.path.join(here, "bench_cpu_select.cpp"), os.path.join(here, "libbench_cpu_select.so")
    try:
        if not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
            subprocess.run(["g++", "-O2", "-fopenmp", "-shared", "-fPIC", src, "-o", lib], check=True)
        L = ctypes.CDLL(lib)
    except Exception as e:                                     # no compiler / no OpenMP: the baseline is optional
        log(f"bench.py: CPU select baseline not available ({e})")
        return None
    L.cpu_select_compress.restype = ctypes.c_double
    L.cpu_select_compress.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)]
    g = grad_host
    r = np.zeros(g.size, np.float32)
    oi, ov = np.empty(k, np.int32), np.empty(k, np.float32)
    threads = ctypes.c_int(0)
    t0 = time.perf_counter()
    L.cpu_select_compress(g.ctypes.data, r.ctypes.data, g.size, k, oi.ctypes.data, ov.ctypes.data, ctypes.byref(threads))
    dt = time.perf_counter() - t0
    return {"value": 4.0 * g.size / dt / 1e9, "unit": "GB/s", "cores": int(threads.value),
            "kind": "std::nth_element on a key copy + OpenMP sweeps (baseline only, not the oracle)",
            "sample": f"one compress call on the full VGG16-shaped gradient, {g.size} elements, {dt:.2f} s"}


class ConfigTimer:
    """Times one compress call of a configuration with the caller's events (gravac_compress_profiled): third
    error-feedback iteration on the same gradient; warm = calls back to back, cold = after a 512 MiB write that
    flushes the caches."""

    def __init__(self, torch, binding):
        self.torch, self.binding = torch, binding
        self.flush = torch.empty(512 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda")
        self.timer = binding.CallTimer()

    def row(self, name, g, cfs, commit, seg=None, res0=None, iters=3, reps=7, modes=("cold",)):
        torch, binding = self.torch, self.binding
        n = g.numel()
        comp = binding.Compressor(n, cfs, commit, seg)
        r = torch.empty(n, dtype=torch.float32, device="cuda")
        rec = {"config": name, "n": n, "cfs": cfs, "commit_cf": cfs[commit], "k": comp.k_total}
        for mode in modes:
            tot, strm, fb = [], [], 0
            for rep in range(reps):
                r.zero_() if res0 is None else r.copy_(res0)
                for it in range(iters):
                    if mode == "cold":
                        self.flush.fill_(1.0)
                    comp(g, r, timer=self.timer)
                    if it == iters - 1 and rep >= 2:   # (the first calls of a layerwise shape allocate staging buffers)
                        tot.append(self.timer.call_ms())
                        strm.append(self.timer.pass_ms())
                st = comp.status()
                fb |= st["any_fallback"]
                assert st["internal_error"] == 0, (name, st)
            t = float(np.median(tot))   # (median of five: one host hiccup does not move the row)
            rec[mode + "_us"] = round(t * 1e3, 1)
            rec[mode + "_max_us"] = round(float(np.max(tot)) * 1e3, 1)
            rec[mode + "_stream_kernel_us"] = round(float(np.median(strm)) * 1e3, 1)
            rec[mode + "_dense_GBps"] = round(4.0 * n / t / 1e6, 1)
            rec[mode + "_call_frac_of_hbm_peak"] = round((ALGO_BYTES_PER_ELEMENT * n + 8.0 * comp.k_total) / t / 1e6 / HBM_PEAK_GBS, 4)
            rec[mode + "_fallback"] = bool(fb)
        log(json.dumps(rec))
        return rec


def time_all_configs(torch, binding, workloads, full_table, vgg_grad=None, only=None):
    """One compress call of every configuration and the W = 8 decompression of configuration 5.  With full_table
    also warm numbers, the 66 M-element LSTM variant and the direct / second-level comparison of Table III.
    `only`: a regular expression that selects the configurations to run (for a profiler run of one of them)."""
    ct = ConfigTimer(torch, binding)
    modes = ("warm", "cold") if full_table else ("cold",)
    rows = []

    def want(name):
        return only is None or re.search(only, name) is not None

    def add(name, make, cfs, commits, seg=None, res0=None):
        if not want(name):
            return
        g = make()
        r0 = res0() if res0 is not None else None
        for c in commits:
            rows.append(ct.row(name, g, cfs, c, seg=seg, res0=r0, modes=modes))

    cache = {}

    def resnet():
        if "g2" not in cache:
            cache["g2"] = torch.from_numpy(workloads.config2_grad(0)).cuda()
        return cache["g2"]

    def resnet_r0():
        if "r2" not in cache:
            cache["r2"] = torch.from_numpy(workloads.config2_residual0()).cuda()
        return cache["r2"]

    def vgg():
        if "g3" not in cache:
            cache["g3"] = vgg_grad if vgg_grad is not None else torch.from_numpy(workloads.config3_grad(0)).cuda()
        return cache["g3"]

    add("1: N = 2^20, Normal(0, 1e-3)", lambda: torch.from_numpy(workloads.config1(0)).cuda(), [100.0], [0])
    add("2: ResNet101-shaped, three CFs in one call", resnet, [10.0, 100.0, 1000.0], [0, 1, 2], res0=resnet_r0)
    add("2: ResNet101-shaped, CF 100 alone", resnet, [100.0], [0], res0=resnet_r0)
    if full_table:
        add("2: ResNet101-shaped, CF 10 alone", resnet, [10.0], [0], res0=resnet_r0)
    cache.pop("g2", None); cache.pop("r2", None)
    add("3: VGG16-shaped, CF 1000", vgg, [1000.0], [0])
    add("3: VGG16-shaped, CF 100", vgg, [100.0], [0])
    add("3: VGG16-shaped, CF 10", vgg, [10.0], [0])
    cache.pop("g3", None)
    add("4: LSTM, listed shapes", lambda: torch.from_numpy(workloads.config4_grad(0)).cuda(), [100.0, 1000.0], [0, 1])
    if full_table:
        add("4: LSTM, 66,034,000-element variant", lambda: torch.from_numpy(workloads.config4_grad(0, 10000, 1500)).cuda(),
            [100.0, 1000.0], [0])
    seg = workloads.offsets_of(workloads.resnet101_tensor_sizes())
    add("5: ResNet101-shaped, 314 tensors, layerwise", lambda: torch.from_numpy(workloads.config5_worker_grad(0)).cuda(),
        [100.0], [0], seg=seg)
    D5, U5 = "5: decompress_accumulate, W = 8", "5: decompress_update, W = 8"
    D2, U2 = "2: decompress_accumulate, W = 8, flat CF 1000 messages", "2: decompress_update, W = 8, flat CF 1000 messages"
    extra = full_table and (only is None or any(re.search(only, x) for x in (U5, D2, U2)))
    if not (want(D5) or extra):
        return rows
    g = torch.from_numpy(workloads.config5_worker_grad(0)).cuda()
    # decompression of the eight workers' messages of configuration 5
    n = g.numel()
    comp = binding.Compressor(n, [100.0], 0, seg)
    k = comp.k_total
    mi = torch.empty(N_WORKERS * k, dtype=torch.int32, device="cuda")
    mv = torch.empty(N_WORKERS * k, dtype=torch.float32, device="cuda")
    for w in range(N_WORKERS):
        gw = g if w == 0 else torch.from_numpy(workloads.config5_worker_grad(w)).cuda()
        r = torch.zeros(n, dtype=torch.float32, device="cuda")
        i, v, _ = comp(gw, r)
        mi[w * k:(w + 1) * k] = i
        mv[w * k:(w + 1) * k] = v
    del g
    dense = torch.zeros(n, dtype=torch.float32, device="cuda")
    dws = torch.empty(binding.gravac_decompress_workspace_bytes(N_WORKERS, n), dtype=torch.uint8, device="cuda")

    def time_decompress(label, mi, mv, k, ws, alpha=None):
        """alpha None: gravac_decompress_accumulate into a zeroed buffer; else gravac_decompress_update of `dense`"""
        rec = {"config": label, "n": n, "pairs": N_WORKERS * k, "workspace": ws is not None}
        for mode in modes:
            ts = []
            for rep in range(10):
                dense.zero_()
                if mode == "cold":
                    ct.flush.fill_(1.0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                if alpha is None:
                    binding.gravac_decompress_accumulate(mi, mv, [k] * N_WORKERS, dense, workspace=ws)
                else:
                    binding.gravac_decompress_update(mi, mv, [k] * N_WORKERS, alpha, dense, workspace=ws)
                e1.record()
                torch.cuda.synchronize()
                if rep >= 2:
                    ts.append(e0.elapsed_time(e1))
            t = float(np.median(ts))
            rec[mode + "_us"] = round(t * 1e3, 1)
            rec[mode + "_algorithmic_GBps"] = round((8.0 * n + 8.0 * N_WORKERS * k) / t / 1e6, 1)
        log(json.dumps(rec))
        rows.append(rec)

    if want(D5):
        for ws in ((None, dws) if full_table else (dws,)):
            time_decompress(D5, mi, mv, k, ws)
    if extra:
        # the update step of Alg. 1 straight from the same messages (eta = 0.1)
        if want(U5):
            time_decompress(U5, mi, mv, k, dws, alpha=-0.1 / N_WORKERS)
        # messages of CF 1000 (flat calls on the eight workers' gradients): few pairs per stretch of dense_out
        comp = binding.Compressor(n, [1000.0], 0)
        k = comp.k_total
        mi = torch.empty(N_WORKERS * k, dtype=torch.int32, device="cuda")
        mv = torch.empty(N_WORKERS * k, dtype=torch.float32, device="cuda")
        for w in range(N_WORKERS):
            gw = torch.from_numpy(workloads.config5_worker_grad(w)).cuda()
            r = torch.zeros(n, dtype=torch.float32, device="cuda")
            i, v, _ = comp(gw, r)
            mi[w * k:(w + 1) * k] = i
            mv[w * k:(w + 1) * k] = v
        if want(D2):
            time_decompress(D2, mi, mv, k, None)
            time_decompress(D2, mi, mv, k, dws)
        if want(U2):
            time_decompress(U2, mi, mv, k, dws, alpha=-0.1 / N_WORKERS)
    if not full_table or only is not None:
        return rows
    # direct compression at each CF against the second-level Top-k on a level-1 message (the comparison of the
    # paper's Table III, on the synthetic gradients)
    for name, g in (("VGG16-shaped", torch.from_numpy(workloads.config3_grad(0)).cuda()),
                    ("ResNet101-shaped", torch.from_numpy(workloads.config2_grad(0)).cuda())):
        n = g.numel()
        rec = {"config": f"multi-level: {name}", "n": n}
        r = torch.empty(n, dtype=torch.float32, device="cuda")
        for cf in (10.0, 100.0, 1000.0):
            comp = binding.Compressor(n, [cf], 0)
            ts = []
            for rep in range(8):
                r.zero_()
                comp(g, r, timer=ct.timer)
                ts.append(ct.timer.call_ms())
            rec[f"direct_cf{int(cf)}_us"] = round(float(np.mean(ts[2:])) * 1e3, 1)
        comp = binding.Compressor(n, [10.0], 0)
        r.zero_()
        i1, v1, _ = comp(g, r)
        torch.cuda.synchronize()

        def level2(i_in, v_in, cf_rel):
            kk = binding.gravac_topk_count(i_in.numel(), cf_rel)
            ws = torch.empty(binding.gravac_workspace_bytes(i_in.numel(), 1, 0), dtype=torch.uint8, device="cuda")
            oi = torch.empty(kk, dtype=torch.int32, device="cuda")
            ov = torch.empty(kk, dtype=torch.float32, device="cuda")
            st = torch.zeros(1, 4, dtype=torch.float64, device="cuda")
            ts = []
            for rep in range(10):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                binding.gravac_recompress(i_in, v_in, cf_rel, None, r, out_idx=oi, out_val=ov, out_stats=st, workspace=ws)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            return oi, ov, round(float(np.mean(ts[2:])) * 1e3, 1)

        i2, v2, rec["level2_10_to_100_us"] = level2(i1, v1, 10.0)
        _, _, rec["level2_100_to_1000_us"] = level2(i2, v2, 10.0)
        _, _, rec["level2_10_to_1000_us"] = level2(i1, v1, 100.0)

        # One iteration of Alg. 1 that evaluates CF 10 and CF 100 and sends the CF 100 message, two ways: the level-1
        # call commits and the level-2 call puts the unselected values back into the residual; or the level-1 call
        # does not commit (GRAVAC_FLAG_NO_COMMIT), the level-2 call leaves the residual alone, and the message that
        # is sent is committed afterwards.  Both leave the same residual.
        kk = binding.gravac_topk_count(i1.numel(), 10.0)
        ws2 = torch.empty(binding.gravac_workspace_bytes(i1.numel(), 1, 0), dtype=torch.uint8, device="cuda")
        oi = torch.empty(kk, dtype=torch.int32, device="cuda")
        ov = torch.empty(kk, dtype=torch.float32, device="cuda")
        st = torch.zeros(1, 4, dtype=torch.float64, device="cuda")
        for key, no_commit in (("iteration_10_and_100_restore_us", False), ("iteration_10_and_100_no_commit_us", True)):
            ts = []
            for rep in range(8):
                r.zero_()
                ct.flush.fill_(1.0)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                a_i, a_v, _ = comp(g, r, flags=binding.FLAG_NO_COMMIT if no_commit else 0)
                binding.gravac_recompress(a_i, a_v, 10.0, None, None if no_commit else r, out_idx=oi, out_val=ov,
                                          out_stats=st, workspace=ws2)
                if no_commit:
                    binding.gravac_commit(oi, r)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            rec[key] = round(float(np.median(ts[2:])) * 1e3, 1)
        log(json.dumps(rec))
        rows.append(rec)
        del g, r, comp, i1, v1, i2, v2
    return rows


def compact(rows):
    """The columns of the configuration table that go into the headline line."""
    out = []
    for r in rows:
        if "pairs" in r:
            out.append({"config": r["config"], "n": r["n"], "pairs": r["pairs"], "cold_us": r["cold_us"],
                        "algorithmic_GBps": r["cold_algorithmic_GBps"]})
        elif "cold_us" in r:
            out.append({"config": r["config"], "n": r["n"], "cfs": r["cfs"], "commit_cf": r["commit_cf"], "k": r["k"],
                        "cold_us": r["cold_us"], "cold_max_us": r["cold_max_us"], "stream_kernel_us": r["cold_stream_kernel_us"],
                        "call_frac": r["cold_call_frac_of_hbm_peak"], "fallback": r["cold_fallback"]})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="leave the table of the other configurations out")
    ap.add_argument("--small", action="store_true", help="1/16-size workload (for a quick functional check)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the same steps replayed from HIP graphs (one graph per gradient of the cycle), "
                         "reported as graph_ms_per_step; the headline value stays the eager one")
    ap.add_argument("--configs", action="store_true",
                    help="instead of the headline step, time one compress call of every configuration (1-5), warm and "
                         "cold, and the decompression of configuration 5, print one JSON line {\"configs\": [...]} and exit")
    ap.add_argument("--filter", default=None,
                    help="with --configs: only the configurations whose name matches this regular expression "
                         "(re.search), e.g. 'VGG16-shaped, CF 10$'")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run 10 plain device copies of the gradient's size (known traffic: 4N read + 4N "
                         "written per copy) so that profiler byte counters can be scaled, then exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build measures the one-GPU share of the path only (no collectives, no sharding); "
            "run it with --gpus 1.")
        sys.exit(2)

    import torch
    from paper_2305_12201_amd import binding, workloads

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.configs:
        print(json.dumps({"configs": time_all_configs(torch, binding, workloads, True, only=args.filter), "data": "synthetic",
                          "note": "times from the caller's HIP events around one gravac_compress call, third "
                                  "error-feedback iteration; call fraction = (12 N + 8 k) / t / 8 TB/s"}), flush=True)
        return

    n_conv, n_fc = workloads.VGG16_N_CONV, workloads.VGG16_N_FC
    if args.small:
        n_conv, n_fc = n_conv // 16, n_fc // 16
    n = n_conv + n_fc
    cf = 1000.0
    if args.copy_calibration:
        a = torch.zeros(n, dtype=torch.float32, device=dev)
        b = torch.ones(n, dtype=torch.float32, device=dev)
        for _ in range(10):
            a.copy_(b)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": 4 * n, "bytes_written_per_copy": 4 * n}))
        return
    k = binding.gravac_topk_count(n, cf)

    log(f"generating {N_GRADS} gradients of {n} elements and {N_WORKERS - 1} peer messages ...")
    comp = binding.Compressor(n, [cf], 0)
    # messages of all workers back to back; slot 0 is rewritten by every step
    msg_idx = torch.empty(N_WORKERS * k, dtype=torch.int32, device=dev)
    msg_val = torch.empty(N_WORKERS * k, dtype=torch.float32, device=dev)
    out_count = torch.zeros(1, dtype=torch.int64, device=dev)
    out_stats = torch.zeros(1, 1, 4, dtype=torch.float64, device=dev)
    residual = torch.zeros(n, dtype=torch.float32, device=dev)
    dense = torch.zeros(n, dtype=torch.float32, device=dev)
    dws = torch.empty(binding.gravac_decompress_workspace_bytes(N_WORKERS, n), dtype=torch.uint8, device=dev)

    def compress(grad, res, slot, timer=None):
        binding.gravac_compress(grad, res, [cf], 0, None, out_idx=msg_idx[slot * k:(slot + 1) * k],
                                out_val=msg_val[slot * k:(slot + 1) * k], out_count=out_count,
                                out_stats=out_stats, workspace=comp.workspace, timer=timer)

    for w in range(1, N_WORKERS):                       # peers: their own gradients, residual zero
        g = torch.from_numpy(workloads.config3_grad(100 + w, n_conv, n_fc)).to(dev)
        scratch = torch.zeros(n, dtype=torch.float32, device=dev)
        compress(g, scratch, w)
        torch.cuda.synchronize()
        del g, scratch
    grad0_host = workloads.config3_grad(0, n_conv, n_fc)
    grads = [torch.from_numpy(grad0_host).to(dev)] + \
            [torch.from_numpy(workloads.config3_grad(i, n_conv, n_fc)).to(dev) for i in range(1, N_GRADS)]
    counts = [k] * N_WORKERS

    def step(i):
        compress(grads[i % N_GRADS], residual, 0)
        binding.gravac_decompress_accumulate(msg_idx, msg_val, counts, dense, workspace=dws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    status = binding.gravac_read_status(comp.workspace)
    assert status["internal_error"] == 0, status

    # ---- the timed region: exactly K steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    status = binding.gravac_read_status(comp.workspace)

    # ---- the last step's message, checked on the device: k pairs, indices strictly ascending and in range, the
    #      residual +0 at every index
    mi, mv = msg_idx[:k], msg_val[:k]
    verified = bool(int(out_count.item()) == k and status["internal_error"] == 0
                    and bool((mi[1:] > mi[:-1]).all()) and int(mi[0]) >= 0 and int(mi[-1]) < n
                    and bool((residual[mi.long()].view(torch.int32) == 0).all())
                    and bool((mv.abs() >= residual.abs().max()).all()))

    # ---- optional: the same K steps replayed from HIP graphs (flat-mode calls are kernel launches only)
    graph_ms = None
    if args.graph:
        graphs = []
        for gi in range(N_GRADS):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                step(gi)
            graphs.append(gr)
        for i in range(5):
            graphs[(args.warmup + args.steps + i) % N_GRADS].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[(args.warmup + args.steps + 5 + i) % N_GRADS].replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / args.steps * 1e3
        assert binding.gravac_read_status(comp.workspace)["internal_error"] == 0

    # ---- per-part timing with HIP events on the launch stream (same steps continued): around the streaming kernel
    #      and the whole compress call (the caller's events, recorded by gravac_compress_profiled), and around the
    #      decompress call, which runs right after compress as in a timed step (the library launches on torch's
    #      current stream, so torch events bracket it)
    timer = binding.CallTimer()
    k_ms, c_ms, d_ms = [], [], []
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(min(args.steps, 50)):
        j = args.warmup + args.steps + i
        compress(grads[j % N_GRADS], residual, 0, timer=timer)
        ev0.record()
        binding.gravac_decompress_accumulate(msg_idx, msg_val, counts, dense, workspace=dws)
        ev1.record()
        ev1.synchronize()
        k_ms.append(timer.pass_ms())
        c_ms.append(timer.call_ms())
        d_ms.append(ev0.elapsed_time(ev1))
    stream_ms = float(np.mean(k_ms))
    compress_ms = float(np.mean(c_ms))
    decompress_ms = float(np.mean(d_ms))
    gain = float(out_stats.cpu()[0, 0, 2])

    achieved = ALGO_BYTES_PER_ELEMENT * n / (stream_ms * 1e-3) / 1e9
    call_bytes = ALGO_BYTES_PER_ELEMENT * n + 8.0 * k
    call_achieved = call_bytes / (compress_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "stream_kernel_vgg16_traffic.json")
    if os.path.exists(tpath) and not args.small:
        try:
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
        except Exception:
            traffic = None

    out = {
        "metric": "dense-gradient GB/s through Top-k+EF compress at CF=100/1000; % of HBM peak",
        "value": 4.0 * n / (ms_per_step * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"VGG16-shaped flat gradient{' (1/16 size: --small)' if args.small else ''}, {n:,} fp32 "
                               f"elements, CF 1000 (k={k:,}), residual carried over {N_GRADS} gradients in turn, thresholds "
                               "sampled in every step (all timed steps alike); step = compress + decompress_accumulate "
                               "of W=8 messages",
                   "n": n, "cf": cf, "k": k, "workers_decompressed": N_WORKERS},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "stream_kernel<0, false, 1> (error feedback + candidate collection, Top-k keys, one CF)",
                     "kernel_ms": stream_ms, "algorithmic_bytes_per_launch": ALGO_BYTES_PER_ELEMENT * n,
                     "kernel_frac": achieved / HBM_PEAK_GBS,
                     "call_frac": call_achieved / HBM_PEAK_GBS, "call_ms": compress_ms,
                     "call_algorithmic_bytes": call_bytes},
        "compress_only": {"ms": compress_ms, "dense_gradient_GBps": 4.0 * n / (compress_ms * 1e-3) / 1e9,
                          "elements_per_s": n / (compress_ms * 1e-3),
                          "algorithmic_frac_of_hbm_peak": call_achieved / HBM_PEAK_GBS},
        "decompress_ms": decompress_ms,
        "compression_gain": gain,
        "fallback_taken": bool(status["any_fallback"]),
        "verified": verified,
    }
    if graph_ms is not None:
        out["graph_ms_per_step"] = graph_ms
    del residual, dense, msg_idx, msg_val
    if not args.no_configs and not args.small:
        log("timing one compress call of every configuration ...")
        vg = grads[0]
        del grads
        out["configs"] = compact(time_all_configs(torch, binding, workloads, False, vgg_grad=vg))
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on the workload's first gradient ...")
        out["cpu_baseline"] = cpu_baseline(grad0_host, cf)
        sel = cpu_select_baseline(grad0_host, k)
        if sel is not None:
            out["cpu_baseline_select"] = sel
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
