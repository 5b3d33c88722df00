#!/usr/bin/env python3
"""Benchmark of the int8 brute-force top-k search on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--nq NQ] [--k 10]

Workload: the 1M x 128 skewed-integer corpus (stand-in for the 128-d descriptor benchmark
of the paper's Table 2), 10 000 queries, squared L2, k = 10, int8 codes, seeded synthetic
data generated on the GPU.  One step = one lpq_search call over the whole query batch
(query encode, contraction + top-k over the whole corpus, merge), with the corpus codes
already resident in HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_OPS = 5.0e15      # MI355X dense int8 matrix peak, op/s
PEAK_HBM = 8.0e12           # MI355X HBM3E, B/s
# HBM bytes of one launch of the main scan kernel on the default workload, from the rocprofv3
# FETCH_SIZE / WRITE_SIZE runs summarised in profiles/search_mfma_kernel_skewed_int_1m_x128_pmc.txt
# (FETCH_SIZE scaled by 2.000, WRITE_SIZE by 1.000 against device copies of known size in the same run).
TRAFFIC_BYTES_DEFAULT_WORKLOAD = 266.7e6
TRAFFIC_SOURCE = ("profiles/search_mfma_kernel_skewed_int_1m_x128_pmc.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                  "runs of this command; a constant taken from that file, not measured in this run)")


def host_info():
    """Logical CPUs of the host and its CPU model string (the oracle's baseline runs there)."""
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return os.cpu_count() or 1, model


class ClockSampler:
    """Samples the shader clock (rocm-smi) from a thread while a GPU loop runs; mean over the samples
    taken between start() and stop(), the first 0.4 s dropped (the clock is still settling)."""

    def __init__(self):
        import threading
        self.samples, self._stop, self._t0 = [], False, 0.0
        self._thread = threading.Thread(target=self._run, daemon=True)
        self._thread.start()

    def _run(self):
        import re
        import subprocess
        while not self._stop:
            t = time.time()
            try:
                out = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=5).stdout
                m = re.search(r'sclk clock speed:"\s*:\s*"\((\d+)Mhz\)', out)
                if m:
                    self.samples.append((t, int(m.group(1))))
            except Exception:
                pass
            time.sleep(0.1)

    def start(self):
        self._t0 = time.time()

    def stop(self):
        t1 = time.time()
        v = [c for t, c in self.samples if self._t0 + 0.4 <= t <= t1 - 0.05]
        return {"mean_mhz": sum(v) / len(v), "min_mhz": min(v), "max_mhz": max(v), "samples": len(v)} if v else None

    def close(self):
        self._stop = True


def time_batches(lpq, torch, index, q, k, metric, reps, warm=10):
    """ms per lpq_search call over `reps` back-to-back calls on one batch, and the per-call time of its
    scan kernel and seeding pass (HIP events around each launch, as in the main timed region)."""
    nq = q.shape[0]
    ids = torch.empty((nq, k), dtype=torch.int32, device="cuda")
    dists = torch.empty_like(ids)
    ws = torch.empty(index.workspace_bytes(nq, k, metric) + 256, dtype=torch.uint8, device="cuda")
    for _ in range(warm):
        index.search(q, k, metric, out=(ids, dists), workspace=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        index.search(q, k, metric, out=(ids, dists), workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    # kernel times from a second, bracketed pass (the event pairs would otherwise sit between the launches timed above)
    lpq.profile_enable(True)
    for _ in range(min(reps, 100)):
        index.search(q, k, metric, out=(ids, dists), workspace=ws)
    torch.cuda.synchronize()
    n_scan, scan_ms = lpq.profile_read(lpq.PROFILE_SCAN)
    _, seed_ms = lpq.profile_read(lpq.PROFILE_SEED)
    lpq.profile_enable(False)
    calls = min(reps, 100)
    return ms, scan_ms / calls, seed_ms / calls, n_scan / calls


def cpu_baseline(oracle, x_host, q_host, params, k, metric, gpu_ids, gpu_dists, sample, bits=8, packed=False):
    """The oracle as it stands, timed on the host cores on `sample` queries; also checks the
    GPU result of those queries bit for bit."""
    import numpy as np
    kq, sb, se, _ = params
    oq = oracle.Quantizer(x_host.shape[1], bits).set_params(kq, sb, se)
    codes = oq.encode(x_host)
    qcodes = oq.encode(q_host[:sample])
    if packed:   # two codes per byte hold -8 .. 7
        codes, qcodes = oracle.nibble_codes(codes), oracle.nibble_codes(qcodes)
    threads = max(1, min(16, oracle.max_threads(), os.cpu_count() or 1))
    t0 = time.perf_counter()
    oids, odists = oracle.search_i8(codes, qcodes, k, metric, threads=threads)
    dt = time.perf_counter() - t0
    ok = bool(np.array_equal(oids, gpu_ids[:sample]) and np.array_equal(odists, gpu_dists[:sample]))
    # the paper measures throughput on a single thread (Section 5.1): the same oracle on one core, fewer queries
    s1 = max(1, min(sample, int(4e9 / (float(codes.shape[0]) * codes.shape[1]))))
    t0 = time.perf_counter()
    oracle.search_i8(codes, qcodes[:s1], k, metric, threads=1)
    dt1 = time.perf_counter() - t0
    host_cores, host_cpu = host_info()
    return {"value": sample / dt, "unit": "queries/s", "cores": threads, "host_cores": host_cores, "host_cpu": host_cpu,
            "kind": "oracle",
            "sample": f"first {sample} queries against the full corpus, {dt:.1f} s wall",
            "gpu_matches_oracle_on_sample": ok,
            "single_thread": {"value": s1 / dt1, "unit": "queries/s", "cores": 1,
                              "sample": f"first {s1} queries against the full corpus, {dt1:.1f} s wall"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The first ~20 searches after an idle period run about 6 % slower (the clocks ramp up), so the
    # default warm-up covers them; 100 timed searches of the default workload take ~0.14 s.
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--ramp", type=int, default=60,
                    help="untimed searches BEFORE the warm-up (reported as ramp_searches): the shader clock needs "
                         "~20 searches (~25 ms of load) after idle to settle, so a short --warmup would time the ramp")
    ap.add_argument("--no-small-batch", action="store_true", help="skip the small-batch (HBM regime) block")
    ap.add_argument("--no-probe", action="store_true", help="skip the attainable-rate probes")
    ap.add_argument("--sample-clocks", action="store_true",
                    help="after the timed region, run ~2 s of searches and ~1 s of each matrix probe while a thread "
                         "samples the shader clock with rocm-smi; reported under `clocks` (evidence for the power limit)")
    ap.add_argument("--nq", type=int, default=0, help="query batch (default: the workload's 10 000)")
    ap.add_argument("--k", type=int, default=10)
    ap.add_argument("--n", type=int, default=0, help="corpus rows (default: the workload's 1 000 000)")
    ap.add_argument("--cpu-sample", type=int, default=512)
    ap.add_argument("--recall-queries", type=int, default=1000)
    ap.add_argument("--path", type=int, default=0, help="0 auto, 1 generic kernel, 2 matrix-core kernel")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--seed-rows", type=int, default=0)
    ap.add_argument("--workload", default="skewed_1m", choices=["tiny", "skewed_1m", "aniso_1m2", "scaled_10m", "product_100m"],
                    help="synthetic workload shape (default: the benchmark configuration)")
    ap.add_argument("--d", type=int, default=0, help="features per vector instead of the workload's (same recipe and seed)")
    ap.add_argument("--bits", type=int, default=8, help="bits per code B of Equation 1 (default 8)")
    ap.add_argument("--packed", action="store_true", help="store two codes per byte (needs --bits <= 4, k <= 16)")
    ap.add_argument("--calib", default="", help="calibration mode instead of the workload's (minmax, absmax, gauss, quantile)")
    ap.add_argument("--scope", default="", help="calibration scope instead of the workload's (per_feature, global, shared_width)")
    ap.add_argument("--calib-arg", type=float, default=1.0, help="sigma multiplier (gauss) or clipped fraction (quantile)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the candidate-list calls (gathered distances, fp32 re-rank), report recall "
                         "before / after the re-rank for a per-feature 6-bit quantizer, and time a small batch on "
                         "4-bit codes stored one and two per byte")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 512 MiB device copy (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; multi-GPU sharding is a design note only "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2110_08919_amd import lpq, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    lpq.lib()
    base = {"tiny": synth.TINY, "skewed_1m": synth.SKEWED_1M, "aniso_1m2": synth.ANISO_1M2,
            "scaled_10m": synth.SCALED_10M, "product_100m": synth.PRODUCT_100M}[args.workload]
    w = base.scaled(n=args.n or None, nq=args.nq or None)
    if args.d:
        w = synth.Workload(f"{w.recipe}_{w.n}_x{args.d}", w.recipe, w.n, args.d, w.nq, w.metric, w.ks, w.calib, w.scope, w.seed)
    k, metric = args.k, w.metric

    # ---- inputs and index build (not part of the timed search step) -------------------
    x = w.corpus("cuda")
    q = w.queries("cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    calib, scope = args.calib or w.calib, args.scope or w.scope
    quant = lpq.Quantizer(w.d, args.bits).calibrate(x, calib, scope, args.calib_arg)
    torch.cuda.synchronize()
    t_cal = time.perf_counter() - t0
    index = lpq.Index(quant, w.n, packed=args.packed)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    index.add_f32(x)
    torch.cuda.synchronize()
    t_enc = time.perf_counter() - t0

    lpq.set_tuning(lpq.TUNE_PATH, args.path)
    lpq.set_tuning(lpq.TUNE_SPLITS, args.splits)
    lpq.set_tuning(lpq.TUNE_SEED_ROWS, args.seed_rows)
    ids = torch.empty((w.nq, k), dtype=torch.int32, device="cuda")
    dists = torch.empty((w.nq, k), dtype=torch.int32, device="cuda")
    ws = torch.empty(index.workspace_bytes(w.nq, k, metric) + 256, dtype=torch.uint8, device="cuda")

    # Clock ramp, disclosed under its own key: searches that are neither warm-up nor timed.  After
    # an idle period the first ~20 searches run ~6 % slower while the shader clock settles, which a
    # 5-search warm-up would put inside the timed region.
    for _ in range(max(args.ramp, 0)):
        index.search(q, k, metric, out=(ids, dists), workspace=ws)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        index.search(q, k, metric, out=(ids, dists), workspace=ws)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` searches ------------------------------------------
    lpq.profile_enable(True)     # creates the event pairs of the per-launch timing here, outside the timed region
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        index.search(q, k, metric, out=(ids, dists), workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    launches, kern_ms = lpq.profile_read(lpq.PROFILE_SCAN)       # the contraction + top-k scan kernel
    seed_launches, seed_ms = lpq.profile_read(lpq.PROFILE_SEED)  # its threshold-seeding pass
    lpq.profile_enable(False)
    if args.copy_calibration:      # a plain copy of known size, for scaling FETCH_SIZE / WRITE_SIZE
        src = torch.ones(512 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Roofline of the dominant kernel, the contraction + top-k scan over the whole corpus: its
    # algorithmic work per launch over its average launch duration (HIP events on the launch
    # stream, recorded inside the library around every launch of the timed region).
    launches_per_step = launches / args.steps
    kern_ms_per_launch = kern_ms / max(launches, 1)
    ops_per_launch = 2.0 * w.nq * w.n * w.d / launches_per_step      # true d, not the padded one
    code_bytes = w.d / 2.0 if args.packed else float(w.d)
    bytes_per_launch = float(w.n) * (code_bytes + 4) / launches_per_step   # corpus codes + norms, streamed once
    mfma_frac = ops_per_launch / (kern_ms_per_launch * 1e-3) / PEAK_INT8_OPS
    hbm_frac = bytes_per_launch / (kern_ms_per_launch * 1e-3) / PEAK_HBM
    if mfma_frac >= hbm_frac:
        roofline = {"bound": "mfma", "achieved": ops_per_launch / (kern_ms_per_launch * 1e-3) / 1e12,
                    "peak": PEAK_INT8_OPS / 1e12, "unit": "TOP/s", "frac": mfma_frac, "traffic": None}
    else:
        roofline = {"bound": "hbm", "achieved": bytes_per_launch / (kern_ms_per_launch * 1e-3) / 1e9,
                    "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": hbm_frac, "traffic": None}
    default_workload = (args.workload == "skewed_1m" and args.n == 0 and args.nq == 0 and args.k == 10 and args.path == 0
                        and args.splits == 0 and args.seed_rows == 0 and args.bits == 8 and not args.packed and args.d == 0
                        and not args.calib and not args.scope)
    roofline["traffic"] = TRAFFIC_BYTES_DEFAULT_WORKLOAD if default_workload else None
    roofline["traffic_source"] = TRAFFIC_SOURCE if default_workload else None
    plan = lpq.search_plan_info(w.d, args.bits, int(args.packed), w.n, int(q.shape[0]), k)
    long_scan = w.d > 256 or (w.d > 128 and plan[3] == 128)   # the scan for long rows (its query tile says so)
    roofline["kernel"] = ("search_long_kernel" if long_scan else "search_mfma_kernel") + \
        ", main scan (contraction + top-k over all corpus rows)"
    roofline["kernel_ms_per_launch"] = kern_ms_per_launch
    roofline["launches_per_step"] = launches_per_step
    roofline["seeding_pass_ms_per_step"] = seed_ms / args.steps
    roofline["frac_with_seeding_pass"] = max(mfma_frac, hbm_frac) * kern_ms / max(kern_ms + seed_ms, 1e-12)
    # the same algorithmic work over the whole step (query encode, seeding pass, scan, selection)
    roofline["frac_end_to_end"] = (2.0 * w.nq * w.n * w.d / (ms_per_step * 1e-3) / PEAK_INT8_OPS if mfma_frac >= hbm_frac
                                   else float(w.n) * (code_bytes + 4) / (ms_per_step * 1e-3) / PEAK_HBM)

    # ---- what the part sustains on the two bounding resources (probes, after the timed region) ----
    attainable = None
    if not args.no_probe:
        gen = torch.Generator(device="cuda").manual_seed(7)
        rnd = torch.randint(-128, 128, (1 << 20,), generator=gen, device="cuda", dtype=torch.int8)
        code_view = quant.encode(x[:min(w.n, 8192)].contiguous()).contiguous()   # codes of this workload's items
        buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 256)
        attainable = {
            "mfma_zero_operands_TOPs": lpq.probe_mfma_i8(None),
            "mfma_random_operands_TOPs": lpq.probe_mfma_i8(rnd),
            "mfma_workload_codes_TOPs": lpq.probe_mfma_i8(code_view),
            "scan_core_loop_workload_codes_TOPs": lpq.probe_scan_core(code_view),
            "stream_global_to_lds_GBps": lpq.probe_stream(buf, 0, 10),
            "stream_register_loads_GBps": lpq.probe_stream(buf, 1, 10),
            "note": "register-resident int8 matrix-instruction loop (operand bits as named; the shader clock falls "
                    "under matrix load: the part is power-limited there), the scan's inner loop alone (matrix "
                    "instructions + filter epilogue + LDS operand reads; no copies, barrier, candidates or query "
                    "padding) and a streaming read of 1 GiB; peaks in `roofline` are the published ones",
        }
        del buf, rnd
        ref = attainable["mfma_workload_codes_TOPs"] * 1e12 if mfma_frac >= hbm_frac else attainable["stream_global_to_lds_GBps"] * 1e9
        roofline["frac_of_attainable"] = roofline["achieved"] * (1e12 if mfma_frac >= hbm_frac else 1e9) / ref

    # ---- shader clock under the search and under the probes (optional) ----------------------------
    clocks = None
    if args.sample_clocks:
        sampler = ClockSampler()
        clocks = {}
        reps = max(200, int(2000.0 / max(ms_per_step, 1e-3)))
        torch.cuda.synchronize()
        sampler.start()
        for _ in range(reps):
            index.search(q, k, metric, out=(ids, dists), workspace=ws)
        torch.cuda.synchronize()
        clocks["search_loop"] = sampler.stop()
        gen = torch.Generator(device="cuda").manual_seed(7)
        rnd = torch.randint(-128, 128, (1 << 20,), generator=gen, device="cuda", dtype=torch.int8)
        codes_ = quant.encode(x[:min(w.n, 8192)].contiguous()).contiguous()
        for name, op in (("mfma_zero_operands", None), ("mfma_workload_codes", codes_), ("mfma_random_operands", rnd)):
            sampler.start()
            tops = [lpq.probe_mfma_i8(op, 1500000) for _ in range(2)]
            clocks[name] = dict(sampler.stop() or {}, TOPs=tops[-1])
        sampler.start()
        tops = [lpq.probe_scan_core(codes_, 250000) for _ in range(2)]
        clocks["scan_core_loop_workload_codes"] = dict(sampler.stop() or {}, TOPs=tops[-1])
        sampler.close()

    # ---- recall@k of the int8 search against fp32 exact search (GPU), on a query subset ----
    rq = min(args.recall_queries, w.nq)
    recall = None
    if rq > 0:
        eids, _ = lpq.search_f32(x, q[:rq], k, metric)
        a, e = ids[:rq].cpu().numpy(), eids.cpu().numpy()
        recall = float(np.mean([len(set(a[i]) & set(e[i])) / k for i in range(rq)]))

    # The headline calibration (global min/max on integer data) makes codes = x - 128, so the recall
    # above is 1 by construction; per-feature min/max on the same data is the informative figure.
    recall_pf = None
    if rq > 0 and default_workload:
        qpf = lpq.Quantizer(w.d, args.bits).calibrate(x, "minmax", "per_feature")
        ipf = lpq.Index(qpf, w.n).add_f32(x)
        pids, _ = ipf.search(q[:rq], k, metric)
        a = pids.cpu().numpy()
        recall_pf = float(np.mean([len(set(a[i]) & set(e[i])) / k for i in range(rq)]))
        del ipf, qpf

    # ---- small batches: the regime bound by corpus bytes (after the timed region) -------------
    small = None
    if default_workload and not args.no_small_batch:
        small = {"note": "ms per lpq_search call over back-to-back calls on one batch; bytes = n (d + 4) corpus bytes "
                         "streamed once per call; fractions of 8 TB/s for the scan kernel alone and end to end; the "
                         "128 MB of the 1M x 128 codes stay in the 256 MB memory-side cache between calls, the "
                         "960 MB of 10M x 96 do not",
                 "cases": []}
        def small_case(name, idx_, qq, n_, d_, reps):
            ms, scan_ms, seed_ms, scans = time_batches(lpq, torch, idx_, qq, k, metric, reps)
            nbytes = float(n_) * (d_ + 4)
            small["cases"].append({"workload": name, "nq": int(qq.shape[0]), "ms_per_batch": ms, "scan_ms": scan_ms,
                                   "seeding_pass_ms": seed_ms, "scan_launches": scans, "bytes": nbytes,
                                   "hbm_frac_scan": nbytes / (scan_ms * 1e-3) / PEAK_HBM if scan_ms > 0 else None,
                                   "hbm_frac_end_to_end": nbytes / (ms * 1e-3) / PEAK_HBM,
                                   "queries_per_s": qq.shape[0] / (ms * 1e-3)})
        for nb in (1, 16, 256):
            small_case(w.name, index, q[:nb], w.n, w.d, 300)
        w4 = synth.SCALED_10M
        x4 = w4.corpus("cuda")
        q4 = w4.queries("cuda")[:16].contiguous()
        quant4 = lpq.Quantizer(w4.d, 8).calibrate(x4, w4.calib, w4.scope)
        index4 = lpq.Index(quant4, w4.n).add_f32(x4)
        del x4
        small_case(w4.name, index4, q4, w4.n, w4.d, 200)
        del index4, quant4

    # ---- candidate-list calls (not part of the timed step) ---------------------------------
    extras = None
    if args.extras and not args.packed:   # (the gathered-distance call takes unpacked indexes only)
        def timed(fn, reps=10):
            fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                out = fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps, out
        m = 100
        gen = torch.Generator(device="cuda").manual_seed(1)
        gids = torch.randint(0, w.n, (w.nq, m), generator=gen, device="cuda", dtype=torch.int32)
        qcodes = quant.encode(q).contiguous()
        g_ms, _ = timed(lambda: index.gather_dist(qcodes, gids, metric))
        rq2 = min(1000, w.nq)
        q6 = lpq.Quantizer(w.d, 6).calibrate(x, "minmax", "per_feature")
        i6 = lpq.Index(q6, w.n).add_f32(x)
        ex, _ = lpq.search_f32(x, q[:rq2], k, metric)
        c_ids, _ = i6.search(q[:rq2], k, metric)
        w_ids, _ = i6.search(q[:rq2], 4 * k, metric)
        r_ms, (f_ids, _) = timed(lambda: lpq.rerank_f32(x, q[:rq2], w_ids, k, metric))
        def rec(a_, e_):
            a_, e_ = a_.cpu().numpy(), e_.cpu().numpy()
            return float(np.mean([len(set(a_[i]) & set(e_[i])) / k for i in range(a_.shape[0])]))
        extras = {"gather_dist": {"pairs": w.nq * m, "ms": g_ms, "Mpairs_per_s": w.nq * m / g_ms / 1e3,
                                  "GBps_rows": w.nq * m * (w.d + 4) / g_ms / 1e6},
                  "rerank_f32": {"queries": rq2, "candidates": 4 * k, "ms": r_ms,
                                 "recall_6bit_per_feature": rec(c_ids, ex), "recall_after_rerank": rec(f_ids, ex)}}

        # 4-bit codes, one per byte against two per byte: the byte-bound small batch
        if k <= 16 and w.d <= 256:
            q4 = lpq.Quantizer(w.d, 4).calibrate(x, "quantile", w.scope, 0.001)
            nb = min(16, w.nq)
            packed = {}
            for name, pk in (("one_code_per_byte", False), ("two_codes_per_byte", True)):
                i4 = lpq.Index(q4, w.n, packed=pk).add_f32(x)
                p_ids, _ = i4.search(q[:rq2], k, metric)
                p_ms, _ = timed(lambda: i4.search(q[:nb], k, metric), reps=20)
                packed[name] = {"ms": p_ms, "batch": nb, "recall": rec(p_ids, ex),
                                "GBps_rows": w.n * (i4.data()[1] + 4) / p_ms / 1e6}
                del i4
            extras["four_bit_quantile_clip"] = packed

    # ---- CPU baseline: the oracle, on a bounded sample -----------------------------------
    cpu = None
    if args.cpu_sample > 0:
        from oracle import lpq_oracle as oracle
        sample = min(args.cpu_sample, w.nq)
        cpu = cpu_baseline(oracle, x.cpu().numpy(), q[:sample].cpu().numpy(), quant.get_params(), k, metric,
                           ids.cpu().numpy(), dists.cpu().numpy(), sample, args.bits, args.packed)

    out = {
        "metric": "queries/sec, int8 brute-force top-%d, %s" % (k, "1M x 128" if args.workload == "skewed_1m" and not args.n else f"{w.n} x {w.d}"),
        "value": w.nq / (ms_per_step * 1e-3),
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 (two per byte, int8 matrix core)" if args.packed else "int8",
        "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "d": w.d, "nq": w.nq, "k": k, "metric": metric,
                   "calibration": f"{calib}/{scope}", "bits": args.bits, "packed": bool(args.packed), "seed": w.seed,
                   "path": {0: "auto", 1: "generic", 2: "matrix-core"}[args.path]},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "ramp_searches": max(args.ramp, 0),
        "attainable": attainable,
        "clocks": clocks,
        "small_batch": small,
        "recall_at_k_vs_fp32": recall,
        "recall_at_k_vs_fp32_per_feature_calibration": recall_pf,
        "recall_queries": rq,
        "index_build": {"calibrate_ms": t_cal * 1e3, "encode_ms": t_enc * 1e3,
                        "encode_GBps": w.n * w.d * 5 / t_enc / 1e9},
        "wall_s_timed_region": wall,
    }
    if extras:
        out["extras"] = extras
    print(json.dumps(out))


if __name__ == "__main__":
    main()
