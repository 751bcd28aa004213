#!/usr/bin/env python3
"""Benchmark of the GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--sweep]

One "step" is one call of the library's dgemm on the headline workload
(m = n = k = 8192, column-major, alpha = 1.5, beta = -0.5, leading dimensions
8200, entries uniform[-1, 1] from a fixed seed), operands already resident in
HBM.  Prints ONE JSON line on stdout.  ``--sweep`` additionally times the other
workload shapes and prints one JSON line per shape on stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "dgemm GFLOP/s and % of FP64 MFMA peak at m=n=k=8192 (1 GPU)"
PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}   # MI355X dense MFMA peaks
HBM_TBPS = 8.0


def time_calls(torch, fn, steps, warmup, per_step=None):
    """Wall time (host clock, synchronised both sides) and device time (events
    on the stream the kernels are launched on) of `steps` calls; with a list as
    `per_step`, also the device time of every single call (events between the calls)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1 if per_step is not None else 2)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        fn()
        if per_step is not None:
            marks[i + 1].record()
    if per_step is None:
        marks[1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if per_step is not None:
        per_step.extend(marks[i].elapsed_time(marks[i + 1]) * 1e-3 for i in range(steps))
    return (t1 - t0) / steps, marks[0].elapsed_time(marks[-1]) * 1e-3 / steps


def device_operands(torch, np, si, dtype, ta, tb, m, n, k, lda, ldb, ldc, seed_cfg, kind="uniform"):
    rng = si.rng_for(seed_cfg, m + n + k)
    gen = si.uniform if kind == "uniform" else si.normal
    ra, ca = si.operand_shape(ta, m, k)
    rb, cb = si.operand_shape(tb, k, n)
    A = gen(rng, ra, ca, lda, dtype, sentinel=0.0)
    B = gen(rng, rb, cb, ldb, dtype, sentinel=0.0)
    C = gen(rng, m, n, ldc, dtype, sentinel=0.0)
    return (A, B, C), tuple(torch.from_numpy(X).cuda() for X in (A, B, C))


def cpu_baseline(np, oracle, host_ops, m, k, lda, ldb, ldc, alpha, beta, budget_s=15.0):
    """Time the oracle (working precision, as it stands) on the first columns
    of the same workload: C[:, :ns] = alpha A B[:, :ns] + beta C[:, :ns]."""
    A, B, C = host_ops
    cores = oracle.num_threads()

    def run(ns):
        Cs = C[:ns].copy()
        t0 = time.perf_counter()
        info = oracle.gemm_work("N", "N", m, ns, k, alpha, A, lda, B, ldb, beta, Cs, ldc)
        dt = time.perf_counter() - t0
        assert info == 0
        return dt

    ns = max(cores, 16)
    dt = run(ns)
    rate = 2.0 * m * ns * k / dt
    ns2 = int(min(C.shape[0], max(ns, budget_s * rate / (2.0 * m * k))))
    ns2 -= ns2 % cores or 0
    ns2 = max(ns2, ns)
    dt2 = run(ns2)
    out = {"value": round(2.0 * m * ns2 * k / dt2 / 1e9, 3), "unit": "GFLOP/s", "cores": cores,
           "kind": "oracle",
           "sample": f"first {ns2} of {C.shape[0]} columns of C of the same dgemm "
                     f"(m={m}, k={k}), {dt2:.1f} s, working-precision triple loop"}
    # the same oracle on one core (n = 1024) and on all cores (n = 4096): leading blocks of the same operands
    also = []
    for nn, threads in ((1024, 1), (4096, cores)):
        if nn > m or nn > C.shape[0]:
            continue
        oracle.set_num_threads(threads)
        Cs = C[:nn].copy()
        t0 = time.perf_counter()
        info = oracle.gemm_work("N", "N", nn, nn, nn, alpha, A, lda, B, ldb, beta, Cs, ldc)
        dt = time.perf_counter() - t0
        assert info == 0
        also.append({"n": nn, "cores": threads, "GFLOP/s": round(2.0 * nn ** 3 / dt / 1e9, 3), "s": round(dt, 2)})
    oracle.set_num_threads(cores)
    out["also"] = also
    return out


def xg_cus(torch):
    return torch.cuda.get_device_properties(0).multi_processor_count


def mfma_probe_tflops(torch, xg, prec, blocks=512, iters=10000):
    """TFLOP/s of xgemm_mfma_peak_probe (32768 flops per wave and round), second of two timed launches."""
    sink = torch.zeros(blocks * 256, dtype=torch.float32 if prec == "s" else torch.float64, device="cuda")
    ms = 0.0
    for _ in range(2):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rc = xg.xgemm_mfma_peak_probe(prec, blocks, iters, sink)
        e1.record()
        torch.cuda.synchronize()
        if rc:
            raise RuntimeError(f"xgemm_mfma_peak_probe returned {rc}")
        ms = e0.elapsed_time(e1)
    return blocks * 4 * iters * 32768 / ms / 1e9


LATENCY_ROWS = [("FP64 fused multiply-add", 8), ("FP32 fused multiply-add", 8), ("FP64 reciprocal square root (+ one add)", 8),
                ("LDS write, read from another lane", 4), ("FP64 16x16x4 matrix instruction, same accumulator", 4),
                ("FP64 matrix instruction -> vector instruction -> matrix instruction", 4),
                ("lane read to scalar registers -> vector instruction", 8), ("FP32 32x32x2 matrix instruction, same accumulator", 4)]


def latencies(torch, xg, iters=4000):
    out = torch.zeros(8, dtype=torch.int64, device="cuda")
    sink = torch.zeros(64, dtype=torch.float64, device="cuda")
    for _ in range(3):                      # the last of three runs is reported (clocks and caches settled)
        rc = xg.xgemm_latency_probe(out, sink, iters)
        if rc:
            raise RuntimeError(f"xgemm_latency_probe returned {rc}")
        torch.cuda.synchronize()
    ticks = out.cpu().tolist()
    rows = []
    for (name, per), t in zip(LATENCY_ROWS, ticks):
        ns = 10.0 * t / (iters * per)
        rows.append({"chain": name, "ns_per_instruction": round(ns, 2), "cycles_at_2.4GHz": round(ns * 2.4, 1)})
    print(json.dumps({"latency_probe": rows, "iters": iters}))


def model_table(torch, np, xg, args):
    """The paper's Sec. 6.1 experiment: predicted against measured efficiency over a family of kernels."""
    from math import gcd
    cus = xg_cus(torch)
    print("| Variant | WG/CU | m x n | rounds | MFMA / slab / wave | loads | LDS reads | LDS writes | stall cycles / slab "
          "| predicted | measured NN | measured NT | better of the two / probe | table | planner uses |")
    print("|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|")
    for prec, dtype, gemm, fkey in (("d", torch.float64, xg.xgemm_dgemm, "f64"), ("s", torch.float32, xg.xgemm_sgemm, "f32")):
        probe = mfma_probe_tflops(torch, xg, prec)
        v = 0
        while xg.xgemm_variant_name(prec, v) is not None:
            name = xg.xgemm_variant_name(prec, v)
            mt_m, mt_n, _kt = (int(x) for x in name.split("_")[1].split("x"))
            wgm, wgn = (int(x) for x in name.split("_")[2][1:].split("x"))
            _rc, o = xg.xgemm_model_predict(prec, v, "N", "N")
            _rc, (e_meas, e_model, e_used) = xg.xgemm_model_efficiency(prec, v)
            wgs = int(o[11] * 4 / (wgm * wgn))
            slots = cus * wgs
            tiles_m = 4096 // mt_m
            q = slots // gcd(slots, tiles_m)
            tiles_n = q * max(1, round(4096 / mt_n / q))
            m, n = tiles_m * mt_m, tiles_n * mt_n
            k = 8192
            lda, ldb = m + 8, max(k, n) + 8
            A = torch.rand(lda * k, dtype=dtype, device="cuda") * 2 - 1
            B = torch.rand(ldb * max(k, n), dtype=dtype, device="cuda") * 2 - 1
            C = torch.zeros(lda * n, dtype=dtype, device="cuda")
            xg.xgemm_force_variant(v)
            xg.xgemm_force_split(1)
            frac = {}
            for tb in ("N", "T"):
                def step():
                    rc = gemm("N", tb, m, n, k, 1.0, A, lda, B, ldb, 1.0, C, lda)
                    if rc:
                        raise RuntimeError(f"{name}: gemm returned {rc}")

                each = []
                time_calls(torch, step, 12, 4, each)
                assert name in xg.xgemm_last_kernel_name(), (name, xg.xgemm_last_kernel_name())
                frac[tb] = 2.0 * m * n * k / sorted(each)[len(each) // 2] / 1e12 / PEAK_TFLOPS[fkey]
            best = max(frac.values())
            print(f"| {name} | {wgs} | {m} x {n} x {k} | {tiles_m * tiles_n // slots} | {o[0]:.0f} | {o[1]:.0f} | {o[2]:.0f} "
                  f"| {o[3]:.0f} | {o[8]:.0f} | {e_model:.3f} | {frac['N']:.3f} | {frac['T']:.3f} "
                  f"| {best * PEAK_TFLOPS[fkey] / probe:.3f} | {e_meas:.3f} | {e_used:.3f} |", flush=True)
            del A, B, C
            v += 1
        print(f"<!-- {prec}: MFMA-only probe {probe:.1f} TFLOP/s = {probe / PEAK_TFLOPS[fkey]:.3f} of the published peak -->")
    xg.xgemm_tuning_reset()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--size", type=int, default=8192, help="m = n = k of the headline dgemm")
    ap.add_argument("--prec", choices=["d", "s"], default="d",
                    help="d: the headline dgemm (default).  s: the sgemm square of the same size "
                         "(alpha = beta = 1, minimal ld) for profiling; reported as its own metric")
    ap.add_argument("--variant", type=int, default=-1, help="force a tile variant (tuning)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--sweep", action="store_true", help="also time the other shapes (stderr)")
    ap.add_argument("--only", default=None, help="with --sweep: only the rows whose name contains this text")
    ap.add_argument("--calib-copy", action="store_true",
                    help="after the timed region, run one plain 1 GiB device-to-device copy kernel "
                         "(a known-size reference for scaling HBM traffic counters under rocprofv3)")
    ap.add_argument("--latencies", action="store_true",
                    help="instead of the benchmark: run the library's latency probe and print what a dependent "
                         "chain of each instruction kind costs a lone wave (ns and cycles at 2.4 GHz)")
    ap.add_argument("--model-table", action="store_true",
                    help="instead of the benchmark: every tile variant forced in turn on a product whose tiles fill "
                         "every CU in every round (k = 4096), its fraction of the MFMA peak beside the analytical "
                         "model's prediction, as a markdown table")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (--gpus 1); "
                 "the GEMM path has no multi-GPU part.")

    import numpy as np
    import torch

    import paper_1611_08035_amd as xg
    import synth_inputs as si

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    xg.lib()
    xg.xgemm_force_variant(args.variant)
    if args.latencies:
        return latencies(torch, xg)
    if args.model_table:
        return model_table(torch, np, xg, args)

    nsz = args.size
    single = args.prec == "s"
    ld = nsz if single else si.padded_ld(nsz)
    alpha, beta = (1.0, 1.0) if single else (1.5, -0.5)
    dtype = np.float32 if single else np.float64
    gemm = xg.xgemm_sgemm if single else xg.xgemm_dgemm
    host_ops, (dA, dB, dC) = device_operands(torch, np, si, dtype, "N", "N", nsz, nsz, nsz, ld, ld, ld,
                                             3 if single else 2)

    def step():
        rc = gemm("N", "N", nsz, nsz, nsz, alpha, dA, ld, dB, ld, beta, dC, ld)
        if rc:
            raise RuntimeError(f"xgemm gemm returned {rc}")

    each = []
    wall, dev = time_calls(torch, step, args.steps, args.warmup, each)
    each.sort()
    kernel = xg.xgemm_last_kernel_name()
    flops = 2.0 * nsz ** 3
    gflops = flops / wall / 1e9
    achieved = flops / dev / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "dgemm_8192_hbm_traffic.json")
    if nsz == 8192 and not single and os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("traffic_bytes_per_launch")
        except Exception:
            traffic = None

    fkey = "f32" if single else "f64"
    peak = PEAK_TFLOPS[fkey]
    metric = METRIC if not single else f"sgemm GFLOP/s and % of FP32 MFMA peak at m=n=k={nsz} (1 GPU)"
    out = {
        "metric": metric, "value": round(gflops, 1), "unit": "GFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall * 1e3, 4),
        "ms_median": round(each[len(each) // 2] * 1e3, 4), "ms_min": round(each[0] * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": fkey,
        "data": "synthetic",
        "config": {"workload": f"{'s' if single else 'd'}gemm NN m=n=k={nsz} alpha={alpha} beta={beta} "
                               f"lda=ldb=ldc={ld} uniform[-1,1]",
                   "kernel": kernel},
        f"pct_of_fp{fkey[1:]}_mfma_peak": round(100.0 * gflops / 1e3 / peak, 2),
        "roofline": {"bound": "mfma", "achieved": round(achieved, 3), "peak": peak,
                     "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "traffic": traffic,
                     "traffic_source": "stored: rocprofv3 FETCH_SIZE / WRITE_SIZE of this command in a run of its own "
                                       "(profiles/dgemm_8192_counters.md), not measured in this run" if traffic else None,
                     "kernel": kernel, "avg_launch_ms": round(dev * 1e3, 4)},
    }
    # the matrix-core rate this device sustains right now (register-resident MFMA loop, no memory
    # traffic), so that the headline can also be read against the clock of the box it ran on
    probe = mfma_probe_tflops(torch, xg, "s" if single else "d")
    out["mfma_probe"] = {"tflops": round(probe, 2), "frac_of_published_peak": round(probe / peak, 4),
                         "headline_frac_of_probe": round(achieved / probe, 4),
                         # matrix-instruction rate of the probe over the flops per cycle of the device (CUs x 4 SIMDs x
                         # 32 or 64 flop): the engine clock the matrix cores sustained just after the timed region
                         "sustained_clock_ghz": round(probe * 1e3 / (xg_cus(torch) * 4 * (64 if single else 32)), 3)}
    if not args.no_cpu and not single:
        import oracle
        out["cpu_baseline"] = cpu_baseline(np, oracle, host_ops, nsz, nsz, ld, ld, ld, alpha, beta)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)

    if args.calib_copy:
        src = torch.ones(1 << 27, dtype=torch.float64, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.sweep:
        del dA, dB, dC, host_ops
        sweep(torch, np, xg, si, args)


def sweep(torch, np, xg, si, args):
    """Other workload shapes, reported the same way (GFLOP/s, fraction of the
    bound that applies: MFMA peak, or HBM for the thin rank-k updates)."""
    rows = []
    for nsz in (512, 1024, 2048, 4096):
        ld = si.padded_ld(nsz)
        rows.append(("d", "N", "N", nsz, nsz, nsz, ld, ld, ld, 1.5, -0.5, 2, "uniform"))
    for nsz in (1024, 4096, 8192, 16384):
        rows.append(("s", "N", "N", nsz, nsz, nsz, nsz, nsz, nsz, 1.0, 1.0, 3, "uniform"))
    for ta, tb in (("N", "T"), ("T", "N"), ("T", "T")):
        rows.append(("s", ta, tb, 4096, 4096, 4096, 4096, 4096, 4096, 1.0, 1.0, 3, "uniform"))
    for mn in (4096, 16384):
        for k in (64, 128, 256):
            rows.append(("d", "N", "N", mn, mn, k, mn, k, mn, -1.0, 1.0, 4, "normal"))
    rows.append(("d", "N", "N", 4097, 3001, 257, 4097, 257, 4097, -1.0, 1.0, 4, "normal"))
    # ragged everywhere (edge tiles along both sides, a partial last slab, a partly filled last round)
    rows.append(("d", "N", "N", 5000, 5000, 5000, 5000, 5000, 5000, 1.5, -0.5, 2, "uniform"))
    rows.append(("d", "T", "N", 7001, 7001, 7001, 7001, 7001, 7001, 1.5, -0.5, 2, "uniform"))
    rows.append(("s", "N", "T", 7001, 7003, 7000, 7001, 7003, 7001, 1.5, -0.5, 3, "uniform"))
    want = lambda name: args.only is None or args.only in name
    for prec, ta, tb, m, n, k, lda, ldb, ldc, alpha, beta, cfg, kind in rows:
        if not want(f"{prec}gemm {ta}{tb} {m}x{n}x{k}"):
            continue
        dtype = np.float64 if prec == "d" else np.float32
        es = 8 if prec == "d" else 4
        _, (dA, dB, dC) = device_operands(torch, np, si, dtype, ta, tb, m, n, k, lda, ldb, ldc, cfg, kind)
        f = xg.xgemm_dgemm if prec == "d" else xg.xgemm_sgemm

        def step():
            rc = f(ta, tb, m, n, k, alpha, dA, lda, dB, ldb, beta, dC, ldc)
            if rc:
                raise RuntimeError(rc)

        flops = 2.0 * m * n * k
        # the device clocks down while the host prepares the next operands:
        # warm up for about 0.2 s of device time before timing a short kernel
        est = max(flops / 60e12, 20e-6)
        steps = max(5, min(200, int(0.1 / est)))
        wall, dev = time_calls(torch, step, steps, max(3, min(400, int(0.2 / est))))
        peak = PEAK_TFLOPS["f64" if prec == "d" else "f32"] * 1e12
        bytes_alg = es * (m * k + k * n + m * n * (2 if beta != 0 else 1))
        bound = min(peak, flops / bytes_alg * HBM_TBPS * 1e12)
        print(json.dumps({"shape": f"{prec}gemm {ta}{tb} {m}x{n}x{k}", "kernel": xg.xgemm_last_kernel_name(),
                          "ms": round(dev * 1e3, 4), "GFLOP/s": round(flops / dev / 1e9, 1),
                          "frac_of_mfma_peak": round(flops / dev / peak, 4),
                          "frac_of_min_mfma_hbm_bound": round(flops / dev / bound, 4),
                          "GB/s_algorithmic": round(bytes_alg / dev / 1e9, 1)}), file=sys.stderr, flush=True)
        del dA, dB, dC
    # the same products on packed operands (pack once, multiply many times): the product alone, and the two
    # packing passes as the HBM traffic they are (read once, written once)
    packed = [("d", "N", "N", 8192, 8192, 8192), ("d", "T", "N", 7001, 7001, 7001), ("d", "N", "N", 16384, 16384, 128),
              ("d", "N", "N", 4096, 4096, 4096), ("s", "N", "N", 8192, 8192, 8192), ("s", "N", "N", 4096, 4096, 4096)]
    for prec, ta, tb, m, n, k in packed:
        if not want(f"{prec}gemm_packed {ta}{tb} {m}x{n}x{k}"):
            continue
        dtype = np.float64 if prec == "d" else np.float32
        tdt = torch.float64 if prec == "d" else torch.float32
        es = 8 if prec == "d" else 4
        ra, rb = (m if ta == "N" else k), (k if tb == "N" else n)
        _, (dA, dB, dC) = device_operands(torch, np, si, dtype, ta, tb, m, n, k, ra, rb, m, 2)
        Ap = torch.empty(xg.xgemm_pack_elems(m, k), dtype=tdt, device="cuda")
        Bp = torch.empty(xg.xgemm_pack_elems(n, k), dtype=tdt, device="cuda")
        pa, pb = getattr(xg, f"xgemm_{prec}pack_a"), getattr(xg, f"xgemm_{prec}pack_b")
        fp, f = getattr(xg, f"xgemm_{prec}gemm_packed"), getattr(xg, f"xgemm_{prec}gemm")
        peak = PEAK_TFLOPS["f64" if prec == "d" else "f32"] * 1e12
        flops = 2.0 * m * n * k

        def check(rc):
            if rc:
                raise RuntimeError(rc)

        est = max(flops / 60e12, 20e-6)
        steps, warm = max(5, min(200, int(0.1 / est))), max(3, min(400, int(0.2 / est)))
        _, t_pa = time_calls(torch, lambda: check(pa(ta, m, k, dA, ra, Ap)), 10, 3)
        _, t_pb = time_calls(torch, lambda: check(pb(tb, k, n, dB, rb, Bp)), 10, 3)
        _, t_plain = time_calls(torch, lambda: check(f(ta, tb, m, n, k, 1.5, dA, ra, dB, rb, -0.5, dC, m)), steps, warm)
        k_plain = xg.xgemm_last_kernel_name()
        _, t_pack = time_calls(torch, lambda: check(fp(m, n, k, 1.5, Ap, Bp, -0.5, dC, m)), steps, warm)
        print(json.dumps({"shape": f"{prec}gemm_packed {ta}{tb} {m}x{n}x{k}", "kernel": xg.xgemm_last_kernel_name(),
                          "ms": round(t_pack * 1e3, 4), "GFLOP/s": round(flops / t_pack / 1e9, 1),
                          "frac_of_mfma_peak": round(flops / t_pack / peak, 4),
                          "plain_ms": round(t_plain * 1e3, 4), "plain_kernel": k_plain,
                          "pack_a_ms": round(t_pa * 1e3, 4), "pack_b_ms": round(t_pb * 1e3, 4),
                          "pack_a_GB/s": round(2.0 * es * m * k / t_pa / 1e9, 1),
                          "pack_b_GB/s": round(2.0 * es * n * k / t_pb / 1e9, 1)}), file=sys.stderr, flush=True)
        del dA, dB, dC, Ap, Bp
    # beyond the configurations: symmetric rank-k updates (n (n + 1) k flops) and
    # shapes whose last round of tiles is nearly empty, plain and with a workspace
    lw = xg.xgemm_workspace_bytes()
    work = torch.zeros(lw, dtype=torch.uint8, device="cuda")
    extra = [("syrk", "d", 8192, 8192, 8192), ("syrk", "d", 16384, 16384, 16384), ("syrk", "d", 4096, 4096, 4096),
             ("syrk", "s", 8192, 8192, 8192), ("syrk", "s", 16384, 16384, 16384),
             ("gemm", "d", 3328, 2560, 2048), ("gemm", "d", 3072, 3072, 3072), ("gemm", "d", 512, 512, 8192),
             ("gemm", "d", 1024, 1024, 1024), ("gemm", "d", 2048, 2048, 2048),
             ("gemm", "s", 3328, 2560, 2048)]
    for op, prec, m, n, k in extra:
        if not (want(f"{prec}{op} {m}x{n}x{k}") or want(f"{prec}{op}_ws {m}x{n}x{k}")):
            continue
        dtype = np.float64 if prec == "d" else np.float32
        ld = si.padded_ld(m)
        _, (dA, dB, dC) = device_operands(torch, np, si, dtype, "N", "T", m, n, k, ld, si.padded_ld(n), ld, 6)
        flops = float(m) * (m + 1) * k if op == "syrk" else 2.0 * m * n * k
        peak = PEAK_TFLOPS["f64" if prec == "d" else "f32"] * 1e12
        for use_ws in (False, True):
            if not want(f"{prec}{op}{'_ws' if use_ws else ''} {m}x{n}x{k}"):
                continue
            if op == "syrk":
                f = getattr(xg, f"xgemm_{prec}syrk_ws")
                call = lambda: f("L", "N", m, k, 1.5, dA, ld, -0.5, dC, ld, work if use_ws else None, lw if use_ws else 0)
            else:
                f = getattr(xg, f"xgemm_{prec}gemm_ws")
                call = lambda: f("N", "T", m, n, k, 1.5, dA, ld, dB, si.padded_ld(n), -0.5, dC, ld,
                                 work if use_ws else None, lw if use_ws else 0)

            def step():
                rc = call()
                if rc:
                    raise RuntimeError(rc)

            est = max(flops / 60e12, 20e-6)
            steps = max(5, min(200, int(0.1 / est)))
            wall, dev = time_calls(torch, step, steps, max(3, min(400, int(0.2 / est))))
            print(json.dumps({"shape": f"{prec}{op}{'_ws' if use_ws else ''} {m}x{n}x{k}",
                              "kernel": xg.xgemm_last_kernel_name(), "pieces": xg.xgemm_last_split(),
                              "ms": round(dev * 1e3, 4), "GFLOP/s": round(flops / dev / 1e9, 1),
                              "frac_of_mfma_peak": round(flops / dev / peak, 4)}), file=sys.stderr, flush=True)
        del dA, dB, dC
    # triangular solves and products (m^2 n flops for side L) and Cholesky factorisations (n^3 / 3):
    # the matrix that is overwritten is restored before every timed call
    def timed_in_place(restore, call, reps=8, skip=3):
        times = []
        for it in range(reps):
            restore()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            rc = call()
            e1.record()
            torch.cuda.synchronize()
            if rc:
                raise RuntimeError(rc)
            if it >= skip:
                times.append(e0.elapsed_time(e1) * 1e-3)
        return sum(times) / len(times)

    for op, prec, side, uplo, trans, msz in (("trsm", "d", "L", "L", "N", 8192), ("trsm", "d", "R", "U", "T", 8192),
                                             ("trsm", "d", "L", "L", "N", 16384), ("trsm", "d", "L", "L", "N", 4096),
                                             ("trsm", "s", "L", "L", "N", 8192), ("trmm", "d", "L", "L", "N", 8192),
                                             ("trmm", "d", "L", "L", "N", 16384)):
        if not want(f"{prec}{op} {side}{uplo}{trans}N {msz}x{msz}"):
            continue
        dtype = np.float64 if prec == "d" else np.float32
        ld = si.padded_ld(msz)
        rng = si.rng_for(7, msz)
        dT = torch.from_numpy(si.triangular(rng, msz, ld, dtype, uplo, False, sentinel=0.0)).cuda()
        dB0 = torch.from_numpy(si.uniform(rng, msz, msz, ld, dtype, sentinel=0.0)).cuda()
        dB = dB0.clone()
        f = getattr(xg, f"xgemm_{prec}{op}")
        dev = timed_in_place(lambda: dB.copy_(dB0), lambda: f(side, uplo, trans, "N", msz, msz, 1.0, dT, ld, dB, ld))
        flops = float(msz) ** 3
        peak = PEAK_TFLOPS["f64" if prec == "d" else "f32"] * 1e12
        print(json.dumps({"shape": f"{prec}{op} {side}{uplo}{trans}N {msz}x{msz}", "ms": round(dev * 1e3, 4),
                          "GFLOP/s": round(flops / dev / 1e9, 1), "frac_of_mfma_peak": round(flops / dev / peak, 4)}),
              file=sys.stderr, flush=True)
        del dT, dB0, dB
    # the two remaining real level-3 routines: symmetric product (2 m^2 n flops) and rank-2k update (2 n (n + 1) k)
    for op, prec, nsz in (("symm", "d", 8192), ("symm", "d", 16384), ("syr2k", "d", 8192), ("symm", "s", 8192),
                          ("syr2k", "s", 8192)):
        if not want(f"{prec}{op} {nsz}"):
            continue
        dtype = np.float64 if prec == "d" else np.float32
        ld = si.padded_ld(nsz)
        rng = si.rng_for(9, nsz)
        dX, dY, dZ = (torch.from_numpy(si.uniform(rng, nsz, nsz, ld, dtype, sentinel=0.0)).cuda() for _ in range(3))
        f = getattr(xg, f"xgemm_{prec}{op}")
        if op == "symm":
            call = lambda: f("L", "L", nsz, nsz, 1.5, dX, ld, dY, ld, -0.5, dZ, ld)
            flops = 2.0 * float(nsz) ** 3
        else:
            call = lambda: f("L", "N", nsz, nsz, 1.5, dX, ld, dY, ld, -0.5, dZ, ld)
            flops = 2.0 * float(nsz) * (nsz + 1) * nsz

        def step():
            rc = call()
            if rc:
                raise RuntimeError(rc)

        wall, dev = time_calls(torch, step, 5, 3)
        peak = PEAK_TFLOPS["f64" if prec == "d" else "f32"] * 1e12
        print(json.dumps({"shape": f"{prec}{op} {nsz}", "ms": round(dev * 1e3, 4), "GFLOP/s": round(flops / dev / 1e9, 1),
                          "frac_of_mfma_peak": round(flops / dev / peak, 4)}), file=sys.stderr, flush=True)
        del dX, dY, dZ
    for prec, uplo, nsz in (("d", "L", 8192), ("d", "L", 16384), ("d", "L", 32768), ("s", "L", 16384)):
        if not want(f"{prec}potrf {uplo} {nsz}"):
            continue
        dtype = np.float64 if prec == "d" else np.float32
        ld = si.padded_ld(nsz)
        dA0 = torch.from_numpy(si.spd(si.rng_for(8, nsz), nsz, ld, dtype, uplo, sentinel=0.0)).cuda()
        dA = dA0.clone()
        dinfo = torch.zeros(1, dtype=torch.int32, device="cuda")
        f = getattr(xg, f"xgemm_{prec}potrf")
        dev = timed_in_place(lambda: dA.copy_(dA0), lambda: f(uplo, nsz, dA, ld, dinfo), reps=5, skip=2)
        if int(dinfo.item()) != 0:
            raise RuntimeError("potrf info %d" % int(dinfo.item()))
        flops = float(nsz) ** 3 / 3.0
        peak = PEAK_TFLOPS["f64" if prec == "d" else "f32"] * 1e12
        print(json.dumps({"shape": f"{prec}potrf {uplo} {nsz}", "ms": round(dev * 1e3, 4),
                          "GFLOP/s": round(flops / dev / 1e9, 1), "frac_of_mfma_peak": round(flops / dev / peak, 4)}),
              file=sys.stderr, flush=True)
        del dA0, dA
    # LU: xgemm_*getrf (base panels shared by all the workgroups their rows need, through the library's own
    # exchange buffer), the same through a caller's buffer (xgemm_*getrf_ws), and held to the leaves of one
    # workgroup each (what a captured call without a buffer gets)
    for prec, nsz, ws in (("d", 4096, 0), ("d", 8192, 0), ("d", 16384, 0), ("d", 32768, 0), ("s", 8192, 0), ("s", 16384, 0), ("s", 32768, 0),
                          ("d", 8192, 1), ("d", 16384, 1), ("s", 8192, 1),
                          ("d", 4096, 2), ("d", 8192, 2), ("d", 16384, 2), ("s", 8192, 2)):
        name = f"{prec}getrf{('', '_ws', ' (leaves only)')[ws]} {nsz}"
        if not want(name):
            continue
        dtype = np.float64 if prec == "d" else np.float32
        ld = si.padded_ld(nsz)
        dA0 = torch.from_numpy(si.uniform(si.rng_for(9, nsz), nsz, nsz, ld, dtype, sentinel=0.0)).cuda()
        dA = dA0.clone()
        dinfo = torch.zeros(1, dtype=torch.int32, device="cuda")
        dpiv = torch.zeros(nsz, dtype=torch.int32, device="cuda")
        xg.xgemm_force_getrf_shared(0 if ws == 2 else -1)
        if ws == 1:
            lwork = xg.xgemm_getrf_workspace_bytes()
            work = torch.empty(lwork, dtype=torch.uint8, device="cuda")
            fw = getattr(xg, f"xgemm_{prec}getrf_ws")
            step = lambda: fw(nsz, nsz, dA, ld, dpiv, dinfo, work, lwork)
        else:
            f = getattr(xg, f"xgemm_{prec}getrf")
            step = lambda: f(nsz, nsz, dA, ld, dpiv, dinfo)
        dev = timed_in_place(lambda: dA.copy_(dA0), step, reps=4, skip=1)
        xg.xgemm_force_getrf_shared(-1)
        if int(dinfo.item()) != 0:
            raise RuntimeError("getrf info %d" % int(dinfo.item()))
        flops = 2.0 * float(nsz) ** 3 / 3.0
        peak = PEAK_TFLOPS["f64" if prec == "d" else "f32"] * 1e12
        print(json.dumps({"shape": name, "ms": round(dev * 1e3, 4),
                          "GFLOP/s": round(flops / dev / 1e9, 1), "frac_of_mfma_peak": round(flops / dev / peak, 4)}),
              file=sys.stderr, flush=True)
        del dA0, dA
    if not want("zgemm"):
        return
    # zgemm 4096^3 on split planes: four real launches, 8 m n k flops
    nsz = 4096
    rng = si.rng_for(5, nsz)
    planes = [torch.from_numpy(si.uniform(rng, nsz, nsz)).cuda() for _ in range(6)]

    def zstep():
        rc = xg.xgemm_zgemm_split("N", "N", nsz, nsz, nsz, (1.0, 0.0), planes[0], planes[1], nsz, planes[2],
                                  planes[3], nsz, (0.0, 0.0), planes[4], planes[5], nsz, None, 0)
        if rc:
            raise RuntimeError(rc)

    wall, dev = time_calls(torch, zstep, 10, 5)
    flops = 8.0 * nsz ** 3
    print(json.dumps({"shape": f"zgemm(4m) NN {nsz}^3", "ms": round(dev * 1e3, 4),
                      "GFLOP/s": round(flops / dev / 1e9, 1),
                      "frac_of_mfma_peak": round(flops / dev / (PEAK_TFLOPS['f64'] * 1e12), 4)}),
          file=sys.stderr, flush=True)
    del planes
    # the same product on interleaved storage: split into planes, real GEMMs, merge (4m and 3m), and the fused
    # form (two packing passes and one real product of twice the rows and depth, written straight into C)
    zs = [torch.from_numpy(si.uniform(rng, 2 * nsz, nsz)).cuda() for _ in range(3)]
    for method, name in ((0, "4m"), (1, "3m"), (2, "fused")):
        lw = xg.xgemm_zgemm_workbytes(nsz, nsz, nsz, method)
        zwork = torch.empty(lw, dtype=torch.uint8, device="cuda")

        def zistep():
            rc = xg.xgemm_zgemm("N", "N", nsz, nsz, nsz, (1.0, 0.0), zs[0], nsz, zs[1], nsz, (0.0, 0.0), zs[2], nsz,
                                method, zwork, lw)
            if rc:
                raise RuntimeError(rc)

        wall, dev = time_calls(torch, zistep, 10, 5)
        own = 6.0 * nsz ** 3 if method == 1 else flops           # what the method itself computes: 3 real products, or 4 (one launch when fused)
        print(json.dumps({"shape": f"zgemm interleaved ({name}) NN {nsz}^3", "ms": round(dev * 1e3, 4),
                          "GFLOP/s": round(own / dev / 1e9, 1),
                          "frac_of_mfma_peak": round(own / dev / (PEAK_TFLOPS['f64'] * 1e12), 4),
                          "flops_counted": "6mnk (three real products)" if method == 1 else "8mnk",
                          "GFLOP/s_as_8mnk": round(flops / dev / 1e9, 1)}),
              file=sys.stderr, flush=True)
        del zwork


if __name__ == "__main__":
    main()
