#!/usr/bin/env python3
"""Benchmark of the GOOM prefix scan on one MI355X.

One "step" is one whole inclusive prefix scan (all three phases: chunk products, carry
chain, fix-up with every output stored) of the long-chain workload: T = 1,048,576 real
64 x 64 matrices with i.i.d. N(0, 1) entries, given as complex64 GOOMs already resident
in HBM; 34 GB in, 34 GB out.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--T N] [--d N] [--chunk-len N]

Everything runs on one GPU; --gpus above 1 is refused.
"""
import argparse
import json
import sys
import time

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix rate, published
MFMA_F64_PEAK_TFLOPS = 78.6    # MI355X dense fp64 matrix rate, published


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--T", type=int, default=1 << 20)
    ap.add_argument("--d", type=int, default=64)
    ap.add_argument("--chunk-len", type=int, default=0)
    ap.add_argument("--cpu-sample-steps", type=int, default=16384,
                    help="leading steps of the chain the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel from rocprofv3 --pmc runs (default: looked up in "
                         "the counter summaries under profiles/ for this kernel and workload, null when there is none)")
    ap.add_argument("--no-extras", action="store_true", help="time the headline scan only")
    ap.add_argument("--only", choices=["tiny", "between", "scan128", "complex128", "lmme", "lyapunov", "recurrence", "large", "backward"], default=None,
                    help="time just one of the other workloads (for profiler runs) and print its figures")
    ap.add_argument("--basic-extras", action="store_true",
                    help="besides the scan, time only a plain device copy of the same size (for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_03426_amd import Goom

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    T, d = args.T, args.d
    dev = torch.device("cuda", 0)
    g = Goom(0)

    if args.only:
        print(json.dumps({"other_workloads": other_workloads(g, torch, dev, args.only)}), flush=True)
        return

    # ---- synthetic input: N(0,1) reals drawn on the device, encoded by the library's codec
    gen = torch.Generator(device=dev)
    gen.manual_seed(251003426 * 10 + 2)
    z = torch.empty((T, d, d), dtype=torch.complex64, device=dev)
    blk = max(1, (1 << 28) // (d * d))
    t_codec = 0.0
    for t0 in range(0, T, blk):
        t1 = min(T, t0 + blk)
        x = torch.randn((t1 - t0, d, d), dtype=torch.float32, device=dev, generator=gen)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        g.to_goom(x, out=z[t0:t1])
        torch.cuda.synchronize()
        t_codec += time.perf_counter() - c0
        del x
    out = torch.empty((T, d, d), dtype=torch.complex64, device=dev)
    print(f"# input ready: {z.numel() * 8 / 1e9:.2f} GB of GOOMs; to_goom ran at "
          f"{z.numel() * 12 / t_codec / 1e9:.0f} GB/s", file=sys.stderr, flush=True)

    def step():
        g.scan(z, chunk_len=args.chunk_len, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # every step bracketed by events on the stream the library launches on (the context's stream is torch's current one)
    stream = torch.cuda.current_stream(dev)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    step_ms = sorted(a.elapsed_time(b) for a, b in ev)
    ms_median = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    products_per_s = T / (ms_per_step * 1e-3)

    # ---- per-kernel durations from HIP events on the library's stream
    g.profile_enable(True)
    kern = {}
    nprof = max(1, min(args.steps, 5))
    for _ in range(nprof):
        step()
        per_call = {}
        for label, ms in g.profile_records():  # a phase may be several launches: add them up
            per_call[label] = per_call.get(label, 0.0) + ms
        for label, ms in per_call.items():
            kern.setdefault(label, []).append(ms)
    g.profile_enable(False)
    kern_avg = {k: sum(v) / len(v) for k, v in kern.items()}
    dominant = max(kern_avg, key=kern_avg.get)
    # algorithmic bytes of the fix-up kernel: every matrix read once (complex64) and every
    # prefix written once (complex64): 2 * 8 * d * d bytes per product
    if dominant.endswith("fixup_outputs") or dominant == "scan_single_chunk":
        alg_bytes = T * 2 * 8 * d * d
    else:
        alg_bytes = T * 8 * d * d
    achieved_gbs = alg_bytes / (kern_avg[dominant] * 1e-3) / 1e9
    # HBM bytes per launch of that kernel as the FETCH_SIZE / WRITE_SIZE counters measured them in separate
    # rocprofv3 --pmc runs of this command: looked up in the tracked counter summaries (profiles/), by kernel and
    # workload; null when no summary covers this run
    traffic, traffic_source = args.traffic_bytes, "--traffic-bytes" if args.traffic_bytes is not None else None
    if traffic is None:
        traffic, traffic_source = traffic_from_profiles(dominant, T, d, args.chunk_len)
    roofline = {
        "bound": "hbm", "kernel": dominant, "achieved": round(achieved_gbs, 1), "peak": HBM_PEAK_GBS,
        "unit": "GB/s", "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
        "traffic": traffic, "traffic_source": traffic_source, "algorithmic_bytes_per_launch": alg_bytes,
        "avg_launch_ms": round(kern_avg[dominant], 4),
    }
    # matrix-core work actually executed: one d^3 product per matrix in phase 1, one per chunk in
    # phase 2, one per matrix in phase 3
    flops_exec = 2.0 * d ** 3 * (2 * T)
    lmme_tflops = flops_exec / (ms_per_step * 1e-3) / 1e12
    phase_tflops = {k: round(2.0 * d ** 3 * T / (v * 1e-3) / 1e12, 2) for k, v in kern_avg.items()
                    if "phase1" in k or "phase3" in k}

    result = {
        "metric": "d\u00d7d GOOM matrix products scanned/sec; LMME TFLOP/s as % of MFMA peak",
        "value": round(products_per_s, 1), "unit": "products/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_events": {"median": round(ms_median, 4), "mean": round(sum(step_ms) / len(step_ms), 4),
                               "min": round(step_ms[0], 4), "max": round(step_ms[-1], 4)},
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"prefix scan of T={T} real {d}x{d} N(0,1) matrices as complex64 GOOMs, "
                               f"in HBM, {T * d * d * 8 / 1e9:.1f} GB in and out",
                   "T": T, "d": d, "chunk_len": args.chunk_len},
        "lmme": {"tflops_executed": round(lmme_tflops, 2), "tflops_useful": round(lmme_tflops / 2, 2),
                 "pct_of_fp32_mfma_peak": round(100 * lmme_tflops / MFMA_F32_PEAK_TFLOPS, 2),
                 "per_phase_tflops": phase_tflops},
        "kernels_ms": {k: round(v, 4) for k, v in kern_avg.items()},
        "roofline": roofline,
    }

    # ---- extras: the reduction variant (final product only), same input
    if not args.no_extras and not args.basic_extras:
        fin = torch.empty((d, d), dtype=torch.complex64, device=dev)
        g.reduce(z, chunk_len=args.chunk_len, out=fin)
        torch.cuda.synchronize()
        r0 = time.perf_counter()
        for _ in range(3):
            g.reduce(z, chunk_len=args.chunk_len, out=fin)
        torch.cuda.synchronize()
        rms = (time.perf_counter() - r0) / 3 * 1e3
        result["reduce"] = {"ms": round(rms, 4), "products_per_s": round(T / (rms * 1e-3), 1),
                            "hbm_gbs": round(T * 8 * d * d / (rms * 1e-3) / 1e9, 1),
                            # every product of a reduction is needed: executed and useful flops coincide
                            "lmme_tflops": round(2.0 * d ** 3 * T / (rms * 1e-3) / 1e12, 2),
                            "pct_of_fp32_mfma_peak": round(2.0 * d ** 3 * T / (rms * 1e-3) / 157.3e12 * 100, 2)}
    if not args.no_extras and not args.basic_extras and d in (32, 64, 128):
        # the same scan fed with the real matrices themselves (4 bytes per entry in instead of 8; an extra of
        # the library, not the configuration `value` is quoted on)
        gen.manual_seed(251003426 * 10 + 2)
        xr = torch.empty((T, d, d), dtype=torch.float32, device=dev)
        for t0 in range(0, T, blk):
            t1 = min(T, t0 + blk)
            xr[t0:t1] = torch.randn((t1 - t0, d, d), dtype=torch.float32, device=dev, generator=gen)
        xsec = timed(torch, lambda: g.scan_real(xr, chunk_len=args.chunk_len, out=out), 3)
        result["scan_of_real_matrices"] = {"ms": round(xsec * 1e3, 4), "products_per_s": round(T / xsec, 1),
                                           "lmme_tflops_executed": round(2.0 * d ** 3 * 2 * T / xsec / 1e12, 2),
                                           "pct_of_fp32_mfma_peak": round(100 * 2.0 * d ** 3 * 2 * T / xsec / 1e12 / MFMA_F32_PEAK_TFLOPS, 2),
                                           "kernels_ms": kernel_times(g, lambda: g.scan_real(xr, chunk_len=args.chunk_len, out=out))}
        del xr
    if not args.no_extras:
        result["to_goom_gbs"] = round(z.numel() * 12 / t_codec / 1e9, 1)
        # the decoder on the first 2^28 inputs (log-magnitudes of N(0,1) draws, all inside float range)
        zc = z.reshape(-1)[: 1 << 28]
        xs = torch.empty(zc.numel(), dtype=torch.float32, device=dev)
        dsec = timed(torch, lambda: g.from_goom(zc, out=xs), 3)
        result["from_goom_gbs"] = round(zc.numel() * 12 / dsec / 1e9, 1)
        del xs
        # what this machine's HBM sustains for a plain device-to-device copy of the same size
        # (read + write bytes over time): the practical ceiling beside the published 8 TB/s
        out.copy_(z)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(3):
            out.copy_(z)
        torch.cuda.synchronize()
        cms = (time.perf_counter() - c0) / 3
        result["hbm_copy_gbs"] = round(2 * z.numel() * 8 / cms / 1e9, 1)
        # the same from the library's own streaming probes (read only, write only, copy): reading alone is
        # the ceiling for phase 1, which writes next to nothing
        for name, mode in (("hbm_read_gbs", 0), ("hbm_write_gbs", 1), ("hbm_probe_copy_gbs", 2)):
            psec = timed(torch, lambda: g.probe_bandwidth(z, out, mode), 3)
            result[name] = round((2 if mode == 2 else 1) * z.numel() * 8 / psec / 1e9, 1)
        # what the float matrix units sustain on this machine for a plain library GEMM (8192^3, float32)
        ga = torch.randn((8192, 8192), device=dev)
        gb = torch.randn((8192, 8192), device=dev)
        gsec = timed(torch, lambda: torch.mm(ga, gb), 5)
        result["sgemm_tflops_measured"] = round(2 * 8192.0 ** 3 / gsec / 1e12, 1)
        del ga, gb
        # and for a kernel that issues nothing but 16 x 16 x 4 matrix instructions (the library's probe)
        sink = torch.zeros(4, device=dev)
        for name, dbl in (("mfma_f32_tflops_measured", False), ("mfma_f64_tflops_measured", True)):
            its = 4096
            msec = timed(torch, lambda: g.probe_matrix_unit(sink, its, dbl), 3)
            result[name] = round(g.PROBE_MATRIX_FLOP_PER_ITER * its / msec / 1e12, 1)

    # ---- the other workloads of the same path, each timed on its own (not part of `value`)
    if not args.no_extras and not args.basic_extras:
        del out
        torch.cuda.empty_cache()
        result["other_workloads"] = other_workloads(g, torch, dev)

    # ---- CPU oracle on a bounded sample of the same workload (reported, not a target)
    if args.cpu_sample_steps > 0:
        from oracle import goom_oracle as oracle
        S = min(T, args.cpu_sample_steps)
        zs = z[:S].cpu().numpy()
        c0 = time.perf_counter()
        re, sg, kap = oracle.scan(zs, return_kappa=True)
        cpu_s = time.perf_counter() - c0
        result["cpu_baseline"] = {
            "value": round(S / cpu_s, 2), "unit": "products/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {S} steps of the same chain (definitional log-sum-exp scan in double), {cpu_s:.1f} s",
        }
        # the GPU result on the sampled prefix must agree with the oracle: every entry whose sum the oracle finds well conditioned
        # (cancellation factor of the last row-by-column sum at most 2^9, as in the parity tests) within 1e-4 relative or 1e-3
        got = g.scan(z[:S]).cpu().numpy()
        finite = np.isfinite(re)
        well = finite & (kap <= 2.0 ** 9)
        err = np.abs(got.real.astype(np.float64) - re)
        tol = np.maximum(1e-3, 1e-4 * np.abs(re))
        result["cpu_baseline"]["ill_conditioned_fraction"] = round(float(1.0 - well.mean()), 6)
        result["cpu_baseline"]["gpu_well_conditioned_entries_within_tolerance"] = round(float(np.mean(err[well] <= tol[well])), 9)
        err, tol = err[finite], tol[finite]
        result["cpu_baseline"]["gpu_entries_within_tolerance"] = round(float(np.mean(err <= tol)), 6)  # ill-conditioned ones included

    print(json.dumps(result), flush=True)


def traffic_from_profiles(kernel_label, T, d, chunk_len):
    """HBM bytes per launch of a kernel from the counter summaries under profiles/: lines of the form
    'traffic_bytes_per_launch kernel=<label> T=<T> d=<d> chunk_len=<L> bytes=<N>'.  Returns (bytes, source) or (None, None)."""
    import glob
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    for path in sorted(glob.glob(os.path.join(here, "profiles", "*.txt"))):
        with open(path) as f:
            for line in f:
                if not line.startswith("traffic_bytes_per_launch "):
                    continue
                kv = dict(item.split("=", 1) for item in line.split()[1:])
                if (kv.get("kernel") == kernel_label and int(kv.get("T", -1)) == T and int(kv.get("d", -1)) == d
                        and int(kv.get("chunk_len", -1)) == chunk_len):
                    return int(kv["bytes"]), ("profiles/" + os.path.basename(path) + ": rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, "
                                              "each scaled by what the same counter reads for a plain copy of known size")
    return None, None


def timed(torch, fn, reps=3):
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def kernel_times(g, fn):
    g.profile_enable(True)
    fn()
    per = {}
    for label, ms in g.profile_records():
        per[label] = round(per.get(label, 0.0) + ms, 4)
    g.profile_enable(False)
    return per


def other_workloads(g, torch, dev, only=None):
    """Scan of 128 x 128 matrices, batched LMME, Lyapunov spectrum, non-diagonal recurrence, tiny scan."""
    import synthetic_inputs as si
    res = {}
    want = lambda name: only is None or only == name
    if want("tiny"):
        res["scan_T256_d8"] = tiny_scan(g, torch, dev, si)
        res.update(small_scans(g, torch, dev, si))
    if want("between"):
        res.update(scans_between_tiles(g, torch, dev, si))
    if want("scan128"):
        res.update(scan128(g, torch, dev, si))
    if want("complex128"):
        res.update(scans_complex128(g, torch, dev, si))
    if want("lmme"):
        res.update(batched_lmme(g, torch, dev, si))
    if want("lyapunov"):
        res.update(lyapunov(g, torch, dev, si))
    if want("recurrence"):
        res.update(recurrence(g, torch, dev, si))
    if want("large"):
        res.update(large_matrices(g, torch, dev, si))
    if want("backward"):
        res.update(scan_backward(g, torch, dev, si))
    return res


def scan_backward(g, torch, dev, si):
    # backward pass of a scan of 64 x 64 matrices, T = 65,536: gradients with respect to every factor's log-magnitudes
    res = {}
    T, d = 1 << 16, 64
    z = torch.empty((T, d, d), dtype=torch.complex64, device=dev)
    for t0, x in si.device_normal_blocks(251003426 * 10 + 6, T, (d, d), dev, 1 << 14):
        g.to_goom(x, out=z[t0:t0 + x.shape[0]])
    p = g.scan(z)
    gp = torch.randn((T, d, d), device=dev, generator=si.device_generator(251003426 * 10 + 7, dev))
    fwd = timed(torch, lambda: g.scan(z, out=p))
    sec = timed(torch, lambda: g.scan_backward(z, p, gp))
    res["scan_backward_T65536_d64"] = {
        "ms": round(sec * 1e3, 3), "forward_ms": round(fwd * 1e3, 3), "products_per_s": round(T / sec, 1),
        "kernels_ms": kernel_times(g, lambda: g.scan_backward(z, p, gp))}
    del z, p, gp
    torch.cuda.empty_cache()
    return res


def tiny_scan(g, torch, dev, si):
    # tiny scan (T = 256, d = 8): latency of one call
    zt = g.to_goom(torch.randn((256, 8, 8), device=dev, generator=si.device_generator(11, dev)))
    return {"us_per_scan": round(timed(torch, lambda: g.scan(zt), 50) * 1e6, 1)}


def small_scans(g, torch, dev, si):
    # long chains of the smallest matrices (T = 2^22 of 8 x 8 and 16 x 16): bound by HBM, if anything
    res = {}
    for d in (8, 16):
        T = 1 << 22
        z = g.to_goom(torch.randn((T, d, d), device=dev, generator=si.device_generator(251003426 * 10 + 80 + d, dev)))
        out = torch.empty_like(z)
        sec = timed(torch, lambda: g.scan(z, out=out), 5)
        byts = 3 * z.numel() * 8  # read, read, write
        res[f"scan_T{T}_d{d}"] = {"ms": round(sec * 1e3, 3), "products_per_s": round(T / sec, 1),
                                  "hbm_gbs_algorithmic": round(byts / sec / 1e9, 1),
                                  "pct_of_hbm_peak": round(100 * byts / sec / 1e9 / HBM_PEAK_GBS, 2),
                                  "kernels_ms": kernel_times(g, lambda: g.scan(z, out=out))}
        del z, out
    return res


def scans_between_tiles(g, torch, dev, si):
    # sizes that are not a tile size (the hot kernel with the padding left out of the product): 48 x 48 and 96 x 96
    res = {}
    for d, T in ((48, 1 << 19), (96, 1 << 17)):
        z = g.to_goom(torch.randn((T, d, d), device=dev, generator=si.device_generator(251003426 * 10 + 90 + d, dev)))
        out = torch.empty_like(z)
        sec = timed(torch, lambda: g.scan(z, out=out), 5)
        byts = 3 * z.numel() * 8  # read, read, write
        fl = 2.0 * d ** 3 * 2 * T
        res[f"scan_T{T}_d{d}"] = {"ms": round(sec * 1e3, 3), "products_per_s": round(T / sec, 1),
                                  "hbm_gbs_algorithmic": round(byts / sec / 1e9, 1),
                                  "lmme_tflops_executed": round(fl / sec / 1e12, 2),
                                  "kernels_ms": kernel_times(g, lambda: g.scan(z, out=out))}
        del z, out
    return res


def scans_complex128(g, torch, dev, si):
    # chains of complex128 GOOMs (double components, fp64 matrix instruction): 8.6 GB of matrices each
    res = {}
    for d, T in ((32, 1 << 19), (64, 1 << 18), (128, 1 << 16)):
        z = g.to_goom(torch.randn((T, d, d), device=dev, dtype=torch.float64, generator=si.device_generator(251003426 * 10 + 100 + d, dev)))
        out = torch.empty_like(z)
        sec = timed(torch, lambda: g.scan(z, out=out), 3)
        byts = 3 * z.numel() * 16  # read, read, write
        fl = 2.0 * d ** 3 * 2 * T
        res[f"scan_T{T}_d{d}_complex128"] = {"ms": round(sec * 1e3, 3), "products_per_s": round(T / sec, 1),
                                             "hbm_gbs_algorithmic": round(byts / sec / 1e9, 1),
                                             "lmme_tflops_executed": round(fl / sec / 1e12, 2),
                                             "pct_of_fp64_mfma_peak": round(100 * fl / sec / 1e12 / MFMA_F64_PEAK_TFLOPS, 2),
                                             "kernels_ms": kernel_times(g, lambda: g.scan(z, out=out))}
        del z, out
        torch.cuda.empty_cache()
    return res


def scan128(g, torch, dev, si):
    # scan of 128 x 128 matrices, T = 262,144 (same bytes as the headline workload)
    res = {}
    T, d = 1 << 18, 128
    z = torch.empty((T, d, d), dtype=torch.complex64, device=dev)
    for t0, x in si.device_normal_blocks(251003426 * 10 + 3, T, (d, d), dev, 1 << 14):
        g.to_goom(x, out=z[t0:t0 + x.shape[0]])
    out = torch.empty_like(z)
    sec = timed(torch, lambda: g.scan(z, out=out))
    fl = 2.0 * d ** 3 * 2 * T
    res["scan_T262144_d128"] = {
        "ms": round(sec * 1e3, 3), "products_per_s": round(T / sec, 1),
        "lmme_tflops_executed": round(fl / sec / 1e12, 2),
        "pct_of_fp32_mfma_peak": round(100 * fl / sec / 1e12 / MFMA_F32_PEAK_TFLOPS, 2),
        "kernels_ms": kernel_times(g, lambda: g.scan(z, out=out))}
    del z, out
    torch.cuda.empty_cache()
    return res


def batched_lmme(g, torch, dev, si):
    # batched LMME: 8192 pairs of 128 x 128, log-magnitudes N(0, 200^2)
    from paper_2510_03426_amd import LMME_EXACT, LMME_FAST
    res = {}
    B, n = 8192, 128
    for ctype, name in ((torch.complex64, "c64"), (torch.complex128, "c128")):
        a = si.device_wide_range_gooms(251003426 * 10 + 31, (B, n, n), 200.0, ctype, dev)
        b = si.device_wide_range_gooms(251003426 * 10 + 32, (B, n, n), 200.0, ctype, dev)
        c = torch.empty_like(a)
        peak = MFMA_F32_PEAK_TFLOPS if name == "c64" else 78.6
        for flags, fname in ((LMME_FAST, "scaled_product"), (LMME_EXACT, "with_repair")):
            sec = timed(torch, lambda: g.lmme(a, b, flags=flags, out=c))
            res[f"lmme_{name}_{fname}"] = {
                "ms": round(sec * 1e3, 3), "pairs_per_s": round(B / sec, 1),
                "tflops": round(2.0 * n ** 3 * B / sec / 1e12, 2),
                "pct_of_mfma_peak": round(100 * 2.0 * n ** 3 * B / sec / 1e12 / peak, 2),
                "hbm_gbs": round(3 * a.numel() * a.element_size() / sec / 1e9, 1),
                "kernels_ms": kernel_times(g, lambda: g.lmme(a, b, flags=flags, out=c))}
        # benign range (entries N(0,1)): nothing to repair
        a = g.to_goom(torch.randn((B, n, n), device=dev, dtype=torch.float32 if name == "c64" else torch.float64))
        b = g.to_goom(torch.randn((B, n, n), device=dev, dtype=torch.float32 if name == "c64" else torch.float64))
        sec = timed(torch, lambda: g.lmme(a, b, flags=LMME_FAST, out=c))
        res[f"lmme_{name}_unit_normal"] = {
            "ms": round(sec * 1e3, 3), "tflops": round(2.0 * n ** 3 * B / sec / 1e12, 2),
            "pct_of_mfma_peak": round(100 * 2.0 * n ** 3 * B / sec / 1e12 / peak, 2),
            "hbm_gbs": round(3 * a.numel() * a.element_size() / sec / 1e9, 1)}
        # its backward pass: gradients with respect to both operands' log-magnitudes (two more products of the same size)
        g.lmme(a, b, flags=LMME_FAST, out=c)
        gc = torch.randn((B, n, n), device=dev, dtype=torch.float32 if name == "c64" else torch.float64)
        sec = timed(torch, lambda: g.lmme_backward(a, b, c, gc))
        res[f"lmme_{name}_unit_normal_backward"] = {
            "ms": round(sec * 1e3, 3), "tflops": round(2 * 2.0 * n ** 3 * B / sec / 1e12, 2),
            "hbm_gbs": round((3 * a.numel() * a.element_size() + 3 * gc.numel() * gc.element_size()) / sec / 1e9, 1),
            "kernels_ms": kernel_times(g, lambda: g.lmme_backward(a, b, c, gc))}
        del a, b, c, gc
        torch.cuda.empty_cache()
    # many rows against a small right operand: the input term of the state-space layer, bias_t = B u_t for all steps at once
    # (8192 heads x 1024 steps, d = 32)
    Bt, n, d = 8192, 1024, 32
    u = g.to_goom(torch.randn((Bt, n, d), device=dev))
    w = g.to_goom(torch.randn((Bt, d, d), device=dev))
    c = torch.empty((Bt, n, d), dtype=torch.complex64, device=dev)
    sec = timed(torch, lambda: g.lmme(u, w, flags=LMME_FAST, out=c))
    res["lmme_tall_8192x1024x32x32"] = {
        "ms": round(sec * 1e3, 3), "tflops": round(2.0 * n * d * d * Bt / sec / 1e12, 2),
        "hbm_gbs": round((u.numel() + w.numel() + c.numel()) * 8 / sec / 1e9, 1),
        "kernels_ms": kernel_times(g, lambda: g.lmme(u, w, flags=LMME_FAST, out=c))}
    del u, w, c
    torch.cuda.empty_cache()
    return res


def lyapunov(g, torch, dev, si):
    # Lyapunov spectrum of Lorenz-96 (d = 32) over T = 131,072 Jacobians, resets every 32 steps
    res = {}
    T, d = 131072, 32
    Jr, _ = si.lorenz96_jacobians(si.BASE_SEED + 4, T, d=d, burn_in=10000)
    Jz = g.to_goom(torch.from_numpy(Jr).to(dev))
    sec = timed(torch, lambda: g.lyapunov_spectrum(Jz, 0.01))
    lam = g.lyapunov_spectrum(Jz, 0.01).cpu().numpy()
    res["lyapunov_lorenz96_d32_T131072"] = {
        "ms": round(sec * 1e3, 3), "jacobians_per_s": round(T / sec, 1), "lambda_1": round(float(lam[0]), 4),
        "kernels_ms": kernel_times(g, lambda: g.lyapunov_spectrum(Jz, 0.01))}
    sec = timed(torch, lambda: g.lyapunov_spectrum(Jz, 0.01, chunk_len=64))
    res["lyapunov_lorenz96_d32_T131072_chunk64"] = {"ms": round(sec * 1e3, 3), "jacobians_per_s": round(T / sec, 1)}
    sec = timed(torch, lambda: g.lyapunov_spectrum_per_step(Jz, 0.01))
    res["lyapunov_per_step_qr_d32_T131072"] = {
        "ms": round(sec * 1e3, 3), "jacobians_per_s": round(T / sec, 1),
        "kernels_ms": kernel_times(g, lambda: g.lyapunov_spectrum_per_step(Jz, 0.01))}
    sec = timed(torch, lambda: g.largest_lyapunov(Jz, 0.01))
    res["largest_lyapunov_d32_T131072"] = {
        "ms": round(sec * 1e3, 3), "jacobians_per_s": round(T / sec, 1),
        "lle": round(float(g.largest_lyapunov(Jz, 0.01).cpu()), 4),
        "kernels_ms": kernel_times(g, lambda: g.largest_lyapunov(Jz, 0.01))}
    sec = timed(torch, lambda: g.scan_reset(Jz))
    res["reset_scan_all_states_d32_T131072"] = {
        "ms": round(sec * 1e3, 3), "jacobians_per_s": round(T / sec, 1),
        "kernels_ms": kernel_times(g, lambda: g.scan_reset(Jz))}
    del Jz
    # the same estimator above 64 x 64 (four waves per batch item in the carry kernel): near-identity Jacobians
    # I + 0.1 N(0, 1/d), d = 128, T = 16,384
    T, d = 16384, 128
    gen = si.device_generator(si.BASE_SEED + 5, dev)
    Jw = torch.eye(d, device=dev)[None] + (0.1 / d ** 0.5) * torch.randn((T, d, d), device=dev, generator=gen)
    Jz = g.to_goom(Jw)
    del Jw
    sec = timed(torch, lambda: g.lyapunov_spectrum(Jz, 0.01))
    res["lyapunov_near_identity_d128_T16384"] = {
        "ms": round(sec * 1e3, 3), "jacobians_per_s": round(T / sec, 1),
        "kernels_ms": kernel_times(g, lambda: g.lyapunov_spectrum(Jz, 0.01))}
    del Jz
    return res


def large_matrices(g, torch, dev, si):
    # matrices beyond the register-resident kernels: LMME of 32 pairs of 1024 x 1024, scans of 1024 x 1024
    # (T = 512) and 256 x 256 (T = 32,768) matrices with N(0,1) entries
    res = {}
    B, n = 32, 1024
    a = g.to_goom(torch.randn((B, n, n), device=dev, generator=si.device_generator(251003426 * 10 + 71, dev)))
    b = g.to_goom(torch.randn((B, n, n), device=dev, generator=si.device_generator(251003426 * 10 + 72, dev)))
    c = torch.empty_like(a)
    sec = timed(torch, lambda: g.lmme(a, b, out=c), 5)
    kt = kernel_times(g, lambda: g.lmme(a, b, out=c))
    res["lmme_32x1024^3"] = {"ms": round(sec * 1e3, 3), "tflops": round(2.0 * n ** 3 * B / sec / 1e12, 2),
                             "pct_of_mfma_peak": round(100 * 2.0 * n ** 3 * B / sec / 1e12 / MFMA_F32_PEAK_TFLOPS, 2),
                             "gemm_tflops": round(2.0 * n ** 3 * B / (kt["lmme_large_gemm"] * 1e-3) / 1e12, 2), "kernels_ms": kt}
    del a, b, c
    # the same product with double components (complex128), on the double-precision matrix instruction
    a = g.to_goom(torch.randn((B, n, n), device=dev, dtype=torch.float64, generator=si.device_generator(251003426 * 10 + 74, dev)))
    b = g.to_goom(torch.randn((B, n, n), device=dev, dtype=torch.float64, generator=si.device_generator(251003426 * 10 + 75, dev)))
    c = torch.empty_like(a)
    sec = timed(torch, lambda: g.lmme(a, b, out=c), 5)
    kt = kernel_times(g, lambda: g.lmme(a, b, out=c))
    res["lmme_32x1024^3_complex128"] = {"ms": round(sec * 1e3, 3), "tflops": round(2.0 * n ** 3 * B / sec / 1e12, 2),
                                        "pct_of_fp64_mfma_peak": round(100 * 2.0 * n ** 3 * B / sec / 1e12 / MFMA_F64_PEAK_TFLOPS, 2),
                                        "gemm_tflops": round(2.0 * n ** 3 * B / (kt["lmme_large_gemm"] * 1e-3) / 1e12, 2), "kernels_ms": kt}
    del a, b, c
    torch.cuda.empty_cache()
    for T, d in ((512, 1024), (32768, 256)):
        z = torch.empty((T, d, d), dtype=torch.complex64, device=dev)
        for t0, x in si.device_normal_blocks(251003426 * 10 + 73, T, (d, d), dev, max(1, (1 << 26) // (d * d))):
            g.to_goom(x, out=z[t0:t0 + x.shape[0]])
        out = torch.empty_like(z)
        sec = timed(torch, lambda: g.scan(z, out=out))
        fl = 2.0 * d ** 3 * 2 * T
        res[f"scan_T{T}_d{d}"] = {"ms": round(sec * 1e3, 3), "products_per_s": round(T / sec, 1),
                                  "lmme_tflops_executed": round(fl / sec / 1e12, 2),
                                  "pct_of_fp32_mfma_peak": round(100 * fl / sec / 1e12 / MFMA_F32_PEAK_TFLOPS, 2),
                                  "kernels_ms": kernel_times(g, lambda: g.scan(z, out=out))}
        del z, out
        torch.cuda.empty_cache()
    # a scan of complex128 matrices above 128: T = 256 of 512 x 512 (the same driver on the fp64 GEMM)
    T, d = 256, 512
    z = g.to_goom(torch.randn((T, d, d), device=dev, dtype=torch.float64, generator=si.device_generator(251003426 * 10 + 76, dev)))
    out = torch.empty_like(z)
    sec = timed(torch, lambda: g.scan(z, out=out), 3)
    fl = 2.0 * d ** 3 * 2 * T
    res[f"scan_T{T}_d{d}_complex128"] = {"ms": round(sec * 1e3, 3), "products_per_s": round(T / sec, 1),
                                         "lmme_tflops_executed": round(fl / sec / 1e12, 2),
                                         "pct_of_fp64_mfma_peak": round(100 * fl / sec / 1e12 / MFMA_F64_PEAK_TFLOPS, 2),
                                         "kernels_ms": kernel_times(g, lambda: g.scan(z, out=out))}
    del z, out
    torch.cuda.empty_cache()
    return res


def recurrence(g, torch, dev, si):
    # non-diagonal recurrence: 8 x 16 sequences of 65,536 tokens, d = 32
    import math
    res = {}
    nseq, T, d = 128, 65536, 32
    az = torch.empty((nseq, T, d, d), dtype=torch.complex64, device=dev)
    for s0, x in si.device_normal_blocks(251003426 * 10 + 51, nseq, (T, d, d), dev, 4, scale=1.05 / math.sqrt(d)):
        g.to_goom(x, out=az[s0:s0 + x.shape[0]])
    bz = g.to_goom(torch.randn((nseq, T, d), device=dev, generator=si.device_generator(251003426 * 10 + 52, dev)))
    h = torch.empty((nseq, T, d), dtype=torch.complex64, device=dev)
    sec = timed(torch, lambda: g.affine_scan(az, bz, out=h))
    kms = kernel_times(g, lambda: g.affine_scan(az, bz, out=h))
    # with this many sequences each is walked start to end and the matrices and inputs are read once; the chunked scan reads them in
    # two of its phases
    reads = 1 if "affine_sequential_walk" in kms else 2
    byts = (reads * az.numel() + reads * bz.numel() + h.numel()) * 8
    res["recurrence_128seq_T65536_d32"] = {
        "ms": round(sec * 1e3, 3), "tokens_per_s": round(nseq * T / sec, 1),
        "hbm_gbs_algorithmic": round(byts / sec / 1e9, 1), "pct_of_hbm_peak": round(100 * byts / sec / 1e9 / HBM_PEAK_GBS, 2),
        "passes_over_the_matrices": reads, "kernels_ms": kms}
    # the same recurrence cut into chunks (what a batch of fewer sequences gets): chunk products, carries, walk
    L = 1024
    sec = timed(torch, lambda: g.affine_scan(az, bz, out=h, chunk_len=L), 2)
    byts2 = (2 * az.numel() + 2 * bz.numel() + h.numel()) * 8
    res["recurrence_128seq_T65536_d32_chunked"] = {
        "ms": round(sec * 1e3, 3), "tokens_per_s": round(nseq * T / sec, 1), "chunk_len": L,
        "hbm_gbs_algorithmic": round(byts2 / sec / 1e9, 1), "kernels_ms": kernel_times(g, lambda: g.affine_scan(az, bz, out=h, chunk_len=L))}
    # its backward pass: gradients with respect to the log-magnitudes of A and of the inputs, given those of the states
    gh = torch.randn((nseq, T, d), device=dev, generator=si.device_generator(251003426 * 10 + 53, dev))
    fn = lambda: g.affine_scan_backward(az, bz, h, gh)
    sec = timed(torch, fn, 2)
    kms = kernel_times(g, fn)
    # algorithmic bytes: A read by the adjoint recurrence (transposed, in place; twice where that runs as a chunked scan), read
    # again for its gradient (reals), which is written
    reads = 2 if "affine_sequential_walk" in kms else 3
    bbytes = az.numel() * (8 * reads + 4)
    res["recurrence_backward_128seq_T65536_d32"] = {
        "ms": round(sec * 1e3, 3), "tokens_per_s": round(nseq * T / sec, 1), "hbm_gbs_algorithmic": round(bbytes / sec / 1e9, 1),
        "passes_over_the_matrices": reads, "kernels_ms": kms}
    del h, gh
    g._ws = None
    torch.cuda.empty_cache()
    # the same recurrence with its states written in scaled floating-point form by the last phase
    sec = timed(torch, lambda: g.affine_scan_scaled(az, bz))
    res["recurrence_scaled_states"] = {"ms": round(sec * 1e3, 3), "tokens_per_s": round(nseq * T / sec, 1)}
    # and with one constant matrix per sequence (no matrix traffic left)
    a1 = az[:, 0].contiguous()
    del az
    torch.cuda.empty_cache()
    h = torch.empty((nseq, T, d), dtype=torch.complex64, device=dev)
    sec = timed(torch, lambda: g.affine_scan(a1, bz, out=h, time_invariant=True))
    res["recurrence_time_invariant"] = {
        "ms": round(sec * 1e3, 3), "tokens_per_s": round(nseq * T / sec, 1),
        "kernels_ms": kernel_times(g, lambda: g.affine_scan(a1, bz, out=h, time_invariant=True))}
    # its backward pass: the adjoint recurrence over the one matrix, the matrix's gradient summed over the steps
    gh = torch.randn((nseq, T, d), device=dev, generator=si.device_generator(251003426 * 10 + 54, dev))
    sec = timed(torch, lambda: g.affine_scan_backward(a1, bz, h, gh, time_invariant=True))
    res["recurrence_time_invariant_backward"] = {
        "ms": round(sec * 1e3, 3), "tokens_per_s": round(nseq * T / sec, 1),
        "kernels_ms": kernel_times(g, lambda: g.affine_scan_backward(a1, bz, h, gh, time_invariant=True))}
    del gh
    g._ws = None
    torch.cuda.empty_cache()
    # one 64 x 64 matrix per sequence: 64 sequences of 32,768 tokens
    a64 = g.to_goom(torch.randn((64, 64, 64), device=dev, generator=si.device_generator(251003426 * 10 + 55, dev)) * (1.02 / 8.0))
    b64 = g.to_goom(torch.randn((64, 32768, 64), device=dev, generator=si.device_generator(251003426 * 10 + 56, dev)))
    h64 = g.affine_scan(a64, b64, time_invariant=True)
    g64 = torch.randn((64, 32768, 64), device=dev, generator=si.device_generator(251003426 * 10 + 57, dev))
    sec = timed(torch, lambda: g.affine_scan(a64, b64, out=h64, time_invariant=True))
    secb = timed(torch, lambda: g.affine_scan_backward(a64, b64, h64, g64, time_invariant=True))
    res["recurrence_time_invariant_d64_64seq_T32768"] = {
        "ms": round(sec * 1e3, 3), "tokens_per_s": round(64 * 32768 / sec, 1), "backward_ms": round(secb * 1e3, 3),
        "kernels_ms": kernel_times(g, lambda: g.affine_scan(a64, b64, out=h64, time_invariant=True))}
    del a64, b64, h64, g64
    g._ws = None
    torch.cuda.empty_cache()
    # the elementwise ends of the recurrence as ops of their own, on the states just computed (nseq x T vectors of d):
    # signed log-add (24 B per element) and scaled exponentiation (12 B per element)
    o = torch.empty_like(h)
    sec = timed(torch, lambda: g.log_add_exp(h, bz, out=o), 5)
    res["log_add_exp_gbs"] = round(24.0 * h.numel() / sec / 1e9, 1)
    sec = timed(torch, lambda: g.scaled_exp(h), 5)
    res["scaled_exp_gbs"] = round(12.0 * h.numel() / sec / 1e9, 1)
    return res


if __name__ == "__main__":
    main()
