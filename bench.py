#!/usr/bin/env python3
"""PCMM benchmark on one MI355X: int8-MFMA TOPS and ms per Llama-3-8B-shaped projection.

One "step" is one pcmm_run over a whole projection: digit split of every residue, int8 MFMA main
loop, recombination and Barrett reduction, for all limbs and both ciphertext components, with W, A
and C resident in HBM.  Plan creation (W packing) is outside the timed region.

Prints ONE JSON line.  `value` is algorithmic int8 TOPS = 2*M*K*Ncols*L*D*S / time with
D = ceil(prime_bits/8) digits and S = w_bits/8 slices; padding or extra issued MFMA work is not credited.
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

INT8_MFMA_PEAK_TOPS = 5000.0      # MI355X dense int8 matrix peak, published
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E peak, published


def _traffic_from_profiles(workload: str):
    """HBM bytes per GEMM launch measured with rocprofv3 --pmc, if a summary for this workload is committed."""
    path = os.path.join(ROOT, "profiles", "gemm_kernel_%s_hbm_traffic.txt" % workload)
    if not os.path.exists(path):
        return None
    with open(path) as f:
        for line in f:
            if line.startswith("traffic_bytes_per_launch="):
                return float(line.split("=", 1)[1])
    return None


def cpu_baseline(wl, W_host, A_dev, C_dev, rows_target_s: float = 20.0):
    """Time the oracle (as it stands) on a bounded sample of the same workload; also checks the GPU rows."""
    import numpy as np

    from oracle import oracle_threads, pcmm_oracle_select

    threads = oracle_threads()
    # size the sample from a short probe so that the oracle runs for roughly rows_target_s seconds
    A_host = A_dev.cpu().numpy().view(np.uint64)
    cols = np.arange(wl.Ncols, dtype=np.int64)
    t0 = time.perf_counter()
    pcmm_oracle_select(W_host, A_host, wl.primes, [0], cols)
    probe = time.perf_counter() - t0
    task = max(probe, 1e-6) / -(-wl.L // threads)            # one (row, limb) task on one thread
    nrows = int(min(wl.M, max(1, rows_target_s * threads / (wl.L * task))))
    rng = np.random.default_rng(12345)
    rows = np.sort(rng.choice(wl.M, size=nrows, replace=False))
    t0 = time.perf_counter()
    want = pcmm_oracle_select(W_host, A_host, wl.primes, rows, cols)
    dt = time.perf_counter() - t0
    macs = nrows * wl.K * wl.Ncols * wl.L
    got = C_dev[:, rows.tolist(), :].cpu().numpy().view(np.uint64)
    exact = bool((got == want).all())
    tops = 2.0 * macs * wl.digits * wl.slices / dt / 1e12
    return {
        "value": tops,
        "unit": "TOPS (int8-equivalent: 2*D*S ops per 128-bit modular MAC)",
        "cores": threads,
        "kind": "oracle",
        "sample": "%d of %d output rows (seeded choice) x all %d columns x all %d limbs, %.1f s wall, "
                  "%.3g modular MAC/s; full projection would take ~%.0f s (extrapolated)"
                  % (nrows, wl.M, wl.Ncols, wl.L, dt, macs / dt, wl.modular_macs / (macs / dt)),
        "gpu_rows_match_oracle": exact,
    }


def ring_switch_rates(pkg, torch, dev, iters: int = 10):
    """The permutation kernels either side of the PCMM (not part of the timed step): HBM GB/s on a batch of
    4 limbs x 2 components x 512 ciphertexts over R_{2^16}, decomposed to R_{2^12} (k = 16) and R_{2^8} (k = 256)."""
    npoly, N = 4 * 2 * 512, 1 << 16
    p = torch.randint(0, 1 << 62, (npoly, N), dtype=torch.int64, device=dev)
    parts = torch.empty_like(p)
    back = torch.empty_like(p)
    stream = torch.cuda.current_stream()
    out = {"workload": "%d polynomials of degree 2^16 (4 limbs x 2 components x 512 ciphertexts), uint64" % npoly,
           "algorithmic_bytes_per_coefficient": 16, "hbm_peak_GBs": HBM_PEAK_GBS}
    for k in (16, 256):
        rates = {}
        for name, fn, src, dst in (("decompose", pkg.pcmm_ring_decompose, p, parts),
                                   ("compose", pkg.pcmm_ring_compose, parts, back)):
            fn(src, dst, N, k, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(iters):
                fn(src, dst, N, k, stream)
            e1.record(stream)
            e1.synchronize()
            ms = e0.elapsed_time(e1) / iters
            rates[name + "_ms"] = ms
            rates[name + "_GBs"] = 16.0 * npoly * N / (ms * 1e-3) / 1e9
            rates[name + "_frac_of_hbm_peak"] = rates[name + "_GBs"] / HBM_PEAK_GBS
        rates["round_trip_exact"] = bool(torch.equal(back, p))
        out["k=%d" % k] = rates
    return out


def library_int8_gemm(torch, dev, wl, iters: int = 5):
    """Context only: the vendor library's plain int8 GEMM (torch._int_mm) on the raw int8 products of the same
    workload, W[M][K] x digit planes [K][Ncols*L*D] -> int32, random int8 data.  No digit split, no recombination,
    no reduction: what 'hand the clear product to a GPU BLAS' costs on this machine for the inner products alone."""
    try:
        n_eq = wl.Ncols * wl.L * wl.digits
        a = torch.randint(-128, 128, (wl.M, wl.K), dtype=torch.int8, device=dev)
        b = torch.randint(-128, 128, (wl.K, n_eq), dtype=torch.int8, device=dev)
        c = torch._int_mm(a, b)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            c = torch._int_mm(a, b)
        e1.record()
        e1.synchronize()
        ms = e0.elapsed_time(e1) / iters
        del a, b, c
        tops = 2.0 * wl.M * wl.K * n_eq / (ms * 1e-3) / 1e12
        return {"what": "torch._int_mm %dx%dx%d int8 -> int32 (inner products only)" % (wl.M, wl.K, n_eq),
                "ms": ms * wl.slices, "tops": tops}
    except Exception as exc:  # the library may not cover a shape; this block is context, not the product
        return {"what": "torch._int_mm unavailable for this shape", "error": str(exc)[:200]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="attn_proj")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ring-switch", action="store_true",
                    help="skip the (untimed-step) measurement of the ring-switch permutation kernels")
    ap.add_argument("--no-library-gemm", action="store_true",
                    help="skip timing the vendor library's plain int8 GEMM on the same int8 work (context only)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2601_18511_amd as pkg
    import pcmm_inputs as pi

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    wl = pi.WORKLOADS[args.workload]

    W_host = pi.gen_W(wl)
    W_dev = torch.from_numpy(W_host).to(dev)
    A_dev = pi.gen_A_torch(wl, dev)
    C_dev = torch.empty((wl.L, wl.M, wl.Ncols), dtype=torch.int64, device=dev)
    plan = pkg.pcmm_plan_create(W_dev, wl.primes, wl.prime_bits, wl.Ncols)
    stream = torch.cuda.current_stream()

    if args.copy_calibration:
        src = torch.ones(1 << 27, dtype=torch.int64, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        pkg.pcmm_run(plan, A_dev, C_dev, stream)
    torch.cuda.synchronize()

    split_ms, gemm_ms = [], []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        s, g = pkg.pcmm_run_profiled(plan, A_dev, C_dev, stream)    # HIP events around each kernel
        split_ms.append(s)
        gemm_ms.append(g)
    torch.cuda.synchronize()
    total = time.perf_counter() - t0

    ms_per_step = total * 1e3 / args.steps
    tops = wl.int8_ops / (ms_per_step * 1e-3) / 1e12
    gemm_avg = sum(gemm_ms) / len(gemm_ms)
    split_avg = sum(split_ms) / len(split_ms)
    gemm_tops = wl.int8_ops / (gemm_avg * 1e-3) / 1e12
    res_bytes = 8.0 * wl.K * wl.Ncols * wl.L
    out_bytes = 8.0 * wl.M * wl.Ncols * wl.L
    split_alg_bytes = res_bytes * (8 + wl.digits) / 8.0
    alg_bytes = res_bytes + out_bytes + wl.M * wl.K * wl.slices

    # the dominant kernel's roofline: int8 MFMA for the projections; HBM where the algorithmic bytes of the
    # launch (digit planes + W + C) take longer at 8 TB/s than its int8 work at 5 POP/s (the wide workload)
    gemm_alg_bytes = wl.K * wl.Ncols * wl.L * wl.digits + wl.M * wl.K * wl.slices + out_bytes
    mfma_floor_s = wl.int8_ops / (INT8_MFMA_PEAK_TOPS * 1e12)
    hbm_floor_s = gemm_alg_bytes / (HBM_PEAK_GBS * 1e9)
    if mfma_floor_s >= hbm_floor_s:
        roofline = {"kernel": "gemm_kernel (int8 MFMA main loop + recombine + Barrett)", "bound": "mfma",
                    "achieved": gemm_tops, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                    "frac": gemm_tops / INT8_MFMA_PEAK_TOPS}
    else:
        gbs = gemm_alg_bytes / (gemm_avg * 1e-3) / 1e9
        roofline = {"kernel": "gemm_kernel (int8 MFMA main loop + recombine + Barrett)", "bound": "hbm",
                    "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                    "mfma_TOPs": gemm_tops}
    roofline["avg_launch_ms"] = gemm_avg
    roofline["algorithmic_bytes_per_launch"] = gemm_alg_bytes
    roofline["traffic"] = _traffic_from_profiles(wl.name)

    result = {
        "metric": "PCMM int8-MFMA TOPS (% of peak) + ms per Llama-3-8B projection, 1 GPU",
        "value": tops,
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "pct_of_int8_peak": 100.0 * tops / INT8_MFMA_PEAK_TOPS,
        "config": {
            "workload": "%s: W %dx%d int%d, A %dx%d uint64 residues, L=%d primes of %d bits, D=%d digits, S=%d"
                        % (wl.name, wl.M, wl.K, wl.w_bits, wl.K, wl.Ncols, wl.L, wl.prime_bits, wl.digits, wl.slices),
            "modular_macs_per_s": wl.modular_macs / (ms_per_step * 1e-3),
            "algorithmic_hbm_GBs": alg_bytes / (ms_per_step * 1e-3) / 1e9,
            "workspace_bytes": pkg.pcmm_plan_workspace_bytes(plan),
        },
        "roofline": roofline,
        "kernels": {
            "gemm_ms_avg": gemm_avg,
            "gemm_ms_min": min(gemm_ms),
            "split_ms_avg": split_avg,
            "split_ms_min": min(split_ms),
            "split_hbm_GBs": split_alg_bytes / (split_avg * 1e-3) / 1e9,
            "split_frac_of_hbm_peak": split_alg_bytes / (split_avg * 1e-3) / 1e9 / HBM_PEAK_GBS,
        },
    }
    # what the matrix cores alone sustain on this machine (no memory traffic): with random and with zero operands
    probe_rand = pkg.pcmm_mfma_probe(0, 200000, True)
    probe_zero = pkg.pcmm_mfma_probe(0, 200000, False)
    result["mfma_probe"] = {
        "random_operands": {"tops": probe_rand[0], "shader_mhz": probe_rand[1]},
        "zero_operands": {"tops": probe_zero[0], "shader_mhz": probe_zero[1]},
        "gemm_frac_of_random_operand_probe": gemm_tops / probe_rand[0],
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, W_host, A_dev, C_dev)
    pkg.pcmm_plan_destroy(plan)
    del A_dev, C_dev, W_dev
    torch.cuda.empty_cache()
    if not args.no_ring_switch:
        result["ring_switch"] = ring_switch_rates(pkg, torch, dev)
    if not args.no_library_gemm:
        result["library_int8_gemm"] = library_int8_gemm(torch, dev, wl)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
