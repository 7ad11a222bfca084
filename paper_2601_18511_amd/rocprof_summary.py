"""rocprofv3 harness: turns rocprofv3 output directories into the short text summaries kept under profiles/.

What it reports for the kernels of one workload (the PCMM path has no counterpart of this in the paper;
the figures are the ones a roofline needs):

  * per kernel: launches, average / minimum / maximum duration (from --kernel-trace, or from the dispatch
    timestamps of a --pmc run when no trace is given);
  * achieved int8 TOP/s of the MFMA kernel against the chip's 5000 TOP/s dense int8 peak, and its
    algorithmic bytes per second against the 8000 GB/s HBM peak;
  * HBM-side traffic: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by what the same counter
    reads for a plain device copy of known size in the same run (bench.py --copy-calibration);
  * MFMA utilisation: SQ_VALU_MFMA_BUSY_CYCLES / (SIMDs x shader cycles), the shader cycles taken from
    GRBM_GUI_ACTIVE (summed over the XCDs) when that counter was collected, else from the kernel's
    duration at the nominal clock -- the denominator used is printed;
  * derived cache and issue figures when their counters are present (L2 hit rate, wait fraction, ...).

Usage (after the rocprofv3 runs named in the summary's "commands" lines):

    python3 -m paper_2601_18511_amd.rocprof_summary --workload attn_proj --trace DIR --pmc DIR [--pmc DIR ...]
            [--command "rocprofv3 ..."]... --out-prefix profiles/

It writes <prefix><kernel>_<workload>_kernel_trace.txt, ..._hbm_traffic.txt (when FETCH_SIZE and WRITE_SIZE
were collected) and ..._counters.txt (when other counters were).  Parsing is plain csv; nothing here
touches the GPU.
"""
from __future__ import annotations

import argparse
import csv
import os
import re
import statistics
import sys
from collections import defaultdict
from typing import Dict, List, Optional, Sequence, Tuple

INT8_MFMA_PEAK_TOPS = 5000.0
HBM_PEAK_GBS = 8000.0
N_SIMD = 1024            # 256 compute units x 4 SIMDs
N_XCD = 8
NOMINAL_GHZ = 2.4
COPY_KERNEL = re.compile(r"copyBuffer|direct_copy_kernel")   # what a plain device-to-device copy runs as
GIB = float(1 << 30)


# --------------------------------------------------------------------------------------------------
# reading rocprofv3 csv output
# --------------------------------------------------------------------------------------------------
def find_csv(directory: str, suffix: str) -> List[str]:
    """All files under `directory` whose name ends in `suffix` (rocprofv3 nests them under <host>/<pid>_...)."""
    out = []
    for base, _dirs, files in os.walk(directory):
        out += [os.path.join(base, f) for f in files if f.endswith(suffix)]
    return sorted(out)


def short_name(kernel: str) -> str:
    """'void (anonymous namespace)::gemm_kernel<4, 4, 2, 5, 1, 0>(GemmArgs)' -> 'gemm_kernel<4, 4, 2, 5, 1, 0>'."""
    k = kernel.strip().strip('"')
    k = re.sub(r"^void\s+", "", k)
    k = k.replace("(anonymous namespace)::", "")
    depth, cut = 0, len(k)
    for i, ch in enumerate(k):                    # cut at the first '(' outside template brackets
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            cut = i
            break
    return k[:cut].strip()


def read_kernel_trace(directory: str) -> Dict[str, List[float]]:
    """kernel name -> durations in ns of every dispatch, from *_kernel_trace.csv."""
    out: Dict[str, List[float]] = defaultdict(list)
    for path in find_csv(directory, "kernel_trace.csv"):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                out[short_name(row["Kernel_Name"])].append(float(row["End_Timestamp"]) - float(row["Start_Timestamp"]))
    return dict(out)


def read_counters(directory: str) -> Tuple[Dict[str, Dict[str, List[float]]], Dict[str, List[float]]]:
    """(kernel -> counter -> value per dispatch, kernel -> duration in ns per dispatch) from *_counter_collection.csv."""
    vals: Dict[str, Dict[str, Dict[str, float]]] = defaultdict(lambda: defaultdict(dict))
    durs: Dict[str, Dict[str, float]] = defaultdict(dict)
    for path in find_csv(directory, "counter_collection.csv"):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                k = short_name(row["Kernel_Name"])
                disp = row["Dispatch_Id"]
                # one row per (dispatch, counter); a counter with several instances appears several times: add up
                vals[k][row["Counter_Name"]][disp] = vals[k][row["Counter_Name"]].get(disp, 0.0) + float(row["Counter_Value"])
                durs[k][disp] = float(row["End_Timestamp"]) - float(row["Start_Timestamp"])
    counters = {k: {c: [v for _, v in sorted(d.items(), key=lambda kv: int(kv[0]))] for c, d in cs.items()}
                for k, cs in vals.items()}
    durations = {k: [v for _, v in sorted(d.items(), key=lambda kv: int(kv[0]))] for k, d in durs.items()}
    return counters, durations


def read_grouped(directory: str, suffix: str):
    """(kernel, Grid_Size) -> {"dur": [ns per dispatch], counter name: [value per dispatch]} from a kernel-trace or
    counter-collection csv: the same kernel launched on different problem sizes stays apart."""
    out: Dict[Tuple[str, int], Dict[str, Dict[str, float]]] = defaultdict(lambda: defaultdict(dict))
    for path in find_csv(directory, suffix):
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if "Grid_Size" in row:          # counter collection: total work-items
                    grid = int(float(row["Grid_Size"]))
                else:                           # kernel trace: work-items per dimension
                    grid = int(float(row["Grid_Size_X"])) * int(float(row["Grid_Size_Y"])) * int(float(row["Grid_Size_Z"]))
                key = (short_name(row["Kernel_Name"]), grid)
                disp = row["Dispatch_Id"]
                out[key]["dur"][disp] = float(row["End_Timestamp"]) - float(row["Start_Timestamp"])
                if "Counter_Name" in row:
                    c = row["Counter_Name"]
                    out[key][c][disp] = out[key][c].get(disp, 0.0) + float(row["Counter_Value"])
    return {k: {c: list(d.values()) for c, d in v.items()} for k, v in out.items()}


def merge_counters(dirs: Sequence[str]):
    """Counters of several --pmc runs in one table.  A kernel's durations are taken from the run that collected
    its issue counters (anything but FETCH_SIZE / WRITE_SIZE) when there is one, so that cycle counts and
    durations of one and the same run are set against each other."""
    counters: Dict[str, Dict[str, List[float]]] = defaultdict(dict)
    durations: Dict[str, List[float]] = {}
    preferred = set()
    for d in dirs:
        c, t = read_counters(d)
        for k, cs in c.items():
            counters[k].update(cs)
            issue_run = any(name not in ("FETCH_SIZE", "WRITE_SIZE") for name in cs)
            if k in t and (k not in durations or (issue_run and k not in preferred)):
                durations[k] = t[k]
                if issue_run:
                    preferred.add(k)
    return dict(counters), durations


def pick(kernels, pattern: str) -> List[str]:
    rx = re.compile(pattern)
    return sorted(k for k in kernels if rx.search(k))


def mean(xs: Sequence[float]) -> float:
    return sum(xs) / len(xs)


# --------------------------------------------------------------------------------------------------
# derived figures
# --------------------------------------------------------------------------------------------------
def copy_scale(directories: Sequence[str], counter: str, copy_kib: float) -> Optional[Tuple[float, float]]:
    """(KiB the counter read for the calibration copy, scale = true KiB / counted KiB), or None without a copy.
    bench.py --copy-calibration runs its plain device copy before anything else, so the calibration copy is the
    FIRST dispatch of a copy kernel that moved a sizeable amount (input generators copy other sizes later)."""
    best = None
    for d in directories:
        for path in find_csv(d, "counter_collection.csv"):
            with open(path, newline="") as f:
                for row in csv.DictReader(f):
                    if row["Counter_Name"] != counter or not COPY_KERNEL.search(row["Kernel_Name"]):
                        continue
                    v, disp = float(row["Counter_Value"]), int(row["Dispatch_Id"])
                    if v >= 0.25 * copy_kib and (best is None or disp < best[0]):
                        best = (disp, v)
    if best is None:
        return None
    return best[1], copy_kib / best[1]


def workload_figures(name: str) -> dict:
    """Algorithmic ops and bytes of a workload of pcmm_inputs (per pcmm_run), and the names of its kernels."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    import pcmm_inputs as pi

    w = pi.WORKLOADS[name]
    digits_bytes = w.K * w.Ncols * w.L * w.digits
    return {
        "desc": "W %dx%d int%d, A %dx%d uint64 residues, L=%d primes of %d bits, D=%d digits, S=%d slices"
                % (w.M, w.K, w.w_bits, w.K, w.Ncols, w.L, w.prime_bits, w.digits, w.slices),
        "int8_ops": float(w.int8_ops),
        "gemm_bytes": float(digits_bytes + w.M * w.K * w.slices + 8 * w.M * w.Ncols * w.L),
        "gemm_parts": (digits_bytes, w.M * w.K * w.slices, 8 * w.M * w.Ncols * w.L),
        "split_bytes": float(w.K * w.Ncols * w.L * (8 + w.digits)),
        "mfma_kernel": "gemm_shortk_kernel" if (w.K <= 128 and w.prime_bits <= 50) else "gemm_kernel",
    }


def trace_summary(workload: str, fig: dict, trace: Dict[str, List[float]], commands: Sequence[str]) -> str:
    mine = pick(trace, r"gemm_kernel|gemm_shortk_kernel|split_kernel|transpose_u64_kernel|mfma_probe_kernel")
    lines = ["rocprofv3 kernel trace of the PCMM kernels on the %s workload" % workload,
             "(%s; one pcmm_run = 1 split_kernel + 1 MFMA-kernel launch)" % fig["desc"], ""]
    lines += ["commands (from /tmp with TMPDIR=/tmp on the MI355X box, R = repository root):"] + ["  " + c for c in commands] + [""]
    lines.append("%-46s %6s %12s %12s %12s" % ("kernel", "calls", "avg_ms", "min_ms", "max_ms"))
    for k in mine:
        d = trace[k]
        lines.append("%-46s %6d %12.4f %12.4f %12.4f" % (k, len(d), mean(d) / 1e6, min(d) / 1e6, max(d) / 1e6))
    lines.append("(every other kernel in the trace belongs to torch: input generators, the calibration copy)")
    g = pick(trace, r"^%s<" % fig["mfma_kernel"])
    if g:
        d = [x for k in g for x in trace[k]]
        avg, lo = mean(d), min(d)
        tops = fig["int8_ops"] / (avg * 1e-9) / 1e12
        gbs = fig["gemm_bytes"] / (avg * 1e-9) / 1e9
        lines += ["",
                  "%s: average %.3f ms (min %.3f ms, median %.3f ms) over %d launches"
                  % (fig["mfma_kernel"], avg / 1e6, lo / 1e6, statistics.median(d) / 1e6, len(d)),
                  "  algorithmic int8 work %.4g ops / average = %.0f TOP/s = %.1f %% of the %.0f TOP/s int8 MFMA peak"
                  % (fig["int8_ops"], tops, 100 * tops / INT8_MFMA_PEAK_TOPS, INT8_MFMA_PEAK_TOPS),
                  "  algorithmic bytes %.2f GiB / average = %.0f GB/s = %.1f %% of the %.0f GB/s HBM peak"
                  % (fig["gemm_bytes"] / GIB, gbs, 100 * gbs / HBM_PEAK_GBS, HBM_PEAK_GBS)]
    s = pick(trace, r"^split_kernel<")
    if s:
        d = [x for k in s for x in trace[k]]
        gbs = fig["split_bytes"] / (mean(d) * 1e-9) / 1e9
        lines += ["split_kernel: average %.3f ms (min %.3f ms); algorithmic bytes %.2f GiB / average = %.0f GB/s = %.1f %% of the HBM peak"
                  % (mean(d) / 1e6, min(d) / 1e6, fig["split_bytes"] / GIB, gbs, 100 * gbs / HBM_PEAK_GBS)]
    lines.append("(averages include the first, cold launch; bench.py reports the HIP-event average of its timed steps)")
    return "\n".join(lines) + "\n"


def traffic_summary(workload: str, fig: dict, counters, commands: Sequence[str], copy_kib: float,
                    directories: Sequence[str]) -> Optional[str]:
    g = pick(counters, r"^%s<" % fig["mfma_kernel"])
    if not g or "FETCH_SIZE" not in counters[g[0]] or "WRITE_SIZE" not in counters[g[0]]:
        return None
    cal_f = copy_scale(directories, "FETCH_SIZE", copy_kib)
    cal_w = copy_scale(directories, "WRITE_SIZE", copy_kib)
    sf = cal_f[1] if cal_f else 1.0
    sw = cal_w[1] if cal_w else 1.0
    lines = ["HBM-side traffic of the PCMM kernels on the %s workload, from rocprofv3 counters" % workload,
             "(%s)" % fig["desc"], "",
             "commands (from /tmp with TMPDIR=/tmp, R = repository root), one counter per run:"] + ["  " + c for c in commands] + [""]
    if cal_f and cal_w:
        lines += ["calibration: bench.py --copy-calibration runs a plain device copy of 1 GiB (reads 2^20 KiB, writes 2^20 KiB).",
                  "  FETCH_SIZE read %.1f KiB for it -> scale %.4f;  WRITE_SIZE read %.1f KiB -> scale %.4f"
                  % (cal_f[0], sf, cal_w[0], sw), ""]
    else:
        lines += ["calibration: no copy kernel in these runs; counters taken at face value (scale 1)", ""]
    lines.append("per launch (average over the profiled launches), counters in KiB, scaled values in GiB:")
    traffic = None
    for pat, label in ((r"^%s<" % fig["mfma_kernel"], fig["mfma_kernel"]), (r"^split_kernel<", "split_kernel")):
        ks = pick(counters, pat)
        if not ks:
            continue
        f = mean([v for k in ks for v in counters[k].get("FETCH_SIZE", [])])
        w = mean([v for k in ks for v in counters[k].get("WRITE_SIZE", [])])
        lines.append("  %-20s FETCH_SIZE %.0f KiB -> %.2f GiB read;   WRITE_SIZE %.0f KiB -> %.2f GiB written"
                     % (label, f, f * sf * 1024 / GIB, w, w * sw * 1024 / GIB))
        if label == fig["mfma_kernel"]:
            traffic = (f * sf + w * sw) * 1024.0
    dp, wp, cp = fig["gemm_parts"]
    lines += ["",
              "algorithmic bytes per launch: %s %.2f GiB (digit planes %.2f + packed W %.3f + C %.2f), split_kernel %.2f GiB"
              % (fig["mfma_kernel"], fig["gemm_bytes"] / GIB, dp / GIB, wp / GIB, cp / GIB, fig["split_bytes"] / GIB),
              "traffic / algorithmic bytes of the MFMA kernel: %.2f" % (traffic / fig["gemm_bytes"]),
              "FETCH_SIZE counts what the L2s request from the fabric: re-reads of W and of digit chunks by different XCDs show up",
              "here even when the Infinity Cache serves them.", "",
              "traffic_bytes_per_launch=%.0f" % traffic]
    return "\n".join(lines) + "\n"


def counter_summary(workload: str, fig: dict, counters, durations, commands: Sequence[str]) -> Optional[str]:
    g = pick(counters, r"^%s<" % fig["mfma_kernel"])
    if not g:
        return None
    c = {name: mean(v) for k in g for name, v in counters[k].items() if name not in ("FETCH_SIZE", "WRITE_SIZE")}
    if not c:
        return None
    dur_ns = mean([x for k in g for x in durations.get(k, [])]) if any(k in durations for k in g) else None
    lines = ["Issue and memory-system counters of %s on the %s workload (rocprofv3 --pmc, per launch, average over the"
             % (", ".join(g), workload), "profiled launches; %s)" % fig["desc"], "",
             "commands (from /tmp with TMPDIR=/tmp, R = repository root), one counter group per run:"]
    lines += ["  " + x for x in commands] + ["", "raw counters:"]
    lines += ["  %-40s %.6g" % (k, v) for k, v in sorted(c.items())]
    lines += ["", "derived:"]
    cycles = None
    if "GRBM_GUI_ACTIVE" in c:
        cycles = c["GRBM_GUI_ACTIVE"] / N_XCD
        lines.append("  shader cycles per launch                 %.4g  (GRBM_GUI_ACTIVE / %d XCDs)" % (cycles, N_XCD))
        if dur_ns:
            lines.append("  mean shader clock                        %.2f GHz  (those cycles / %.3f ms, the launch's duration in this run)"
                         % (cycles / dur_ns, dur_ns / 1e6))
    elif dur_ns:
        cycles = dur_ns * NOMINAL_GHZ
        lines.append("  shader cycles per launch                 %.4g  (duration %.3f ms x the nominal %.1f GHz; GRBM_GUI_ACTIVE not collected)"
                     % (cycles, dur_ns / 1e6, NOMINAL_GHZ))
    if cycles and "SQ_VALU_MFMA_BUSY_CYCLES" in c:
        lines.append("  MFMA busy                                %.1f %%  (SQ_VALU_MFMA_BUSY_CYCLES / (%d SIMDs x shader cycles))"
                     % (100 * c["SQ_VALU_MFMA_BUSY_CYCLES"] / (N_SIMD * cycles), N_SIMD))
    if dur_ns:
        tops = fig["int8_ops"] / (dur_ns * 1e-9) / 1e12
        lines.append("  achieved int8 rate in this run           %.0f TOP/s = %.1f %% of the %.0f TOP/s peak"
                     % (tops, 100 * tops / INT8_MFMA_PEAK_TOPS, INT8_MFMA_PEAK_TOPS))
    if "SQ_INSTS_VALU_MFMA_I8" in c:
        lines.append("  int8 MFMA instructions issued            %.6g  (16x16x64: 32768 ops each -> %.4g ops; algorithmic %.4g)"
                     % (c["SQ_INSTS_VALU_MFMA_I8"], c["SQ_INSTS_VALU_MFMA_I8"] * 32768, fig["int8_ops"]))
    if "SQ_WAIT_INST_ANY" in c and "SQ_WAVE_CYCLES" in c:
        lines.append("  waves waiting on a counter               %.1f %%  (SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES)"
                     % (100 * c["SQ_WAIT_INST_ANY"] / c["SQ_WAVE_CYCLES"]))
    if "SQ_ACTIVE_INST_VALU" in c and "SQ_WAVE_CYCLES" in c:
        lines.append("  waves issuing vector-ALU work            %.1f %%  (SQ_ACTIVE_INST_VALU / SQ_WAVE_CYCLES)"
                     % (100 * c["SQ_ACTIVE_INST_VALU"] / c["SQ_WAVE_CYCLES"]))
    if "TCC_HIT_sum" in c and "TCC_MISS_sum" in c:
        lines.append("  L2 hit rate                              %.1f %%  (TCC_HIT / (TCC_HIT + TCC_MISS))"
                     % (100 * c["TCC_HIT_sum"] / (c["TCC_HIT_sum"] + c["TCC_MISS_sum"])))
    if "TCP_TCC_READ_REQ_sum" in c:
        lines.append("  L2 -> L1 read traffic                    %.2f GiB  (TCP_TCC_READ_REQ x 64 B)"
                     % (c["TCP_TCC_READ_REQ_sum"] * 64 / GIB))
        if "TCP_TOTAL_CACHE_ACCESSES_sum" in c and c["TCP_TOTAL_CACHE_ACCESSES_sum"] > 0:
            lines.append("  L1 hit rate                              %.1f %%  (1 - TCP_TCC_READ_REQ / TCP_TOTAL_CACHE_ACCESSES)"
                         % (100 * (1 - c["TCP_TCC_READ_REQ_sum"] / c["TCP_TOTAL_CACHE_ACCESSES_sum"])))
    if "TCP_TCC_READ_REQ_LATENCY_sum" in c and c.get("TCP_TCC_READ_REQ_sum"):
        lines.append("  mean L2 round trip of a read             %.0f clk  (TCP_TCC_READ_REQ_LATENCY / TCP_TCC_READ_REQ)"
                     % (c["TCP_TCC_READ_REQ_LATENCY_sum"] / c["TCP_TCC_READ_REQ_sum"]))
    if "TCP_TCC_WRITE_REQ_LATENCY_sum" in c and c.get("TCP_TCC_WRITE_REQ_sum"):
        lines.append("  mean L2 round trip of a write            %.0f clk  (TCP_TCC_WRITE_REQ_LATENCY / TCP_TCC_WRITE_REQ)"
                     % (c["TCP_TCC_WRITE_REQ_LATENCY_sum"] / c["TCP_TCC_WRITE_REQ_sum"]))
    if "TCC_EA0_RDREQ_LEVEL_sum" in c and c.get("TCC_EA0_RDREQ_sum"):
        lines.append("  mean fabric round trip of an L2 miss     %.0f clk  (TCC_EA0_RDREQ_LEVEL / TCC_EA0_RDREQ)"
                     % (c["TCC_EA0_RDREQ_LEVEL_sum"] / c["TCC_EA0_RDREQ_sum"]))
    return "\n".join(lines) + "\n"


STREAMING = re.compile(r"^(split_kernel|transpose_u64_kernel|slot_rearrange_kernel|ntt\w*_kernel|mac_intt\w*|pack_w_kernel)")


def streaming_summary(trace_dir: Optional[str], fetch_dir: str, write_dir: str, commands: Sequence[str],
                      copy_kib: float, notes: Sequence[str]) -> str:
    """The HBM-bound kernels beside the MFMA kernels: per (kernel, grid size) the launch time and the bytes the L2s
    exchanged with the fabric (FETCH_SIZE + WRITE_SIZE, scaled by the calibration copy), hence the achieved GB/s."""
    f = read_grouped(fetch_dir, "counter_collection.csv")
    w = read_grouped(write_dir, "counter_collection.csv")
    t = read_grouped(trace_dir, "kernel_trace.csv") if trace_dir else {}
    cal_f, cal_w = copy_scale([fetch_dir], "FETCH_SIZE", copy_kib), copy_scale([write_dir], "WRITE_SIZE", copy_kib)
    sf, sw = (cal_f[1] if cal_f else 1.0), (cal_w[1] if cal_w else 1.0)
    lines = ["HBM-side traffic and achieved rates of the streaming kernels (rocprofv3), per launch, by kernel and grid size", "",
             "commands (from /tmp with TMPDIR=/tmp, R = repository root):"] + ["  " + c for c in commands] + [""]
    lines.append("calibration copy (1 GiB each way): FETCH_SIZE scale %.4f, WRITE_SIZE scale %.4f" % (sf, sw))
    lines += list(notes) + ["", "%-34s %12s %6s %10s %10s %12s %12s %10s" %
                            ("kernel", "grid", "calls", "avg_ms", "min_ms", "read GiB", "written GiB", "GB/s")]
    for key in sorted(set(f) & set(w)):
        if not STREAMING.search(key[0]):
            continue
        rd = mean(f[key]["FETCH_SIZE"]) * sf * 1024.0
        wr = mean(w[key]["WRITE_SIZE"]) * sw * 1024.0
        dur = t.get(key, f[key])["dur"]              # durations of the un-instrumented trace when there is one
        lines.append("%-34s %12d %6d %10.4f %10.4f %12.3f %12.3f %10.0f" %
                     (key[0], key[1], len(dur), mean(dur) / 1e6, min(dur) / 1e6, rd / GIB, wr / GIB,
                      (rd + wr) / (mean(dur) * 1e-9) / 1e9))
    lines.append("(GB/s = (read + written) / average duration; %.0f GB/s is the HBM peak)" % HBM_PEAK_GBS)
    return "\n".join(lines) + "\n"


# --------------------------------------------------------------------------------------------------
def main(argv: Optional[Sequence[str]] = None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workload", required=True, help="name in pcmm_inputs.WORKLOADS")
    ap.add_argument("--trace", help="output directory of a rocprofv3 --kernel-trace run")
    ap.add_argument("--pmc", action="append", default=[], help="output directory of a rocprofv3 --pmc run (repeatable)")
    ap.add_argument("--command", action="append", default=[], help="a command line to quote in the summaries (repeatable)")
    ap.add_argument("--copy-kib", type=float, default=float(1 << 20), help="KiB the calibration copy reads (and writes)")
    ap.add_argument("--out-prefix", default="profiles/", help="prefix of the files written")
    ap.add_argument("--streaming-out", help="also write the summary of the HBM-bound kernels beside the MFMA kernels "
                                            "(needs --pmc directories of a FETCH_SIZE and a WRITE_SIZE run, in that order)")
    ap.add_argument("--note", action="append", default=[], help="a line to add to the streaming summary (repeatable)")
    args = ap.parse_args(argv)

    fig = workload_figures(args.workload)
    stem = "%s%s_%s" % (args.out_prefix, fig["mfma_kernel"], args.workload)
    written = []

    def put(suffix: str, text: Optional[str]):
        if text:
            with open(stem + suffix, "w") as f:
                f.write(text)
            written.append(stem + suffix)

    trace_cmds = [c for c in args.command if "--kernel-trace" in c]
    pmc_cmds = [c for c in args.command if "--pmc" in c]
    if args.trace:
        put("_kernel_trace.txt", trace_summary(args.workload, fig, read_kernel_trace(args.trace), trace_cmds))
    if args.pmc:
        counters, durations = merge_counters(args.pmc)
        put("_hbm_traffic.txt", traffic_summary(args.workload, fig, counters,
                                                [c for c in pmc_cmds if "FETCH_SIZE" in c or "WRITE_SIZE" in c], args.copy_kib,
                                                args.pmc))
        put("_counters.txt", counter_summary(args.workload, fig, counters, durations,
                                             [c for c in pmc_cmds if "FETCH_SIZE" not in c and "WRITE_SIZE" not in c]))
    if args.streaming_out:
        if len(args.pmc) < 2:
            ap.error("--streaming-out needs the FETCH_SIZE and the WRITE_SIZE run directories")
        with open(args.streaming_out, "w") as f:
            f.write(streaming_summary(args.trace, args.pmc[0], args.pmc[1], args.command, args.copy_kib, args.note))
        written.append(args.streaming_out)
    for w in written:
        print(w)
    return 0 if written else 1


if __name__ == "__main__":
    sys.exit(main())
