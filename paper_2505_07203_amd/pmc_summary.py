#!/usr/bin/env python3
"""Turns rocprofv3 output of `bench.py` runs into the short text summaries kept under profiles/.

    python -m paper_2505_07203_amd.pmc_summary --workload llama8b_32k \\
        --trace DIR --fetch DIR --write DIR [--sq DIR] --out-dir profiles

DIRs are the `-d` folders of four rocprofv3 runs of the SAME bench command (the command lines are printed into the
summaries): `--kernel-trace --stats`, `--pmc FETCH_SIZE`, `--pmc WRITE_SIZE` and, optionally, a pass of SQ / GRBM
counters.  FETCH_SIZE and WRITE_SIZE count KiB per dispatch; each is scaled by what the same counter reads for the
copy kernel of known size that `bench.py --copy-calibration` launches (stream_copy_kernel: 2^30 bytes read, 2^30
written).  The traffic summary ends with machine-readable lines

    traffic_bytes_per_launch<TAB>class<TAB>kernel function<TAB>bytes
    kernel_sources_sha256<TAB>hex

which bench.py reads back for `roofline.traffic`; it ignores them when the kernel sources have changed since.
"""
import argparse
import collections
import csv
import glob
import hashlib
import os

HERE = os.path.dirname(os.path.abspath(__file__))
KERNEL_SOURCES = ("gemm_mfma.hip", "gemm_common.h", "attn_mfma.hip", "kernels_basic.hip")

# kernel class -> substring of the kernel's demangled name
CLASSES = collections.OrderedDict([
    ("attention", "attn_fwd64_kernel"),
    ("gate_up", "gemm_bf16_mfma_kernel<2, "),          # either tile height
    ("residual", "gemm_bf16_mfma_kernel<1, "),
    ("qkv", "gemm_bf16_mfma_kernel<3, "),
    ("attention_redo", "attn_fwd_kernel<128, 1, 8, false>"),
    ("rmsnorm", "rmsnorm_bf16_vec_kernel"),
    ("lm_head", "lm_head_kernel"),
    ("embed", "embed_kernel"),
    ("copy_calibration", "stream_copy_kernel"),
])


def kernel_sources_sha256():
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(HERE, "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def classify(name):
    for cls, sub in CLASSES.items():
        if sub in name:
            return cls
    return None


def read_counters(d):
    """-> {class: {counter: [values per dispatch]}}"""
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
        with open(f, newline="") as fh:
            for row in csv.DictReader(fh):
                cls = classify(row["Kernel_Name"])
                if cls:
                    out[cls][row["Counter_Name"]].append(float(row["Counter_Value"]))
    return out


def short_name(name):
    """A kernel's demangled name without return type, namespaces and argument list (template arguments kept)."""
    for drop in ("void ", "(anonymous namespace)::", "po::"):
        name = name.replace(drop, "")
    depth = 0
    for i, ch in enumerate(name):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return name[:i]
    return name


def read_stats(d):
    """-> [(short kernel name, class or '', calls, average ns, min ns, max ns)] from the kernel-trace statistics"""
    out = []
    for f in glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True):
        with open(f, newline="") as fh:
            for row in csv.DictReader(fh):
                out.append((short_name(row["Name"]), classify(row["Name"]) or "", int(row["Calls"]),
                            float(row["AverageNs"]), float(row["MinNs"]), float(row["MaxNs"])))
    return out


def mean(v):
    return sum(v) / len(v) if v else float("nan")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="llama8b_32k")
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--sq")
    common = "--copy-calibration --no-cpu-baseline --no-phase-timing --no-clock-sample --no-extras"
    ap.add_argument("--bench-flags", default="--steps 1 --warmup 0 " + common,
                    help="bench.py flags of the counter passes (one prefill: counter collection serialises dispatches)")
    ap.add_argument("--trace-flags", default="--steps 3 --warmup 1 " + common,
                    help="bench.py flags of the kernel-trace pass")
    ap.add_argument("--tag", default="", help="suffix of the summaries' file names, e.g. fp8 for a run with --fp8")
    ap.add_argument("--stem", default="", help="file-name stem of the summaries (default prefill_<workload>[_<tag>])")
    ap.add_argument("--trace-cmd", default="", help="the whole traced command, when it is not a --workload run of bench.py")
    ap.add_argument("--trace-log", default="", help="stdout of the traced command: its JSON line is quoted under the table")
    ap.add_argument("--out-dir", default=os.path.join(os.path.dirname(HERE), "profiles"))
    a = ap.parse_args()
    os.makedirs(a.out_dir, exist_ok=True)
    stem = a.stem or f"prefill_{a.workload}" + (f"_{a.tag}" if a.tag else "")
    trace_cmd = a.trace_cmd or f"python3 bench.py --workload {a.workload} {a.trace_flags}"
    cmd = f"python3 bench.py --workload {a.workload} {a.bench_flags}"
    if a.trace:
        st = read_stats(a.trace)
        path = os.path.join(a.out_dir, stem + "_kernel_trace.txt")
        with open(path, "w") as f:
            f.write(f"rocprofv3 kernel trace summary: {trace_cmd}\n")
            f.write("command (from the repository root, on the MI355X box):\n  rocprofv3 --kernel-trace --stats "
                    f"--output-format csv -d <dir> -- {trace_cmd}\n")
            f.write("then: python3 -m paper_2505_07203_amd.pmc_summary --trace <dir> [--trace-log <stdout of that run>] "
                    "[--stem / --tag / --trace-cmd / --trace-flags as above]\n")
            f.write("(every prefill of the run is in the table, warm-up included, and the kernels of the model load; microseconds)\n\n")
            f.write(f"{'kernel':44s} {'class':16s} {'calls':>6s} {'average us':>11s} {'min us':>9s} {'max us':>9s} {'total ms':>9s} {'%':>6s}\n")
            tot = sum(c * ns for _, _, c, ns, _, _ in st)
            for name, cls, calls, ns, lo, hi in sorted(st, key=lambda r: -r[2] * r[3]):
                f.write(f"{name[:44]:44s} {cls:16s} {calls:6d} {ns / 1e3:11.1f} {lo / 1e3:9.1f} {hi / 1e3:9.1f} "
                        f"{calls * ns / 1e6:9.2f} {100.0 * calls * ns / tot:6.2f}\n")
            f.write(f"\nsum over all kernels: {tot / 1e6:.2f} ms\n")
            if a.trace_log:
                # what the traced command itself printed (bench.py's JSON line), for the throughput under the profiler
                import json
                with open(a.trace_log) as lf:
                    lines = [l for l in lf if l.startswith('{"metric"')]
                if lines:
                    d = json.loads(lines[-1])
                    e, h = d.get("end_to_end", {}), d.get("peak_hbm_bytes", {})
                    f.write(f"\nthe traced run's own bench line: {d['value']:.0f} {d['unit']}, {d['ms_per_step']:.1f} ms per step, "
                            f"{e.get('frac_of_bf16_mfma_peak', float('nan')):.3f} of the nominal bf16 peak, weights "
                            f"{h.get('weights_arena', 0) / 1e9:.2f} GB + workspace {h.get('workspace_arena', 0) / 1e9:.2f} GB\n")
        print("wrote", path)
    if a.fetch and a.write:
        fe, wr = read_counters(a.fetch), read_counters(a.write)
        sq = read_counters(a.sq) if a.sq else {}
        cal_f = mean(fe["copy_calibration"]["FETCH_SIZE"])
        cal_w = mean(wr["copy_calibration"]["WRITE_SIZE"])
        kib = float(1 << 20)                                  # the calibration kernel moves 2^20 KiB each way
        ff, fw = kib / cal_f, kib / cal_w
        path = os.path.join(a.out_dir, stem + "_pmc_counters.txt")
        with open(path, "w") as f:
            f.write(f"rocprofv3 counter summary: whole prefill path, workload {a.workload}\n")
            f.write("commands (from the repository root, on the MI355X box; one pass per run, counters only):\n")
            f.write(f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <fetch dir> -- {cmd}\n")
            f.write(f"  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <write dir> -- {cmd}\n")
            if a.sq:
                f.write(f"  rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE "
                        f"SQ_ACTIVE_INST_VALU SQ_INSTS_VALU GRBM_GUI_ACTIVE --output-format csv -d <sq dir> -- {cmd}\n")
            f.write("then: python3 -m paper_2505_07203_amd.pmc_summary --fetch <fetch dir> --write <write dir> [--sq <sq dir>]\n")
            f.write("(one prefill is counted; values are means per dispatch of each kernel; counter collection serialises dispatches)\n\n")
            f.write("calibration (stream_copy_kernel: 2^30 bytes read, 2^30 bytes written)\n")
            f.write(f"  FETCH_SIZE reads {cal_f:12.1f} for 1048576 KiB fetched  -> true KiB = {ff:.5f} x counter\n")
            f.write(f"  WRITE_SIZE reads {cal_w:12.1f} for 1048576 KiB written  -> true KiB = {fw:.5f} x counter\n\n")
            f.write(f"{'kernel class':18s} {'launches':>8s} {'FETCH_SIZE':>12s} {'WRITE_SIZE':>12s} {'traffic GB':>11s}\n")
            traffic = {}
            for cls in CLASSES:
                if cls == "copy_calibration" or cls not in fe:
                    continue
                f_kib, w_kib = mean(fe[cls]["FETCH_SIZE"]), mean(wr[cls]["WRITE_SIZE"])
                traffic[cls] = (f_kib * ff + w_kib * fw) * 1024.0
                f.write(f"{cls:18s} {len(fe[cls]['FETCH_SIZE']):8d} {f_kib:12.1f} {w_kib:12.1f} {traffic[cls] / 1e9:11.3f}\n")
            if sq:
                f.write("\nmatrix-core and LDS counters (SQ counters are sums over the chip, GRBM_GUI_ACTIVE over the 8 XCDs)\n")
                f.write(f"{'kernel class':18s} {'GUI cycles/8':>13s} {'MFMA busy/1024 SIMDs':>21s} {'MFMA busy / GUI':>16s} "
                        f"{'VALU insts':>11s} {'LDS conflict / LDS active':>26s}\n")
                for cls in ("attention", "gate_up", "residual", "qkv"):
                    if cls not in sq:
                        continue
                    c = {k: mean(v) for k, v in sq[cls].items()}
                    gui = c.get("GRBM_GUI_ACTIVE", float("nan")) / 8
                    mf = c.get("SQ_VALU_MFMA_BUSY_CYCLES", float("nan")) / 1024
                    lds = c.get("SQ_LDS_BANK_CONFLICT", 0.0) / max(c.get("SQ_LDS_IDX_ACTIVE", 1.0), 1.0)
                    f.write(f"{cls:18s} {gui:13.4g} {mf:21.4g} {mf / gui:16.3f} {c.get('SQ_INSTS_VALU', float('nan')):11.4g} {lds:26.4f}\n")
            f.write("\n")
            for cls in ("attention", "gate_up", "residual", "qkv"):
                if cls in traffic:
                    f.write(f"traffic_bytes_per_launch\t{cls}\t{CLASSES[cls]}\t{traffic[cls]:.0f}\n")
            f.write(f"kernel_sources_sha256\t{kernel_sources_sha256()}\n")
        print("wrote", path)


if __name__ == "__main__":
    main()
