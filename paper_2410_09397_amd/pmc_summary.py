"""Condenses rocprofv3 output of `bench.py` into the short text summaries kept under profiles/.

Inputs are the CSV files of three profiler runs of the same bench command:
  --stats DIR   rocprofv3 --kernel-trace --stats   (per-kernel durations)
  --fetch DIR   rocprofv3 --pmc FETCH_SIZE         (with bench.py --calibrate-copy)
  --write DIR   rocprofv3 --pmc WRITE_SIZE         (with bench.py --calibrate-copy)
The byte counters are scaled by what they read for the plain 1 GiB device copy that
`--calibrate-copy` adds to the run.  Writes profiles/<kernel group>_<workload>.md and updates
profiles/hbm_traffic.json (HBM bytes of one backward call, stamped with a hash of the kernel
sources they were measured on), which bench.py reports as roofline.traffic and marks stale when
the sources have changed since.
"""
import argparse
import collections
import csv
import glob
import hashlib
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = float(1 << 30)  # bytes read, and bytes written, by the calibration copy
BWD_KERNELS = ("delta_kernel", "bwd_dkdv", "bwd_dq", "ld_scores_kernel<2>", "ld_scores_kernel<(attn::ScoreMode)2>", "ld_gemm_kernel", "generic_delta",
               "generic_dq", "generic_dkdv", "block_len_kernel", "block_order_kernel", "block_order_fused_kernel", "bwd_prep_kernel",
               "bwd_onepass_kernel", "bwd_splitd_kernel")


def source_hash():
    """sha256 over the kernel sources and the C header (names and contents, sorted): what a stored
    byte count was measured on."""
    h = hashlib.sha256()
    for d in (os.path.join(ROOT, "paper_2410_09397_amd", "csrc"), os.path.join(ROOT, "include")):
        for name in sorted(os.listdir(d)):
            path = os.path.join(d, name)
            if os.path.isfile(path):
                h.update(name.encode())
                with open(path, "rb") as fh:
                    h.update(fh.read())
    return h.hexdigest()[:16]


def traffic_key(workload, tiling):
    return workload if not tiling else "%s@tiling%d" % (workload, tiling)
FWD_KERNELS = ("fwd_kernel", "ld_scores_kernel<0>", "ld_scores_kernel<1>", "ld_scores_kernel<(attn::ScoreMode)0>",
               "ld_scores_kernel<(attn::ScoreMode)1>", "ld_lse_combine", "generic_fwd")


def _one(pattern):
    files = glob.glob(pattern, recursive=True)
    if not files:
        raise FileNotFoundError(pattern)
    return files[0]


def short(name):
    return name.replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "").replace("attn::", "")


def kernel_stats(d):
    rows = {}
    with open(_one(os.path.join(d, "**", "*kernel_stats.csv"))) as fh:
        for r in csv.DictReader(fh):
            rows[short(r["Name"])] = (int(r["Calls"]), float(r["AverageNs"]))
    return rows


COPIES = 3  # device copies that bench.py --calibrate-copy issues (the runtime may split each in several dispatches)


def counter_avg(d, counter):
    """Average counter value per dispatch and per kernel; for the calibration copy, per copy."""
    acc = collections.defaultdict(list)
    with open(_one(os.path.join(d, "**", "*counter_collection.csv"))) as fh:
        for r in csv.DictReader(fh):
            if r["Counter_Name"] == counter:
                acc[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: (sum(v) / COPIES if "copyBuffer" in k else sum(v) / len(v)) for k, v in acc.items()}


def per_call_weights(name, calls, base_calls, four_phase_bwd=True):
    """(launches per attn_bwd call, launches per attn_fwd call) of a kernel."""
    if "ld_gemm_kernel<false>" in name:  # dQ = dS K in the four-phase backward, O = P V in the large-d forward
        return (1.0, 1.0) if four_phase_bwd else (0.0, calls / float(base_calls))
    k = calls / float(base_calls)
    return (k, 0.0) if is_in(name, BWD_KERNELS) else (0.0, k)


def is_in(name, group):
    return any(g in name for g in group)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True, help="workload name as printed in bench.py's config.workload")
    ap.add_argument("--workload-index", type=int, required=True)
    ap.add_argument("--shape", default=None, help="the --shape string given to bench.py, if any")
    ap.add_argument("--extra-frac", type=float, default=None, help="the --extra-frac given to bench.py, if any")
    ap.add_argument("--tiling", type=int, default=0, help="the --tiling given to bench.py, if any")
    ap.add_argument("--stats", required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--bench-json", default=None, help="file holding the bench.py JSON line of the stats run")
    ap.add_argument("--line-only", action="store_true",
                    help="print one line (time, bytes read and written by one attn_bwd call) and write no file: sweeps")
    args = ap.parse_args()

    stats = kernel_stats(args.stats)
    fetch = counter_avg(args.fetch, "FETCH_SIZE")
    write = counter_avg(args.write, "WRITE_SIZE")
    copy_f = [v for k, v in fetch.items() if "copyBuffer" in k]
    copy_w = [v for k, v in write.items() if "copyBuffer" in k]
    if not copy_f or not copy_w:
        raise RuntimeError("calibration copy kernel not found: run bench.py with --calibrate-copy")
    # counters are in KiB-like units per dispatch: bytes = value * factor * 1024
    f_r = COPY_BYTES / 1024.0 / copy_f[0]
    f_w = COPY_BYTES / 1024.0 / copy_w[0]

    lines = []
    w = args.workload_index
    shape = (" --shape %s" % args.shape) if args.shape else ""
    if args.extra_frac is not None:
        shape += " --extra-frac %g" % args.extra_frac
    if args.tiling:
        shape += " --tiling %d" % args.tiling
    lines.append("# rocprofv3 summary: attention kernels, workload %s\n" % args.workload)
    lines.append("Commands (from the repository root, on one MI355X; `cd /tmp && export TMPDIR=/tmp` first):\n")
    lines.append("```")
    lines.append("rocprofv3 --kernel-trace --stats -d %s -o w%d --output-format csv -- python bench.py --workload %d%s "
                 "--steps 5 --warmup 2 --sustain 0 --no-kernel-split --no-cpu-baseline" % (args.stats, w, w, shape))
    for c, d in (("FETCH_SIZE", args.fetch), ("WRITE_SIZE", args.write)):
        lines.append("rocprofv3 --pmc %s -d %s -o pmc --output-format csv -- python bench.py --workload %d%s --steps 3 "
                     "--warmup 1 --sustain 0 --no-kernel-split --no-cpu-baseline --calibrate-copy" % (c, d, w, shape))
    lines.append("python -m paper_2410_09397_amd.pmc_summary --workload %s --workload-index %d%s --stats %s --fetch %s "
                 "--write %s" % (args.workload, w, shape, args.stats, args.fetch, args.write))
    lines.append("```\n")
    measured_hash = source_hash()  # replaced by the hash the profiled run itself reports, when it does
    if args.bench_json and os.path.exists(args.bench_json):
        for l in open(args.bench_json):
            if l.startswith("{"):
                j = json.loads(l)
                measured_hash = j.get("source_hash", measured_hash)
                lines.append("bench.py line of the kernel-trace run: value %.1f %s, bwd %.3f ms, fwd %.3f ms, "
                             "ms_per_step %.3f\n" % (j["value"], j["unit"], j["bwd_ms"], j["fwd_ms"], j["ms_per_step"]))
    lines.append("Calibration (plain 1 GiB device copy in the same run): FETCH_SIZE reads %.1f -> factor %.3f; "
                 "WRITE_SIZE reads %.1f -> factor %.3f (bytes = counter x factor x 1024).\n"
                 % (copy_f[0], f_r, copy_w[0], f_w))
    lines.append("| kernel | calls | avg duration (us) | HBM read (MB) | HBM written (MB) |")
    lines.append("|---|---|---|---|---|")
    tot = {"bwd": [0.0, 0.0, 0.0], "fwd": [0.0, 0.0, 0.0]}
    base_calls = max(1, min(c for n, (c, _) in stats.items() if is_in(n, BWD_KERNELS + FWD_KERNELS)))
    for name, (calls, avg) in sorted(stats.items(), key=lambda kv: -kv[1][1]):
        if not (is_in(name, BWD_KERNELS) or is_in(name, FWD_KERNELS)):
            continue
        rd = fetch.get(name, 0.0) * f_r * 1024.0
        wr = write.get(name, 0.0) * f_w * 1024.0
        # a kernel launched more than once per call (the large-d GEMM) counts that many times
        wb, wf = per_call_weights(name, calls, base_calls, any("ld_scores_kernel<2>" in n or "ScoreMode)2>" in n for n in stats))
        for grp, k in (("bwd", wb), ("fwd", wf)):
            tot[grp][0] += avg * k
            tot[grp][1] += rd * k
            tot[grp][2] += wr * k
        lines.append("| %s | %d | %.1f | %.1f | %.1f |" % (name, calls, avg / 1e3, rd / 1e6, wr / 1e6))
    lines.append("")
    for grp, label in (("bwd", "attn_bwd call (all its kernels)"), ("fwd", "attn_fwd call")):
        t = tot[grp]
        lines.append("%s: %.3f ms, HBM read %.1f MB + written %.1f MB = %.1f MB" %
                     (label, t[0] / 1e6, t[1] / 1e6, t[2] / 1e6, (t[1] + t[2]) / 1e6))
    from paper_2410_09397_amd import io_bound, synth
    wl = synth.workload(w)
    if args.shape:
        wl = synth.reshaped(wl, args.shape)
    if args.extra_frac is not None:
        wl = synth.with_density(wl, args.extra_frac)
    y = io_bound.yardstick(wl)
    bwd_bytes = tot["bwd"][1] + tot["bwd"][2]
    lines.append("\nPaper's I/O yardstick for the backward (max{compulsory, Theta-term at M = 160 KB}): %.1f MB; "
                 "measured / yardstick = %.2f" % (y / 1e6, bwd_bytes / y))
    lines.append("Algorithmic backward FLOPs %.4g -> %.1f TFLOP/s over the summed kernel durations (%.1f %% of the "
                 "2500 TFLOP/s dense bf16 MFMA peak)." % (wl.bwd_flops(), wl.bwd_flops() / (tot["bwd"][0] * 1e-9) * 1e-12,
                                                           wl.bwd_flops() / (tot["bwd"][0] * 1e-9) * 1e-12 / 25.0))
    out_dir = os.path.join(ROOT, "profiles")
    os.makedirs(out_dir, exist_ok=True)
    if args.line_only:
        print("%s tiling %d: attn_bwd %.3f ms, HBM read %.1f MB, written %.1f MB, total %.1f MB = %.2f x yardstick %.1f MB"
              % (args.workload, args.tiling, tot["bwd"][0] / 1e6, tot["bwd"][1] / 1e6, tot["bwd"][2] / 1e6, bwd_bytes / 1e6,
                 bwd_bytes / y, y / 1e6))
        return
    key = traffic_key(args.workload, args.tiling)
    lines.append("Kernel sources: hash %s (paper_2410_09397_amd.pmc_summary.source_hash)." % measured_hash)
    with open(os.path.join(out_dir, "attn_kernels_%s.md" % key.replace("@", "_")), "w") as fh:
        fh.write("\n".join(lines) + "\n")
    tpath = os.path.join(out_dir, "hbm_traffic.json")
    traffic = json.load(open(tpath)) if os.path.exists(tpath) else {}
    traffic[key] = {"bytes": bwd_bytes, "read": tot["bwd"][1], "written": tot["bwd"][2], "bwd_ms_summed": tot["bwd"][0] / 1e6,
                    "source_hash": measured_hash}
    with open(tpath, "w") as fh:
        json.dump(traffic, fh, indent=1, sort_keys=True)
    print("\n".join(lines))




# ------------------------------------------------------------------ compiler resource usage
def kernel_resources(sources=None):
    """Registers, scratch and occupancy of every kernel in the given sources (default: all of the library's), from
    hipcc -Rpass-analysis=kernel-resource-usage: a list of dicts with the compiler's field names plus "kernel"."""
    import re
    import subprocess
    from concurrent.futures import ThreadPoolExecutor
    from paper_2410_09397_amd import build as hip_build

    def one(src):
        cmd = ["hipcc", *hip_build.FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c",
               os.path.join(hip_build.CSRC, src), "-o", os.devnull]
        return subprocess.run(cmd, capture_output=True, text=True).stderr

    srcs = list(sources or hip_build.SOURCES)
    with ThreadPoolExecutor(max_workers=4) as pool:
        outputs = list(pool.map(one, srcs))
    rows = []
    for err in outputs:
        cur = None
        for line in err.splitlines():
            m = re.search(r"remark: (?:Function Name: (\S+)|\s+(\S[^:]*): (\S+))", line)
            if not m:
                continue
            if m.group(1):
                name = subprocess.run(["c++filt", m.group(1)], capture_output=True, text=True).stdout.strip()
                if name.startswith("_Z"):  # c++filt does not know the bf16 type code
                    name = re.sub(r"^_ZN4attn\d+(\w+?)IDF16bEEv.*$", r"\1<bf16>", name)
                cur = {"kernel": short(name)}
                rows.append(cur)
            elif cur is not None:
                cur[m.group(2).strip()] = m.group(3)
    return rows


def resources_main():
    """python -m paper_2410_09397_amd.pmc_summary resources  -> markdown table of registers, scratch and
    occupancy of every kernel, from hipcc -Rpass-analysis=kernel-resource-usage on the committed sources."""
    rows = kernel_resources()
    print("## Compiler resource usage (`hipcc -Rpass-analysis=kernel-resource-usage`, gfx950)\n")
    print("| kernel | VGPRs | AGPRs | scratch (bytes/lane) | occupancy (waves/SIMD) |")
    print("|---|---|---|---|---|")
    for r in rows:
        print("| %s | %s | %s | %s | %s |" % (r["kernel"], r.get("VGPRs", "?"), r.get("AGPRs", "?"),
                                         r.get("ScratchSize [bytes/lane]", "?"), r.get("Occupancy [waves/SIMD]", "?")))


# ------------------------------------------------------------------------------ SQ counters
SQ_PASSES = (
    "SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_VALU "
    "SQ_VALU_MFMA_BUSY_CYCLES SQ_ACTIVE_INST_LDS",
    "SQ_INSTS_VALU SQ_INSTS_MFMA SQ_INSTS_LDS SQ_INSTS_SALU SQ_INSTS_VALU_TRANS_F32 SQ_INST_LEVEL_LDS SQ_INSTS_VMEM "
    "SQ_LDS_BANK_CONFLICT",
    "SQ_LDS_IDX_ACTIVE SQ_LDS_ADDR_CONFLICT SQ_LDS_DATA_FIFO_FULL SQ_LDS_CMD_FIFO_FULL SQ_BUSY_CU_CYCLES "
    "SQ_ACTIVE_INST_ANY SQ_VALU_MFMA_COEXEC_CYCLES SQ_ACTIVE_INST_MISC",
)


def sq_main(argv):
    """python -m paper_2410_09397_amd.pmc_summary sq --workload NAME --bench-args "..." DIR1 DIR2 DIR3
    -> profiles/sq_counters_<NAME>.md from the three rocprofv3 --pmc passes listed in SQ_PASSES."""
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--bench-args", default="")
    ap.add_argument("--resources", default=None, help="file with the compiler's kernel-resource-usage table to append")
    ap.add_argument("dirs", nargs=3)
    args = ap.parse_args(argv)
    vals = collections.defaultdict(dict)
    for d in args.dirs:
        acc = collections.defaultdict(list)
        with open(_one(os.path.join(d, "**", "*counter_collection.csv"))) as fh:
            for r in csv.DictReader(fh):
                acc[(short(r["Kernel_Name"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
        for (k, c), v in acc.items():
            vals[k][c] = sum(v) / len(v)
    kernels = [k for k in vals if is_in(k, BWD_KERNELS + FWD_KERNELS + ("mfma_ceiling_kernel",)) and vals[k].get("SQ_INSTS_MFMA", 0) > 0]
    lines = ["# SQ counters of the attention kernels, workload %s\n" % args.workload,
             "Three `rocprofv3 --pmc` passes of the same command (8 SQ counters each; from the repository root on one MI355X,",
             "after `cd /tmp && export TMPDIR=/tmp`), then this summary:\n", "```"]
    for i, p in enumerate(SQ_PASSES):
        lines.append("rocprofv3 --pmc %s -d %s -o pmc --output-format csv -- python bench.py %s --steps 3 --warmup 1 --sustain 0 "
                     "--no-kernel-split --no-cpu-baseline" % (p, args.dirs[i], args.bench_args))
    lines.append("python -m paper_2410_09397_amd.pmc_summary sq --workload %s --bench-args \"%s\" %s" %
                 (args.workload, args.bench_args, " ".join(args.dirs)))
    lines.append("```\n")
    lines.append("Values are averages per dispatch, summed over the device.  `mfma_ceiling_kernel` is the library's register-only MFMA loop")
    lines.append("(two waves per SIMD, nothing but MFMAs), which `bench.py` runs at the end: its row shows what the counters read for a matrix")
    lines.append("pipe that is never idle.\n")
    counters = [c for p in SQ_PASSES for c in p.split()]
    lines.append("| counter | " + " | ".join(kernels) + " |")
    lines.append("|---|" + "---|" * len(kernels))
    for c in counters:
        lines.append("| %s | " % c + " | ".join("%.4g" % vals[k].get(c, float("nan")) for k in kernels) + " |")
    lines.append("\nDerived:\n")
    lines.append("| ratio | " + " | ".join(kernels) + " |")
    lines.append("|---|" + "---|" * len(kernels))

    def ratio(a, b, scale=1.0):
        return " | ".join("%.3f" % (scale * vals[k].get(a, float("nan")) / vals[k][b]) if vals[k].get(b) else "-" for k in kernels)
    lines.append("| MFMA busy cycles / (4 SIMDs x CU busy cycles) | %s |" % ratio("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES", 0.25))
    lines.append("| VALU instructions (incl. MFMA) per MFMA | %s |" % ratio("SQ_INSTS_VALU", "SQ_INSTS_MFMA"))
    lines.append("| transcendental instructions per MFMA | %s |" % ratio("SQ_INSTS_VALU_TRANS_F32", "SQ_INSTS_MFMA"))
    lines.append("| LDS instructions per MFMA | %s |" % ratio("SQ_INSTS_LDS", "SQ_INSTS_MFMA"))
    lines.append("| SALU instructions per MFMA | %s |" % ratio("SQ_INSTS_SALU", "SQ_INSTS_MFMA"))
    lines.append("| LDS bank-conflict cycles / LDS active cycles | %s |" % ratio("SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE"))
    lines.append("| LDS data-FIFO-full cycles / CU busy cycles | %s |" % ratio("SQ_LDS_DATA_FIFO_FULL", "SQ_BUSY_CU_CYCLES"))
    lines.append("| wave cycles waiting on LDS instructions / wave cycles | %s |" % ratio("SQ_WAIT_INST_LDS", "SQ_WAVE_CYCLES"))
    lines.append("| wave cycles waiting on any instruction / wave cycles | %s |" % ratio("SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES"))
    lines.append("| MFMA and VALU co-executing cycles / MFMA busy cycles | %s |" % ratio("SQ_VALU_MFMA_COEXEC_CYCLES", "SQ_VALU_MFMA_BUSY_CYCLES"))
    if args.resources and os.path.exists(args.resources):
        lines.append("\n" + open(args.resources).read().rstrip())
    lines.append("\nKernel sources: hash %s." % source_hash())
    out = os.path.join(ROOT, "profiles", "sq_counters_%s.md" % args.workload)
    with open(out, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    import sys
    if len(sys.argv) > 1 and sys.argv[1] == "sq":
        sq_main(sys.argv[2:])
    elif len(sys.argv) > 1 and sys.argv[1] == "resources":
        resources_main()
    else:
        main()
