"""Benchmark of the attention hot path on one MI355X.

A step is one pass of the whole path on one batch of seeded synthetic input that is already
resident in HBM: attn_fwd (O, LSE) followed by attn_bwd / attn_bwd_blocksparse (delta, dK/dV,
dQ).  The reported value is the metric's attention-backward TFLOP/s: algorithmic backward
FLOPs (five n x n x d contractions over visible pairs) divided by the backward's share of the
timed steps, measured with HIP events on the launch stream; ms_per_step covers forward plus
backward.  Prints one JSON line.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "attention-backward TFLOP/s (bf16, 1 GPU) + HBM bytes vs paper I/O bound"
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}  # MI355X dense MFMA bf16; fp32 vector


def cpu_baseline(w, seconds_hint=20.0):
    """The oracle's backward, timed on a bounded sample of the workload on the host cores."""
    import numpy as np
    from oracle import attn_oracle as orc
    from paper_2410_09397_amd import synth
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    n_s = min(w.n, 8192 if w.d <= 128 else 2048)  # about 10-30 s of host work at the larger shapes
    heads_s = max(1, min(w.batch * w.heads, 2 * cores))
    ws = w.small(name=w.name + "_cpu_sample", batch=1, heads=heads_s, n=n_s)
    inp = synth.make_inputs(ws)
    m = dict(causal=ws.causal, keep=inp["keep"], block=ws.block)
    O, LSE = orc.attn_fwd(inp["Q"], inp["K"], inp["V"], ws.scale, **m)
    t0 = time.perf_counter()
    orc.attn_bwd(inp["Q"], inp["K"], inp["V"], O, inp["dO"], LSE, ws.scale, **m)
    dt = time.perf_counter() - t0
    return {"value": ws.bwd_flops() / dt * 1e-12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "oracle float64 backward on %d heads of the same workload %s "
                      "(d=%d, %s%s), %.1f s" % (heads_s, "at its full n=%d" % n_s if n_s == w.n else
                                                "with n cut to %d" % n_s, ws.d,
                                                "causal" if ws.causal else "non-causal",
                                                ", block-sparse" if ws.sparse else "", dt)}


def load_traffic(name, tiling):
    """HBM bytes of one backward call from the committed rocprofv3 --pmc summary, if there is one for this
    workload and tiling, and whether the kernel sources have changed since it was measured.  The counters cannot be
    read from inside this process: the figure is a recorded one (profiles/attn_kernels_<workload>.md gives the
    commands that refresh it), and it is reported as stale when the hash stored with it no longer matches."""
    from paper_2410_09397_amd import pmc_summary
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None, None
    with open(path) as fh:
        entry = json.load(fh).get(pmc_summary.traffic_key(name, tiling))
    if entry is None:
        return None, None
    if not isinstance(entry, dict):  # a bare number: measured before hashes were stored
        return float(entry), True
    return float(entry["bytes"]), entry.get("source_hash") != pmc_summary.source_hash()


def quick_workload(index, steps=10, warmup=3):
    """One of the metric's other configurations, timed briefly with the library's own choices: median backward
    and forward time over `steps` steps (HIP events around each call)."""
    import torch
    from paper_2410_09397_amd import attn, io_bound, synth
    w = synth.workload(index)
    dt = {"bf16": torch.bfloat16, "f32": torch.float32}[w.dtype]
    inp = synth.make_inputs(w)
    Q, K, V, dO = (torch.from_numpy(inp[t]).to("cuda").to(dt) for t in ("Q", "K", "V", "dO"))
    mask = attn.BlockMask(inp["keep"], w.block, w.n) if w.sparse else None
    O, LSE = torch.empty_like(Q), torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(Q) for _ in range(3))
    ws = torch.empty(max(attn.attn_workspace_bytes(attn._desc(Q, w.scale, w.causal), mask), 256), dtype=torch.uint8, device="cuda")
    fwd_t, bwd_t = [], []
    for k in range(warmup + steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        attn.attn_fwd(Q, K, V, w.scale, causal=w.causal, mask=mask, out=(O, LSE), workspace=ws)
        e[1].record()
        if mask is not None:
            attn.attn_bwd_blocksparse(Q, K, V, O, dO, LSE, w.scale, mask, causal=w.causal, out=grads, workspace=ws)
        else:
            attn.attn_bwd(Q, K, V, O, dO, LSE, w.scale, causal=w.causal, out=grads, workspace=ws)
        e[2].record()
        torch.cuda.synchronize()
        if k >= warmup:
            fwd_t.append(e[0].elapsed_time(e[1]))
            bwd_t.append(e[1].elapsed_time(e[2]))
    fwd_ms, bwd_ms = sorted(fwd_t)[steps // 2], sorted(bwd_t)[steps // 2]
    traffic, stale = load_traffic(w.name, 0)
    tf = w.bwd_flops() / (bwd_ms * 1e-3) * 1e-12
    return {"workload": w.name, "dtype": w.dtype, "steps": steps, "bwd_ms": bwd_ms, "fwd_ms": fwd_ms, "bwd_tflops": tf,
            "frac": tf / PEAK_TFLOPS[w.dtype], "fwd_tflops": w.fwd_flops() / (fwd_ms * 1e-3) * 1e-12,
            "traffic": traffic, "traffic_stale": stale,
            "traffic_over_yardstick": (traffic / io_bound.report(w)["yardstick_bytes"]) if traffic else None}


def mfma_ceiling(attn, torch, zero_operands, iters=150000):
    """Rate and clock of the library's register-only MFMA loop: a short warm-up launch, then `iters`
    iterations (about 40 ms at the clock random operands allow)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    attn.attn_mfma_ceiling(20000, zero_operands)
    torch.cuda.synchronize()
    e0.record()
    clock, flops = attn.attn_mfma_ceiling(iters, zero_operands)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    return {"tflops": flops / (ms * 1e-3) * 1e-12, "clock_ghz": float(clock.item()), "ms": ms, "iters": iters}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3, help="1..5, index into the metric's configurations")
    ap.add_argument("--shape", default=None, help="batch,heads,n,d[,causal]: replace the workload's sizes (sweeps); "
                                                  "the JSON line then names the derived workload")
    ap.add_argument("--extra-frac", type=float, default=None,
                    help="block-sparse workload only: share of non-diagonal key blocks kept per query-block row")
    ap.add_argument("--per-head-masks", action="store_true",
                    help="block-sparse workload: a different block mask for every (batch, head) pair (sweeps)")
    ap.add_argument("--tiling", type=int, default=0,
                    help="attn_bwd_tiling of include/attn_mi355x.h (0 = the library's choice, 1 = two kernels, "
                         "2 / 3 = one pass with 64 / 128 keys per workgroup, 6 = four-phase scheme, 7 = fused split-d)")
    ap.add_argument("--sustain", type=float, default=1.0,
                    help="seconds of back-to-back steps after the timed ones for the `sustained` figure (0 = none)")
    ap.add_argument("--no-kernel-split", action="store_true",
                    help="do not time the two kernels of the two-kernel tiling one at a time (profiling runs: "
                         "every launch of the run then belongs to a whole step)")
    ap.add_argument("--other-workloads", dest="other_workloads", action="store_true", default=None,
                    help="also time the metric's other configurations briefly (10 steps each) and report them in "
                         "\"other_workloads\" (default: only beside the plain default run)")
    ap.add_argument("--no-other-workloads", dest="other_workloads", action="store_false")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--wgrad", action="store_true",
                    help="also time attn_bwd_wgrad (the paper's weight gradient) on the same shape and "
                         "report it in an extra \"wgrad\" object (bf16, d <= 256, no block mask only)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy, so that HBM byte counters read in the "
                         "same profiler run can be scaled by a transfer of known size")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="diagnostic: time the register-only MFMA loop of the library on random and on zero "
                         "operands (the power-limited ceiling of the matrix pipe), print one JSON line and exit")
    ap.add_argument("--zero-operands", action="store_true",
                    help="diagnostic: run the workload on all-zero Q, K, V, dO (same instruction stream, no "
                         "switching activity); the line is marked and is not a benchmark result")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2410_09397_amd import attn, io_bound, pmc_summary, synth
    if args.mfma_ceiling:
        print(json.dumps({"probe": "mfma_ceiling", "unit": "TFLOP/s", "nominal_peak": PEAK_TFLOPS["bf16"],
                          **{kind: mfma_ceiling(attn, torch, mode) for kind, mode in
                             (("random", 0), ("zeros", 1), ("random_b_operand_from_lds", 2),
                              ("random_b_from_lds_plus_vector_arithmetic", 3), ("dkdv_tile_loop_without_dependencies", 4))}}))
        return
    w = synth.workload(args.workload)
    if args.shape:
        w = synth.reshaped(w, args.shape)
    if args.extra_frac is not None:
        w = synth.with_density(w, args.extra_frac)
    if args.per_head_masks:
        if not w.sparse:
            sys.exit("--per-head-masks applies to the block-sparse workload")
        w = dataclasses.replace(w, name=w.name + "_masks_per_head", per_head_masks=True)
    dt = {"bf16": torch.bfloat16, "f32": torch.float32}[w.dtype]
    inp = synth.make_inputs(w)
    Q, K, V, dO = (torch.from_numpy(inp[t]).to("cuda").to(dt) for t in ("Q", "K", "V", "dO"))
    if args.zero_operands:
        for t in (Q, K, V, dO):
            t.zero_()
    mask = attn.BlockMask(inp["keep"], w.block, w.n) if w.sparse else None
    O = torch.empty_like(Q)
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(Q) for _ in range(3))
    desc = attn._desc(Q, w.scale, w.causal, args.tiling)
    ws = torch.empty(max(attn.attn_workspace_bytes(desc, mask), 256), dtype=torch.uint8, device="cuda")

    def bwd(tiling):
        if mask is not None:
            attn.attn_bwd_blocksparse(Q, K, V, O, dO, LSE, w.scale, mask, causal=w.causal, out=grads, workspace=ws,
                                      tiling=tiling)
        else:
            attn.attn_bwd(Q, K, V, O, dO, LSE, w.scale, causal=w.causal, out=grads, workspace=ws, tiling=tiling)

    def step(ev=None):
        attn.attn_fwd(Q, K, V, w.scale, causal=w.causal, mask=mask, out=(O, LSE), workspace=ws)
        if ev:
            ev[0].record()
        bwd(args.tiling)
        if ev:
            ev[1].record()

    for _ in range(args.warmup):
        step()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    bwd_times = sorted(a.elapsed_time(b) for a, b in events)
    bwd_ms_mean = sum(bwd_times) / args.steps
    bwd_ms = bwd_times[args.steps // 2] if args.steps % 2 else 0.5 * (bwd_times[args.steps // 2 - 1] + bwd_times[args.steps // 2])

    # the same step back to back for at least a second after the timed steps: the clock of the part follows its
    # power draw, and a window of a few milliseconds still sees the clock the idle part started from
    sustained = None
    if args.sustain > 0:
        sev, t1 = [], time.perf_counter()
        while time.perf_counter() - t1 < args.sustain and len(sev) < 20000:
            batch = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
            for ev in batch:
                step(ev)
            torch.cuda.synchronize()
            sev += batch
        st = sorted(a.elapsed_time(b) for a, b in sev)
        sustained = {"seconds": time.perf_counter() - t1, "steps": len(sev), "bwd_ms_median": st[len(st) // 2],
                     "bwd_ms_mean": sum(st) / len(st),
                     "bwd_tflops": w.bwd_flops() / (st[len(st) // 2] * 1e-3) * 1e-12}

    # the two kernels of the two-kernel tiling one at a time (the library runs one of them alone on request)
    kernels = None
    if (not args.no_kernel_split and w.dtype == "bf16" and w.d in (64, 128, 256) and args.tiling in (0, 1)
            and (not w.sparse or w.block == 128)):
        kernels = []
        pairs = w.batch * w.heads * float(w.n) * w.n * w.kept_fraction()  # visible (query, key) pairs
        for name, part, mults in (("bwd_dq_kernel (+ delta)", attn.ATTN_BWD_PART_DQ, 6), ("bwd_dkdv_kernel", attn.ATTN_BWD_PART_DKDV, 8)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            bwd(part)
            e0.record()
            for _ in range(args.steps):
                bwd(part)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            ex = mults * w.d * pairs / (ms * 1e-3) * 1e-12
            kernels.append({"kernel": name, "ms": ms, "flops_per_pair_executed": "%dd" % mults,
                            "executed_tflops": ex, "frac_executed": ex / PEAK_TFLOPS["bf16"]})
        bwd(args.tiling)  # leave the outputs of a whole call behind
    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    fwd_ms = ms_per_step - bwd_ms_mean
    bwd_tflops = w.bwd_flops() / (bwd_ms * 1e-3) * 1e-12

    peak = PEAK_TFLOPS[w.dtype]
    traffic, traffic_stale = load_traffic(w.name, args.tiling)
    bound = io_bound.report(w)
    out = {
        "metric": METRIC, "value": bwd_tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype,
        "data": "all-zero operands (diagnostic, not a benchmark result)" if args.zero_operands else "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "heads": w.heads, "n": w.n, "d": w.d,
                   "causal": w.causal, "block_sparse": w.sparse, "step": "attn_fwd + attn_bwd",
                   "bwd_tiling": args.tiling},
        "value_is": "median over the timed steps of (algorithmic backward FLOPs / time between the HIP events around attn_bwd)",
        "value_mean": w.bwd_flops() / (bwd_ms_mean * 1e-3) * 1e-12,
        "bwd_ms": bwd_ms, "bwd_ms_mean": bwd_ms_mean, "bwd_ms_min": bwd_times[0], "bwd_ms_max": bwd_times[-1],
        "sustained": sustained,
        "fwd_ms": fwd_ms, "fwd_tflops": w.fwd_flops() / (fwd_ms * 1e-3) * 1e-12,
        "step_tflops": (w.fwd_flops() + w.bwd_flops()) / (ms_per_step * 1e-3) * 1e-12,
        "roofline": {"bound": "mfma" if w.dtype == "bf16" else "alu", "kernel": "attn_bwd (all kernels of one call)",
                     "achieved": bwd_tflops, "peak": peak, "unit": "TFLOP/s", "frac": bwd_tflops / peak,
                     "traffic": traffic, "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc, recorded)",
                     "traffic_stale": traffic_stale, "kernels": kernels},
        "io_bound": bound,
        "source_hash": pmc_summary.source_hash(),  # of csrc/ and include/: what this line was measured on
        "traffic_over_yardstick": (traffic / bound["yardstick_bytes"]) if traffic else None,
    }
    if w.dtype == "bf16":
        # context for `frac`: what a register-only MFMA loop sustains on this GPU for random operands
        # (the clock under matrix load follows the power the data draws; `peak` assumes 2.4 GHz)
        out["mfma_ceiling_random_operands"] = mfma_ceiling(attn, torch, 0)
    if args.wgrad and w.dtype == "bf16" and w.d in (64, 128, 256) and not w.sparse:
        del grads, O, ws
        wi = synth.make_wgrad_inputs(w)
        A1, A2, A3, X, Y, G = (torch.from_numpy(wi[t]).to("cuda").to(dt) for t in ("A1", "A2", "A3", "X", "Y", "dO"))
        g = torch.empty((w.batch, w.heads, w.d, w.d), dtype=torch.float32, device="cuda")
        wws = torch.empty(attn.attn_wgrad_workspace_bytes(desc), dtype=torch.uint8, device="cuda")
        for _ in range(args.warmup):
            attn.attn_bwd_wgrad(A1, A2, A3, X, Y, G, scale=1.0, causal=w.causal, out=g, workspace=wws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            attn.attn_bwd_wgrad(A1, A2, A3, X, Y, G, scale=1.0, causal=w.causal, out=g, workspace=wws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        # the paper's algorithm: A = S A_2^T, q = dO h^T, T = A_1^T p (n x n x d each, over visible pairs) and
        # S = A_1 X, h = A_3 Y, g = T A_2 (n x d x d each)
        bh = w.batch * w.heads
        flops = bh * (6.0 * w.n * w.n * w.d * w.kept_fraction() + 6.0 * w.n * w.d * w.d)
        out["wgrad"] = {"ms": ms, "algorithmic_tflops": flops / (ms * 1e-3) * 1e-12,
                        "note": "projections + forward + dQ kernel + A_1^T dQ; executes 10 n^2 d per pair"}
    if args.other_workloads is None:  # by default only beside the plain default run
        args.other_workloads = (args.workload == 3 and not args.shape and args.extra_frac is None and not args.tiling and not args.per_head_masks
                                and not args.zero_operands and not args.calibrate_copy and not args.no_kernel_split)
    if args.other_workloads:
        out["other_workloads"] = [quick_workload(i) for i in (1, 2, 4, 5) if i != args.workload]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
