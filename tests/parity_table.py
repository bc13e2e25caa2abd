"""Turns the JSON lines that the GPU parity tests record (ATTN_PARITY_RECORD=<file>, one line per
checked tensor) into the table kept as profiles/parity_errors.md:
    ATTN_PARITY_RECORD=gpurun_out/parity.jsonl ATTN_PARITY_RECORD_ONLY=1 python -m pytest tests -m gpu -q
    python -m tests.parity_table gpurun_out/parity.jsonl > profiles/parity_errors.md
"""
import collections
import json
import sys


def main(path):
    rows = [json.loads(l) for l in open(path)]
    out = ["# Observed parity errors of the GPU path against the float64 oracle\n",
           "Made by `python -m tests.parity_table` from the lines the GPU tests record (commands in that file's",
           "docstring).  Two figures per checked tensor: `max|x - ref| / max|ref|` (the gate: <= 2e-2 for bf16, <= 1e-4 for fp32)",
           "and the elementwise relative error `max(|x - ref| / max(|ref|, 1e-3 max|ref|))`.  Isolated = the backward is fed the",
           "oracle's O (rounded to the storage type) and LSE on both sides; chained = the GPU backward consumes the GPU",
           "forward's own bf16 O and fp32 LSE while the oracle chains its exact ones.\n",
           "## Largest error per output and kind of comparison\n",
           "| storage | tensor | comparison | tensors checked | max-normalised (worst case) | elementwise, floor 1e-3 max (worst case) |",
           "|---|---|---|---|---|---|"]
    groups = collections.defaultdict(list)
    for r in rows:
        kind = "forward" if r["tensor"] == "O" else ("chained" if r.get("chained") else "isolated")
        groups[(r["dtype"], r["tensor"], kind)].append(r)
    for key in sorted(groups):
        v = groups[key]
        a = max(v, key=lambda r: r["max_normalised"])
        b = max(v, key=lambda r: r["elementwise"])
        out.append("| %s | %s | %s | %d | %.2e (%s) | %.2e (%s) |" % (*key, len(v), a["max_normalised"], a["case"],
                                                                     b["elementwise"], b["case"]))
    out.append("\n## The five workloads of the metric at full size (sampled rows of three heads; chained)\n")
    out.append("| workload | tensor | max-normalised | elementwise, floor 1e-3 max |")
    out.append("|---|---|---|---|")
    full = collections.defaultdict(list)
    for r in rows:
        if r["case"].startswith("cfg") and " head " in r["case"]:
            full[(r["case"].split(" head ")[0], r["tensor"])].append(r)
    for key in sorted(full):
        v = full[key]
        out.append("| %s | %s | %.2e | %.2e |" % (*key, max(r["max_normalised"] for r in v), max(r["elementwise"] for r in v)))
    print("\n".join(out))


if __name__ == "__main__":
    main(sys.argv[1])
