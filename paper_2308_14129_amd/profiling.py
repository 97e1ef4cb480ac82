"""Turns rocprofv3 output of `bench.py` runs into the short text summaries kept under profiles/.

    python -m paper_2308_14129_amd.profiling kernels  <workload> <precision> <batch> \
        <dir of a --kernel-trace --stats run> <out.md> [--note TEXT]
    python -m paper_2308_14129_amd.profiling counters <workload> <precision> <batch> <out.md> \
        --fetch <dir> --write <dir> [--mfma <dir>] [--note TEXT]

Both write one "- `key`: value" line per figure, among them the hash of the kernel sources the
run was measured on; bench.py takes `roofline.traffic`, the MFMA-busy figures and the trace
durations it quotes from these files, and only while the sources are still those.

HBM bytes: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by what the same counter
reads for the plain 256 MiB device copies that `bench.py --pmc-calibration` appends to the run.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import os
import re
import sys
from collections import defaultdict

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
# (a name that is the beginning of another comes after it: the first match names the kernel)
STEP_KERNELS = ("k_scatter", "k_select", "k_prepare", "k_gru", "k_embed", "k_centrality", "k_topk_keys", "k_topk_flags",
                "k_tr_gather", "k_rowgemm", "k_tr_attn_fwd", "k_tr_attn_bwd", "k_tr_scatter", "k_tr_pairs", "k_tr_logit",
                "k_tr_pair_scatter", "k_tr_gru_gates", "k_tr_gru_time", "k_gemm_tn", "k_colsum", "k_gemm64",
                "k_pack_gru", "k_pack", "k_transpose", "k_tr_update",
                "k_mod_msgsum", "k_mod_update", "k_mod_commit", "k_mod_simple", "k_mod_hop2", "k_mr_items", "k_mr_attn",
                "k_mod_decode")
COPY_KIB = 256 * 1024  # one calibration copy reads and writes this much
XCDS = 8                # accelerator dies of one MI355X


# the sources the step's kernels are compiled from (the partitioner, the epoch machinery, the training
# step and the C API's host code can change without touching what the step's profiles measured)
STEP_SOURCES = ("k_embed.hip", "k_gru.hip", "decode.h", "prepare.h", "lookup.h", "winners.h", "kernels_common.h",
                "step_small.hip", "step_launch.hip", "pack.hip")


def kernel_source_id() -> str:
    h = hashlib.sha256()
    for name in STEP_SOURCES:
        h.update(name.encode())
        h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()[:16]


def short_name(full: str) -> str | None:
    for k in STEP_KERNELS:
        if f"::{k}" in full or full.startswith(k):
            return k
    return None


def _one(pattern: str) -> str:
    hits = sorted(glob.glob(pattern, recursive=True))
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[0]


def read_counters(run_dir: str):
    """{counter: {kernel short name or full name: [values per dispatch]}} in dispatch order."""
    path = _one(os.path.join(run_dir, "**", "*counter_collection.csv"))
    out = defaultdict(lambda: defaultdict(list))
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            name = short_name(row["Kernel_Name"]) or row["Kernel_Name"]
            out[row["Counter_Name"]][name].append(float(row["Counter_Value"]))
    return out


def copy_scale(per_kernel: dict, counter: str) -> float:
    """KiB of HBM traffic per counter unit, from the last calibration copy of the run."""
    cands = [(n, v) for n, v in per_kernel.items() if short_name(n) is None and v and
             ("copy" in n.lower() or "elementwise" in n.lower())]
    best = None
    for n, v in cands:
        if v[-1] > 0.25 * COPY_KIB / 4 and (best is None or abs(v[-1] - COPY_KIB) < abs(best - COPY_KIB)):
            best = v[-1]
    if best is None:
        raise SystemExit(f"{counter}: no calibration copy found (run bench.py with --pmc-calibration)")
    return COPY_KIB / best


def cmd_kernels(args):
    path = _one(os.path.join(args.run_dir, "**", "*kernel_stats.csv"))
    rows = []
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            k = short_name(row["Name"])
            if k:
                m = re.search(r"(k_[a-z_0-9]+(?:<[^>]*>)?)", row["Name"])
                tmpl = m.group(1) if m else k
                rows.append((tmpl, int(row["Calls"]), float(row["AverageNs"]) / 1e3, float(row["MinNs"]) / 1e3,
                             float(row["MaxNs"]) / 1e3, float(row["StdDev"]) / 1e3))
    rows.sort(key=lambda r: -r[1] * r[2])
    with open(args.out, "w") as f:
        f.write(f"# Step kernels, workload {args.workload}, {args.precision}, batch {args.batch}: "
                f"rocprofv3 --kernel-trace --stats\n\n{args.note}\n\n")
        f.write(f"- `kernel_source_id`: {kernel_source_id()}\n- `workload`: {args.workload}\n"
                f"- `precision`: {args.precision}\n- `batch`: {args.batch}\n")
        seen = set()
        for r in rows:  # the variant with the most time per kernel
            k = short_name(r[0])
            if k not in seen:
                seen.add(k)
                f.write(f"- `{k}_trace_avg_us`: {r[2]:.2f}\n")
        f.write("\n")
        f.write("| kernel | calls | avg us | min us | max us | stddev us |\n|---|---|---|---|---|---|\n")
        for r in rows:
            f.write(f"| `{r[0]}` | {r[1]} | {r[2]:.2f} | {r[3]:.2f} | {r[4]:.2f} | {r[5]:.2f} |\n")
    print(open(args.out).read())


def cmd_counters(args):
    lines = [f"- `kernel_source_id`: {kernel_source_id()}", f"- `workload`: {args.workload}",
             f"- `precision`: {args.precision}", f"- `batch`: {args.batch}"]
    table = []
    fetch = read_counters(args.fetch)["FETCH_SIZE"]
    write = read_counters(args.write)["WRITE_SIZE"]
    fs, ws = copy_scale(fetch, "FETCH_SIZE"), copy_scale(write, "WRITE_SIZE")
    lines += [f"- `fetch_scale`: {fs:.4f}", f"- `write_scale`: {ws:.4f}"]
    for k in STEP_KERNELS:
        if k in fetch and k in write:
            # steady state: the second half of the launches (the first ones include warm-up steps)
            fv, wv = fetch[k][len(fetch[k]) // 2:], write[k][len(write[k]) // 2:]
            fb = sum(fv) / len(fv) * fs * 1024
            wb = sum(wv) / len(wv) * ws * 1024
            lines.append(f"- `{k}_hbm_bytes_per_launch`: {fb + wb:.0f}")
            table.append((k, len(fetch[k]), fb / 1e6, wb / 1e6))
    if args.mfma:
        c = read_counters(args.mfma)
        for k in ("k_gru", "k_embed"):
            busy, tot = c["SQ_VALU_MFMA_BUSY_CYCLES"].get(k), c["SQ_BUSY_CYCLES"].get(k)
            mops = c["SQ_INSTS_VALU_MFMA_MOPS_BF16"].get(k) or c["SQ_INSTS_VALU_MFMA_MOPS_F32"].get(k)
            act = c["GRBM_GUI_ACTIVE"].get(k)
            h = lambda v: v[len(v) // 2:]
            if mops:
                lines.append(f"- `{k}_mfma_flop_per_launch`: {sum(h(mops)) / len(h(mops)) * 512:.0f}")
            if busy and act:
                # SQ_VALU_MFMA_BUSY_CYCLES comes summed over all 1024 SIMDs (256 units x 4) and
                # GRBM_GUI_ACTIVE summed over the 8 XCDs (one eighth of it, at 2.4 GHz, is the
                # kernel's duration under the profiler): mean share of a SIMD's cycles with the
                # matrix core busy
                frac = (sum(h(busy)) / len(h(busy))) / (sum(h(act)) / len(h(act)) / XCDS * 4 * 256)
                lines.append(f"- `{k}_mfma_busy_frac`: {frac:.5f}")
            if busy and tot:
                lines.append(f"- `{k}_mfma_busy_cycles_per_launch`: {sum(h(busy)) / len(h(busy)):.0f}")
                lines.append(f"- `{k}_sq_busy_cycles_per_launch`: {sum(h(tot)) / len(h(tot)):.0f}")
            if act:
                lines.append(f"- `{k}_gpu_active_cycles_per_launch`: {sum(h(act)) / len(h(act)):.0f}")
    with open(args.out, "w") as f:
        f.write(f"# Counter figures, workload {args.workload}, {args.precision}, batch {args.batch}\n\n")
        f.write(args.note + "\n\n")
        f.write("\n".join(lines) + "\n\n")
        f.write("| kernel | launches | HBM read MB / launch | HBM written MB / launch |\n|---|---|---|---|\n")
        for k, n, fb, wb in table:
            f.write(f"| `{k}` | {n} | {fb:.2f} | {wb:.2f} |\n")
    print(open(args.out).read())


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    k = sub.add_parser("kernels")
    k.add_argument("workload")
    k.add_argument("precision")
    k.add_argument("batch")
    k.add_argument("run_dir")
    k.add_argument("out")
    k.add_argument("--note", default="")
    c = sub.add_parser("counters")
    c.add_argument("workload")
    c.add_argument("precision")
    c.add_argument("batch")
    c.add_argument("out")
    c.add_argument("--fetch", required=True)
    c.add_argument("--write", required=True)
    c.add_argument("--mfma")
    c.add_argument("--note", default="")
    args = ap.parse_args()
    {"kernels": cmd_kernels, "counters": cmd_counters}[args.cmd](args)


if __name__ == "__main__":
    sys.exit(main())
