#!/usr/bin/env python3
"""Benchmark of the per-GPU GCN hot path on one MI355X.

Default workload (the one the headline metric is quoted on): configs[3], ONE GPU's SHARD of a
billion-edge graph -- a 7M x 28M double-permuted adjacency block with ~200M stored entries,
feature slice 28M x 32, weight slice 32 x 128 (fp32).  One "step" = one GCN layer forward +
backward over it (every row of the hot path: sparse product, dense product, activation, activation
gradient, transposed sparse product, the two backward dense products), run in the paper's order
(Eq. 2.1 then 2.2: aggregate at width 32, then combine).  `--workload tiny|social|copurchase|road`
times a whole L-layer network forward + backward (with the loss head) on one of the four graph
workloads instead.  Inputs are synthetic, seeded, generated on the GPU and resident in HBM
before the timed region.

Prints ONE JSON line.  `value` is the first of `--trials` repetitions of K steps timed with the
per-kernel event timing OFF; the per-kernel figures come from K more steps with it on.  Besides the
contract keys the line carries
  "roofline":     the dominant kernel against 8 TB/s: `achieved` = MEASURED HBM bytes per launch (rocprofv3
                  FETCH_SIZE + WRITE_SIZE, from the committed counter summary of this workload) / its average
                  duration (HIP events around every launch, this run); beside it the same duration under the
                  two algorithmic byte counts (no reuse of gathered rows: an upper bound on traffic that can
                  exceed the peak; perfect reuse: the lower bound),
  "cpu_baseline": the CPU oracle timed on a bounded sample of the same workload,
  "parity":       (default workload) the GPU results of one more step against the oracle values the
                  cpu_baseline leg computed on its sample: max-norm and element-wise relative errors,
  "spmm_calls":   each sparse product of one step (all its kernels together): ms, GFLOP/s = 2 nnz D / t
                  (Eq. 4.3), measured HBM GB/s and its fraction of 8 TB/s, the two algorithmic rates, the
                  share of gathers served from cache and the regime that follows from it,
  "kernels":      per-kernel ms, measured GB/s and fraction of 8 TB/s, TFLOP/s and fraction of the matrix peak,
  "trials":       ms per step of the repetitions (mean and min).

`--launch-log FILE` writes the names of the timed launches in order (for matching a profiler's dispatch
list); `--summarize-counters DIR --name NAME` turns rocprofv3 output collected with it into
profiles/traffic_NAME.json (what "traffic" above reads) and profiles/counters_NAME.md.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}     # dense matrix-core peaks of the part
METRIC = "GCN layer fwd+bwd ms; SpMM achieved HBM GB/s (% roofline) on 1 MI355X"
CSRC = os.path.join(ROOT, "paper_2505_04083_amd", "csrc")
PROFILES = os.path.join(ROOT, "profiles")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", choices=["shard", "tiny", "social", "copurchase", "road", "shard_sparse", "road_full"],
                    default="shard")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (testing only; <1 is not the metric)")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32",
                    help="storage type of activations / gradients (the headline metric is f32)")
    ap.add_argument("--trials", type=int, default=3, help="repetitions of the K timed steps (the first one is `value`)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-div", type=int, default=0,
                    help="oracle sample = 1/div of the workload (0: 2 for the shard, 1 for tiny, 4 for social / copurchase, 32 for road)")
    ap.add_argument("--cpu-one-core", action="store_true",
                    help="graph workloads: also time the oracle on ONE core (on a sample 8 times smaller than the all-core one)")
    ap.add_argument("--mask", choices=["bits", "values"], default="bits",
                    help="what the backward pass reads for the ReLU derivative: one sign bit per element written by the "
                         "forward pass, or the activated output itself")
    ap.add_argument("--fused-aggregation", action="store_true",
                    help="aggregate-first forward with the combination in the sparse kernels' epilogue (a measured alternative, off by default)")
    ap.add_argument("--windows", type=int, default=0, help="column windows of the sparse product (0 = the library's default)")
    ap.add_argument("--no-input-grad", action="store_true",
                    help="graph workloads only: leave out the gradient with respect to the input features (Eq. 2.6-2.7 of the "
                         "first layer, which no weight update needs); NOT the headline configuration, named in config.workload")
    ap.add_argument("--graph", action="store_true",
                    help="graph workloads only: also record the step into a HIP graph and time K replays (graph_ms_per_step)")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run plain device copies of known size (reference dispatch for counter scaling)")
    ap.add_argument("--launch-log", default="", help="write the names of the timed launches, in order, to this file and skip "
                                                      "everything after the timed steps (profiler runs)")
    ap.add_argument("--summarize-counters", default="", metavar="DIR",
                    help="no GPU work: read rocprofv3 output under DIR (fetch/, write/, optionally trace/, each with the launch "
                         "log of its run) and write profiles/traffic_NAME.json and profiles/counters_NAME.md")
    ap.add_argument("--name", default="", help="NAME for --summarize-counters (default: <workload>_<dtype>)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------
# cost model of a timing label
# ------------------------------------------------------------------------------------------------

def mfma_peak_of(name):
    """(matrix-core peak in TFLOP/s a dense kernel is measured against, the reason if it is not its storage type's)."""
    if "]x3" in name:                                 # fp32 product = six bf16 matrix products: the pipe that binds is the bf16 one
        return MFMA_PEAK_TFLOPS["bf16"] / 6.0, "bf16 / 6 (six bf16 products per fp32 product)"
    if "]w32" in name:                                # bf16 storage widened on load, multiplied by the fp32 instructions
        return MFMA_PEAK_TFLOPS["f32"], "fp32 (bf16 inputs widened on load)"
    return MFMA_PEAK_TFLOPS["bf16" if "<bf16>" in name else "f32"], None


def kernel_cost(name, bins, names=()):
    """(no-reuse bytes, perfect-reuse bytes, flops) of one launch, from the sizes in the timing label.

    Sparse product over `rows` rows holding `entries` stored entries at width d: 8 B of CSR per entry (value +
    column), a 4 B row pointer and one s*d-byte output row per row, and the gathered operand rows: one per
    entry without reuse (what the double permutation leaves between neighbouring entries), one per DISTINCT
    column at most with perfect reuse.  Dense products: every operand and result once (both counts equal)."""
    m = re.match(r"spmm_(subwave|wave|split)<(f32|bf16),G\d+,VW\d+,d(\d+)>\[(A|At)\]", name)
    if m:
        kind, dt, d, o = m.groups()
        s, d = (4 if dt == "f32" else 2), int(d)
        rows, ent = bins[o]
        cols = sum(bins["At" if o == "A" else "A"][0])
        i = {"subwave": 0, "wave": 1, "split": 2}[kind]
        e, r = ent[i], rows[i]
        if kind == "split" and name.replace("spmm_split", "spmm_wave") not in names:
            e, r = e + ent[1], r + rows[1]       # column windows on: the segment kernels take every row of 256+ entries
        fixed = e * 8 + r * (4 + s * d)
        return fixed + e * s * d, fixed + min(e, cols) * s * d, 2 * e * d
    m = re.match(r"spmm_subwave_combine<f32,d(\d+),N(\d+)>\[(A|At)\]", name)
    if m:       # the short rows' sparse product plus, per row, the N-wide result (and its sign bits) instead of a re-read of H
        d, N, o = int(m.group(1)), int(m.group(2)), m.group(3)
        rows, ent = bins[o]
        cols = sum(bins["At" if o == "A" else "A"][0])
        e, r = ent[0], rows[0]
        fixed = e * 8 + r * (4 + 4 * d + 4 * N + 4 * ((N + 31) // 32))
        return fixed + e * 4 * d, fixed + min(e, cols) * 4 * d, 2 * e * d + 2 * r * d * N
    m = re.match(r"gemm_(nn|nt)<(f32|bf16)>\[M(\d+),N(\d+),K(\d+)\]", name)
    if m:
        s = 4 if m.group(2) == "f32" else 2
        M, N, K = map(int, m.groups()[2:])
        nxt = re.search(r"next(\d+)$", name)              # also writes T = result x Wn[N x dn] for the following layer
        dn = int(nxt.group(1)) if nxt else 0
        b = s * (M * K + M * N + M * dn) + 4 * K * N
        return b, b, 2 * M * N * (K + dn)
    m = re.match(r"gemm_tn<(f32|bf16)>\[R(\d+),M(\d+),N(\d+)\]", name)
    if m:
        s = 4 if m.group(1) == "f32" else 2
        R, M, N = map(int, m.groups()[1:])
        b = s * R * (M + N) + 4 * M * N
        return b, b, 2 * R * M * N
    m = re.match(r"bwd_dense<(f32|bf16)>\[R(\d+),M(\d+),N(\d+)\](.*)", name)
    if m:       # reads the gradient (or its factor dT), the mask source (values, or one bit per element) and P; writes dOut
        s = 4 if m.group(1) == "f32" else 2
        R, M, N = map(int, m.groups()[1:4])
        tail = m.group(5)
        mask = 0 if "nomask" in tail else (4 * R * ((N + 31) // 32) if "bits" in tail else s * R * N)
        f = re.search(r"fact(\d+)", tail)
        dn = int(f.group(1)) if f else 0
        grad = s * R * (dn if f else N)
        dout = 0 if "dWonly" in tail else 1
        b = grad + s * R * M * (1 + dout) + mask + 4 * M * N
        return b, b, 2 * R * M * N * (1 + dout) + 2 * R * N * dn
    m = re.match(r"(relu|relu_bwd|softmax_ce)\[R(\d+),C(\d+)\]", name)
    if m:
        R, C = int(m.group(2)), int(m.group(3))
        b = 4 * R * C * {"relu": 2, "relu_bwd": 3, "softmax_ce": 2}[m.group(1)]
        return b, b, 0
    return None, None, None


# ------------------------------------------------------------------------------------------------
# measured HBM traffic: committed rocprofv3 counter summaries, stamped with the kernel sources
# ------------------------------------------------------------------------------------------------

# which source files a timing label's kernels are compiled from (a summary is current while these are unchanged)
_SOURCES = [
    (r"spmm_", ["spmm.hip"]),
    (r"gemm_|dw_partials_reduce", ["gemm.hip", "dense_bf16.hip", "bf16_frag.h", "buffer_addr.h"]),
    (r"bwd_dense", ["dense_bwd.hip", "dense_bf16.hip", "bf16_frag.h", "buffer_addr.h"]),
    (r"", ["elementwise.hip"]),
]
# kernels a timed launch may consist of: (label prefix, kernel-name prefixes, most kernels; 0 = any number)
_SYMBOLS = [
    ("spmm_subwave_combine", ["k_spmm_subwave_combine"], 1), ("rows_combine", ["k_rows_combine"], 1),
    ("spmm_subwave", ["k_spmm_subwave"], 1), ("spmm_wave", ["k_spmm_wave"], 1),
    ("spmm_split", ["k_spmm_segment", "k_spmm_combine"], 2),
    ("gemm_tn", ["k_gemm_tn"], 1), ("gemm_n", ["k_gemm_f32", "k_gemm_deep", "k_gemm_small"], 1),
    ("bwd_dense", ["k_bwd_dense"], 1), ("dw_partials_reduce", ["k_reduce_partials"], 0),
    ("relu_bwd_bits", ["k_relu_bwd_bits"], 1), ("relu_bwd", ["k_relu_bwd"], 1), ("relu", ["k_relu"], 1),
    ("sign_bits", ["k_bits_from_act"], 1), ("softmax_ce", ["k_softmax_ce", "k_sum_level"], 0),
]


def source_sha():
    out = {}
    for f in sorted(os.listdir(CSRC)):
        if f.endswith((".hip", ".h")):
            out[f] = hashlib.sha256(open(os.path.join(CSRC, f), "rb").read()).hexdigest()[:16]
    return out


def sources_of(label):
    for pat, files in _SOURCES:
        if re.match(pat, label):
            return files
    return []


class Traffic:
    """profiles/traffic_<workload>_<dtype>.json: measured HBM bytes per launch of every timing label."""

    def __init__(self, workload, dtype, usable=True):
        self.path = os.path.join(PROFILES, f"traffic_{workload}_{dtype}.json")
        self.rel = os.path.relpath(self.path, ROOT)
        self.data = json.load(open(self.path)) if (usable and os.path.exists(self.path)) else None
        self.now = source_sha()

    def of(self, label):
        """(bytes per launch, None) or (None, why not)."""
        if self.data is None:
            return None, "no counter summary for this workload"
        e = self.data["labels"].get(label)
        if e is None:
            return None, "label not in the counter summary"
        stale = [f for f in sources_of(label) if self.data["source_sha"].get(f) != self.now.get(f)]
        if stale:
            return None, "counter summary is older than " + ", ".join(stale)
        return e["fetch_bytes"] + e["write_bytes"], None


def short_symbol(n):
    n = n.replace("(anonymous namespace)::", "").replace("plx::", "")
    n = re.sub(r"^void ", "", n)
    return re.match(r"([^(]*)", n).group(1)


def match_launches(labels, symbols):
    """Assign the LAST dispatches of `symbols` (kernel names in dispatch order) to `labels` (timed launches in
    order), walking both backwards; returns one list of dispatch indices per label."""
    out = [None] * len(labels)
    j = len(symbols) - 1
    for i in range(len(labels) - 1, -1, -1):
        rule = next((r for r in _SYMBOLS if labels[i].startswith(r[0])), None)
        if rule is None:
            raise SystemExit(f"no kernel rule for the timing label {labels[i]}")
        got = []
        while j >= 0 and any(symbols[j].startswith(p) for p in rule[1]) and (rule[2] == 0 or len(got) < rule[2]):
            got.append(j); j -= 1
        if not got:
            raise SystemExit(f"dispatch list and launch log disagree at {labels[i]} (next dispatch: {symbols[j] if j >= 0 else None})")
        out[i] = got[::-1]
    return out


def read_dispatches(path, value_col=None):
    """plx kernels of a rocprofv3 CSV in dispatch order: [(kernel name, value or (start, end))], and the counter
    value of the reference dispatch (a plain 4 GiB device copy)."""
    rows, copies = [], []
    for r in csv.DictReader(open(path)):
        name = r["Kernel_Name"]
        if "copyBuffer" in name and value_col:
            copies.append((int(r["Dispatch_Id"]), float(r[value_col])))
        if "plx::" not in name:
            continue
        v = float(r[value_col]) if value_col else (int(r["Start_Timestamp"]), int(r["End_Timestamp"]))
        rows.append((int(r["Dispatch_Id"]), short_symbol(name), v))
    rows.sort()
    # --copy-ref issues its four 4 GiB copies after every set-up copy and before the first step: the last four
    ref = sorted(v for _, v in sorted(copies)[-4:])
    return [(s, v) for _, s, v in rows], (ref[len(ref) // 2] if len(ref) == 4 else None)


def newest(files):
    """A directory that several profiler runs wrote into holds one file per run: only the latest one counts."""
    return sorted(files, key=os.path.getmtime, reverse=True)[:1]


def summarize_counters(args):
    """DIR/fetch and DIR/write: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script with --copy-ref and
    --launch-log DIR/<kind>/launches.txt; DIR/trace (optional): a --kernel-trace --stats run with its launch log."""
    d = args.summarize_counters
    name = args.name or f"{args.workload}_{args.dtype}"
    per_label = {}
    scale = {}
    for kind, counter in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        f = newest(glob.glob(os.path.join(d, kind, "**", "*counter_collection.csv"), recursive=True))
        if not f:
            raise SystemExit(f"no counter_collection.csv under {d}/{kind}")
        disp, copy = read_dispatches(f[0], "Counter_Value")
        if copy is None:
            raise SystemExit(f"{kind}: no reference copy dispatch (run with --copy-ref)")
        scale[kind] = 4 * (1 << 30) / 1024 / copy          # the copy reads and writes 4 GiB; counters are in KiB
        labels = open(os.path.join(d, kind, "launches.txt")).read().split()
        for lab, idx in zip(labels, match_launches(labels, [s for s, _ in disp])):
            e = per_label.setdefault(lab, {"fetch": [], "write": [], "symbols": sorted({disp[i][0] for i in idx})})
            e[kind].append(sum(disp[i][1] for i in idx) * 1024 * scale[kind])
    trace_us, stats_lines = {}, []
    tf = newest(glob.glob(os.path.join(d, "trace", "**", "*kernel_trace.csv"), recursive=True))
    if tf:
        disp, _ = read_dispatches(tf[0])
        labels = open(os.path.join(d, "trace", "launches.txt")).read().split()
        for lab, idx in zip(labels, match_launches(labels, [s for s, _ in disp])):
            trace_us.setdefault(lab, []).append(sum(disp[i][1][1] - disp[i][1][0] for i in idx) / 1e3)
        for sf in newest(glob.glob(os.path.join(d, "trace", "**", "*kernel_stats.csv"), recursive=True)):
            for r in csv.DictReader(open(sf)):
                if "plx::" in r["Name"]:
                    stats_lines.append((float(r["Percentage"]), f"| `{short_symbol(r['Name'])}` | {r['Calls']} | "
                                        f"{float(r['AverageNs']) / 1e3:.1f} | {r['Percentage']} |"))
    out = {"command": f"see profiles/counters_{name}.md", "fetch_scale": scale["fetch"], "write_scale": scale["write"],
           "source_sha": source_sha(), "labels": {}}
    lines = []
    for lab, e in per_label.items():
        fb = sum(e["fetch"]) / max(len(e["fetch"]), 1); wb = sum(e["write"]) / max(len(e["write"]), 1)
        out["labels"][lab] = {"fetch_bytes": int(fb), "write_bytes": int(wb), "symbols": e["symbols"]}
        us = trace_us.get(lab)
        avg = sum(us) / len(us) if us else None
        if avg:
            out["labels"][lab]["rocprof_avg_us"] = round(avg, 1)
        lines.append((-(avg or 0), f"| `{lab}` | {', '.join(e['symbols'])} | {'' if not avg else f'{avg:.1f}'} | {fb / 1e9:.3f} | "
                      f"{wb / 1e9:.3f} | {'' if not avg else f'{(fb + wb) / avg / 1e3:.0f}'} | "
                      f"{'' if not avg else f'{(fb + wb) / avg / 1e3 / HBM_PEAK_GBS * 100:.0f}'} |"))
    os.makedirs(PROFILES, exist_ok=True)
    json.dump(out, open(os.path.join(PROFILES, f"traffic_{name}.json"), "w"), indent=1)
    w, dt = args.workload, args.dtype
    run = f"python3 bench.py --workload {w} --dtype {dt} --no-cpu-baseline --trials 1 --steps 2 --warmup 1 --copy-ref"
    with open(os.path.join(PROFILES, f"counters_{name}.md"), "w") as fo:
        fo.write(f"# HBM traffic and kernel times per launch: workload `{w}`, {dt}\n\n"
                 "One MI355X, rocprofv3 (ROCm 7.2.0).  Commands, from the repository root (`cd /tmp && export TMPDIR=/tmp` first,\n"
                 "outputs under `D=gpurun_out/prof_" + name + "`):\n\n"
                 f"    rocprofv3 --kernel-trace --stats --output-format csv -d $D/trace -- {run.replace(' --copy-ref', '')} --launch-log $D/trace/launches.txt\n"
                 f"    rocprofv3 --pmc FETCH_SIZE --kernel-include-regex 'plx|copyBuffer' --output-format csv -d $D/fetch -- {run} --launch-log $D/fetch/launches.txt\n"
                 f"    rocprofv3 --pmc WRITE_SIZE --kernel-include-regex 'plx|copyBuffer' --output-format csv -d $D/write -- {run} --launch-log $D/write/launches.txt\n"
                 f"    python3 bench.py --workload {w} --dtype {dt} --summarize-counters $D --name {name}\n\n"
                 "Counters are KiB per dispatch, scaled by what the same counter reads for a plain 4 GiB device copy in the same run\n"
                 f"(FETCH_SIZE x {scale['fetch']:.3f}, WRITE_SIZE x {scale['write']:.3f}).  A row is one timed launch of the library (the label\n"
                 "`bench.py` reports), matched to the profiler's dispatches through the launch log; values are averages over the\n"
                 "timed steps.\n\n"
                 "| launch | kernels | avg us (kernel trace) | fetched GB | written GB | GB/s | % of 8 TB/s |\n|---|---|---|---|---|---|---|\n")
        fo.write("\n".join(l for _, l in sorted(lines)) + "\n")
        if stats_lines:
            fo.write("\n`rocprofv3 --kernel-trace --stats` summary of the same run (all dispatches incl. warm-up):\n\n"
                     "| kernel | calls | avg us | % of GPU time |\n|---|---|---|---|\n")
            fo.write("\n".join(l for _, l in sorted(stats_lines, reverse=True)[:24]) + "\n")
    print(f"wrote profiles/traffic_{name}.json and profiles/counters_{name}.md ({len(per_label)} launches)")


def note(msg):
    """progress line on stderr (the JSON line on stdout stays alone)"""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    args = parse()
    if args.summarize_counters:
        return summarize_counters(args)
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus {args.gpus} is not "
              "supported. value is one GPU's throughput; run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_04083_amd as plx
    from paper_2505_04083_amd.network import GcnNetwork, aligned_rows
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    cfg = synth.CONFIGS[args.workload]
    if args.scale != 1.0:
        cfg = cfg.scaled(args.scale)
    tdt = torch.float32 if args.dtype == "f32" else torch.bfloat16
    code = plx.PLX_F32 if args.dtype == "f32" else plx.PLX_BF16
    side = torch.cuda.Stream(device=dev) if args.graph else None      # graph capture needs a non-default stream
    ctx = plx.plx_ctx(0, stream=side.cuda_stream) if side else plx.plx_ctx(0)
    if args.windows:
        plx.plx_ctx_set_column_windows(ctx, args.windows)
    if args.fused_aggregation:
        plx.plx_ctx_set_fused_aggregation(ctx, True)
    shard_state = None

    t0 = time.time()
    if cfg.kind == "shard":
        din, dout = cfg.dims
        rowptr, col, val = synth.shard_block(cfg.seed, cfg.m, cfg.k, cfg.n_samples, dev)
        torch.cuda.synchronize()
        t_gen = time.time() - t0
        X = synth.normal(cfg.seed, synth.S_FEAT, cfg.k, din, dev, tdt)
        dF = synth.normal(cfg.seed, synth.S_AUX, cfg.m, dout, dev, tdt)
        W = synth.glorot(cfg.seed, 0, din, dout, dev)
        t0 = time.time()
        csr = plx.plx_csr_import(ctx, cfg.m, cfg.k, rowptr, col, val)
        t_build = time.time() - t0
        order = plx.PLX_ORDER_AGG_FIRST
        ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, code, plx.PLX_ACT_RELU, order),
                         dtype=torch.uint8, device=dev)
        F = torch.empty(cfg.m, dout, device=dev, dtype=tdt)   # the activated output, and its sign as one bit per element (Eq. 2.4)
        act = plx.PLX_ACT_RELU if args.mask == "values" else plx.PLX_ACT_RELU_BITS
        Zm = F if args.mask == "values" else torch.empty(cfg.m, (dout + 31) // 32, device=dev, dtype=torch.int32)
        saved = torch.empty(cfg.m, din, device=dev, dtype=tdt)
        dX = torch.empty(cfg.k, din, device=dev, dtype=tdt); dW = torch.empty(din, dout, device=dev)

        def step(grad=dF):
            plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, None if args.mask == "values" else Zm, F, saved, ws, act=act, order=order)
            plx.plx_gcn_layer_bwd(ctx, csr, False, X, W, Zm, grad, saved, dX, dW, ws, act=act, order=order)

        shard_state = dict(rowptr=rowptr, col=col, val=val, X=X, W=W, dF=dF, F=F, saved=saved, dX=dX, dW=dW, step=step)
        workload = (f"configs[3]: one GPU's 7M x 28M shard block of a billion-edge graph, {args.dtype}, "
                    "layer 32 -> 128, aggregate-first")
        if args.workload == "shard_sparse":
            workload = workload.replace("configs[3]:", "configs[3], secondary row with ~50 M entries:")
        unit = "ms per GCN layer fwd+bwd"
        shape = {"m": cfg.m, "k": cfg.k, "din": din, "dout": dout, "order": "agg_first"}
    else:
        src, dst = cfg.edges(dev)
        pr, pc = cfg.perms(dev)
        torch.cuda.synchronize()
        t_gen = time.time() - t0
        t0 = time.time()
        csr = plx.plx_build_csr(ctx, cfg.n, src, dst, pr, pc)
        t_build = time.time() - t0
        del src, dst
        # random rows: any order is P_c order; stored like every matrix of the network, rows padded to 16 bytes
        H0 = aligned_rows(cfg.n, cfg.dims[0], tdt, dev)
        H0.copy_(synth.normal(cfg.seed, synth.S_FEAT, cfg.n, cfg.dims[0], dev, tdt))
        Ws = cfg.weights(dev)
        y = cfg.labels(dev)
        net = GcnNetwork(ctx, csr, Ws, dtype=tdt, sign_bits=args.mask == "bits", input_grad=not args.no_input_grad)

        def step():
            net.step(H0, y)

        idx = {"tiny": 0, "social": 1, "copurchase": 2, "road": 4, "road_full": 4}[args.workload]
        workload = (f"configs[{idx}]: {args.workload} graph, {args.dtype}, {len(Ws)}-layer GCN "
                    + "-".join(map(str, cfg.dims)) + ", whole forward + backward with loss head, AUTO order"
                    + (", WITHOUT the gradient of the input features" if args.no_input_grad else ""))
        unit = f"ms per {len(Ws)}-layer network fwd+bwd"
        shape = {"n": cfg.n, "dims": cfg.dims}
    if args.scale != 1.0:
        workload += f" (SHRUNK x{args.scale})"

    note(f"inputs generated in {t_gen:.1f} s, adjacency handle built (nnz = {csr.nnz})")
    stream_ref = None
    if args.copy_ref:
        # 2^30 fp32 read + 2^30 fp32 written by a plain copy: the known-size dispatch the
        # FETCH_SIZE / WRITE_SIZE counters are scaled by; its rate and a plain fill's rate are also
        # the practical ceilings a streaming kernel can be compared with
        ref_src = torch.ones(1 << 30, dtype=torch.float32, device=dev)
        ref_dst = torch.empty_like(ref_src)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ref_dst.copy_(ref_src); ref_dst.fill_(2.0)
        ev[0].record()
        for _ in range(3):
            ref_dst.copy_(ref_src)
        ev[1].record()
        for _ in range(3):
            ref_dst.fill_(2.0)
        ev[2].record()
        torch.cuda.synchronize()
        gib4 = 4 * (1 << 30)
        stream_ref = {"copy_GBps_read_plus_write": round(2 * gib4 * 3 / ev[0].elapsed_time(ev[1]) / 1e6, 1),
                      "fill_GBps": round(gib4 * 3 / ev[1].elapsed_time(ev[2]) / 1e6, 1), "bytes_each_way": gib4}
        del ref_src, ref_dst
    for _ in range(args.warmup):
        step()
    plx.plx_sync(ctx)
    torch.cuda.synchronize()
    note(f"{args.warmup} warm-up steps done")

    # ---- the timed region: K steps, nothing but the library's launches (event timing off) -------------
    trial_ms = []
    for _ in range(max(1, args.trials)):
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        plx.plx_sync(ctx)
        torch.cuda.synchronize()
        trial_ms.append((time.perf_counter() - t0) * 1e3 / args.steps)
    ms_per_step = trial_ms[0]
    note(f"{len(trial_ms)} x {args.steps} timed steps done: {ms_per_step:.3f} ms per step")

    # ---- K more steps with an event pair around every launch: the per-kernel figures ---------------------
    plx.plx_timing_enable(ctx, True)
    for _ in range(args.steps):
        step()
    trace = plx.plx_timing_trace(ctx)
    plx.plx_timing_enable(ctx, False)
    timing = {}
    for name, ms in trace:
        c, t = timing.get(name, (0, 0.0))
        timing[name] = (c + 1, t + ms)
    if args.launch_log:
        os.makedirs(os.path.dirname(os.path.abspath(args.launch_log)), exist_ok=True)
        with open(args.launch_log, "w") as fo:
            fo.write("\n".join(n for n, _ in trace) + "\n")

    graph_ms = None
    if args.graph and cfg.kind != "shard" and not args.launch_log:
        graph = net.capture(H0, y, side)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- per-kernel accounting ------------------------------------------------------------------------
    traffic = Traffic(args.workload, args.dtype, usable=args.scale == 1.0 and not args.windows and not args.fused_aggregation)
    bins = {"A": plx.plx_csr_bins(csr, False), "At": plx.plx_csr_bins(csr, True)}
    cost = {name: kernel_cost(name, bins, timing) for name in timing}
    meas = {name: traffic.of(name) for name in timing}
    kernels = {}
    for name, (count, total_ms) in timing.items():
        avg = total_ms / max(count, 1)
        b_hi, b_lo, fl = cost[name]
        b_meas, why = meas[name]
        k = {"launches_per_step": count / args.steps, "avg_ms": round(avg, 4)}
        if b_meas is not None:
            k["hbm_bytes_measured"] = int(b_meas)
            k["GBps_measured"] = round(b_meas / avg / 1e6, 1)
            k["frac_hbm"] = round(b_meas / avg / 1e6 / HBM_PEAK_GBS, 4)
        elif b_hi:
            k["traffic_note"] = why
        if b_hi:
            k["GBps_no_reuse_count"] = round(b_hi / avg / 1e6, 1)
            if b_lo != b_hi:
                k["GBps_perfect_reuse_count"] = round(b_lo / avg / 1e6, 1)
        if fl:
            k["GFLOPs"] = round(fl / avg / 1e6, 1)
        if fl and not name.startswith("spmm_"):      # dense products run on the matrix cores
            peak, why_peak = mfma_peak_of(name)
            if why_peak:
                k["mfma_peak_used"] = why_peak
            k["frac_mfma"] = round(fl / avg / 1e9 / peak, 4)
            hbm_frac = k.get("frac_hbm", b_hi / avg / 1e6 / HBM_PEAK_GBS)      # dense kernels: both byte counts coincide
            k["binding"] = "hbm" if hbm_frac >= k["frac_mfma"] else "mfma"
            ai = fl / b_hi
            balance = peak * 1e3 / HBM_PEAK_GBS
            if ai < balance:                        # below the machine balance HBM binds whatever the kernel does
                k["mfma_ceiling_at_full_hbm_rate"] = round(ai / balance, 3)
        kernels[name] = k
    dominant = max((n for n in timing if cost[n][0]), key=lambda n: timing[n][1])
    d_avg = timing[dominant][1] / timing[dominant][0]
    b_hi, b_lo, d_fl = cost[dominant]
    b_meas, why = meas[dominant]
    roofline = {"bound": "hbm", "kernel": dominant, "peak": HBM_PEAK_GBS, "unit": "GB/s", "avg_launch_ms": round(d_avg, 4)}
    if b_meas is not None:
        roofline.update({"achieved": round(b_meas / d_avg / 1e6, 1), "frac": round(b_meas / d_avg / 1e6 / HBM_PEAK_GBS, 4),
                         "traffic": int(b_meas),
                         "basis": f"measured HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, {traffic.rel}) / this run's launch time"})
    else:       # no current counter summary: the perfect-reuse count is the only basis that cannot overstate the rate
        roofline.update({"achieved": round(b_lo / d_avg / 1e6, 1), "frac": round(b_lo / d_avg / 1e6 / HBM_PEAK_GBS, 4),
                         "traffic": None, "basis": f"perfect-reuse byte count (a LOWER bound on traffic; {why})"})
    roofline.update({"no_reuse_upper_bound": {"bytes_per_launch": int(b_hi), "GBps": round(b_hi / d_avg / 1e6, 1)},
                     "perfect_reuse_lower_bound": {"bytes_per_launch": int(b_lo), "GBps": round(b_lo / d_avg / 1e6, 1)}})
    if kernels[dominant].get("binding") == "mfma":     # a dense product nearer its matrix-core peak than its HBM peak
        peak = round(mfma_peak_of(dominant)[0], 1)
        tf = d_fl / d_avg / 1e9
        roofline.update({"bound": "mfma", "achieved": round(tf, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4),
                         "algorithmic_flops_per_launch": int(d_fl),
                         "basis": "flops of the product (2 M N K per product) / this run's launch time"})

    # the sparse products: one entry per (orientation, width), its kernels together; and all of them together
    calls = {}
    for n, (c, t) in timing.items():
        m_ = re.match(r"spmm_\w+<(f32|bf16),G\d+,VW\d+,d(\d+)>\[(A|At)\]", n)
        if not m_:
            continue
        e = calls.setdefault((m_.group(3), int(m_.group(2)), m_.group(1)),
                             {"ms": 0.0, "hi": 0.0, "flops": 0.0, "meas": 0.0, "meas_ok": True, "launches": 0.0})
        e["ms"] += t / args.steps; e["hi"] += cost[n][0] * c / args.steps; e["flops"] += cost[n][2] * c / args.steps
        e["launches"] = max(e["launches"], c / args.steps)
        if meas[n][0] is None:
            e["meas_ok"] = False
        else:
            e["meas"] += meas[n][0] * c / args.steps
    spmm_calls = []
    tot = {"ms": 0.0, "hi": 0.0, "lo": 0.0, "flops": 0.0, "meas": 0.0, "meas_ok": True}
    for (o, d, dt), e in sorted(calls.items()):
        rows_o = sum(bins[o][0]); cols_o = sum(bins["At" if o == "A" else "A"][0]); s_ = 4 if dt == "f32" else 2
        b_min = (8 * csr.nnz + 4 * (rows_o + 1) + s_ * d * (rows_o + cols_o)) * e["launches"]
        c_ = {"matrix": o, "width": d, "dtype": dt, "calls_per_step": e["launches"], "ms": round(e["ms"], 4),
              "GFLOPs": round(e["flops"] / e["ms"] / 1e6, 1)}
        if e["meas_ok"]:
            hit = 1.0 - e["meas"] / e["hi"]
            c_.update({"hbm_bytes_measured": int(e["meas"]), "GBps_measured": round(e["meas"] / e["ms"] / 1e6, 1),
                       "frac_of_8TBps": round(e["meas"] / e["ms"] / 1e6 / HBM_PEAK_GBS, 4),
                       "share_of_no_reuse_bytes_not_fetched": round(hit, 3),
                       "regime": ("HBM gather with over-fetch (operand rows shorter than the fetch granule: more bytes move than the no-reuse count charges)"
                                  if hit < -0.05 else "HBM gather (most operand rows come from HBM)" if hit < 0.5 else
                                  "cache-served gather (most operand rows come from the Infinity Cache / L2)")})
        c_.update({"GBps_no_reuse_count": round(e["hi"] / e["ms"] / 1e6, 1),
                   "GBps_perfect_reuse_count": round(b_min / e["ms"] / 1e6, 1)})
        spmm_calls.append(c_)
        tot["ms"] += e["ms"]; tot["hi"] += e["hi"]; tot["lo"] += b_min; tot["flops"] += e["flops"]; tot["meas"] += e["meas"]
        tot["meas_ok"] = tot["meas_ok"] and e["meas_ok"]
    spmm = None
    if tot["ms"] > 0:
        spmm = {"ms_per_step": round(tot["ms"], 4), "GFLOPs": round(tot["flops"] / tot["ms"] / 1e6, 1),
                "GBps_no_reuse_count": round(tot["hi"] / tot["ms"] / 1e6, 1),
                "GBps_perfect_reuse_count": round(tot["lo"] / tot["ms"] / 1e6, 1)}
        if tot["meas_ok"]:
            spmm.update({"GBps_measured": round(tot["meas"] / tot["ms"] / 1e6, 1),
                         "frac_of_8TBps": round(tot["meas"] / tot["ms"] / 1e6 / HBM_PEAK_GBS, 4)})

    out = {
        "metric": METRIC, "value": round(ms_per_step, 4), "unit": unit,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": workload, **shape, "nnz": csr.nnz,
                   "rows_entries_by_bin(<256,<4096,>=4096)": {k_: [list(v[0]), list(v[1])] for k_, v in bins.items()}},
        "roofline": roofline, "cpu_baseline": None, "spmm": spmm, "spmm_calls": spmm_calls, "kernels": kernels,
        "trials": {"ms_per_step": [round(x, 4) for x in trial_ms], "mean": round(sum(trial_ms) / len(trial_ms), 4),
                   "min": round(min(trial_ms), 4)},
        "setup_s": {"generate": round(t_gen, 2), "csr_build_transpose_bins": round(t_build, 2)},
    }
    if stream_ref:
        out["stream_ref"] = stream_ref
    if graph_ms is not None:
        out["graph_ms_per_step"] = round(graph_ms, 4)

    if not args.no_cpu_baseline and not args.launch_log:
        div = args.cpu_sample_div or {"shard": 2, "shard_sparse": 1, "tiny": 1, "road": 32, "road_full": 32}.get(args.workload, 4)
        if cfg.kind == "shard":
            out["cpu_baseline"], out["parity"] = cpu_baseline_and_parity(cfg, ctx, shard_state, div, args.dtype)
        else:
            out["cpu_baseline"] = cpu_baseline_network(cfg, div, unit, args.cpu_one_core)
    print(json.dumps(out))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def errors(gpu, ref):
    """(max-norm relative error, element-wise relative error with a floor of 1e-3 of the largest magnitude)"""
    import numpy as np
    g = gpu.detach().double().cpu().numpy()
    top = float(np.abs(ref).max())
    if top == 0.0:
        return float(np.abs(g).max()), float(np.abs(g).max())
    diff = np.abs(g - ref)
    return float(diff.max() / top), float((diff / np.maximum(np.abs(ref), 1e-3 * top)).max())


def cpu_baseline_and_parity(cfg, ctx, st, div, dtype):
    """The oracle as it stands, on 1/div of the block: rows [0, m/div) for Eq. 2.1-2.6 and output rows [0, k/div)
    for Eq. 2.7 of the gradient those rows produce; each part's time is scaled by div.  Then one more GPU step on
    the same sample (the gradient is zero in the other rows, so dW and dX depend on the sample alone) and the
    comparison of its results with the oracle's values.  Gradient entries whose pre-activation lies within
    1e-5 (bf16: 2e-2) of the largest one of zero are zeroed on both sides: there the two summation orders may
    take the integer decision of Eq. 2.4 differently."""
    import numpy as np
    import torch
    import oracle
    import paper_2505_04083_amd as plx
    rowptr, col, val, X, W, dF = st["rowptr"], st["col"], st["val"], st["X"], st["W"], st["dF"]
    mb, kb = max(1, cfg.m // div), max(1, cfg.k // div)
    rp = rowptr.cpu().numpy(); c = col.cpu().numpy(); v = val.cpu().numpy()
    X64 = X.float().cpu().numpy().astype(np.float64)
    Wh = W.cpu().numpy().astype(np.float64)
    dFh = dF[:mb].float().cpu().numpy().astype(np.float64)
    nb = int(rp[mb])
    row_b = np.repeat(np.arange(mb, dtype=np.int64), np.diff(rp[:mb + 1]))
    col_b = c[:nb].astype(np.int64); val_b = v[:nb].astype(np.float64)
    # entries of the sample rows that land in output rows [0, kb) of the transposed product
    keep = c[:nb] < kb
    row_t = row_b[keep]; col_t = col_b[keep]; val_t = val_b[keep]
    t = {}
    t0 = time.perf_counter(); H = oracle.spmm_coo(mb, row_b, col_b, val_b, X64); t["spmm"] = time.perf_counter() - t0
    t0 = time.perf_counter(); Q = oracle.gemm(H, Wh); t["gemm_nn"] = time.perf_counter() - t0
    band = (1e-5 if dtype == "f32" else 2e-2) * float(np.abs(Q).max())
    shaky = np.abs(Q) < band
    dFh[shaky] = 0.0
    t0 = time.perf_counter(); Fo = oracle.relu(Q); dQ = oracle.relu_bwd(Q, dFh); t["act"] = time.perf_counter() - t0
    t0 = time.perf_counter(); dWo = oracle.gemm(H, dQ, ta=True); t["gemm_tn"] = time.perf_counter() - t0
    t0 = time.perf_counter(); dS = oracle.gemm(dQ, Wh, tb=True); t["gemm_nt"] = time.perf_counter() - t0
    # Eq. 2.7 over ALL rows of the block costs the oracle the same per entry; here its sample is the entries of the
    # sample rows (the others carry a zero gradient), so this part is scaled by the share of entries it covered
    t0 = time.perf_counter(); dXo = oracle.spmm_t_coo(kb, row_t, col_t, val_t, dS); t["spmm_t"] = time.perf_counter() - t0
    share_t = max(len(row_t), 1) / float(len(c))
    total = sum(t.values())
    scaled = sum(v_ for k_, v_ in t.items() if k_ != "spmm_t") * div + t["spmm_t"] / share_t
    cpu = {"value": round(scaled * 1e3, 1), "unit": "ms per GCN layer fwd+bwd", "cores": oracle.num_threads(),
           "cpu": cpu_model(), "kind": "oracle",
           "sample": f"1/{div} of the block (rows [0,{mb}) for Eq. 2.1-2.6, scaled by {div}; Eq. 2.7 on the {len(row_t)} entries of "
                     f"those rows in output rows [0,{kb}), scaled by {1 / share_t:.2f} to all {len(c)} entries), {total:.1f} s of CPU work",
           "parts_s": {k_: round(v_, 3) for k_, v_ in t.items()}}
    # ---- the same sample through the GPU path ----------------------------------------------------------
    grad = torch.zeros_like(dF)
    grad[:mb] = torch.as_tensor(dFh, dtype=torch.float32).to(dF.device).to(dF.dtype)
    st["step"](grad)
    plx.plx_sync(ctx)
    par = {"sample": f"rows [0,{mb}) of the block, dense gradient (zero in the other rows and where |Q| < {band:.2e}: "
                     f"{int((shaky & (Q != 0)).sum())} entries with an ill-conditioned sign, {int((Q == 0).sum())} exact zeros of rows "
                     f"without entries, of {shaky.size}); dX on output rows [0,{kb})",
           "tolerance_max_norm": 1e-4 if dtype == "f32" else 2e-2, "tensors": {}}
    for name, g, o in (("H = A X (Eq. 2.1)", st["saved"][:mb], H), ("F = ReLU(H W) (Eq. 2.2-2.3)", st["F"][:mb], Fo),
                       ("dW = H^T dQ (Eq. 2.4-2.5)", st["dW"], dWo), ("dX = A^T (dQ W^T) (Eq. 2.6-2.7)", st["dX"][:kb], dXo)):
        e_max, e_elt = errors(g, o)
        par["tensors"][name] = {"max_norm_rel_err": float(f"{e_max:.3e}"), "elementwise_rel_err": float(f"{e_elt:.3e}")}
    par["ok"] = all(v_["max_norm_rel_err"] <= par["tolerance_max_norm"] for v_ in par["tensors"].values())
    return cpu, par


def cpu_baseline_network(cfg, div, unit, one_core=False):
    """The oracle's whole-network forward + backward (Eq. 2.1-2.7 and the loss head) on the same
    recipe shrunk to 1/div of the nodes and edges (same degree distribution and widths); time
    scaled by div.  one_core: the same once more on one thread, on a sample 8 times smaller."""
    import oracle
    from oracle import gcn as ogcn

    def run(d):
        small = cfg if d == 1 else cfg.scaled(1.0 / d)
        src, dst = small.edges()
        F0 = small.features().numpy()
        Ws = [w.numpy() for w in small.weights()]
        y = small.labels().numpy()
        adj = oracle.adjacency(small.n, src.numpy(), dst.numpy())
        t0 = time.perf_counter()
        ogcn.forward_backward(adj, F0, Ws, y)
        return time.perf_counter() - t0, small.n, adj.nnz

    total, n, nnz = run(div)
    out = {"value": round(total * div * 1e3, 1), "unit": unit, "cores": oracle.num_threads(), "cpu": cpu_model(), "kind": "oracle",
           "sample": f"same generator at 1/{div} of the nodes and edges (n = {n}, nnz = {nnz}), "
                     f"{total:.1f} s of CPU work, scaled by {div}"}
    if one_core:
        threads = oracle.num_threads()
        oracle.set_num_threads(1)
        t1, n1, nnz1 = run(div * 8)
        oracle.set_num_threads(threads)
        out["one_core"] = {"value": round(t1 * div * 8 * 1e3, 1), "unit": unit, "cores": 1,
                           "sample": f"1/{div * 8} of the nodes and edges (n = {n1}, nnz = {nnz1}), {t1:.1f} s, scaled by {div * 8}"}
    return out


if __name__ == "__main__":
    main()
