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

Prints ONE JSON line.  Besides the contract keys it carries
  "roofline":     the dominant kernel's algorithmic HBM bytes / its average duration (HIP events
                  recorded around every launch inside the timed steps) against 8 TB/s,
  "cpu_baseline": the CPU oracle timed on a bounded sample of the same workload (default workload),
  "spmm_calls":   each sparse product of one step (all its kernels together): ms, GFLOP/s = 2 nnz D / t
                  (Eq. 4.3) and GB/s on the no-reuse byte count and on the perfect-reuse lower bound,
  "kernels":      per-kernel ms, GB/s, TFLOP/s and the fraction of the HBM and matrix-core peaks,
  "trials":       ms per step of `--trials` repetitions of the K timed steps (mean and min).
"""
from __future__ import annotations

import argparse
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
    ap.add_argument("--mask", choices=["bits", "values"], default="bits",
                    help="what the backward pass reads for the ReLU derivative: one sign bit per element written by the "
                         "forward pass, or the activated output itself")
    ap.add_argument("--windows", type=int, default=0, help="column windows of the sparse product (0 = the library's default)")
    ap.add_argument("--graph", action="store_true",
                    help="graph workloads only: also record the step into a HIP graph and time K replays (graph_ms_per_step)")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run plain device copies of known size (reference dispatch for counter scaling)")
    return ap.parse_args()


def mfma_peak_of(name):
    """(matrix-core peak in TFLOP/s a dense kernel is measured against, the reason if it is not its storage type's)."""
    if "]x3" in name:                                 # fp32 product = six bf16 matrix products: the pipe that binds is the bf16 one
        return MFMA_PEAK_TFLOPS["bf16"] / 6.0, "bf16 / 6 (six bf16 products per fp32 product)"
    if "]w32" in name:                                # bf16 storage widened on load, multiplied by the fp32 instructions
        return MFMA_PEAK_TFLOPS["f32"], "fp32 (bf16 inputs widened on load)"
    return MFMA_PEAK_TFLOPS["bf16" if "<bf16>" in name else "f32"], None


def kernel_cost(name, bins, names=()):
    """(algorithmic HBM bytes, flops) of one launch, from the sizes in the timing label.

    Sparse product over `rows` rows holding `entries` stored entries at width d: 8 B of CSR per
    entry (value + column), one s*d-byte gathered operand row per entry (the double permutation
    leaves no reuse between entries), a 4 B row pointer and one s*d-byte output row per row.
    Dense products: every operand and result once."""
    m = re.match(r"spmm_(subwave|wave|split)<(f32|bf16),G\d+,VW\d+,d(\d+)>\[(A|At)\]", name)
    if m:
        kind, dt, d, o = m.groups()
        s, d = (4 if dt == "f32" else 2), int(d)
        rows, ent = bins[o]
        i = {"subwave": 0, "wave": 1, "split": 2}[kind]
        e, r = ent[i], rows[i]
        if kind == "split" and name.replace("spmm_split", "spmm_wave") not in names:
            e, r = e + ent[1], r + rows[1]       # column windows on: the segment kernels take every row of 256+ entries
        return e * (8 + s * d) + r * (4 + s * d), 2 * e * d
    m = re.match(r"gemm_(nn|nt)<(f32|bf16)>\[M(\d+),N(\d+),K(\d+)\]", name)
    if m:
        s = 4 if m.group(2) == "f32" else 2
        M, N, K = map(int, m.groups()[2:])
        nxt = re.search(r"next(\d+)$", name)              # also writes T = result x Wn[N x dn] for the following layer
        dn = int(nxt.group(1)) if nxt else 0
        return s * (M * K + M * N + M * dn) + 4 * K * N, 2 * M * N * (K + dn)
    m = re.match(r"gemm_tn<(f32|bf16)>\[R(\d+),M(\d+),N(\d+)\]", name)
    if m:
        s = 4 if m.group(1) == "f32" else 2
        R, M, N = map(int, m.groups()[1:])
        return s * R * (M + N) + 4 * M * N, 2 * R * M * N
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
        return grad + s * R * M * (1 + dout) + mask + 4 * M * N, 2 * R * M * N * (1 + dout) + 2 * R * N * dn
    m = re.match(r"(relu|relu_bwd|softmax_ce)\[R(\d+),C(\d+)\]", name)
    if m:
        R, C = int(m.group(2)), int(m.group(3))
        return 4 * R * C * {"relu": 2, "relu_bwd": 3, "softmax_ce": 2}[m.group(1)], 0
    return None, None


def measured_traffic(name):
    """HBM bytes per launch of the kernel behind a timing label, from the committed rocprofv3
    FETCH_SIZE / WRITE_SIZE summary of the default workload (profiles/traffic_layer_shard_f32.json,
    counters already scaled by a plain 4 GiB copy); None if the summary has no such kernel."""
    path = os.path.join(ROOT, "profiles", "traffic_layer_shard_f32.json")
    if not os.path.exists(path):
        return None
    k = json.load(open(path))["kernels"]
    m = re.match(r"spmm_(subwave|wave|split)<f32,G(\d+),VW(\d+),d\d+>\[(A|At)\]", name)
    keys = []
    if m:
        kind, g, vw, o = m.groups()
        base = {"subwave": "k_spmm_subwave", "wave": "k_spmm_wave", "split": "k_spmm_segment"}[kind]
        keys = [f"{base}<float, {g}, {vw}> [{o}]"]
        if kind == "split":
            keys.append(f"k_spmm_combine<float> [{o}]")
    elif name.startswith("gemm_nn<f32>"):
        keys = [x for x in k if x.startswith("k_gemm_small_f32") or x.startswith("k_gemm_f32")]
    elif name.startswith("bwd_dense<f32>"):
        keys = [x for x in k if x.startswith("k_bwd_dense_f32")]
    if not keys or any(x not in k for x in keys):
        return None
    return sum(k[x]["fetch_bytes"] + k[x]["write_bytes"] for x in keys)


def note(msg):
    """progress line on stderr (the JSON line on stdout stays alone)"""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    args = parse()
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
    cpu_inputs = None

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

        def step():
            plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, None if args.mask == "values" else Zm, F, saved, ws, act=act, order=order)
            plx.plx_gcn_layer_bwd(ctx, csr, False, X, W, Zm, dF, saved, dX, dW, ws, act=act, order=order)

        cpu_inputs = (rowptr, col, val, X, W, dF)
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
        net = GcnNetwork(ctx, csr, Ws, dtype=tdt, sign_bits=args.mask == "bits")

        def step():
            net.step(H0, y)

        idx = {"tiny": 0, "social": 1, "copurchase": 2, "road": 4, "road_full": 4}[args.workload]
        workload = (f"configs[{idx}]: {args.workload} graph, {args.dtype}, {len(Ws)}-layer GCN "
                    + "-".join(map(str, cfg.dims)) + ", whole forward + backward with loss head, AUTO order")
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
    plx.plx_timing_enable(ctx, True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    plx.plx_sync(ctx)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    timing = plx.plx_timing_report(ctx)
    plx.plx_timing_enable(ctx, False)
    ms_per_step = elapsed * 1e3 / args.steps
    trial_ms = [ms_per_step]
    for _ in range(args.trials - 1):
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        plx.plx_sync(ctx)
        torch.cuda.synchronize()
        trial_ms.append((time.perf_counter() - t0) * 1e3 / args.steps)

    note(f"{args.trials} x {args.steps} timed steps done: {ms_per_step:.3f} ms per step")
    graph_ms = None
    if args.graph and cfg.kind != "shard":
        graph = net.capture(H0, y, side)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # ---- per-kernel accounting (algorithmic bytes / flops of one launch) -------------------------
    bins = {"A": plx.plx_csr_bins(csr, False), "At": plx.plx_csr_bins(csr, True)}
    cost = {name: kernel_cost(name, bins, timing) for name in timing}
    kernels = {}
    for name, (count, total_ms) in timing.items():
        avg = total_ms / max(count, 1)
        b, fl = cost[name]
        kernels[name] = {"launches_per_step": count / args.steps, "avg_ms": round(avg, 4),
                         "GBps": None if not b else round(b / avg / 1e6, 1),
                         "GFLOPs": None if not fl else round(fl / avg / 1e6, 1)}
        if b:
            kernels[name]["frac_hbm"] = round(b / avg / 1e6 / HBM_PEAK_GBS, 4)
        if fl and not name.startswith("spmm_"):      # dense products run on the matrix cores
            peak, why = mfma_peak_of(name)
            if why:
                kernels[name]["mfma_peak_used"] = why
            kernels[name]["frac_mfma"] = round(fl / avg / 1e9 / peak, 4)
            kernels[name]["binding"] = "hbm" if kernels[name]["frac_hbm"] >= kernels[name]["frac_mfma"] else "mfma"
    dominant = max((n for n in timing if cost[n][0]), key=lambda n: timing[n][1])
    d_avg = timing[dominant][1] / timing[dominant][0]
    d_bytes = cost[dominant][0]
    achieved = d_bytes / d_avg / 1e6
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(dominant) if (args.scale == 1.0 and args.workload == "shard" and args.dtype == "f32") else None,
                "algorithmic_bytes_per_launch": int(d_bytes), "avg_launch_ms": round(d_avg, 4)}
    if kernels[dominant].get("binding") == "mfma":     # a dense product nearer its matrix-core peak than its HBM peak
        peak = round(mfma_peak_of(dominant)[0], 1)
        tf = cost[dominant][1] / d_avg / 1e9
        roofline.update({"bound": "mfma", "achieved": round(tf, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4),
                         "algorithmic_flops_per_launch": int(cost[dominant][1])})
    if roofline["bound"] == "hbm" and achieved > HBM_PEAK_GBS:
        roofline["note"] = ("above the HBM peak: the algorithmic count charges one operand row per stored entry, but the "
                            "column windows (or an operand that fits the Infinity Cache) serve part of the gathers from cache")
    # all sparse-product kernels together, the figure the metric names
    sp = [(n, c, t) for n, (c, t) in timing.items() if n.startswith("spmm_")]
    sp_ms = sum(t for _, _, t in sp) / args.steps
    sp_by = sum(cost[n][0] * c for n, c, _ in sp) / args.steps
    sp_fl = sum(cost[n][1] * c for n, c, _ in sp) / args.steps
    spmm = {"ms_per_step": round(sp_ms, 4), "GBps": round(sp_by / sp_ms / 1e6, 1),
            "frac_of_8TBps": round(sp_by / sp_ms / 1e6 / HBM_PEAK_GBS, 4), "GFLOPs": round(sp_fl / sp_ms / 1e6, 1)}

    # one entry per sparse product (orientation, width): its kernels together
    calls = {}
    for n, c, t in sp:
        m_ = re.match(r"spmm_\w+<(f32|bf16),G\d+,VW\d+,d(\d+)>\[(A|At)\]", n)
        key = (m_.group(3), int(m_.group(2)), m_.group(1))
        e = calls.setdefault(key, {"ms": 0.0, "bytes": 0.0, "flops": 0.0, "launches": 0.0})
        e["ms"] += t / args.steps; e["bytes"] += cost[n][0] * c / args.steps; e["flops"] += cost[n][1] * c / args.steps
        e["launches"] = max(e["launches"], c / args.steps)
    spmm_calls = []
    for (o, d, dt), e in sorted(calls.items()):
        rows_o = sum(bins[o][0]); cols_o = sum(bins["At" if o == "A" else "A"][0]); s_ = 4 if dt == "f32" else 2
        b_min = (8 * csr.nnz + 4 * (rows_o + 1) + s_ * d * (rows_o + cols_o)) * e["launches"]
        spmm_calls.append({"matrix": o, "width": d, "dtype": dt, "calls_per_step": e["launches"], "ms": round(e["ms"], 4),
                           "GFLOPs": round(e["flops"] / e["ms"] / 1e6, 1),
                           "GBps_no_reuse": round(e["bytes"] / e["ms"] / 1e6, 1),
                           "frac_of_8TBps": round(e["bytes"] / e["ms"] / 1e6 / HBM_PEAK_GBS, 4),
                           "GBps_perfect_reuse_bound": round(b_min / e["ms"] / 1e6, 1)})

    cpu = None
    if not args.no_cpu_baseline:
        div = args.cpu_sample_div or {"shard": 2, "shard_sparse": 1, "tiny": 1, "road": 32, "road_full": 32}.get(args.workload, 4)
        if cfg.kind == "shard":
            rowptr, col, val, X, W, dF = cpu_inputs
            cpu = cpu_baseline(cfg, rowptr, col, val, X.float(), W, dF.float(), div)
        else:
            cpu = cpu_baseline_network(cfg, div, unit)

    out = {
        "metric": METRIC, "value": round(ms_per_step, 4), "unit": unit,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": workload, **shape, "nnz": csr.nnz,
                   "rows_entries_by_bin(<256,<4096,>=4096)": {k_: [list(v[0]), list(v[1])] for k_, v in bins.items()}},
        "roofline": roofline, "cpu_baseline": cpu, "spmm": spmm, "spmm_calls": spmm_calls, "kernels": kernels,
        "trials": {"ms_per_step": [round(x, 4) for x in trial_ms], "mean": round(sum(trial_ms) / len(trial_ms), 4),
                   "min": round(min(trial_ms), 4)},
        "setup_s": {"generate": round(t_gen, 2), "csr_build_transpose_bins": round(t_build, 2)},
    }
    if stream_ref:
        out["stream_ref"] = stream_ref
    if graph_ms is not None:
        out["graph_ms_per_step"] = round(graph_ms, 4)
    print(json.dumps(out))


def cpu_baseline(cfg, rowptr, col, val, X, W, dF, div):
    """The oracle as it stands, on 1/div of the block: rows [0, m/div) for Eq. 2.1-2.6 and output
    rows [0, k/div) for Eq. 2.7; each part's time is scaled by div."""
    import numpy as np
    import oracle
    mb, kb = max(1, cfg.m // div), max(1, cfg.k // div)
    rp = rowptr.cpu().numpy(); c = col.cpu().numpy(); v = val.cpu().numpy()
    Xh = X.cpu().numpy(); Wh = W.cpu().numpy().astype(np.float64); dFh = dF[:mb].cpu().numpy().astype(np.float64)
    nb = int(rp[mb])
    row_b = np.repeat(np.arange(mb, dtype=np.int64), np.diff(rp[:mb + 1]))
    col_b = c[:nb].astype(np.int64); val_b = v[:nb].astype(np.float64)
    X64 = Xh.astype(np.float64)
    # entries of the whole block that land in output rows [0, kb) of the transposed product
    keep = c < kb
    row_t = np.repeat(np.arange(cfg.m, dtype=np.int64), np.diff(rp))[keep]
    col_t = c[keep].astype(np.int64); val_t = v[keep].astype(np.float64)
    dS_full = np.random.default_rng(0).standard_normal((cfg.m, cfg.dims[0]))
    t = {}
    t0 = time.perf_counter(); H = oracle.spmm_coo(mb, row_b, col_b, val_b, X64); t["spmm"] = time.perf_counter() - t0
    t0 = time.perf_counter(); Q = oracle.gemm(H, Wh); t["gemm_nn"] = time.perf_counter() - t0
    t0 = time.perf_counter(); oracle.relu(Q); dQ = oracle.relu_bwd(Q, dFh); t["act"] = time.perf_counter() - t0
    t0 = time.perf_counter(); oracle.gemm(H, dQ, ta=True); t["gemm_tn"] = time.perf_counter() - t0
    t0 = time.perf_counter(); oracle.gemm(dQ, Wh, tb=True); t["gemm_nt"] = time.perf_counter() - t0
    t0 = time.perf_counter(); oracle.spmm_t_coo(kb, row_t, col_t, val_t, dS_full); t["spmm_t"] = time.perf_counter() - t0
    total = sum(t.values())
    return {"value": round(total * div * 1e3, 1), "unit": "ms per GCN layer fwd+bwd", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"1/{div} of the block (rows [0,{mb}) for Eq. 2.1-2.6, output rows [0,{kb}) for Eq. 2.7), "
                      f"{total:.1f} s of CPU work, each part scaled by {div}",
            "parts_s": {k_: round(v_, 3) for k_, v_ in t.items()}}


def cpu_baseline_network(cfg, div, unit):
    """The oracle's whole-network forward + backward (Eq. 2.1-2.7 and the loss head) on the same
    recipe shrunk to 1/div of the nodes and edges (same degree distribution and widths); time
    scaled by div."""
    import oracle
    from oracle import gcn as ogcn
    small = cfg if div == 1 else cfg.scaled(1.0 / div)
    src, dst = small.edges()
    F0 = small.features().numpy()
    Ws = [w.numpy() for w in small.weights()]
    y = small.labels().numpy()
    adj = oracle.adjacency(small.n, src.numpy(), dst.numpy())
    t0 = time.perf_counter()
    ogcn.forward_backward(adj, F0, Ws, y)
    total = time.perf_counter() - t0
    return {"value": round(total * div * 1e3, 1), "unit": unit, "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"same generator at 1/{div} of the nodes and edges (n = {small.n}, nnz = {adj.nnz}), "
                      f"{total:.1f} s of CPU work, scaled by {div}"}


if __name__ == "__main__":
    main()
