#!/usr/bin/env python3
"""Benchmark of the per-GPU GCN hot path on one MI355X.

One "step" = one GCN layer forward + backward (every row of the hot path: sparse product,
dense product, activation, activation gradient, transposed sparse product, the two backward
dense products) on the workload the headline metric is quoted on: ONE GPU's SHARD of a
billion-edge graph -- a 7M x 28M double-permuted adjacency block with ~200M stored entries,
feature slice 28M x 32, weight slice 32 x 128 (fp32), run in the paper's order (Eq. 2.1 then
2.2: aggregate at width 32, then combine).  Inputs are synthetic, seeded, generated on the GPU
and resident in HBM before the timed region.

Prints ONE JSON line.  Besides the contract keys it carries
  "roofline":     the dominant kernel's algorithmic HBM bytes / its average duration (HIP events
                  recorded around every launch inside the timed steps) against 8 TB/s,
  "cpu_baseline": the CPU oracle timed on a bounded sample of the same workload,
  "kernels":      per-kernel ms / GB/s / GFLOP/s of one step (information only).
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

HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3
METRIC = "GCN layer fwd+bwd ms; SpMM achieved HBM GB/s (% roofline) on 1 MI355X"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (testing only; <1 is not the metric)")
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32",
                    help="storage type of activations / gradients (the headline metric is f32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-div", type=int, default=2, help="oracle sample = 1/div of the rows")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run one plain device copy of known size (reference dispatch for counter scaling)")
    return ap.parse_args()


ELT = 4   # bytes per dense element (set from --dtype)


def spmm_bytes(rows, entries, d, s=None):
    """Algorithmic bytes of a sparse product over `rows` rows holding `entries` stored entries:
    8 B of CSR per entry (value + column), one s*d-byte gathered operand row per entry (the
    double permutation leaves no reuse between entries), a 4 B row pointer and one s*d-byte
    output row per row."""
    s = ELT if s is None else s
    return entries * (8 + s * d) + rows * (4 + s * d)


def measured_traffic(name):
    """HBM bytes per launch of the kernel behind a timing label, from the committed rocprofv3
    FETCH_SIZE / WRITE_SIZE summary of this same workload (profiles/traffic_layer_shard_f32.json,
    counters already scaled by a plain 4 GiB copy); None if the summary has no such kernel."""
    path = os.path.join(ROOT, "profiles", "traffic_layer_shard_f32.json")
    if not os.path.exists(path):
        return None
    k = json.load(open(path))["kernels"]
    import re
    m = re.match(r"spmm_(subwave|wave|split)<(f32|bf16),G(\d+),VW(\d+)>\[(A|At)\]", name)
    keys = []
    if m:
        kind, dt, g, vw, o = m.groups()
        t = "float" if dt == "f32" else "unsigned short"
        base = {"subwave": ["k_spmm_subwave"], "wave": ["k_spmm_wave"], "split": ["k_spmm_segment"]}[kind]
        keys = [f"{b}<{t}, {g}, {vw}> [{o}]" for b in base]
        if kind == "split":
            keys.append(f"k_spmm_combine<{t}> [{o}]")
    elif name.startswith("gemm_nn"):
        keys = [x for x in k if x.startswith("k_gemm_small_f32") or x.startswith("k_gemm_f32")]
    elif name.startswith("bwd_dense"):
        keys = [x for x in k if x.startswith("k_bwd_dense_f32")]
    if not keys or any(x not in k for x in keys):
        return None
    return sum(k[x]["fetch_bytes"] + k[x]["write_bytes"] for x in keys)


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus {args.gpus} is not "
              "supported. value is one GPU's throughput; run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_04083_amd as plx
    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    cfg = synth.CONFIGS["shard"]
    if args.scale != 1.0:
        cfg = cfg.scaled(args.scale)
    din, dout = cfg.dims
    global ELT
    tdt = torch.float32 if args.dtype == "f32" else torch.bfloat16
    ELT = 4 if args.dtype == "f32" else 2
    code = plx.PLX_F32 if args.dtype == "f32" else plx.PLX_BF16

    t0 = time.time()
    rowptr, col, val = synth.shard_block(cfg.seed, cfg.m, cfg.k, cfg.n_samples, dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t0
    nnz = int(col.numel())
    X = synth.normal(cfg.seed, synth.S_FEAT, cfg.k, din, dev, tdt)
    dF = synth.normal(cfg.seed, synth.S_AUX, cfg.m, dout, dev, tdt)
    W = synth.glorot(cfg.seed, 0, din, dout, dev)

    ctx = plx.plx_ctx(0)
    t0 = time.time()
    csr = plx.plx_csr_import(ctx, cfg.m, cfg.k, rowptr, col, val)
    t_import = time.time() - t0
    order = plx.PLX_ORDER_AGG_FIRST
    ws = torch.empty(plx.plx_gcn_layer_workspace(csr, False, din, dout, code, plx.PLX_ACT_RELU, order),
                     dtype=torch.uint8, device=dev)
    F = torch.empty(cfg.m, dout, device=dev, dtype=tdt)   # only the activated output is stored (its sign serves Eq. 2.4)
    saved = torch.empty(cfg.m, din, device=dev, dtype=tdt)
    dX = torch.empty(cfg.k, din, device=dev, dtype=tdt); dW = torch.empty(din, dout, device=dev)

    def step():
        plx.plx_gcn_layer_fwd(ctx, csr, False, X, W, None, F, saved, ws, act=plx.PLX_ACT_RELU, order=order)
        plx.plx_gcn_layer_bwd(ctx, csr, False, X, W, F, dF, saved, dX, dW, ws, act=plx.PLX_ACT_RELU, order=order)

    if args.copy_ref:
        # 2^30 fp32 read + 2^30 fp32 written by one plain copy kernel: the known-size dispatch the
        # FETCH_SIZE / WRITE_SIZE counters are scaled by
        ref_src = torch.ones(1 << 30, dtype=torch.float32, device=dev)
        ref_dst = torch.empty_like(ref_src)
        for _ in range(3):
            ref_dst.copy_(ref_src)
        torch.cuda.synchronize()
        del ref_src, ref_dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
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

    # ---- per-kernel accounting (algorithmic bytes / flops of one launch) -------------------------
    (rows_f, ent_f), (rows_b, ent_b) = plx.plx_csr_bins(csr, False), plx.plx_csr_bins(csr, True)
    m, k = cfg.m, cfg.k
    alg = {}
    for name in timing:
        b = fl = None
        if name.startswith("spmm_"):
            rows, ent = (rows_b, ent_b) if name.endswith("[At]") else (rows_f, ent_f)
            i = {"spmm_subwave": 0, "spmm_wave": 1, "spmm_split": 2}[name.split("<")[0]]
            b, fl = spmm_bytes(rows[i], ent[i], din), 2 * ent[i] * din
        elif name.startswith("gemm_nn"):
            b, fl = ELT * (m * din + m * dout) + 4 * din * dout, 2 * m * din * dout
        elif name.startswith("bwd_dense"):       # reads dF, F (mask), saved; writes dS; two products
            b, fl = ELT * (2 * m * dout + 2 * m * din) + 4 * din * dout, 4 * m * din * dout
        elif name.startswith("gemm_nt"):
            b, fl = 4 * (m * dout + din * dout + m * din), 2 * m * din * dout
        elif name.startswith("gemm_tn<"):
            b, fl = 4 * (m * din + m * dout + din * dout), 2 * m * din * dout
        elif name == "relu":
            b, fl = 4 * 2 * m * dout, 0
        elif name == "relu_bwd":
            b, fl = 4 * 3 * m * dout, 0
        alg[name] = (b, fl)
    kernels = {}
    for name, (count, total_ms) in timing.items():
        avg = total_ms / max(count, 1)
        b, fl = alg.get(name, (None, None))
        kernels[name] = {"launches_per_step": count / args.steps, "avg_ms": round(avg, 4),
                         "GBps": None if not b else round(b / avg / 1e6, 1),
                         "GFLOPs": None if not fl else round(fl / avg / 1e6, 1)}
    dominant = max(timing, key=lambda n: timing[n][1])
    d_avg = timing[dominant][1] / timing[dominant][0]
    d_bytes = alg[dominant][0]
    achieved = d_bytes / d_avg / 1e6
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(dominant) if (args.scale == 1.0 and args.dtype == "f32") else None,
                "algorithmic_bytes_per_launch": int(d_bytes), "avg_launch_ms": round(d_avg, 4)}
    # whole sparse products (all their kernels), the figure the metric names
    def spmm_total(tag, rows, ent):
        ms = sum(t / c for n, (c, t) in timing.items() if n.startswith("spmm_") and n.endswith(tag))
        by = sum(spmm_bytes(rows[i], ent[i], din) for i in range(3))
        return {"ms": round(ms, 4), "GBps": round(by / ms / 1e6, 1), "frac_of_8TBps": round(by / ms / 1e6 / HBM_PEAK_GBS, 4),
                "GFLOPs": round(2 * sum(ent) * din / ms / 1e6, 1)}
    spmm = {"A_x_X": spmm_total("[A]", rows_f, ent_f), "At_x_G": spmm_total("[At]", rows_b, ent_b)}

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, rowptr, col, val, X.float(), W, dF.float(), args.cpu_sample_div)

    out = {
        "metric": METRIC, "value": round(ms_per_step, 4), "unit": "ms per GCN layer fwd+bwd",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"configs[3]: one GPU's 7M x 28M shard block of a billion-edge graph, {args.dtype}, "
                               "layer 32 -> 128, aggregate-first" + ("" if args.scale == 1.0 else f" (SHRUNK x{args.scale})"),
                   "m": m, "k": k, "nnz": nnz, "din": din, "dout": dout, "order": "agg_first",
                   "rows_entries_by_bin(<256,<4096,>=4096)": {"A": [list(rows_f), list(ent_f)], "At": [list(rows_b), list(ent_b)]}},
        "roofline": roofline, "cpu_baseline": cpu, "spmm": spmm, "kernels": kernels,
        "setup_s": {"generate": round(t_gen, 2), "csr_import_transpose_bins": round(t_import, 2)},
    }
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


if __name__ == "__main__":
    main()
