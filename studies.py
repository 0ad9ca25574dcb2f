#!/usr/bin/env python3
"""Two measurement studies on one MI355X, analogues of the paper's Table 3 and Table 2 on the
synthetic workloads (the paper's datasets are not available).  Each prints one JSON object.

  python studies.py balance [--workload road] [--scale 1.0]
      Block balance under no / single / double permutation (Table 3: max / mean of the stored
      entries over an 8 x 8 tiling), plus the sparse product's time on each of the three stored
      matrices at width 64 -- what the double permutation costs in locality on ONE GPU.

  python studies.py skinny
      Tall-skinny sensitivity (Sec. 4.1, Table 2): at equal flops, configuration U_g (the
      adjacency block has K/g columns, the dense operand keeps width 128) against V_g (full K,
      dense operand 128/g wide), g = 1, 4, 16, 64.

  python studies.py skinny --launch-log DIR/<run>/launches.txt   (under rocprofv3 --pmc), then
  python studies.py skinny-table --dir DIR
      The same cases with hardware counters per case: HBM bytes read and written, L2 hit rate, wavefronts launched.

  python studies.py blocks [--scale 1.0]
      Blocked aggregation (Sec. 5.2) on the shard block: the forward product at width 32 and the
      transposed product (also width 32, as in the layer's backward pass) with the rows cut into 1, 2, 4, 8, 16, 32 blocks -- the
      one-GPU cost of issuing the aggregation as separate per-block launches, which is what a
      multi-GPU run overlaps with the per-block all-reduce.

  python studies.py windows [--workload shard|social|copurchase]
      Column windows of the sparse product: time of A X and A^T G with the rows of 256+ entries
      cut into 1 (off), 2, 4, 8, 16, 32 column windows, at the widths the workload uses.
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

import torch

import paper_2505_04083_amd as plx
import synth

DEV = torch.device("cuda", 0)


def time_spmm(ctx, csr, X, Y, reps=5):
    plx.plx_spmm(ctx, csr, X, Y)
    plx.plx_sync(ctx)
    t0 = time.perf_counter()
    for _ in range(reps):
        plx.plx_spmm(ctx, csr, X, Y)
    plx.plx_sync(ctx)
    return (time.perf_counter() - t0) * 1e3 / reps


def spmm_bytes(csr, d, transposed=False):
    rows, ent = plx.plx_csr_bins(csr, transposed)
    return sum(ent) * (8 + 4 * d) + sum(rows) * (4 + 4 * d)


def block_ratio(ctx, csr, n, blocks=8):
    """max / mean of the entry counts over a blocks x blocks tiling of the stored matrix."""
    rowptr, col, _ = plx.plx_csr_export(ctx, csr)
    edges = (torch.arange(blocks + 1, device=DEV, dtype=torch.int64) * n) // blocks
    row_block = torch.bucketize(torch.arange(n, device=DEV), edges[1:], right=True)
    rb = torch.repeat_interleave(row_block, rowptr[1:] - rowptr[:-1])
    cb = torch.bucketize(col.to(torch.int64), edges[1:], right=True)
    cnt = torch.bincount(rb * blocks + cb, minlength=blocks * blocks).double()
    return float(cnt.max() / cnt.mean())


def balance(args):
    cfg = synth.CONFIGS[args.workload]
    if args.scale != 1.0:
        cfg = cfg.scaled(args.scale)
    ctx = plx.plx_ctx(0)
    src, dst = cfg.edges(DEV)
    pr, pc = cfg.perms(DEV)
    d = 64
    X = synth.normal(cfg.seed, synth.S_FEAT, cfg.n, d, DEV)
    Y = torch.empty(cfg.n, d, device=DEV)
    out = {"study": "block balance and locality under permutation (Table 3 analogue)", "workload": cfg.name,
           "n": cfg.n, "blocks": "8x8", "width": d, "cases": {}}
    for name, (a, b) in {"original": (None, None), "single_permutation": (pr, pr), "double_permutation": (pr, pc)}.items():
        csr = plx.plx_build_csr(ctx, cfg.n, src, dst, a, b)
        ms = time_spmm(ctx, csr, X, Y)
        by = spmm_bytes(csr, d)
        out["cases"][name] = {"max_over_mean": round(block_ratio(ctx, csr, cfg.n), 4), "spmm_ms": round(ms, 3),
                              "algorithmic_GBps": round(by / ms / 1e6, 1)}
        out["nnz"] = csr.nnz
        csr.close()
    nnz, n, B = out["nnz"], cfg.n, 8
    out["single_permutation_closed_form"] = round(((nnz - n) / B**2 + n / B) / (nnz / B**2), 4)
    print(json.dumps(out))


def skinny(args):
    ctx = plx.plx_ctx(0)
    m, k, samples, width = 2_000_000, 8_000_000, 64_000_000, 128
    out = {"study": "tall-skinny sensitivity at equal flops (Table 2 analogue)", "m": m, "k": k, "cases": []}
    log = open(args.launch_log, "w") if args.launch_log else None       # profiler runs: ONE product per case, its launches named
    for g in (1, 4, 16, 64):
        for label, kk, ss, d in (("U", k // g, samples // g, width), ("V", k, samples, width // g)):
            if g == 1 and label == "V":
                continue
            rowptr, col, val = synth.shard_block(synth.BASE_SEED + 40 + g, m, kk, ss, DEV)
            csr = plx.plx_csr_import(ctx, m, kk, rowptr, col, val)
            X = synth.normal(7, synth.S_FEAT, kk, d, DEV)
            Y = torch.empty(m, d, device=DEV)
            if log:
                plx.plx_timing_enable(ctx, True)
                plx.plx_spmm(ctx, csr, X, Y)
                for name, ms in plx.plx_timing_trace(ctx):
                    log.write(f"{label}_{g} {name} {ms:.4f}\n")
                plx.plx_timing_enable(ctx, False)
                csr.close()
                del rowptr, col, val, X, Y
                continue
            ms = time_spmm(ctx, csr, X, Y)
            out["cases"].append({"config": f"{label}_{g}", "cols": kk, "nnz": csr.nnz, "width": d,
                                 "GFLOP": round(2 * csr.nnz * d / 1e9, 2), "spmm_ms": round(ms, 3),
                                 "GFLOPs": round(2 * csr.nnz * d / ms / 1e6, 1),
                                 "algorithmic_GBps": round(spmm_bytes(csr, d) / ms / 1e6, 1)})
            csr.close()
            del rowptr, col, val, X, Y
    if log:
        log.close()
        return
    print(json.dumps(out))


def skinny_table(args):
    """Table 2 analogue from profiler output: DIR/a and DIR/b hold `rocprofv3 --pmc ... --kernel-include-regex k_spmm` runs of
    `studies.py skinny --launch-log DIR/<run>/launches.txt` (a: FETCH_SIZE SQ_WAVES, b: WRITE_SIZE TCC_HIT_sum TCC_MISS_sum)."""
    import csv
    import glob
    import re
    d = args.dir
    per_case = {}
    for run in ("a", "b"):
        f = glob.glob(os.path.join(d, run, "**", "*counter_collection.csv"), recursive=True)[0]
        disp = {}
        for r in csv.DictReader(open(f)):
            if "k_spmm" not in r["Kernel_Name"]:
                continue
            e = disp.setdefault(int(r["Dispatch_Id"]), {"kernel": re.sub(r".*(k_spmm_\w+).*", r"\1", r["Kernel_Name"]), "grid": int(r["Grid_Size"])})
            e[r["Counter_Name"]] = float(r["Counter_Value"])
        disp = [disp[i] for i in sorted(disp)]
        i = 0
        for line in open(os.path.join(d, run, "launches.txt")):
            case, name, ms = line.split()
            n = 2 if name.startswith("spmm_split") else 1           # segment + combine kernels
            c = per_case.setdefault(case, {"ms": 0.0, "grid": 0})
            if run == "a":
                c["ms"] += float(ms)
            for e in disp[i:i + n]:
                kind = name.split("<")[0].replace("spmm_", "")
                assert {"subwave": "k_spmm_subwave", "wave": "k_spmm_wave", "split": "k_spmm_"}[kind] in e["kernel"], (case, name, e)
                for k_, v in e.items():
                    if k_ not in ("kernel", "grid"):
                        c[k_] = c.get(k_, 0.0) + v
                if run == "a":
                    c["grid"] += e["grid"]
            i += n
        assert i == len(disp), (run, i, len(disp))
    print("| case | ms (one product, under the profiler) | HBM read GB | HBM written GB | HBM GB/s | % of 8 TB/s | L2 hit % | wavefronts | work-items launched |")
    print("|---|---|---|---|---|---|---|---|---|")
    for case, c in per_case.items():
        rd, wr = c["FETCH_SIZE"] * 1024 * 2.0, c["WRITE_SIZE"] * 1024          # FETCH_SIZE counts half of what a plain copy reads
        hit = c["TCC_HIT_sum"] / max(c["TCC_HIT_sum"] + c["TCC_MISS_sum"], 1.0)
        bw = (rd + wr) / c["ms"] / 1e6
        print(f"| {case} | {c['ms']:.3f} | {rd / 1e9:.2f} | {wr / 1e9:.2f} | {bw:.0f} | {bw / 80:.0f} | {hit * 100:.0f} | "
              f"{int(c['SQ_WAVES'])} | {c['grid']} |")


def blocks(args):
    ctx = plx.plx_ctx(0)
    cfg = synth.CONFIGS["shard"]
    m, k, samples = (int(cfg.m * args.scale), int(cfg.k * args.scale), int(cfg.n_samples * args.scale))
    rowptr, col, val = synth.shard_block(cfg.seed, m, k, samples, DEV)
    csr = plx.plx_csr_import(ctx, m, k, rowptr, col, val)
    del rowptr, col, val
    X = synth.normal(cfg.seed, synth.S_FEAT, k, 32, DEV)
    Y = torch.empty(m, 32, device=DEV)
    G = synth.normal(cfg.seed, synth.S_AUX, m, 32, DEV)
    Gt = torch.empty(k, 32, device=DEV)
    out = {"study": "blocked aggregation, per-block launches on one GPU (Sec. 5.2)", "m": m, "k": k, "nnz": csr.nnz,
           "cases": []}
    for nb in (1, 2, 4, 8, 16, 32):
        plx.plx_csr_set_row_blocks(ctx, csr, nb)
        fwd = time_spmm(ctx, csr, X, Y)
        plx.plx_spmm_t(ctx, csr, G, Gt); plx.plx_sync(ctx)
        reps = 5
        t0 = time.perf_counter()
        for _ in range(reps):
            plx.plx_spmm_t(ctx, csr, G, Gt)
        plx.plx_sync(ctx)
        bwd = (time.perf_counter() - t0) * 1e3 / reps
        per_block = []
        for b in range(nb):
            plx.plx_spmm_block(ctx, csr, False, b, X, Y); plx.plx_sync(ctx)
            t0 = time.perf_counter()
            plx.plx_spmm_block(ctx, csr, False, b, X, Y); plx.plx_sync(ctx)
            per_block.append((time.perf_counter() - t0) * 1e3)
        out["cases"].append({"n_blocks": nb, "spmm_d32_ms": round(fwd, 3), "spmm_t_d32_ms": round(bwd, 3),
                             "block_ms_min": round(min(per_block), 3), "block_ms_max": round(max(per_block), 3)})
    print(json.dumps(out))


def windows(args):
    cfg = synth.CONFIGS[args.workload if args.workload in ("shard", "social", "copurchase") else "shard"]
    ctx = plx.plx_ctx(0)
    if cfg.kind == "shard":
        rowptr, col, val = synth.shard_block(cfg.seed, cfg.m, cfg.k, cfg.n_samples, DEV)
        m, k, widths = cfg.m, cfg.k, [cfg.dims[0]]
    else:
        src, dst = cfg.edges(DEV)
        pr, pc = cfg.perms(DEV)
        m = k = cfg.n
        widths = sorted(set(min(a, b) for a, b in zip(cfg.dims[:-1], cfg.dims[1:])))    # the narrower side of every layer
    out = {"study": "column windows of the sparse product", "workload": cfg.name, "rows": m, "cols": k, "cases": []}
    for nw in (1, 2, 4, 8, 16, 32):
        plx.plx_ctx_set_column_windows(ctx, nw)
        if cfg.kind == "shard":
            csr = plx.plx_csr_import(ctx, m, k, rowptr, col, val)
        else:
            csr = plx.plx_build_csr(ctx, cfg.n, src, dst, pr, pc)
        case = {"n_windows": nw}
        for d in widths:
            ld = -(-d // 16) * 16                    # rows padded to 64 bytes
            X = torch.zeros(k, ld, device=DEV)[:, :d]; X.copy_(synth.normal(cfg.seed, synth.S_FEAT, k, d, DEV))
            G = torch.zeros(m, ld, device=DEV)[:, :d]; G.copy_(synth.normal(cfg.seed, synth.S_AUX, m, d, DEV))
            Y = torch.empty(m, ld, device=DEV)[:, :d]
            Yt = torch.empty(k, ld, device=DEV)[:, :d]
            case[f"AX_d{d}_ms"] = round(time_spmm(ctx, csr, X, Y), 3)
            plx.plx_spmm_t(ctx, csr, G, Yt); plx.plx_sync(ctx)
            t0 = time.perf_counter()
            for _ in range(5):
                plx.plx_spmm_t(ctx, csr, G, Yt)
            plx.plx_sync(ctx)
            case[f"AtG_d{d}_ms"] = round((time.perf_counter() - t0) * 1e3 / 5, 3)
            del X, Y, G, Yt
        out["nnz"] = csr.nnz
        out["cases"].append(case)
        csr.close()
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("study", choices=["balance", "skinny", "skinny-table", "blocks", "windows"])
    ap.add_argument("--launch-log", default="", help="skinny: run ONE product per case and write its timed launches here (profiler runs)")
    ap.add_argument("--dir", default="", help="skinny-table: directory with the profiler output")
    ap.add_argument("--workload", default="road", choices=["tiny", "social", "copurchase", "road", "shard"])
    ap.add_argument("--scale", type=float, default=1.0)
    args = ap.parse_args()
    if args.study == "skinny-table":
        return skinny_table(args)
    assert torch.cuda.is_available(), "studies.py needs a GPU"
    torch.cuda.set_device(DEV)
    {"balance": balance, "skinny": skinny, "blocks": blocks, "windows": windows}[args.study](args)


if __name__ == "__main__":
    main()
