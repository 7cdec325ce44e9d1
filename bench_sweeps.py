#!/usr/bin/env python3
"""Side measurements that are not the benchmark (bench.py is): each prints one JSON line.

  --paper-sweep   the shape of the paper's kernel-scaling experiment (Sec. 5.1): B=32, 4 heads, C=64,
                  sequence lengths 1K..16K, every method, 5 warm-up + 20 timed launches with the cache
                  cleared (a 512 MiB read) before each, HIP events around the single launch, median
  --vendor-ref    torch.linalg.solve_triangular (the ROCm libraries' batched triangular solve) on the
                  chunk matrices of a workload, beside this library's forward substitution
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def paper_sweep(tri, si, torch, np, dev):
    flush = torch.empty(1 << 27, dtype=torch.float32, device=dev).normal_()
    rows = []
    variants = [("fwd_subst", 0, 0), ("block_recursive", 1, 2), ("mixed", 3, 2), ("mixed_b32", 6, 2), ("block_direct", 4, 2),
                ("neumann", 2, 2), ("newton_schulz", 5, 2)]
    for Tlen in (1024, 2048, 4096, 8192, 16384):
        ws = si.workload(2, B=32, Tlen=Tlen, H=4)
        si_inp = si.make_inputs(ws)
        K, beta, g = si_inp["K"].to(dev), si_inp["beta"].to(dev), si_inp["g"].to(dev)
        T = torch.empty((ws.n_mat, 64, 64), device=dev)
        A32 = tri.gdn_chunk_build_A(K, beta, g, 64, op_dtype=tri.F32)
        for name, method, op in variants:
            for entry in ("fused", "standalone"):
                ms = []
                for i in range(25):
                    sink = flush.sum()  # noqa: F841  (the read that clears the caches)
                    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    a.record()
                    if entry == "fused":
                        tri.gdn_chunk_tri_inv_ex(K, beta, g, 64, T=T, method=method, op_dtype=op)
                    else:
                        tri.tri_inv_ex(A32, T=T, method=method, op_dtype=op)
                    b.record()
                    torch.cuda.synchronize()
                    if i >= 5:
                        ms.append(a.elapsed_time(b))
                rows.append({"Tlen": Tlen, "n_mat": ws.n_mat, "method": name, "op": tri.DTYPE_NAMES[op], "entry": entry,
                             "us_median": float(np.median(ms)) * 1e3, "us_min": float(np.min(ms)) * 1e3,
                             "matrices_per_s": ws.n_mat / (float(np.median(ms)) * 1e-3)})
        del K, beta, g, T, A32
    return {"paper_sweep": rows, "protocol": "B=32, H=4, d_k=128, C=64, bf16 keys, scalar gate; per point 5 warm-up + 20 "
            "timed launches, a 512 MiB read before each to clear the caches, HIP events around the single launch, median"}


def vendor_ref(tri, si, torch, dev, workload):
    w = si.WORKLOADS[workload]
    inp = si.make_inputs(w)
    K, beta = inp["K"].to(dev), inp["beta"].to(dev)
    g = None if inp["g"] is None else inp["g"].to(dev)
    n_mat, C = w.n_mat, w.C
    A32 = tri.gdn_chunk_build_A(K, beta, g, C, gate_kind=w.gate_kind, op_dtype=tri.F32)
    M = A32 + torch.eye(C, device=dev)
    eye = torch.eye(C, device=dev).expand(n_mat, C, C).contiguous()
    for _ in range(2):
        Tv = torch.linalg.solve_triangular(M, eye, upper=False, unitriangular=True)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        Tv = torch.linalg.solve_triangular(M, eye, upper=False, unitriangular=True)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 5
    Tours = tri.tri_inv_ex(A32, method=tri.FWD_SUBST)
    torch.cuda.synchronize()
    return {"vendor_ref": {"call": "torch.linalg.solve_triangular(I + A, I, upper=False, unitriangular=True), fp32",
                           "workload": w.index, "ms": ms, "matrices_per_s": n_mat / (ms * 1e-3),
                           "max_abs_diff_to_tri_inv_fwd_subst": float((Tv - Tours).abs().max())}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--paper-sweep", action="store_true")
    ap.add_argument("--vendor-ref", action="store_true")
    ap.add_argument("--workload", type=int, default=2)
    args = ap.parse_args()

    import numpy as np
    import torch

    import synth_inputs as si
    import paper_2605_21325_amd as tri

    if not torch.cuda.is_available():
        print("bench_sweeps.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    out = {}
    if args.paper_sweep:
        out.update(paper_sweep(tri, si, torch, np, dev))
    if args.vendor_ref:
        out.update(vendor_ref(tri, si, torch, dev, args.workload))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
