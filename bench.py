#!/usr/bin/env python3
"""Benchmark of the batched triangular-inversion hot path on one MI355X.

A "step" is one pass of the whole hot path -- load keys/beta/g, Gram on the matrix cores,
gate + mask, inversion, store of T -- over one batch of synthetic input, i.e. one call of the
fused C-ABI entry point `gdn_chunk_tri_inv_ex` on workload 2 (B=8, T=8192, H=16, d_k=128, C=64:
16 384 chunk matrices, bf16 keys, scalar gate).  Inputs are resident in HBM before the timed
region.  The timed steps rotate over several distinct input/output buffer sets so that no step
finds its data in the 256 MB last-level cache left by the previous one.

Prints ONE JSON line: the contract fields plus
  roofline      achieved algorithmic GB/s of the kernel (HIP events on the launch stream) vs 8 TB/s
  cpu_baseline  the fp64 oracle timed on the host cores on the same batch
  parity        sampled outputs of the timed configuration checked against the oracle
  methods       (with --table) matrices/s for every method / operand type, standalone and fused
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
METRIC = "64x64 tri-inversions/sec + effective TFLOP/s & GB/s vs roofline; rel error"

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command (the counters
# cannot be read from inside the process): a profiled constant with the summary it was read from, keyed by
# (workload index, method, op_dtype).  Absent = not profiled for that configuration (reported as null).
PROFILED_TRAFFIC = {(2, 1, 2): (545.4e6, "profiles/k_gdn_tri_inv_block_bf16_workload2.txt"),
                    (3, 1, 2): (2150.0e6, "profiles/k_kda_tri_inv_block_bf16_workload3.txt"),
                    (4, 1, 2): (810.0e6, "profiles/k_gdn_tri_inv_c128_block_bf16_workload4.txt")}


def algorithmic_bytes_per_matrix(w, fused: bool, in_bytes: int = 4, out_bytes: int = 4) -> int:
    C, d = w.C, w.d_k
    out = out_bytes * C * C
    if not fused:
        return in_bytes * C * (C - 1) // 2 + out          # strictly-lower A in, dense fp32 T out
    kb = 2 if w.k_dtype == "bf16" else 4
    n = C * d * kb + 4 * C + out                          # K, beta, T
    if w.gate_kind == 0:
        n += 4 * C
    elif w.gate_kind == 1:
        n += 4 * C * d
    return n


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", type=int, default=2)
    ap.add_argument("--method", type=int, default=1, help="0 fwd, 1 block recursive, 2 neumann, 3 mixed, 4 block direct")
    ap.add_argument("--op", type=int, default=2, help="operand type: 0 f32, 1 f16, 2 bf16")
    ap.add_argument("--out", default="f32", choices=["f32", "f16", "bf16"],
                    help="element type of T (the contract's fp32, or a 16-bit result: TRIINV_FLAG_OUT_*)")
    ap.add_argument("--chunk", type=int, default=0, help="override the workload's chunk size C (16, 32, 64, 128)")
    ap.add_argument("--nbuf", type=int, default=4, help="distinct buffer sets the steps rotate over")
    ap.add_argument("--table", action="store_true", help="also time every method / operand type")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--solve-rhs", type=int, default=1, choices=[1, 2],
                    help="with --solve: right-hand sides per launch (2 = two D_X-column tensors sharing one inversion)")
    ap.add_argument("--solve", type=int, default=0, metavar="D_X",
                    help="also time gdn_chunk_tri_solve (the inverse applied to D_X right-hand-side columns instead of stored)")
    ap.add_argument("--accuracy", action="store_true",
                    help="instead of timing: error and residual of every method / operand type against the oracle on "
                         "sampled matrices of the full-size workload, fused entry point and (scalar / no gate) standalone")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run plain device copies of 1 GiB in the same process (under rocprofv3 --pmc their FETCH_SIZE / "
                         "WRITE_SIZE readings give the factors that scale the kernels' readings to bytes)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the chunk matrices are independent; sharding is "
              "a plain split of the batch with no exchange). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import synth_inputs as si
    import paper_2605_21325_amd as tri
    from paper_2605_21325_amd import build as tri_build

    if not os.path.exists(tri.binding.LIB_PATH):
        tri_build.build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    out_torch = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[args.out]
    out_bytes = 4 if args.out == "f32" else 2
    w = si.WORKLOADS[args.workload]
    if args.chunk:
        w = si.workload(args.workload, C=args.chunk)
    inp = si.make_inputs(w)
    n_mat, C = w.n_mat, w.C
    sets = []
    for _ in range(max(1, args.nbuf)):
        K = inp["K"].to(dev)
        beta = inp["beta"].to(dev)
        g = None if inp["g"] is None else inp["g"].to(dev)
        T = torch.empty((n_mat, C, C), dtype=out_torch, device=dev)
        sets.append((K, beta, g, T))
    torch.cuda.synchronize()

    if args.accuracy:
        import oracle
        from oracle import metrics

        rng = np.random.default_rng(2605)
        sel = np.unique(np.concatenate([[0, n_mat - 1], rng.integers(0, n_mat, size=254)])).tolist()
        A_ref = oracle.build_A(inp["K"], inp["beta"], inp["g"], w.gate_kind, C, sel=sel)
        T_ref = oracle.tri_inv(A_ref)
        A32 = torch.from_numpy(A_ref.astype(np.float32)).to(dev)
        T32_ref = oracle.tri_inv(A32.cpu())
        A32_ref = A32.cpu().numpy().astype(np.float64)
        K, beta, g, T = sets[0]
        rows = []

        def stats(Tg, Tr, Ar):
            Tg = Tg.float().cpu().numpy().astype(np.float64)
            e = metrics.forward_errors(Tr, Tg)
            r = metrics.residual(Ar, Tg)
            bad = int((~np.isfinite(e["rel_fro"])).sum())
            with np.errstate(invalid="ignore"):
                return {"rel_fro_max": float(np.nanmax(e["rel_fro"])) if bad < len(sel) else float("nan"),
                        "rel_fro_median": float(np.nanmedian(e["rel_fro"])) if bad < len(sel) else float("nan"),
                        "max_abs_max": float(np.nanmax(e["max_abs"])) if bad < len(sel) else float("nan"),
                        "residual_abs_max": float(np.nanmax(r["abs"])) if bad < len(sel) else float("nan"),
                        "residual_normalised_max": float(np.nanmax(r["normalised"])) if bad < len(sel) else float("nan"),
                        "non_finite_matrices": bad, "structure_ok": bool(metrics.structure_ok(Tg))}

        for method in (0, 1, 4, 3, 6, 2, 5):
            for op in (0, 1, 2):
                if method == 0 and op != 0:
                    continue
                for flags, tag in ((0, ""), (tri.FLAG_REFINE1, "+refine")):
                    if flags and method == 0:
                        continue
                    row = {"method": tri.METHOD_NAMES[method] + tag, "op": tri.DTYPE_NAMES[op]}
                    try:
                        tri.gdn_chunk_tri_inv_ex(K, beta, g, C, T=T, gate_kind=w.gate_kind, method=method, op_dtype=op, flags=flags)
                        torch.cuda.synchronize()
                        row["fused"] = stats(T[sel], T_ref, A_ref)
                    except tri.TriInvError as e:
                        row["fused"] = {"error": str(e)}
                    try:
                        Ts = tri.tri_inv_ex(A32, method=method, op_dtype=op, flags=flags)
                        torch.cuda.synchronize()
                        row["standalone"] = stats(Ts, T32_ref, A32_ref)
                    except tri.TriInvError as e:
                        row["standalone"] = {"error": str(e)}
                    rows.append(row)
        # the inverse applied to right-hand sides: W = (I + A)^{-1} diag(s) X, first batch entry, against the oracle's solve
        solve_rows = []
        d_x = 128
        for op in (0, 1, 2):
            xdt = {0: torch.float32, 1: torch.float16, 2: torch.bfloat16}[op]
            rhs = si.make_rhs(w, d_x, xdt)
            X1, s1 = rhs["X"][:1].contiguous(), rhs["row_scale"][:1].contiguous()
            W_ref = oracle.gdn_chunk_tri_solve(inp["K"][:1], inp["beta"][:1], None if inp["g"] is None else inp["g"][:1], X1, s1,
                                               w.gate_kind, C)
            den = np.sqrt((W_ref ** 2).sum(axis=(1, 3)))
            for method in (1, 3):
                row = {"method": tri.METHOD_NAMES[method], "op": tri.DTYPE_NAMES[op]}
                try:
                    Wg = tri.gdn_chunk_tri_solve(K[:1].contiguous(), beta[:1].contiguous(), None if g is None else g[:1].contiguous(),
                                                 X1.to(dev), C, row_scale=s1.to(dev), gate_kind=w.gate_kind, method=method)
                    torch.cuda.synchronize()
                    Wg = Wg.float().cpu().numpy().astype(np.float64)
                    rel = np.sqrt(((Wg - W_ref) ** 2).sum(axis=(1, 3))) / den          # per head
                    row.update({"rel_fro_max": float(rel.max()), "rel_fro_median": float(np.median(rel)),
                                "max_abs": float(np.abs(Wg - W_ref).max()), "non_finite": int((~np.isfinite(Wg)).sum())})
                except tri.TriInvError as e:
                    row["error"] = str(e)
                solve_rows.append(row)
        print(json.dumps({"accuracy": rows, "solve_accuracy": solve_rows, "solve_d_x": d_x, "sampled_matrices": len(sel),
                          "workload": f"configs[{w.index}] {w.name}: B={w.B} T={w.Tlen} H={w.H} d_k={w.d_k} C={w.C} -> {n_mat} matrices",
                          "tolerances": {"f32": 1e-5, "f16": 2e-2, "bf16": 2e-2},
                          "note": "fused: against the oracle on the stored keys; standalone: A built by the oracle in fp64, "
                                  "stored fp32, inverted by tri_inv_ex and compared with the oracle on those stored values"}))
        return 0

    def step(i: int, method: int, op: int):
        K, beta, g, T = sets[i % len(sets)]
        tri.gdn_chunk_tri_inv_ex(K, beta, g, C, T=T, gate_kind=w.gate_kind, method=method, op_dtype=op)

    def timed(method: int, op: int, steps: int, warmup: int):
        for i in range(warmup):
            step(i, method, op)
        torch.cuda.synchronize()
        # HIP events on the launch stream (torch's current stream is the one the library is given)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            step(i, method, op)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, e0.elapsed_time(e1) / steps

    copy_ref = None
    if args.copy_ref:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        copy_ref = {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4, "ms": ms,
                    "GBps": 2 * src.numel() * 4 / (ms * 1e-3) / 1e9}
        del src, dst

    wall, avg_kernel_ms = timed(args.method, args.op, args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    value = n_mat * args.steps / wall
    bytes_per_launch = algorithmic_bytes_per_matrix(w, fused=True, out_bytes=out_bytes) * n_mat
    achieved = bytes_per_launch / (avg_kernel_ms * 1e-3) / 1e9
    flops_inv = C ** 3 / 3.0
    flops_gram = C * C * w.d_k

    # ---- the paper's kernel-timing protocol (Sec. 5.1): 5 warm-up + 20 timed launches, the data
    # cache cleared before each one (a 512 MiB fill), per-launch HIP events; median and min --------
    flush = torch.empty(1 << 27, dtype=torch.float32, device=dev)
    cold_ms = []
    for i in range(25):
        flush.fill_(float(i))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        step(i, args.method, args.op)
        b.record()
        torch.cuda.synchronize()
        if i >= 5:
            cold_ms.append(a.elapsed_time(b))
    # the same with the cache cleared by READING 512 MiB instead (the caches then hold clean lines of an unrelated
    # buffer; after a fill they hold 256 MB of dirty lines whose write-back is charged to the timed launch)
    cold_clean_ms = []
    for i in range(25):
        sink = flush.sum()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        step(i, args.method, args.op)
        b.record()
        torch.cuda.synchronize()
        if i >= 5:
            cold_clean_ms.append(a.elapsed_time(b))
    del sink
    # plain device-to-device copy of the same volume, same event timing: the practical HBM ceiling
    src_c = torch.empty(bytes_per_launch // 8, dtype=torch.float32, device=dev).normal_()
    dst_c = torch.empty_like(src_c)
    dst_c.copy_(src_c)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        dst_c.copy_(src_c)
    b.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * src_c.numel() * 4 / (a.elapsed_time(b) / 10 * 1e-3) / 1e9
    del src_c, dst_c, flush

    # ---- parity of the timed configuration on sampled outputs ------------------------------
    import oracle
    from oracle import metrics

    rng = np.random.default_rng(12345)
    sel = np.unique(np.concatenate([[0, n_mat - 1], rng.integers(0, n_mat, size=62)])).tolist()
    T_ref = oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], inp["g"], w.gate_kind, C, sel=sel)
    T_gpu = sets[(args.steps - 1) % len(sets)][3][sel].float().cpu().numpy().astype(np.float64)
    err = metrics.forward_errors(T_ref, T_gpu)["rel_fro"]
    A_ref = oracle.build_A(inp["K"], inp["beta"], inp["g"], w.gate_kind, C, sel=sel)
    res = metrics.residual(A_ref, T_gpu)["normalised"]
    tol = (1e-5 if (args.op == 0 or args.method == 0) else 2e-2) + {"f32": 0.0, "f16": 2.0 ** -11, "bf16": 2.0 ** -8}[args.out]
    parity = {"sampled_matrices": len(sel), "rel_fro_max": float(np.max(err)), "residual_max": float(np.max(res)),
              "tolerance": tol, "ok": bool(np.max(err) <= tol and metrics.structure_ok(T_gpu))}

    # ---- the oracle timed on the host cores -----------------------------------------------
    cpu_baseline = None
    if not args.no_cpu:
        cores = oracle.hw_threads()
        # bounded sample: whole-batch passes on all host threads until ~5 s of wall time have been spent
        # (at least 2 passes), then a one-thread leg over the first 2048 matrices
        passes, t0 = 0, time.perf_counter()
        while passes < 2 or (time.perf_counter() - t0 < 5.0 and passes < 200):
            oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], inp["g"], w.gate_kind, C, n_threads=cores)
            passes += 1
        dt = (time.perf_counter() - t0) / passes
        n1 = min(n_mat, 2048)
        sel1 = list(range(n1))
        t0 = time.perf_counter()
        oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], inp["g"], w.gate_kind, C, sel=sel1, n_threads=1)
        dt1 = time.perf_counter() - t0
        cpu_baseline = {"value": n_mat / dt, "unit": "matrices/s", "cores": cores, "kind": "oracle",
                        "sample": f"{passes} passes over the whole batch ({n_mat} matrices, fused build + fp64 forward "
                                  f"substitution), {dt:.3f} s wall per pass on {cores} threads",
                        "one_thread_value": n1 / dt1, "one_thread_sample": f"first {n1} matrices, {dt1:.2f} s"}

    traffic = PROFILED_TRAFFIC.get((w.index, args.method, args.op)) if args.out == "f32" and not args.chunk else None
    traffic = (traffic[0], f"profiled constant, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, {traffic[1]}") \
        if traffic else (None, None)
    out = {
        "metric": METRIC, "value": value, "unit": "matrices/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": {0: "f32", 1: "f16", 2: "bf16"}[args.op],
        "data": "synthetic",
        "config": {"workload": f"configs[{w.index}] {w.name}: B={w.B} T={w.Tlen} H={w.H} d_k={w.d_k} C={w.C} "
                               f"-> {n_mat} matrices, fused gdn_chunk_tri_inv_ex",
                   "method": tri.METHOD_NAMES[args.method], "op_dtype": tri.DTYPE_NAMES[args.op],
                   "k_dtype": w.k_dtype, "out_dtype": args.out, "buffer_sets": len(sets)},
        "effective": {"GBps": achieved, "TFLOPs_inversion": flops_inv * n_mat / (avg_kernel_ms * 1e-3) / 1e12,
                      "TFLOPs_with_gram": (flops_inv + flops_gram) * n_mat / (avg_kernel_ms * 1e-3) / 1e12,
                      "kernel_ms_avg": avg_kernel_ms,
                      "cold_cache_ms_median": float(np.median(cold_ms)), "cold_cache_ms_min": float(np.min(cold_ms)),
                      "cold_cache_read_flush_ms_median": float(np.median(cold_clean_ms)),
                      "cold_cache_read_flush_ms_min": float(np.min(cold_clean_ms)),
                      "device_copy_same_bytes_GBps": copy_gbps},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic[0], "traffic_source": traffic[1]},
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    if copy_ref is not None:
        out["copy_ref"] = copy_ref

    if args.solve:
        # W = (I + A)^{-1} diag(s) X with X, W [B, Tlen, H, d_x] in the operand type: same rotation over buffer sets
        d_x = args.solve
        xdt = {0: torch.float32, 1: torch.float16, 2: torch.bfloat16}[args.op]
        rhs = si.make_rhs(w, d_x, xdt)
        n_rhs = args.solve_rhs
        Xs = [rhs["X"].to(dev) for _ in sets]
        Ws = [torch.empty_like(x) for x in Xs]
        scale = rhs["row_scale"].to(dev)
        if n_rhs == 2:      # a second right-hand side of the same shape, with its own values, scale and result
            rhs2 = si.make_rhs(w, d_x, xdt, seed_offset=1)
            X2s = [rhs2["X"].to(dev) for _ in sets]
            W2s = [torch.empty_like(x) for x in X2s]
            scale2 = rhs2["row_scale"].to(dev)

        def solve_step(i):
            K, beta, g, _ = sets[i % len(sets)]
            j = i % len(sets)
            if n_rhs == 1:
                tri.gdn_chunk_tri_solve(K, beta, g, Xs[j], C, row_scale=scale, W=Ws[j], gate_kind=w.gate_kind, method=args.method)
            else:
                tri.gdn_chunk_tri_solve_multi(K, beta, g, [Xs[j], X2s[j]], C, row_scales=[scale, scale2], Ws=[Ws[j], W2s[j]],
                                              gate_kind=w.gate_kind, method=args.method)

        for i in range(args.warmup):
            solve_step(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.steps):
            solve_step(i)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        esz = 4 if args.op == 0 else 2
        # inputs of the fused kernel (everything but T) + the row scale + X in + W out
        bpm = algorithmic_bytes_per_matrix(w, True) - 4 * C * C + n_rhs * (4 * C + 2 * C * d_x * esz)
        # sampled check against the oracle: the first and the last batch entry's rows
        b_sel = sorted({0, w.B - 1})
        W_ref = oracle.gdn_chunk_tri_solve(inp["K"][b_sel], inp["beta"][b_sel], None if inp["g"] is None else inp["g"][b_sel],
                                           rhs["X"][b_sel], rhs["row_scale"][b_sel], w.gate_kind, C)
        W_gpu = Ws[(args.steps - 1) % len(sets)][b_sel].float().cpu().numpy().astype(np.float64)
        rel = float((np.sqrt(((W_gpu - W_ref) ** 2).sum(axis=(1, 3))) / np.sqrt((W_ref ** 2).sum(axis=(1, 3)))).max())
        if n_rhs == 2:
            W2_ref = oracle.gdn_chunk_tri_solve(inp["K"][b_sel], inp["beta"][b_sel], None if inp["g"] is None else inp["g"][b_sel],
                                                rhs2["X"][b_sel], rhs2["row_scale"][b_sel], w.gate_kind, C)
            W2_gpu = W2s[(args.steps - 1) % len(sets)][b_sel].float().cpu().numpy().astype(np.float64)
            rel = max(rel, float((np.sqrt(((W2_gpu - W2_ref) ** 2).sum(axis=(1, 3))) / np.sqrt((W2_ref ** 2).sum(axis=(1, 3)))).max()))
        out["solve"] = {"entry": "gdn_chunk_tri_solve" if n_rhs == 1 else "gdn_chunk_tri_solve_multi", "n_rhs": n_rhs, "d_x": d_x, "x_dtype": tri.DTYPE_NAMES[args.op], "kernel_ms_avg": ms,
                        "matrices_per_s": n_mat / (ms * 1e-3), "algorithmic_bytes_per_matrix": bpm,
                        "GBps": bpm * n_mat / (ms * 1e-3) / 1e9, "hbm_frac": bpm * n_mat / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "rel_fro_max_sampled": rel, "tolerance": 1e-5 if args.op == 0 else 2e-2,
                        "ok": bool(rel <= (1e-5 if args.op == 0 else 2e-2))}
        del Xs, Ws

    if args.table:
        table = []
        # input of the standalone entry point: the same chunk matrices, written out once by the library's own
        # gdn_chunk_build_A outside any timed region
        K, beta, g, _ = sets[0]
        A32 = tri.gdn_chunk_build_A(K, beta, g, C, gate_kind=w.gate_kind, op_dtype=tri.F32)
        torch.cuda.synchronize()
        # one copy per buffer set, so that no timed launch finds its input in the last-level cache
        A32s = [A32] + [A32.clone() for _ in range(len(sets) - 1)]
        for method in (0, 1, 4, 3, 6, 2, 5):
            for op in (0, 1, 2):
                if method == 0 and op != 0:
                    continue
                row = {"method": tri.METHOD_NAMES[method], "op": tri.DTYPE_NAMES[op]}
                try:
                    _, km = timed(method, op, 10, 3)
                    row["fused_matrices_per_s"] = n_mat / (km * 1e-3)
                    row["fused_GBps"] = algorithmic_bytes_per_matrix(w, True) * n_mat / (km * 1e-3) / 1e9
                except tri.TriInvError as e:
                    row["fused_error"] = str(e)
                if A32 is not None:
                    try:
                        Ts = [s[3] for s in sets]
                        for i in range(3):
                            tri.tri_inv_ex(A32s[i % len(Ts)], T=Ts[i % len(Ts)], method=method, op_dtype=op)
                        torch.cuda.synchronize()
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        for i in range(10):
                            tri.tri_inv_ex(A32s[i % len(Ts)], T=Ts[i % len(Ts)], method=method, op_dtype=op)
                        e1.record()
                        torch.cuda.synchronize()
                        ms = e0.elapsed_time(e1) / 10
                        row["standalone_matrices_per_s"] = n_mat / (ms * 1e-3)
                        row["standalone_GBps"] = algorithmic_bytes_per_matrix(w, False) * n_mat / (ms * 1e-3) / 1e9
                    except tri.TriInvError as e:
                        row["standalone_error"] = str(e)
                table.append(row)
                if method == 0 and C == 64 and A32 is not None:
                    # the same baseline with A broadcast by wavefront shuffles instead of through LDS (standalone only)
                    Ts = [s[3] for s in sets]
                    for i in range(3):
                        tri.tri_inv_ex(A32s[i % len(Ts)], T=Ts[i % len(Ts)], method=0, flags=tri.FLAG_FWD_SHUFFLE)
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for i in range(10):
                        tri.tri_inv_ex(A32s[i % len(Ts)], T=Ts[i % len(Ts)], method=0, flags=tri.FLAG_FWD_SHUFFLE)
                    e1.record()
                    torch.cuda.synchronize()
                    ms = e0.elapsed_time(e1) / 10
                    table.append({"method": "fwd_subst_shuffle", "op": "f32", "standalone_matrices_per_s": n_mat / (ms * 1e-3),
                                  "standalone_GBps": algorithmic_bytes_per_matrix(w, False) * n_mat / (ms * 1e-3) / 1e9})
        out["methods"] = table

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
