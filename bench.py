#!/usr/bin/env python3
"""Benchmark of the 4x1 structured-sparse INT8 SpMM on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|base|mini]

One "step" is one pass of the whole hot path (pack is done once, outside) over the
workload's SpMM calls: for the default `large` workload the BERT-Large layer shapes
(1024x1024, 4096x1024, 1024x4096) at 90 % and 80 % 4x1-block sparsity with
M = 16 x 384 = 6144 tokens, fused bias + GELU + int8 requantisation (table path).
Inputs are seeded synthetic tensors already resident in HBM; each call rotates through
several distinct activation/output buffers so that repeated launches do not hit in the
last-level cache.  Prints ONE JSON line.

metric  : dense-equivalent TOPS = sum(2*N*K*M) / time (the dense GEMM work the sparse
          kernel replaces); non-zero TOPS (2 * 4 * nnz_blocks * M, padding excluded) and
          the fraction of the binding roofline are reported beside it.
roofline: algorithmic bytes per launch = K*M (X once) + N*M*sizeof(out) + 6 B per non-zero
          4x1 block (4 int8 values + 2-byte index) + 4*(N/4+1) (block-row pointers)
          + 12*N (scale, bias, row sum), divided by the average launch duration measured
          here with HIP events, against 8 TB/s; t_int8 = non-zero ops / 5 POP/s never binds
          for these shapes and is printed per shape for reference.
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
INT8_MFMA_PEAK_TOPS = 5000.0
# the benchmark's metric, verbatim; `value` is its effective (dense-equivalent) TOPS, the roofline
# share is in the `roofline` object
METRIC = "SpMM effective TOPS + % of HBM/int8 roofline at 70\u201390% sparsity, BERT shapes"
METRIC_DETAIL = "dense-equivalent TOPS = 2NKM / time (4x1 block-sparse INT8, fused epilogue); nonzero_tops beside it"
ROTATE = 3   # distinct X/out buffer sets per SpMM (6 calls x 3 sets x ~30 MB > 256 MB of cache)

TRAFFIC_PROFILE = os.path.join("profiles", "spmm_rowtile_mfma_bert_large_hbm_traffic.txt")


def measured_traffic():
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE from two rocprofv3 --pmc runs, each scaled by a plain
    copy of known size in the same run) per kernel instantiation, read from the committed summary of those
    runs: {kernel name: bytes}, and the file they came from.  Not measured by this run."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    table = {}
    try:
        tail = open(path).read().split("# per kernel instantiation", 1)[1]
    except (OSError, IndexError):
        return table, None
    for ln in tail.splitlines()[1:]:
        ln = ln.strip()
        if ln.endswith("bytes") and "(" in ln:
            name, rest = ln.rsplit(")", 1)
            table[name + ")"] = int(rest.split()[0])
    return table, TRAFFIC_PROFILE


def algorithmic_bytes(N, K, M, nnz_blocks, out_elem):
    return K * M + N * M * out_elem + 6 * nnz_blocks + 4 * (N // 4 + 1) + 12 * N


def run_grid(args, np, torch, sp, wl) -> int:
    """The kernel benchmark the paper reports as geometric means over its GEMM shapes (Section 5.1 and its
    table of sparse-against-dense speed-ups per sparsity ratio): every case of the 92-shape grid, one at a time, as a back-to-back loop of `steps` launches of
    the sparse kernel (int8 requantised output) and of the dense int8 GEMM of the same shape."""
    import math
    sps = tuple(float(v) for v in args.sparsities.split(",")) if args.sparsities else wl.SPARSITIES
    Ms = (args.tokens,) if args.tokens else wl.GRID_M
    cases = wl.grid_cases(out_type="s8", sparsities=sps, Ms=Ms)
    if args.only:
        cases = [c for c in cases if args.only in c.name]
    stream = torch.cuda.current_stream().cuda_stream
    steps = max(5, args.steps)

    def loop_us(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / steps

    dense_us, rows = {}, []
    ops = t_sparse = 0.0
    nnz_total = padded_total = 0
    for case in cases:
        d = wl.make(case)
        # (timing only: the row order of scale and bias does not matter here)
        h = sp.spmm_pack_ex(d["W"], case.orientation, reorder_rows=True) if args.reorder else sp.spmm_pack(d["W"], case.orientation)
        info = sp.spmm_info(h)
        nnz_total += info[2]
        padded_total += info[3]
        ws, bias, X = (torch.from_numpy(d[k]).cuda() for k in ("w_scale", "bias", "X"))
        out = torch.empty((case.N, case.M), dtype=torch.int8, device="cuda")
        ep = sp.make_epilogue(ws, d["x_scale"], 0, bias, "none", "s8", d["out_scale"], 0)
        us = loop_us(sp.spmm_run_bound(h, X, case.M, case.M, ep, out, case.M, stream))
        key = (case.N, case.K, case.M)
        if key not in dense_us and not args.no_dense:
            a = torch.randint(-128, 127, (case.M, case.K), dtype=torch.int8, device="cuda")
            b = torch.randint(-128, 127, (case.N, case.K), dtype=torch.int8, device="cuda").t()
            dense_us[key] = loop_us(lambda: torch._int_mm(a, b))
        sp.spmm_destroy(h)
        ops += 2.0 * case.N * case.K * case.M
        t_sparse += us
        rows.append((case, us, dense_us.get(key)))
    table = {}
    for s in sps:
        for M in Ms:
            r = [dn / us for c, us, dn in rows if c.sparsity == s and c.M == M and dn]
            if r:
                table.setdefault("s%d" % round(s * 100), {})["m%d" % M] = {
                    "geomean": round(math.exp(sum(math.log(v) for v in r) / len(r)), 2),
                    "min": round(min(r), 2), "max": round(max(r), 2), "shapes": len(r)}
    print(json.dumps({
        "metric": METRIC, "metric_detail": METRIC_DETAIL,
        "value": round(ops / t_sparse / 1e6, 2), "unit": "TOPS", "n_gpus": 1, "steps": steps, "warmup": 3,
        "ms_per_step": round(t_sparse / 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "shape_grid_%d_cases_s8" % len(rows) + ("[rows reordered]" if args.reorder else ""),
                   "launch_mode": "eager_back_to_back"},
        "padded_over_nnz_blocks": round(padded_total / max(1, nnz_total), 3),
        "speedup_vs_dense_gemm": table,
        "slowest_vs_dense": [{"case": c.name, "us": round(us, 2), "dense_us": round(dn, 2)}
                             for c, us, dn in sorted([r for r in rows if r[2]], key=lambda r: r[2] / r[1])[:5]],
    }))
    return 0


def time_base_f32(np, torch, sp, wl, steps, with_dense):
    """BERT-Base layer shapes (768x768, 3072x768, 768x3072) at 90 % and 80 %, M = 32 x 128 = 4096 tokens, fp32
    output (bias, no GELU): per call, a back-to-back loop of `steps` launches over rotating buffers, the share of
    the HBM roofline and the ratio to the dense int8 GEMM of the same shape timed the same way."""
    stream = torch.cuda.current_stream().cuda_stream
    rows, dense_us = [], {}

    def loop_us(fn, n):
        for it in range(3):
            fn(it)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for it in range(n):
            fn(it)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    for case in wl.base_cases(batches=(32,), sparsities=(0.9, 0.8)):
        d = wl.make(case)
        h = sp.spmm_pack(d["W"], case.orientation)
        N, K, nnzb, _, _ = sp.spmm_info(h)
        ws, bias = torch.from_numpy(d["w_scale"]).cuda(), torch.from_numpy(d["bias"]).cuda()
        ep = sp.make_epilogue(ws, d["x_scale"], 0, bias, case.postop, case.out_type, d["out_scale"], 0, d["mid_scale"])
        Xs = [torch.from_numpy(d["X"]).cuda() for _ in range(ROTATE)]
        outs = [torch.empty((N, case.M), dtype=torch.float32, device="cuda") for _ in range(ROTATE)]
        runs = [sp.spmm_run_bound(h, Xs[j], case.M, case.M, ep, outs[j], case.M, stream) for j in range(ROTATE)]
        us = loop_us(lambda it: runs[it % ROTATE](), steps)
        key = (N, K)
        if with_dense and key not in dense_us:
            a = torch.randint(-128, 127, (case.M, K), dtype=torch.int8, device="cuda")
            b = torch.randint(-128, 127, (N, K), dtype=torch.int8, device="cuda").t()
            dense_us[key] = loop_us(lambda it: torch._int_mm(a, b), 20)
        nbytes = algorithmic_bytes(N, K, case.M, nnzb, 4)
        rows.append({"case": case.name, "us_back_to_back": round(us, 2), "algorithmic_bytes": int(nbytes),
                     "roofline_frac": round(nbytes / (HBM_PEAK_GBS * 1e9) * 1e6 / us, 4),
                     "dense_equiv_tops": round(2.0 * N * K * case.M / us / 1e6, 1),
                     "kernel": sp.spmm_kernel_variant(h, case.M, case.out_type, case.postop),
                     "speedup_vs_dense_gemm": round(dense_us[key] / us, 2) if key in dense_us else None})
        sp.spmm_destroy(h)
    return {"workload": "bert_base_layers_m4096_s90_s80_f32", "launch_mode": "eager_back_to_back", "per_call": rows}


def make_bufs(torch, sp, d, case, N, prev, flags):
    """ROTATE device copies of the activations and ROTATE output buffers of one call, in the layout `flags` names
    (SPMM_TILED_X / SPMM_TILED_OUT).  A chained call (d["X"] is None) reads the previous call's output buffers of
    the same layout."""
    tdt = {"s32": torch.int32, "f32": torch.float32, "s8": torch.int8, "u8": torch.uint8}
    if d["X"] is None:
        xs = prev["bufs"][flags | (sp.binding.SPMM_TILED_OUT if flags & sp.binding.SPMM_TILED_X else 0)][1]
    else:
        xh = sp.tile_major(d["X"]) if flags & sp.binding.SPMM_TILED_X else d["X"]
        xs = [torch.from_numpy(xh).cuda() for _ in range(ROTATE)]
    if flags & sp.binding.SPMM_TILED_OUT:
        outs = [torch.empty(((case.M + 31) // 32) * N * 32, dtype=tdt[case.out_type], device="cuda") for _ in range(ROTATE)]
    else:
        outs = [torch.empty((N, case.M), dtype=tdt[case.out_type], device="cuda") for _ in range(ROTATE)]
    return xs, outs


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large", choices=["large", "base", "mini", "mini_chain", "large_chain", "large_sum", "grid", "clustered"],
                    help="large_sum: the two BERT-Large Linears that feed a residual add (attention output and "
                         "second feed-forward), with the Sum post-operator and fp32 output; mini_chain: the BERT-Mini "
                         "feed-forward pair chained on the device (GELU -> uint8 code of launch 1 is the activation "
                         "matrix of launch 2); grid: the 92-shape grid "
                         "(int8 output), geometric-mean speed-up over the dense int8 GEMM per sparsity and token count")
    ap.add_argument("--tokens", type=int, default=0,
                    help="workload base only: token count M (default 4096 = 32 sequences of 128)")
    ap.add_argument("--sparsities", default="", help="workload base only: comma list, e.g. 0.7,0.8,0.9")
    ap.add_argument("--reorder", action="store_true",
                    help="pack with SPMM_PACK_REORDER_ROWS (rows clustered by k overlap); outputs and per-row "
                         "operands are then in the library's row order")
    ap.add_argument("--layout", default="tile_major", choices=["tile_major", "row_major"],
                    help="activation layout of the timed steps: token-tile-major [M/32][rows][32] for X and for 1-byte "
                         "outputs (the library's own layout between layers: spmm_run_tiled), or plain row-major")
    ap.add_argument("--no-other-layout", action="store_true", help="skip the extra timing of the same steps in the other layout")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--tuning", default="", help="token_tile,variant override passed to spmm_set_tuning")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches only")
    ap.add_argument("--profile", action="store_true",
                    help="for profiler runs: warm-up and the event-timed steps only (no graph, no back-to-back loops)")
    ap.add_argument("--only", default="", help="keep only the calls whose case name contains this substring")
    ap.add_argument("--qkv", action="store_true",
                    help="also time the three attention projections (N = K of the first shape) as three launches and "
                         "as one launch of the stacked [3N, K] weight")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 256 MiB device copy (profiling aid: scales FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the SpMM shards trivially over tokens or output "
              "channels with no communication); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2306_16601_amd as sp
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sp.lib()   # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    if args.workload == "grid":
        return run_grid(args, np, torch, sp, wl)
    if args.workload == "large":
        cases = wl.large_cases()
        wname = "bert_large_layers_m6144_s90_s80_gelu_s8"
    elif args.workload == "base":
        sps = tuple(float(v) for v in args.sparsities.split(",")) if args.sparsities else (0.9, 0.8)
        cases = [c for c in wl.base_cases(batches=(32,), sparsities=sps)]
        wname = "bert_base_layers_m4096_s90_s80_f32"
        if args.tokens or args.sparsities:
            M = args.tokens or 4096
            cases = [c.with_(M=M, name=c.name.replace("_m4096_", "_m%d_" % M)) for c in cases]
            wname = "bert_base_layers_m%d_s%s_f32" % (M, "_".join(str(int(round(v * 100))) for v in sps))
    elif args.workload == "large_sum":
        cases = [c.with_(out_type="f32", postop="none") for c in wl.large_cases() if c.N == 1024]
        wname = "bert_large_residual_linears_m6144_s90_s80_sum_f32"
    elif args.workload == "mini_chain":
        cases = wl.chain_cases()
        wname = "bert_mini_ffn_pair_chained_u8_m1024_s80"
    elif args.workload == "large_chain":
        cases = wl.chain_cases(large=True)
        wname = "bert_large_ffn_pair_chained_u8_m6144_s90"
    elif args.workload == "clustered":
        cases = wl.clustered_cases()
        wname = "clustered32_4096x1024_m6144_s90_s80_gelu_s8"
    else:
        cases = wl.mini_cases()
        wname = "bert_mini_ffn_pair_m1024_s80"
    made = wl.make_chain(cases) if args.workload in ("mini_chain", "large_chain") else None
    if args.reorder:
        wname += "[rows reordered]"
    if args.only:
        cases = [c for c in cases if args.only in c.name]
        wname += "[" + args.only + "]"
        if not cases:
            print("bench.py: --only matched no case", file=sys.stderr)
            return 2
    out_elem = {"s32": 4, "f32": 4, "s8": 1, "u8": 1}
    tdt = {"s32": torch.int32, "f32": torch.float32, "s8": torch.int8, "u8": torch.uint8}

    # ------------------------------------------------------------------ set up (not timed)
    calls = []
    for case_i, case in enumerate(cases):
        d = made[case_i] if made is not None else wl.make(case)
        if args.reorder:
            if made is not None:
                print("bench.py: --reorder is not available for the chained pair", file=sys.stderr)
                return 2
            h = sp.spmm_pack_ex(d["W"], case.orientation, reorder_rows=True)
            # from here on the problem is the one the handle stands for: rows in the library's order
            order = sp.spmm_row_order(h)
            d["W"] = np.ascontiguousarray(d["W"][order])
            d["w_scale"] = np.ascontiguousarray(d["w_scale"][order])
            if d["bias"] is not None:
                d["bias"] = np.ascontiguousarray(d["bias"][order])
        else:
            h = sp.spmm_pack(d["W"], case.orientation)
        if args.tuning:
            tm, r = (int(v) for v in args.tuning.split(","))
            sp.spmm_set_tuning(h, tm, r)
        N, K, nnzb, padded, dev_bytes = sp.spmm_info(h)
        ws = torch.from_numpy(d["w_scale"]).cuda()
        bias = torch.from_numpy(d["bias"]).cuda() if d["bias"] is not None else None
        lut = None
        if case.postop == "gelu" and case.out_type in ("s8", "u8"):
            lut = torch.from_numpy(sp.spmm_make_gelu_lut(d["mid_scale"], d["out_scale"], d["out_zero_point"],
                                                         case.out_type)).cuda()
        Rs = None
        if args.workload == "large_sum":
            R = (wl.rng_for(97, case.N, case.M).standard_normal((case.N, case.M)) *
                 wl.preact_sigma(case.K, case.sparsity)).astype(np.float32)
            d["R"] = R
            Rs = [torch.from_numpy(R).cuda() for _ in range(ROTATE)]
            eps = [sp.make_epilogue(ws, d["x_scale"], 0, bias, case.postop, case.out_type, d["out_scale"], 0,
                                    d["mid_scale"], lut, Rs[j], case.M) for j in range(ROTATE)]
        else:
            eps = [sp.make_epilogue(ws, d["x_scale"], d["x_zero_point"], bias, case.postop, case.out_type,
                                    d["out_scale"], d["out_zero_point"], d["mid_scale"], lut)] * ROTATE
        ep = eps[0]
        # (chained pair: the second launch reads the first launch's output buffers)
        # layout flags of this call: tile-major X, and tile-major output where it is a 1-byte one
        tiled = 0
        if args.layout == "tile_major":
            tiled = sp.binding.SPMM_TILED_X | (sp.binding.SPMM_TILED_OUT if case.out_type in ("s8", "u8") else 0)

        prev = calls[-1] if calls else None
        Xs, outs = make_bufs(torch, sp, d, case, N, prev, tiled)
        calls.append(dict(case=case, d=d, h=h, ep=ep, eps=eps, keep=(ws, bias, lut, Rs), Xs=Xs, outs=outs, N=N, K=K,
                          tiled=tiled, bufs={tiled: (Xs, outs)}, prev=prev,
                          M=case.M, nnzb=nnzb, padded=padded, dev_bytes=dev_bytes,
                          bytes=algorithmic_bytes(N, K, case.M, nnzb, out_elem[case.out_type]) +
                          (4 * N * case.M if Rs else 0),
                          dense_ops=2.0 * N * K * case.M, nnz_ops=2.0 * 4 * nnzb * case.M,
                          plan=sp.spmm_plan(h, case.M, case.out_type)))

    # arguments marshalled once per (call, rotation): a launch is then one C call
    stream = torch.cuda.current_stream().cuda_stream
    for c in calls:
        c["run"] = [sp.spmm_run_tiled_bound(c["h"], c["Xs"][j], c["M"], c["M"], c["eps"][j], c["outs"][j], c["M"],
                                            c["tiled"], stream) for j in range(ROTATE)]

    def launch(c, it):
        if c["run"][it % ROTATE]() != 0:
            raise RuntimeError("spmm_run failed")

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)          # one plain copy kernel moving 256 MiB each way
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ warm-up
    for it in range(args.warmup):
        for c in calls:
            launch(c, it)
    torch.cuda.synchronize()
    nc = len(calls)

    # ------------------------------------------------------------------ timed region A: K steps, eager launches,
    # HIP events on the launch stream around every kernel (per-kernel durations for the roofline)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(nc + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(args.steps):
        ev[it][0].record()
        for ci, c in enumerate(calls):
            launch(c, it)
            ev[it][ci + 1].record()
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    eager_ms_per_step = ev[0][0].elapsed_time(ev[args.steps - 1][nc]) / args.steps
    per_call_us = np.array([[ev[it][ci].elapsed_time(ev[it][ci + 1]) * 1e3 for ci in range(nc)]
                            for it in range(args.steps)])
    avg_us = per_call_us.mean(axis=0)
    med_us = np.median(per_call_us, axis=0)
    min_us = per_call_us.min(axis=0)

    # ------------------------------------------------------------------ timed region B: the same K steps replayed from
    # HIP graphs (one graph per buffer rotation; spmm_run allocates nothing and never synchronises, so it
    # captures as is).  Launch-bound sequences of 10-50 us kernels are what graphs are for; this is `value`.
    graph_ms_per_step = None
    if not args.no_graph and not args.profile:
        try:
            graphs = []
            for j in range(ROTATE):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    cap = torch.cuda.current_stream().cuda_stream      # the capturing stream
                    for c in calls:
                        sp.spmm_run_tiled(c["h"], c["Xs"][j], c["M"], c["M"], c["eps"][j], c["outs"][j], c["M"], c["tiled"], cap)
                graphs.append(g)
            for it in range(max(2, args.warmup // 2)):
                graphs[it % ROTATE].replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for it in range(args.steps):
                graphs[it % ROTATE].replay()
            e1.record()
            torch.cuda.synchronize()
            graph_ms_per_step = e0.elapsed_time(e1) / args.steps
        except Exception as exc:   # fall back to the eager figure
            print("bench.py: graph capture unavailable (%r); reporting eager launches" % (exc,), file=sys.stderr)

    # ------------------------------------------------------------------ timed region C: the same K steps as plain eager
    # launches, back to back on the stream with nothing between them.  Kernels of a few microseconds (short
    # batches) run faster this way than as graph nodes; `value` takes the faster of B and C and says which.
    stream_ms_per_step = eager_ms_per_step
    if not args.profile:
        for it in range(max(2, args.warmup // 2)):
            for c in calls:
                launch(c, it)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for it in range(args.steps):
            for c in calls:
                launch(c, it)
        e1.record()
        torch.cuda.synchronize()
        stream_ms_per_step = e0.elapsed_time(e1) / args.steps
    # each call on its own, the same way (what the dense comparator below is timed like)
    b2b_us = [float(v) for v in avg_us] if args.profile else []
    for c in ([] if args.profile else calls):
        for it in range(3):
            launch(c, it)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for it in range(args.steps):
            launch(c, it)
        e1.record()
        torch.cuda.synchronize()
        b2b_us.append(e0.elapsed_time(e1) * 1e3 / args.steps)
    # ------------------------------------------------------------------ extra: the same steps in the OTHER activation
    # layout (row-major when the timed steps are tile-major and vice versa), eager back to back + events per launch
    other_layout = None
    if not args.profile and not args.no_other_layout:
        other = "row_major" if args.layout == "tile_major" else "tile_major"

        def flags_of(c):
            if other == "row_major":
                return 0
            return sp.binding.SPMM_TILED_X | (sp.binding.SPMM_TILED_OUT if c["case"].out_type in ("s8", "u8") else 0)
        for c in calls:
            f = flags_of(c)
            if f not in c["bufs"]:
                c["bufs"][f] = make_bufs(torch, sp, c["d"], c["case"], c["N"], c["prev"], f)
            xs, os_ = c["bufs"][f]
            c["run_o"] = [sp.spmm_run_tiled_bound(c["h"], xs[j], c["M"], c["M"], c["eps"][j], os_[j], c["M"], f, stream)
                          for j in range(ROTATE)]
        for it in range(max(2, args.warmup // 2)):
            for c in calls:
                c["run_o"][it % ROTATE]()
        torch.cuda.synchronize()
        # the two layouts hold the same values
        same = True
        for c in calls:
            launch(c, 0)
        for c in calls:
            c["run_o"][0]()
        torch.cuda.synchronize()
        for c in calls:
            def rows(buf, flags):
                a_ = buf.cpu().numpy()
                return sp.from_tile_major(a_.reshape(-1, c["N"], 32), c["M"]) if flags & sp.binding.SPMM_TILED_OUT else a_
            same &= bool(np.array_equal(rows(c["outs"][0], c["tiled"]).view(np.uint8),
                                        rows(c["bufs"][flags_of(c)][1][0], flags_of(c)).view(np.uint8)))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for it in range(args.steps):
            for c in calls:
                c["run_o"][it % ROTATE]()
        e1.record()
        torch.cuda.synchronize()
        t_ms = e0.elapsed_time(e1) / args.steps
        evt = [[torch.cuda.Event(enable_timing=True) for _ in range(nc + 1)] for _ in range(args.steps)]
        for it in range(args.steps):
            evt[it][0].record()
            for ci, c in enumerate(calls):
                c["run_o"][it % ROTATE]()
                evt[it][ci + 1].record()
        torch.cuda.synchronize()
        t_ev_ms = evt[0][0].elapsed_time(evt[args.steps - 1][nc]) / args.steps
        t_call = np.array([[evt[it][ci].elapsed_time(evt[it][ci + 1]) * 1e3 for ci in range(nc)]
                           for it in range(args.steps)]).mean(axis=0) * (t_ms / t_ev_ms)
        # the timed layout once more, right after: sustained load lowers the clocks, so a later measurement reads a
        # few percent slower than the first; this is the like-for-like partner of the figure above
        for it in range(2):
            for c in calls:
                launch(c, it)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for it in range(args.steps):
            for c in calls:
                launch(c, it)
        e1.record()
        torch.cuda.synchronize()
        again_ms = e0.elapsed_time(e1) / args.steps
        other_layout = {"layout": other, "ms_per_step": round(t_ms, 5),
                        "timed_layout_remeasured_after_it_ms_per_step": round(again_ms, 5),
                        "value": round(sum(c["dense_ops"] for c in calls) / (t_ms * 1e-3) / 1e12, 2),
                        "same_values_in_both_layouts": same,
                        "per_call_us_in_step": {c["case"].name: round(float(t_call[i]), 2) for i, c in enumerate(calls)},
                        "per_call_roofline_frac_in_step": {c["case"].name: round(c["bytes"] / (float(t_call[i]) * 1e-6) / (HBM_PEAK_GBS * 1e9), 4)
                                                           for i, c in enumerate(calls)}}
        for c in calls:
            del c["run_o"]

    # `value` and the roofline use ONE launch mode: plain eager launches back to back on the stream (what a
    # caller of spmm_run gets; graph replay of the same steps is reported beside it)
    ms_per_step, launch_mode = stream_ms_per_step, "eager_back_to_back"
    # Kernel durations inside the step: the events around every launch (region A) also bracket the dispatch
    # gap between kernels, so each launch's event interval is scaled by (back-to-back step time / event-timed
    # step time); the scaled figures are what rocprofv3's kernel trace of the same command shows.
    gap_scale = min(1.0, stream_ms_per_step / eager_ms_per_step) if eager_ms_per_step > 0 else 1.0

    dense_ops = sum(c["dense_ops"] for c in calls)
    nnz_ops = sum(c["nnz_ops"] for c in calls)
    value = dense_ops / (ms_per_step * 1e-3) / 1e12
    nnz_tops = nnz_ops / (ms_per_step * 1e-3) / 1e12

    # ------------------------------------------------------------------ dense int8 GEMM of the same shapes (vendor BLAS)
    dense = {}
    if not args.no_dense:
        for (N, K) in sorted({(c["N"], c["K"]) for c in calls}):
            M = calls[0]["M"]
            try:
                a = torch.randint(-128, 127, (M, K), dtype=torch.int8, device="cuda")
                b = torch.randint(-128, 127, (N, K), dtype=torch.int8, device="cuda").t()
                for _ in range(5):
                    torch._int_mm(a, b)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(20):
                    torch._int_mm(a, b)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / 20
                dense["%dx%d" % (N, K)] = {"us": round(us, 2), "tops": round(2.0 * N * K * M / us / 1e6, 1)}
            except Exception as exc:   # the comparator is context only
                dense["%dx%d" % (N, K)] = {"error": repr(exc)[:120]}

    # ------------------------------------------------------------------ Q, K, V projections sharing one X: three launches
    # against one launch of the stacked weight (same outputs, see tests)
    qkv = None
    if args.qkv:
        c0 = calls[0]
        case0 = c0["case"]
        parts = [wl.make(case0.with_(keys=(case0.keys + (i,)))) for i in range(3)]
        hs = [sp.spmm_pack(p["W"], case0.orientation) for p in parts]
        hb = sp.spmm_pack(np.concatenate([p["W"] for p in parts]), case0.orientation)
        ws3 = torch.from_numpy(np.concatenate([p["w_scale"] for p in parts])).cuda()
        b3 = torch.from_numpy(np.concatenate([p["bias"] for p in parts])).cuda()
        N0, M0 = c0["N"], c0["M"]
        eps = [sp.make_epilogue(ws3[i * N0:(i + 1) * N0], c0["d"]["x_scale"], 0, b3[i * N0:(i + 1) * N0], case0.postop,
                                case0.out_type, c0["d"]["out_scale"], 0, c0["d"]["mid_scale"], c0["keep"][2])
               for i in range(3)]
        epb = sp.make_epilogue(ws3, c0["d"]["x_scale"], 0, b3, case0.postop, case0.out_type, c0["d"]["out_scale"], 0,
                               c0["d"]["mid_scale"], c0["keep"][2])
        o3 = [torch.empty((3 * N0, M0), dtype=tdt[case0.out_type], device="cuda") for _ in range(ROTATE)]
        ob = [torch.empty((3 * N0, M0), dtype=tdt[case0.out_type], device="cuda") for _ in range(ROTATE)]
        st = torch.cuda.current_stream().cuda_stream

        def three(it):
            j = it % ROTATE
            for i in range(3):
                sp.spmm_run(hs[i], c0["Xs"][j], M0, M0, eps[i], o3[j][i * N0:(i + 1) * N0], M0, st)

        def one(it):
            j = it % ROTATE
            sp.spmm_run(hb, c0["Xs"][j], M0, M0, epb, ob[j], M0, st)

        res = {}
        for name, fn in (("three_launches_us", three), ("stacked_launch_us", one)):
            for it in range(6):
                fn(it)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for it in range(30):
                fn(it)
            e1.record()
            torch.cuda.synchronize()
            res[name] = round(e0.elapsed_time(e1) * 1e3 / 30, 2)
        res["identical_outputs"] = bool(torch.equal(o3[0], ob[0]))
        res["shape"] = "3 x %dx%d, M=%d, %s" % (N0, c0["K"], M0, case0.name)
        qkv = res
        for h in hs + [hb]:
            sp.spmm_destroy(h)

    # ------------------------------------------------------------------ per-shape rows + roofline of the SpMM kernel
    rows = []
    for ci, c in enumerate(calls):
        t_hbm = c["bytes"] / (HBM_PEAK_GBS * 1e9) * 1e6
        t_int8 = c["nnz_ops"] / (INT8_MFMA_PEAK_TOPS * 1e12) * 1e6
        t = float(avg_us[ci])
        key = "%dx%d" % (c["N"], c["K"])
        rows.append({
            "case": c["case"].name, "us_avg": round(t, 2), "us_median": round(float(med_us[ci]), 2),
            "us_min": round(float(min_us[ci]), 2),
            "dense_equiv_tops": round(c["dense_ops"] / t / 1e6, 1), "nonzero_tops": round(c["nnz_ops"] / t / 1e6, 1),
            "algorithmic_bytes": int(c["bytes"]), "t_hbm_us": round(t_hbm, 2), "t_int8_us": round(t_int8, 2),
            "bound": "hbm" if t_hbm >= t_int8 else "mfma", "roofline_frac": round(max(t_hbm, t_int8) / t, 4),
            "nnz_blocks": int(c["nnzb"]), "padded_blocks": int(c["padded"]),
            "plan": {"token_tile": c["plan"][0], "rows_per_wg": c["plan"][1], "workgroups": c["plan"][2]},
            "us_in_step": round(t * gap_scale, 2), "roofline_frac_in_step": round(max(t_hbm, t_int8) / (t * gap_scale), 4),
            "us_back_to_back": round(b2b_us[ci], 2),
            "speedup_vs_dense_gemm": (round(dense[key]["us"] / b2b_us[ci], 2)
                                      if key in dense and "us" in dense[key] else None),
            "sha256": {"W": wl.sha256(c["d"]["W"])[:16],
                       "X": wl.sha256(c["d"]["X"])[:16] if c["d"]["X"] is not None else "output of the previous call"},
        })
    # roofline of the dominant kernel instantiation (largest share of the step): algorithmic bytes of
    # its launches / their summed durations = bytes per launch / average launch duration
    by_kernel = {}
    for ci, c in enumerate(calls):
        name = sp.spmm_kernel_variant(c["h"], c["M"], c["case"].out_type, c["case"].postop, c["tiled"])
        k = by_kernel.setdefault(name, {"bytes": 0.0, "us": 0.0, "launches": 0, "nnz_ops": 0.0})
        k["bytes"] += c["bytes"]
        k["us"] += float(avg_us[ci]) * gap_scale
        k["us_events"] = k.get("us_events", 0.0) + float(avg_us[ci])
        k["launches"] += 1
        k["nnz_ops"] += c["nnz_ops"]
    dom_name = max(by_kernel, key=lambda n: by_kernel[n]["us"])
    dom = by_kernel[dom_name]
    achieved = dom["bytes"] / (dom["us"] * 1e-6) / 1e9
    traffic_table, traffic_file = measured_traffic()
    # measured ceilings of the two candidate multiply instructions (registers only), beside the data-sheet peak
    peaks = {}
    if not args.profile:
        try:
            peaks = {"mfma_i32_16x16x64_i8": round(sp.spmm_measure_peak(0), 1), "dot4_i32_i8": round(sp.spmm_measure_peak(1), 1)}
        except Exception as exc:
            peaks = {"error": repr(exc)[:120]}
    roofline = {
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic_table.get(dom_name),
        "traffic_source": (("%s (rocprofv3 --pmc summary, not measured by this run)" % traffic_file)
                           if dom_name in traffic_table else
                           "no entry for this kernel in %s" % (traffic_file or TRAFFIC_PROFILE)),
        "kernel": dom_name, "launches_per_step": dom["launches"],
        "avg_launch_us": round(dom["us"] / dom["launches"], 3),
        "algorithmic_bytes_per_launch": int(dom["bytes"] / dom["launches"]),
        "int8_mfma_frac": round(dom["nnz_ops"] / (dom["us"] * 1e-6) / (INT8_MFMA_PEAK_TOPS * 1e12), 4),
        "avg_launch_us_between_events": round(dom["us_events"] / dom["launches"], 3),
        "timing": "HIP events on the launch stream around every launch of the timed steps, scaled by the ratio of the "
                  "back-to-back step time to the event-timed step time (the events also bracket the dispatch gap)",
        "int8_mfma_measured_tops": peaks.get("mfma_i32_16x16x64_i8"), "int8_dot4_measured_tops": peaks.get("dot4_i32_i8"),
        "int8_mfma_peak_tops": INT8_MFMA_PEAK_TOPS,
        "other_kernels": {n: {"avg_launch_us": round(v["us"] / v["launches"], 3),
                              "frac": round(v["bytes"] / (v["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                              "traffic": traffic_table.get(n)}
                          for n, v in by_kernel.items() if n != dom_name},
    }

    # ------------------------------------------------------------------ CPU baseline: the oracle on the host cores
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sample = [c for c in calls if abs(c["case"].sparsity - calls[0]["case"].sparsity) < 1e-9]
        ops, secs, parity = 0.0, 0.0, True
        prev_ref = None
        for c in sample:
            d, case = c["d"], c["case"]
            launch(c, 0)
            torch.cuda.synchronize()
            got = c["outs"][0].cpu().numpy()
            if c["tiled"] & sp.binding.SPMM_TILED_OUT:
                got = sp.from_tile_major(got.reshape(-1, c["N"], 32), c["M"])
            t1 = time.perf_counter()
            ref = oracle.spmm(d["W"], d["X"] if d["X"] is not None else prev_ref, d["w_scale"], d["x_scale"], d["bias"],
                              case.postop, case.out_type, d["out_scale"], d["out_zero_point"], d["mid_scale"],
                              d["x_zero_point"], sum=d.get("R"))
            prev_ref = ref
            secs += time.perf_counter() - t1
            ops += c["dense_ops"]
            if case.out_type == "f32" and case.postop == "gelu":
                parity &= bool(np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-7))
            else:
                parity &= bool(np.array_equal(got, ref))
        # the same oracle on ONE thread, on the first call of the sample
        one = None
        try:
            c = sample[0]
            d, case = c["d"], c["case"]
            nthreads = oracle.num_threads()
            oracle.set_num_threads(1)
            t1 = time.perf_counter()
            oracle.spmm(d["W"], d["X"], d["w_scale"], d["x_scale"], d["bias"], case.postop, case.out_type,
                        d["out_scale"], d["out_zero_point"], d["mid_scale"], d["x_zero_point"], sum=d.get("R"))
            s1 = time.perf_counter() - t1
            oracle.set_num_threads(nthreads)
            one = {"value": round(c["dense_ops"] / s1 / 1e12, 5), "seconds": round(s1, 2), "sample": case.name}
        except Exception as exc:
            one = {"error": repr(exc)[:120]}
        cpu = {"value": round(ops / secs / 1e12, 5), "unit": "TOPS (dense-equivalent)", "cores": oracle.num_threads(),
               "one_thread": one,
               "kind": "oracle", "seconds": round(secs, 2),
               "sample": "%d SpMM calls of the workload (%s), one run each" % (
                   len(sample), ", ".join(c["case"].name for c in sample)),
               "gpu_matches_oracle": parity}

    for c in calls:
        sp.spmm_destroy(c["h"])

    # the second family of shapes the target names (BERT-Base, fp32 output), beside the headline workload
    base_f32 = None
    if args.workload == "large" and not args.profile and not args.only and not args.tuning:
        base_f32 = time_base_f32(np, torch, sp, wl, max(10, args.steps // 2), not args.no_dense)

    line = {
        "metric": METRIC, "metric_detail": METRIC_DETAIL,
        "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": wname, "calls_per_step": nc, "tokens": calls[0]["M"], "orientation": "n4k1",
                   "buffer_rotation": ROTATE,
                   "activation_layout": ("token-tile-major [M/32][rows][32]: X, and the 1-byte outputs a next layer reads "
                                         "(spmm_run_tiled)") if args.layout == "tile_major" else "row-major"},
        "nonzero_tops": round(nnz_tops, 2),
        "roofline": roofline, "cpu_baseline": cpu, "dense_int8_gemm": dense, "qkv_stacked": qkv, "per_call": rows,
        "base_f32": base_f32,
        "other_layout": other_layout,
        "ms_per_step_eager_with_events": round(eager_ms_per_step, 5),
        "ms_per_step_graph": (round(graph_ms_per_step, 5) if graph_ms_per_step is not None else None),
        "ms_per_step_eager_back_to_back": round(stream_ms_per_step, 5),
        "launch_mode": launch_mode,
        "host_wall_s_eager": round(wall_s, 4),
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
