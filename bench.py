#!/usr/bin/env python3
"""Benchmark of the ROAST hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of seeded synthetic input:
  * ROAST-MM on the BERT-base-FFN configuration (bf16 activations, fp32 accumulation, two chained
    layers 768->3072->768 sharing one M at 100x compression, 8192 tokens): forward of both layers,
    then dX and dM of both layers (6 calls);
  * the ROAST lookup on the DLRM-shaped configuration (26 tables, 10M rows x 128, chunks of 32 hashed
    into 1.28M slots, 65536 x 26 Zipf(1.05) lookups): forward and gradient scatter-add (2 calls).
All inputs are resident in HBM before the timed region.  `value` is the ROAST-MM fwd+bwd rate in
TFLOP/s (3 x 2*I*H*O per layer over the time of the six MM calls); the lookup's GB/s is reported
next to it under "embedding".  Per-call times are measured with HIP events on the launch stream.

Prints ONE JSON line.  The CPU oracle is timed beside it on a bounded sample (cpu_baseline).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # 256 CU x 4096 bf16 FLOP/clk/CU x 2.4 GHz, dense
PEAK_HBM_GBS = 8000.0

TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_default_pmc_hbm_traffic.txt")


def load_measured_traffic(path=TRAFFIC_PROFILE):
    """HBM-side bytes per call of the default workload, read from the committed rocprofv3 summary
    (FETCH_SIZE + WRITE_SIZE of two --pmc runs of this script, each scaled by what the counter reads
    for a plain 256 MiB copy).  The summary carries one line per call of the step:
        traffic: <call> | <kernel(s) that serve it> | <fetched bytes> | <written bytes>
    Returns {call: {"kernels": str, "fetch": bytes, "write": bytes}}.  A missing file or a malformed
    line is an error: a roofline without its traffic figure would silently go stale."""
    rows = {}
    with open(path) as f:
        for line in f:
            if not line.startswith("traffic:"):
                continue
            parts = [x.strip() for x in line[len("traffic:"):].split("|")]
            if len(parts) != 4 or not parts[1]:
                raise ValueError(f"{path}: malformed traffic line: {line!r}")
            rows[parts[0]] = {"kernels": parts[1], "fetch": float(parts[2]), "write": float(parts[3])}
    if not rows:
        raise ValueError(f"{path}: no 'traffic:' lines")
    return rows


def traffic_of(rows, calls, kernel_substr):
    """Sum of fetched + written bytes over `calls`; every call must be in the summary and be served by a
    kernel whose name contains `kernel_substr` (else the summary belongs to another build)."""
    total = 0.0
    for c in calls:
        if c not in rows:
            raise KeyError(f"{TRAFFIC_PROFILE}: no traffic line for call {c!r}")
        if kernel_substr not in rows[c]["kernels"]:
            raise KeyError(f"{TRAFFIC_PROFILE}: call {c!r} is listed with kernels {rows[c]['kernels']!r}, "
                           f"expected {kernel_substr!r}")
        total += rows[c]["fetch"] + rows[c]["write"]
    return total


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=50)
    p.add_argument("--warmup", type=int, default=10)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--mm-only", action="store_true", help="profiling aid: skip the lookup calls")
    p.add_argument("--embed-only", action="store_true", help="profiling aid: skip the ROAST-MM calls")
    p.add_argument("--hot-path-only", action="store_true",
                   help="profiling aid: skip the secondary timings made outside the timed steps (optimizer step, "
                        "pooled lookup), so that a trace holds the hot path's kernels only")
    p.add_argument("--reduce", choices=["atomic", "deterministic"], default="atomic")
    p.add_argument("--workload", choices=["default", "cfg1_single_f32", "cfg2_bert_ffn_bf16", "cfg3_bert_stack_bf16", "cfg5_large_bf16",
                                           "dim_sweep_b512"],
                   default="default",
                   help="default = the headline step (cfg2 ROAST-MM + cfg4 lookup); the others time forward, dX and "
                        "dM of every layer of another ROAST-MM configuration (a secondary figure, same JSON shape); "
                        "dim_sweep_b512 = square Dim x Dim layers at batch 512 with a dense bf16 GEMM beside each")
    p.add_argument("--dtype", choices=["config", "f32"], default="config",
                   help="cfg* workloads only: f32 runs the configuration's shapes with fp32 tensors (through the "
                        "workspace entry points, i.e. on the matrix cores from bfloat16 planes)")
    p.add_argument("--no-f32-workspace", action="store_true",
                   help="fp32 workloads: call without workspaces (vector-ALU fp32 kernels)")
    p.add_argument("--dm-workspace", action="store_true",
                   help="atomic mode only: give roast_mm_bwd_dM its optional scratch (contraction parts x H x O "
                        "floats per call); about 7 %% faster dM, but a buffer of the size of the virtual weights, "
                        "which the method otherwise never needs")
    p.add_argument("--graph", action="store_true",
                   help="--workload cfg*: capture one step in a HIP graph and time replays (what a launch-bound "
                        "loop like config 1 gains from it)")
    p.add_argument("--calibration-copy", action="store_true",
                   help="profiling aid: also launch one plain 256 MiB device copy per step, the kernel of known "
                        "size that the FETCH_SIZE / WRITE_SIZE counters are scaled by")
    return p.parse_args()


def time_optimizer(roast, torch, M, dM, Mb):
    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {}
    big_n = 64 << 20
    big = [torch.zeros(big_n, dtype=torch.float32, device="cuda") for _ in range(4)]
    big_b = torch.empty(roast.roast_m_shadow_bytes(big_n) // 2, dtype=torch.bfloat16, device="cuda")
    small = [torch.zeros_like(M) for _ in range(2)]
    Mc, dMc = M.clone(), dM.clone()
    # bytes per parameter: M read+write, dM read+write (cleared), states read+write, shadow 2 x 2 written
    per_param = {"sgd": 4 * 4 + 4, "adagrad": 6 * 4 + 4, "adam": 8 * 4 + 4}
    for name, kind in (("sgd", roast.ROAST_OPT_SGD), ("adagrad", roast.ROAST_OPT_ADAGRAD), ("adam", roast.ROAST_OPT_ADAM)):
        d = roast.optim_desc(kind, 1e-3, step=3, eps=1e-8)
        ms_small = timed(lambda: roast.roast_optim_step(d, Mc, dMc, small[0], small[1], Mb))
        ms_big = timed(lambda: roast.roast_optim_step(d, big[0], big[1], big[2], big[3], big_b), reps=5)
        out[name] = {"cfg2_M_ms": ms_small, "M_64Mi_ms": ms_big,
                     "M_64Mi_GBs": per_param[name] * big_n / (ms_big * 1e-3) / 1e9}
    return out


def bench_mm_config(args, roast, wl, torch, np, to_dev, mode, workload=None, steps=None, warmup=None):
    """Forward, dX and dM of every layer of one ROAST-MM configuration, all layers sharing M and dM."""
    cfg = wl.CONFIGS[workload or args.workload]
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    if args.dtype == "f32":
        import dataclasses
        cfg = dataclasses.replace(cfg, dtype="f32")
    inp = wl.make_mm_inputs(cfg)
    bf16 = cfg.dtype == "bf16"
    M = to_dev(inp.M)
    Mb = roast.roast_m_shadow_bf16(M) if bf16 else (None if args.no_f32_workspace else roast.roast_m_planes_bf16(M))
    dM = torch.zeros(cfg.m_size, dtype=torch.float32, device="cuda")
    layers = []
    tensors = {}
    fill_rng = np.random.default_rng(cfg.seed + 1)
    for l in cfg.layers:
        d = roast.mm_desc(l.H, l.O, cfg.Z1, cfg.Z2, cfg.m_size, l.layer_id, cfg.lam, inp.hash)
        key = (l.H, l.O)
        if key not in tensors:      # one X / dY per distinct shape, reused by the layers of that shape
            # a chained configuration draws only its first X and last dY: the rest is drawn here
            Xn = inp.X[l.name] if l.name in inp.X else wl.draw_act(fill_rng, cfg.I, l.H, cfg.dtype)
            dYn = inp.dY[l.name] if l.name in inp.dY else wl.draw_act(fill_rng, cfg.I, l.O, cfg.dtype)
            X, dY = to_dev(Xn), to_dev(dYn)
            tensors[key] = (X, dY, torch.empty_like(dY), torch.empty_like(X))
        layers.append((d, l) + tensors[key])
    ws = None
    if mode == roast.ROAST_REDUCE_DETERMINISTIC or args.dm_workspace:
        ws = torch.empty(max(max(roast.roast_mm_bwd_dM_workspace(d, cfg.I, mode) for d, *_ in layers), 1),
                         dtype=torch.uint8, device="cuda")

    wf = wx = None
    if not bf16 and not args.no_f32_workspace:
        # fp32: the workspaces with which the three products run on the matrix cores
        nbytes = lambda f: max(max(f(d) for d, *_ in layers), 16)
        wf = torch.empty(nbytes(lambda d: roast.roast_mm_fwd_workspace(d, torch.float32, cfg.I)), dtype=torch.uint8,
                         device="cuda")
        wx = torch.empty(nbytes(lambda d: roast.roast_mm_bwd_dx_workspace(d, torch.float32, cfg.I)), dtype=torch.uint8,
                         device="cuda")
        if mode == roast.ROAST_REDUCE_ATOMIC:
            ws = torch.empty(nbytes(lambda d: roast.roast_mm_bwd_dM_workspace_f32(d, cfg.I)), dtype=torch.uint8,
                             device="cuda")

    def step():
        if bf16:
            roast.roast_m_shadow_bf16(M, Mb)
        elif Mb is not None:
            roast.roast_m_planes_bf16(M, Mb)
        for d, l, X, dY, Y, dX in layers:
            roast.roast_mm_fwd(d, X, M, Y, M_bf16=Mb, ws=wf)
        for d, l, X, dY, Y, dX in reversed(layers):
            roast.roast_mm_bwd_dx(d, dY, M, dX, M_bf16=Mb, ws=wx)
            roast.roast_mm_bwd_dM(d, X, dY, dM, mode, ws)

    for _ in range(warmup):
        step()
    run = step
    if args.graph:
        # the library only launches kernels (no allocation, no synchronisation, no memset), so a step
        # can be captured once its kernels have been configured by the warm-up calls above
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
        for _ in range(3):
            run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = e0.elapsed_time(e1) / steps
    flop = 3.0 * sum(2.0 * cfg.I * l.H * l.O for l in cfg.layers)
    peak = PEAK_BF16_TFLOPS if bf16 else 157.3
    tflops = flop / (ms * 1e-3) / 1e12
    return {"metric": "ROAST-MM fwd+bwd TFLOP/s (% MFMA peak)", "unit": "TFLOP/s", "value": tflops, "n_gpus": 1,
            "steps": steps, "warmup": warmup, "ms_per_step": (t1 - t0) * 1e3 / steps, "mm_ms": ms,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32",
            "data": "synthetic", "pct_mfma_peak": 100.0 * tflops / peak,
            "config": {"workload": f"{cfg.name}: I={cfg.I}, {len(cfg.layers)} layer call(s), {cfg.Z1}x{cfg.Z2} tiles, "
                                   f"|M|={cfg.m_size}, {cfg.dtype}", "reduce": args.reduce, "dm_workspace": ws is not None,
                       "f32_on_matrix_cores": wf is not None, "hip_graph": bool(args.graph)},
            "roofline": {"kernel": "whole step (all MM kernels)", "bound": "mfma" if bf16 else "alu", "achieved": tflops,
                         "peak": peak, "unit": "TFLOP/s", "frac": tflops / peak, "traffic": None}}


def bench_dim_sweep(args, roast, wl, torch, np):
    """Square Dim x Dim ROAST-MM layers at batch 512 (the shape family of the paper's Table 1 and
    Appendix B), |M| from 4 MB to 512 MB, bf16 with 64x64 tiles: forward, dX, dM and the optimizer
    step, each timed alone, with the vendor dense bf16 GEMM of the same shape beside them.  The
    printed Dim 8096 is run as printed (126.5 tiles per side: ragged last tile and last contraction step)."""
    I, Z = 512, 64
    f32 = args.dtype == "f32"
    tdt = torch.float32 if f32 else torch.bfloat16
    dims = [512, 1024, 2048, 4096, 8096, 10240, 20480]
    m_sizes = [1 << 20, 16 << 20, 128 << 20]
    g = torch.Generator(device="cuda").manual_seed(2207)
    hp = wl.draw_hash(np.random.default_rng(10702), use_sign=True, align=1)

    def timed(fn, reps, warm=None):
        for _ in range(max(2, args.warmup // 3) if warm is None else warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    rows = []
    Ms = {m: torch.randn(m, dtype=torch.float32, device="cuda", generator=g) * 0.02 for m in m_sizes}
    # made once per M, as after an optimizer step: the bf16 shadow, or for fp32 the three bfloat16 planes
    shadows = {m: (roast.roast_m_planes_bf16(Ms[m]) if f32 else roast.roast_m_shadow_bf16(Ms[m])) for m in m_sizes}
    dM = torch.zeros(max(m_sizes), dtype=torch.float32, device="cuda")
    for dim in dims:
        reps = max(5, min(args.steps, int(4e6 / dim)))
        X = torch.randn((I, dim), dtype=torch.float32, device="cuda", generator=g).to(tdt)
        dY = torch.randn((I, dim), dtype=torch.float32, device="cuda", generator=g).to(tdt)
        Y, dX = torch.empty_like(X), torch.empty_like(X)
        W = (torch.randn((dim, dim), dtype=torch.float32, device="cuda", generator=g) * 0.02).to(tdt)
        dW = torch.empty_like(W)
        row = {"Dim": dim, "GFLOP_per_product": 2.0 * I * dim * dim / 1e9,
               "dense_fwd_ms": timed(lambda: torch.matmul(X, W, out=Y), reps),
               "dense_dx_ms": timed(lambda: torch.matmul(dY, W.t(), out=dX), reps),
               "dense_dw_ms": timed(lambda: torch.matmul(X.t(), dY, out=dW), reps), "roast": {}}
        del W, dW
        for m in m_sizes:
            d = roast.mm_desc(dim, dim, Z, Z, m, 0, 1.0, hp)
            nbytes = max(roast.roast_mm_fwd_workspace(d, tdt, I), roast.roast_mm_bwd_dx_workspace(d, tdt, I),
                         roast.roast_mm_bwd_dM_workspace_f32(d, I) if f32 else 0, 16)
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            M, Mb, dMv = Ms[m], shadows[m], dM[:m]
            wsm = ws if f32 else None
            r = {"fwd_ms": timed(lambda: roast.roast_mm_fwd(d, X, M, Y, M_bf16=Mb, ws=ws), reps),
                 "fwd_no_ws_ms": timed(lambda: roast.roast_mm_fwd(d, X, M, Y, M_bf16=Mb), reps),
                 "dx_ms": timed(lambda: roast.roast_mm_bwd_dx(d, dY, M, dX, M_bf16=Mb, ws=ws), reps),
                 "dM_ms": timed(lambda: roast.roast_mm_bwd_dM(d, X, dY, dMv, roast.ROAST_REDUCE_ATOMIC, wsm), reps),
                 "workspace_MB": nbytes / 1e6}
            row["roast"][f"{m * 4 >> 20}MB"] = r
            del ws
        # element-wise hashing (1x1 tiles, one hash per virtual weight): the HashedNet-style map the
        # paper compares against, through the same entry points and the same matrix-core kernels -- only
        # the staging of the weight operand differs (a gather through the hash per element instead of a
        # contiguous tile) -- with the same split-contraction workspace (bf16; fp32 runs it on the
        # vector ALUs)
        row["elementwise_1x1"] = {}
        for m in (m_sizes[0], m_sizes[-1]):
            d = roast.mm_desc(dim, dim, 1, 1, m, 0, 1.0, hp)
            M, dMv = Ms[m], dM[:m]
            nbytes = max(roast.roast_mm_fwd_workspace(d, tdt, I), roast.roast_mm_bwd_dx_workspace(d, tdt, I), 16)
            ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
            row["elementwise_1x1"][f"{m * 4 >> 20}MB"] = {
                "fwd_ms": timed(lambda: roast.roast_mm_fwd(d, X, M, Y, ws=ws), 3, 1),
                "dx_ms": timed(lambda: roast.roast_mm_bwd_dx(d, dY, M, dX, ws=ws), 3, 1),
                "dM_ms": timed(lambda: roast.roast_mm_bwd_dM(d, X, dY, dMv, roast.ROAST_REDUCE_ATOMIC), 3, 1)}
            del ws
        rows.append(row)
        print(f"# Dim {dim}: dense fwd {row['dense_fwd_ms']:.3f} ms; ROAST fwd "
              + " / ".join(f"{v['fwd_ms']:.3f}" for v in row["roast"].values()) + " ms; 1x1 tiles fwd "
              + " / ".join(f"{v['fwd_ms']:.3f}" for v in row["elementwise_1x1"].values()) + " ms",
              file=sys.stderr, flush=True)
    last = rows[-1]
    best = last["roast"]["4MB"]["fwd_ms"]
    tflops = last["GFLOP_per_product"] / best
    avg = lambda key, m: sum(r["roast"][m][key] for r in rows) / len(rows)
    return {"metric": "ROAST-MM forward TFLOP/s at Dim 20480, batch 512, |M| 4 MB", "unit": "TFLOP/s", "value": tflops,
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": best, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32" if f32 else "bf16", "data": "synthetic",
            "config": {"workload": "dim_sweep_b512: square Dim x Dim, batch 512, 64x64 tiles, |M| 4 / 64 / 512 MB, "
                                   + ("fp32 on the matrix cores (bfloat16 planes)" if f32 else "bf16")},
            "averages_ms": {m: {k: avg(k, m) for k in ("fwd_ms", "dx_ms", "dM_ms")} for m in last["roast"]},
            "dense_averages_ms": {k: sum(r[k] for r in rows) / len(rows)
                                  for k in ("dense_fwd_ms", "dense_dx_ms", "dense_dw_ms")},
            "elementwise_over_tiled_fwd": {m: sum(r["elementwise_1x1"][m]["fwd_ms"] for r in rows)
                                           / sum(r["roast"][m]["fwd_ms"] for r in rows) for m in ("4MB", "512MB")},
            "table": rows,
            "roofline": {"kernel": "roast_mm_fwd at Dim 20480", "bound": "mfma", "achieved": tflops,
                         "peak": 157.3 if f32 else PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": tflops / (157.3 if f32 else PEAK_BF16_TFLOPS), "traffic": None}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); the hot path has no multi-GPU leg.",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2207_10702_amd import binding as roast, workloads as wl
    from paper_2207_10702_amd.checks import to_dev

    roast.load()
    torch.cuda.set_device(0)
    mode = roast.ROAST_REDUCE_ATOMIC if args.reduce == "atomic" else roast.ROAST_REDUCE_DETERMINISTIC
    if args.workload == "dim_sweep_b512":
        print(json.dumps(bench_dim_sweep(args, roast, wl, torch, np)))
        return
    if args.workload != "default":
        print(json.dumps(bench_mm_config(args, roast, wl, torch, np, to_dev, mode)))
        return

    # ------------------------------------------------------------------ inputs (resident before timing)
    mcfg = wl.CONFIGS["cfg2_bert_ffn_bf16"]
    mi = wl.make_mm_inputs(mcfg)
    l1, l2 = mcfg.layers
    d1 = roast.mm_desc(l1.H, l1.O, mcfg.Z1, mcfg.Z2, mcfg.m_size, l1.layer_id, mcfg.lam, mi.hash)
    d2 = roast.mm_desc(l2.H, l2.O, mcfg.Z1, mcfg.Z2, mcfg.m_size, l2.layer_id, mcfg.lam, mi.hash)
    M = to_dev(mi.M)
    Mb = torch.empty(roast.roast_m_shadow_bytes(mcfg.m_size) // 2, dtype=torch.bfloat16, device="cuda")
    X = to_dev(mi.X[l1.name])
    dY = to_dev(mi.dY[l2.name])
    I = mcfg.I
    H1 = torch.empty((I, l1.O), dtype=torch.bfloat16, device="cuda")
    Y = torch.empty((I, l2.O), dtype=torch.bfloat16, device="cuda")
    dH1 = torch.empty((I, l1.O), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((I, l1.H), dtype=torch.bfloat16, device="cuda")
    dM = torch.zeros(mcfg.m_size, dtype=torch.float32, device="cuda")
    # workspace: required by the deterministic mode, optional in the atomic mode (off by default:
    # nothing of the size of the virtual weight matrix is then ever allocated)
    ws = None
    if args.reduce == "deterministic" or args.dm_workspace:
        ws_bytes = max(roast.roast_mm_bwd_dM_workspace(d1, I, mode), roast.roast_mm_bwd_dM_workspace(d2, I, mode), 1)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    ecfg = wl.CONFIGS["cfg4_dlrm_embed_f32"]
    ei = wl.make_embed_inputs(ecfg)
    ed = roast.embed_desc(ecfg.D, ecfg.Z, ecfg.m_size, ecfg.lam, ei.hash)
    eM = to_dev(ei.M)
    rows, tables, dOut = to_dev(ei.rows), to_dev(ei.tables), to_dev(ei.dOut)
    N = ecfg.N
    out = torch.empty((N, ecfg.D), dtype=torch.float32, device="cuda")
    edM = torch.zeros(ecfg.m_size, dtype=torch.float32, device="cuda")
    ews = torch.empty(max(roast.roast_embed_bwd_workspace(ed, N, mode), 1), dtype=torch.uint8, device="cuda")

    cal_src = cal_dst = None
    if args.calibration_copy:
        cal_src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        cal_dst = torch.empty_like(cal_src)

    names = []
    if not args.embed_only:
        names += ["m_shadow", "mm_fwd_l1", "mm_fwd_l2", "mm_bwd_dx_l2", "mm_bwd_dM_l2", "mm_bwd_dx_l1", "mm_bwd_dM_l1"]
    if not args.mm_only:
        names += ["embed_fwd", "embed_bwd"]

    def step(ev=None, sec=None):
        """One pass of the hot path.  ev: events recorded around every call (the instrumented pass);
        sec: events at the three section boundaries only (the timed pass)."""
        k = 0

        def mark():
            nonlocal k
            if ev is not None:
                ev[k].record()
            k += 1

        def section(i):
            if sec is not None:
                sec[i].record()

        mark()
        section(0)
        if not args.embed_only:
            roast.roast_m_shadow_bf16(M, Mb); mark()       # once per step: M changes once per step
            roast.roast_mm_fwd(d1, X, M, H1, M_bf16=Mb); mark()
            roast.roast_mm_fwd(d2, H1, M, Y, M_bf16=Mb); mark()
            roast.roast_mm_bwd_dx(d2, dY, M, dH1, M_bf16=Mb); mark()
            roast.roast_mm_bwd_dM(d2, H1, dY, dM, mode, ws); mark()
            roast.roast_mm_bwd_dx(d1, dH1, M, dX, M_bf16=Mb); mark()
            roast.roast_mm_bwd_dM(d1, X, dH1, dM, mode, ws); mark()
        section(1)
        if not args.mm_only:
            roast.roast_embed_fwd(ed, rows, tables, eM, out); mark()
        section(2)
        if not args.mm_only:
            roast.roast_embed_bwd(ed, rows, tables, dOut, edM, mode, ews); mark()
        section(3)
        if cal_src is not None:
            cal_dst.copy_(cal_src)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Instrumented pass (before the timed one): the same K steps with an event around every call, for
    # the per-call figures and the per-kernel rooflines.  An event between two launches keeps the second
    # from starting under the tail of the first and costs a few microseconds per call (about 6 % of the
    # ROAST-MM section), so `value` is not taken from this pass.
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for _ in range(args.steps)]
    for s in range(args.steps):
        step(evs[s])
    torch.cuda.synchronize()
    samples = {n: np.array([evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(args.steps)])
               for i, n in enumerate(names)}                        # ms per call, one sample per step
    per_call = {n: float(np.mean(v)) for n, v in samples.items()}
    # Kernel pass for the ROAST-MM calls: each call launched K times in a row between two events.  A
    # call here is one launch of one kernel, so elapsed / K is that kernel's own duration -- what a
    # kernel trace reports -- without the few microseconds an event costs on each side of a single
    # launch.  The per-kernel roofline is taken from this figure.
    launch_ms = {}
    if not args.embed_only:
        mm_launch = {"mm_fwd_l1": lambda: roast.roast_mm_fwd(d1, X, M, H1, M_bf16=Mb),
                     "mm_fwd_l2": lambda: roast.roast_mm_fwd(d2, H1, M, Y, M_bf16=Mb),
                     "mm_bwd_dx_l2": lambda: roast.roast_mm_bwd_dx(d2, dY, M, dH1, M_bf16=Mb),
                     "mm_bwd_dM_l2": lambda: roast.roast_mm_bwd_dM(d2, H1, dY, dM, mode, ws),
                     "mm_bwd_dx_l1": lambda: roast.roast_mm_bwd_dx(d1, dH1, M, dX, M_bf16=Mb),
                     "mm_bwd_dM_l1": lambda: roast.roast_mm_bwd_dM(d1, X, dH1, dM, mode, ws)}
        for n, fn in mm_launch.items():
            k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fn()
            k0.record()
            for _ in range(args.steps):
                fn()
            k1.record()
            torch.cuda.synchronize()
            launch_ms[n] = k0.elapsed_time(k1) / args.steps
    # Timed pass: exactly K steps between two synchronisations, calls back to back as a training loop
    # issues them; events only where the step passes from ROAST-MM to the lookup and from the lookup's
    # forward to its gradient, to split the step's time between the two metrics.
    secs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(sec=secs[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    sec_ms = [float(np.mean([secs[s][i].elapsed_time(secs[s][i + 1]) for s in range(args.steps)])) for i in range(3)]
    # zeroing dM is the caller's job and outside the step; its cost is reported beside it
    z0, z1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    z0.record()
    for _ in range(20):
        dM.zero_()
    z1.record()
    torch.cuda.synchronize()

    result = {"metric": "ROAST-MM fwd+bwd TFLOP/s (% MFMA peak); ROAST-embedding GB/s (% HBM peak)",
              "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
              "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
              "dtype": "bf16", "data": "synthetic",
              "config": {"workload": "cfg2_bert_ffn_bf16 (ROAST-MM 8192x768x3072 + 8192x3072x768, 64x64 tiles, "
                                     "|M|=47185) + cfg4_dlrm_embed_f32 (1703936 lookups x 128, chunk 32, |M|=1.28M)",
                         "reduce": args.reduce, "dm_workspace": ws is not None},
              "timing": "value, mm_ms, the embedding GB/s and ms_per_step come from the timed pass (K steps, calls back to "
                        "back, events at the two section boundaries only); per_call_* come from an instrumented pass of the "
                        "same K steps run before it (an event around every call); kernel_ms and the ROAST-MM per-kernel "
                        "rooflines from a kernel pass (each call K times in a row between two events)",
              "section_ms": {"roast_mm (shadow + 6 calls)": sec_ms[0], "embed_fwd": sec_ms[1], "embed_bwd": sec_ms[2]},
              "per_call_ms": per_call,
              "per_call_median_ms": {n: float(np.median(v)) for n, v in samples.items()},
              "per_call_min_ms": {n: float(np.min(v)) for n, v in samples.items()},
              "dM_zero_ms": z0.elapsed_time(z1) / 20}

    # The weight update of a training step (outside `value`): one fused pass that applies the rule,
    # clears dM and refreshes the bf16 shadow.  Timed on config 2's M and on a 64 Mi-entry M (config 5's).
    if not args.embed_only and not args.hot_path_only:
        result["optimizer"] = time_optimizer(roast, torch, M, dM, Mb)

    flop_layer = {"l1": 2.0 * I * l1.H * l1.O, "l2": 2.0 * I * l2.H * l2.O}
    if not args.embed_only:
        mm_ms = sec_ms[0]                                   # timed pass: shadow + the six calls, back to back
        mm_flop = 3.0 * (flop_layer["l1"] + flop_layer["l2"])
        result["mm_ms_instrumented"] = sum(v for k, v in per_call.items() if k.startswith("mm_") or k == "m_shadow")
        tflops = mm_flop / (mm_ms * 1e-3) / 1e12
        result["value"] = tflops
        result["mm_ms"] = mm_ms
        result["pct_mfma_peak"] = 100.0 * tflops / PEAK_BF16_TFLOPS
        # Per-call rooflines.  A forward / dX / dM call in this configuration (bf16 shadow, atomic dM
        # without workspace) is exactly one launch of one instantiation of the MFMA kernel template,
        # so the kernel pass's time per launch on the launch stream is that kernel's duration.
        mm_calls = [k for k in per_call if k.startswith("mm_")]
        result["roofline_per_call"] = {
            k: {"achieved": flop_layer[k[-2:]] / (launch_ms[k] * 1e-3) / 1e12, "unit": "TFLOP/s",
                "frac": flop_layer[k[-2:]] / (launch_ms[k] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                "launch_us": 1e3 * launch_ms[k], "call_us_instrumented": 1e3 * per_call[k]} for k in mm_calls}
        # The dominant kernel = the instantiation with the largest total time per step: the dM
        # product (MODE 2, two launches per step, one per layer; both 38.65 GFLOP).
        by_kind = {"k_roast_mfma<MODE_DM> (mm_bwd_dM_l1 + mm_bwd_dM_l2)": ["mm_bwd_dM_l1", "mm_bwd_dM_l2"],
                   "k_roast_mfma<MODE_FWD> (mm_fwd_l1 + mm_fwd_l2)": ["mm_fwd_l1", "mm_fwd_l2"],
                   "k_roast_mfma<MODE_DX> (mm_bwd_dx_l1 + mm_bwd_dx_l2)": ["mm_bwd_dx_l1", "mm_bwd_dx_l2"]}
        dom = max(by_kind, key=lambda k: sum(launch_ms[c] for c in by_kind[k]))
        calls = by_kind[dom]
        ach = sum(flop_layer[c[-2:]] for c in calls) / (sum(launch_ms[c] for c in calls) * 1e-3) / 1e12
        traffic = None
        if args.reduce == "atomic" and ws is None:       # the configuration the committed summary was taken in
            traffic = traffic_of(load_measured_traffic(), calls, "k_roast_mfma") / len(calls)
        result["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                              "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS, "traffic": traffic,
                              "launches_per_step": len(calls),
                              "avg_launch_us": 1e3 * sum(launch_ms[c] for c in calls) / len(calls),
                              "avg_call_us_instrumented": 1e3 * sum(per_call[c] for c in calls) / len(calls)}
        result["kernel_ms"] = launch_ms
    if not args.mm_only:
        # compulsory HBM bytes: output (or dOut) once, ids once, M (and dM read+write) once
        ids = N * (8 + 4)
        bytes_fwd = N * ecfg.D * 4 + ids + ecfg.m_size * 4
        bytes_bwd = N * ecfg.D * 4 + ids + 2 * ecfg.m_size * 4
        # one call each, so the section times of the timed pass are the calls' times
        gbs_f = bytes_fwd / (sec_ms[1] * 1e-3) / 1e9
        gbs_b = bytes_bwd / (sec_ms[2] * 1e-3) / 1e9
        tot = (bytes_fwd + bytes_bwd) / ((sec_ms[1] + sec_ms[2]) * 1e-3) / 1e9
        tr = load_measured_traffic() if args.reduce == "atomic" else None
        result["embedding"] = {"value": tot, "unit": "GB/s", "pct_hbm_peak": 100.0 * tot / PEAK_HBM_GBS,
                               "fwd_GBs": gbs_f, "bwd_GBs": gbs_b, "bytes_fwd": bytes_fwd, "bytes_bwd": bytes_bwd,
                               # the gradient is the larger consumer of the two (and of the whole step):
                               # its kernels together (zero + route + accumulate = one call) are the
                               # dominant HBM-bound work
                               "roofline": {"kernel": "k_embed_zero + k_embed_route + k_embed_accum (embed_bwd)",
                                            "bound": "hbm", "achieved": gbs_b, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                            "frac": gbs_b / PEAK_HBM_GBS,
                                            "traffic": traffic_of(tr, ["embed_bwd"], "k_embed_accum") if tr else None},
                               "roofline_fwd": {"kernel": "k_embed (embed_fwd)", "bound": "hbm", "achieved": gbs_f,
                                                "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs_f / PEAK_HBM_GBS,
                                                "traffic": traffic_of(tr, ["embed_fwd"], "k_embed") if tr else None}}
        if not args.hot_path_only:
            # the pooled reading of "gather-sum": one output row per sample = the sum of its 26 lookups
            nb = N // ecfg.n_tables
            bag_off = torch.arange(nb + 1, dtype=torch.int64, device="cuda") * ecfg.n_tables
            pout = torch.empty((nb, ecfg.D), dtype=torch.float32, device="cuda")
            pdOut = dOut[:nb]
            pws = torch.empty(max(roast.roast_embed_bag_bwd_workspace(ed, N, nb, mode), 1), dtype=torch.uint8, device="cuda")

            def timed(fn, reps=20):
                for _ in range(3):
                    fn()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps

            pf = timed(lambda: roast.roast_embed_bag_fwd(ed, rows, tables, bag_off, eM, pout))
            pb = timed(lambda: roast.roast_embed_bag_bwd(ed, rows, tables, bag_off, pdOut, edM, mode, pws))
            edM.zero_()
            result["embedding"]["pooled_sum_of_26"] = {
                "bags": nb, "fwd_ms": pf, "bwd_ms": pb, "lookups_per_s_fwd": N / (pf * 1e-3),
                "lookups_per_s_bwd": N / (pb * 1e-3),
                # what the gathers deliver: every lookup reads D floats of M (cache-resident) / of dOut
                "gathered_GBs_fwd": N * ecfg.D * 4 / (pf * 1e-3) / 1e9, "gathered_GBs_bwd": N * ecfg.D * 4 / (pb * 1e-3) / 1e9}
        if args.embed_only:
            result["value"] = tot
            result["unit"] = "GB/s"
            result["dtype"] = "f32"
            result["roofline"] = result["embedding"]["roofline"]

    # The other ROAST-MM configurations (outside `value`): forward, dX and dM of every layer, timed
    # as a whole step each, with their fraction of the MFMA peak (fp32 for config 1: it runs on the
    # bf16 matrix cores from bfloat16 planes and is priced against the fp32 MFMA peak).
    if not args.embed_only and not args.hot_path_only and not args.mm_only and args.reduce == "atomic" and ws is None:
        del X, dY, H1, Y, dH1, dX, out, dOut, rows, tables
        torch.cuda.empty_cache()
        others = {}
        for name, st, wu in (("cfg1_single_f32", 50, 10), ("cfg3_bert_stack_bf16", 8, 2), ("cfg5_large_bf16", 8, 2)):
            r = bench_mm_config(args, roast, wl, torch, np, to_dev, mode, workload=name, steps=st, warmup=wu)
            others[name] = {"workload": r["config"]["workload"], "ms_per_step": r["mm_ms"], "TFLOPs": r["value"],
                            "dtype": r["dtype"], "peak_TFLOPs": r["roofline"]["peak"], "frac": r["roofline"]["frac"],
                            "steps": st, "warmup": wu}
            torch.cuda.empty_cache()
        result["other_configs"] = others

    if not args.no_cpu_baseline and not args.embed_only:
        import oracle
        # bounded sample: the first `rows_s` tokens through forward, dX and dW (+ scatter) of both layers
        rows_s = I     # the whole configuration: about 10 s on 16 host threads
        Xs = wl.act_as_f64(mi.X[l1.name][:rows_s])
        dYs = wl.act_as_f64(mi.dY[l2.name][:rows_s])
        lam = float(np.float32(mcfg.lam))
        c0 = time.perf_counter()
        W1 = oracle.materialize_w(mi.hash, l1.layer_id, l1.H, l1.O, mcfg.Z1, mcfg.Z2, lam, mi.M)
        W2 = oracle.materialize_w(mi.hash, l2.layer_id, l2.H, l2.O, mcfg.Z1, mcfg.Z2, lam, mi.M)
        h1 = oracle.mm_fwd(Xs, W1)
        oracle.mm_fwd(h1, W2)
        dh1 = oracle.mm_bwd_dx(dYs, W2)
        g = oracle.mm_bwd_dm(mi.hash, l2.layer_id, mcfg.Z1, mcfg.Z2, mcfg.m_size, lam, h1, dYs)
        oracle.mm_bwd_dx(dh1, W1)
        oracle.mm_bwd_dm(mi.hash, l1.layer_id, mcfg.Z1, mcfg.Z2, mcfg.m_size, lam, Xs, dh1, dM=g)
        c1 = time.perf_counter()
        flop_s = 3.0 * (flop_layer["l1"] + flop_layer["l2"]) * rows_s / I
        result["cpu_baseline"] = {"value": flop_s / (c1 - c0) / 1e12, "unit": "TFLOP/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "cpu_model": cpu_model(), "host_logical_cpus": os.cpu_count(),
                                  "sample": f"{rows_s} of {I} tokens of cfg2 through fwd, dX and dM of both layers "
                                            f"(W materialised element by element, fp64 triple loops, OpenMP over "
                                            f"rows, {oracle.num_threads()} threads), {c1 - c0:.1f} s wall"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
