#!/usr/bin/env python3
"""Benchmark of the one-GPU MoE hot path.

A step is one pass of the whole path over one batch of synthetic input:
moe_route -> moe_dispatch -> moe_expert_ffn (resident experts only) -> moe_combine
(the training configuration adds moe_combine_bwd -> moe_expert_ffn_bwd -> moe_dispatch_bwd).
Inputs are resident in HBM before the timed region; rows of the packed output that belong
to other ranks are pre-filled outside it.

Prints ONE JSON line: tokens/s of the layer, per-call times, the roofline of the dominant
kernel (the MFMA gate/up grouped GEMM, timed with HIP events on its own stream inside the
timed steps), HBM-bandwidth fractions of dispatch and combine, and the CPU oracle timed on
a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # fp32 vector
PEAK_HBM_GBS = 8000.0


def traffic_from_profile(workload: str, kernel: str):
    """HBM-side bytes per launch of `kernel` (read + written) as the committed rocprofv3
    summary of this workload has them: profiles/hotpath_<workload>_kernel_trace_and_traffic.md,
    table of the two --pmc passes (FETCH_SIZE and WRITE_SIZE, already scaled by the factors of
    the plain 512 MiB copy: columns 'read MB' and 'written MB').  None when there is no such
    file or row."""
    path = os.path.join(ROOT, "profiles", f"hotpath_{workload}_kernel_trace_and_traffic.md")
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return None
    in_table = False
    for line in lines:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 5 and cells[1].startswith("FETCH_SIZE") and cells[2].startswith("read MB"):
            in_table = True
            continue
        if in_table and len(cells) >= 5 and cells[0].startswith(kernel):
            try:
                return (float(cells[2]) + float(cells[4])) * 1e6
            except ValueError:
                continue
    return None


def measure_ceilings(n_loc: int, d: int, f: int, x_packed, W1_0):
    """What the part gives, measured in this process by committed code: a plain copy kernel
    with dispatch's 1:2 read:write mix (and 1:1), the bare MFMA issue loop (zero and varied
    operands), and the library's dense GEMM of the gate/up shape on the workload's data (one
    torch.matmul of [n_loc, d] x [d, 2f]; not grouped, no SwiGLU)."""
    import torch
    import paper_2510_19470_amd as moe
    dev = x_packed.device
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, reps):
        fn()
        fn()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps
    out = {}
    n = 512 << 20
    src = torch.empty(n, dtype=torch.uint8, device=dev)
    src.fill_(1)
    dst = torch.empty(2 * n, dtype=torch.uint8, device=dev)
    t = timed(lambda: moe.moe_measure_copy(src, dst, 2), 10)
    out["copy_read1_write2_gbs"] = 3 * n / (t * 1e-3) / 1e9
    t = timed(lambda: moe.moe_measure_copy(src, dst, 1), 10)
    out["copy_read1_write1_gbs"] = 2 * n / (t * 1e-3) / 1e9
    out["copy_bytes_read"] = n
    del src, dst
    blocks = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.empty(blocks * 512, dtype=torch.float32, device=dev)
    for rnd, key in ((False, "mfma_issue_zero_operands_tflops"), (True, "mfma_issue_varied_operands_tflops")):
        fl = [0.0]

        def go():
            fl[0] = moe.moe_measure_mfma(sink, blocks, 4000, rnd)
        t = timed(go, 5)
        out[key] = fl[0] / (t * 1e-3) / 1e12
    del sink
    # library GEMM of the gate/up shape on the workload data: x_packed rows of the compute
    # region against one expert's W1 repeated to 2f rows
    A = x_packed[:n_loc]
    reps_w = max(1, (2 * f + W1_0.shape[0] - 1) // W1_0.shape[0])
    Wt = W1_0.repeat(reps_w, 1)[:2 * f].contiguous().t()       # [2f, d] in memory, as the experts are
    C = torch.empty((n_loc, 2 * f), dtype=A.dtype, device=dev)
    t = timed(lambda: torch.matmul(A, Wt, out=C), 5)
    out["library_gemm_tflops"] = 2.0 * n_loc * d * 2 * f / (t * 1e-3) / 1e12
    out["library_gemm_shape"] = [int(n_loc), int(d), int(2 * f)]
    del C, Wt
    out["note"] = ("measured in this run: moe_measure_copy (512 MiB read, one 16-byte piece per "
                   "thread), moe_measure_mfma (8 wavefronts per compute unit issuing "
                   "v_mfma_f32_32x32x16_bf16 from registers), torch.matmul bf16 on the workload's "
                   "packed tokens")
    return out


def cpu_baseline(cfg, inp, sample_tokens: int):
    """The oracle as it stands on a bounded sample: the first `sample_tokens` tokens of the
    same workload (same d, E, k, f, placement; resident experts only)."""
    import moe_workloads as wl
    from oracle import moe_oracle as orc
    T = min(sample_tokens, cfg.T)
    f32 = lambda a: None if a is None else wl.stored_to_f32(a, cfg.dtype)
    x = f32(inp.x)[:T]
    Wg = f32(inp.Wg)
    W1 = [f32(w) for w in inp.W1]
    W3 = [f32(w) for w in inp.W3] if cfg.gated else None
    W2 = [f32(w) for w in inp.W2]
    t0 = time.perf_counter()
    res = orc.layer_forward(x, Wg, inp.bias, cfg.k, inp.dest_rank, cfg.R, W1, W3, W2)
    if cfg.backward:
        dout = f32(inp.dOut)[:T]
        dy, _ = orc.combine_bwd(dout, res["y_packed"], res["slot_to_row"], res["topk_w"])
        if cfg.gated:
            dxp = orc.expert_ffn_bwd(dy, res["x_packed"], res["G"], res["U"], res["expert_counts"],
                                     res["expert_offsets"], W1, W3, W2)[0]
        else:
            dxp = orc.expert_ffn2_bwd(dy, res["x_packed"], res["G"], res["expert_counts"],
                                      res["expert_offsets"], W1, W2)[0]
        orc.dispatch_bwd(dxp, res["slot_to_row"], T, cfg.k)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": T / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "host_cpu_count": os.cpu_count(),
            "sample": f"first {T} of {cfg.T} tokens of '{cfg.name}', NumPy oracle computing in "
                      f"float64 on the stored bf16 values (upcast exactly through float32), "
                      f"resident experts only, {dt:.2f} s; cores = BLAS threads used, "
                      f"host_cpu_count = os.cpu_count()"}


def sr_compression_bench(ctx, rows: int, cols: int, cr: int = 50, reps: int = 10):
    """Shared/residual expert compression (paper Sec. 4.2) on one weight matrix of the
    workload's expert shape: encode and decode timed with events, outside the timed steps.
    Synthetic weights drawn on the device: shared ~ N(0, 1/cols); residual = a dense part of
    5 % of that scale plus, on 2 % of the entries, a part of the full scale."""
    import torch
    import paper_2510_19470_amd as moe
    g = torch.Generator(device="cuda")
    g.manual_seed(4242)
    sd = cols ** -0.5
    S = (torch.randn(rows, cols, device="cuda", generator=g) * sd).to(torch.bfloat16)
    R = torch.randn(rows, cols, device="cuda", generator=g) * (0.05 * sd)
    big = torch.rand(rows, cols, device="cuda", generator=g) < 0.02
    R = R + big * (torch.randn(rows, cols, device="cuda", generator=g) * sd)
    W = (S.float() + R).to(torch.bfloat16)
    del R, big
    n = rows * cols
    k = moe.moe_sr_keep_count(n, cr)
    vals, idx = moe.moe_sr_encode(ctx, W, S, k)
    out = moe.moe_sr_decode(ctx, S, vals, idx)

    def timed(fn):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    t_enc = timed(lambda: moe.moe_sr_encode(ctx, W, S, k, vals, idx))
    t_dec = timed(lambda: moe.moe_sr_decode(ctx, S, vals, idx, out))
    by_enc = 2 * n * 2 + k * 6          # expert + shared read once, list written
    by_dec = 2 * n * 2 + k * 6          # shared read, expert written, list read
    return {"matrix": f"{rows}x{cols} bf16", "cr": cr, "kept": int(k),
            "encode_ms": t_enc, "decode_ms": t_dec,
            "encode_algorithmic_gbs": by_enc / (t_enc * 1e-3) / 1e9,
            "encode_streamed_gbs": (5 * 2 * n * 2 + k * 6) / (t_enc * 1e-3) / 1e9,
            "decode_gbs": by_dec / (t_dec * 1e-3) / 1e9,
            "decode_frac_of_hbm_peak": by_dec / (t_dec * 1e-3) / 1e9 / PEAK_HBM_GBS}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10,
                    help="untimed steps first (the clock of an idle GPU takes tens of ms to ramp up)")
    ap.add_argument("--config", default="mixtral",
                    help="workload: tiny | small | mixtral | finegrained | train | paper (a layer "
                         "of the paper's own sweep with its two-matrix expert) | paper_train "
                         "(the same layer, forward + backward)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0,
                    help="tokens of the oracle baseline sample (0 = sized for ~10-30 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the other configurations (small, finegrained, train) and the "
                         "measured ceilings that the default run adds outside the timed region")
    ap.add_argument("--no-sr", action="store_true",
                    help="skip the shared/residual compression measurement (one expert matrix, "
                         "outside the timed steps)")
    ap.add_argument("--chunks", type=int, default=0,
                    help="also time the chunked overlap schedule (moe_pipeline_forward) with this "
                         "many chunks on --chunk-streams streams, outside the timed steps")
    ap.add_argument("--chunk-streams", type=int, default=2)
    ap.add_argument("--graph", action="store_true",
                    help="also capture one step into a HIP graph and time its replays (outside the "
                         "timed steps)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 512 MiB device copy (a kernel of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--table3-sweep", action="store_true",
                    help="instead of one workload: the paper's layer shapes (Table 3: K, B*L, H, M "
                         "varied one at a time around K=2, B*L=8192, H=1024, M=4096; E=32, "
                         "two-matrix expert, forward + backward), one JSON line with a row per shape")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import moe_workloads as wl
    import paper_2510_19470_amd as moe
    from paper_2510_19470_amd.layer import layer_from_inputs, to_device

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    if args.table3_sweep:
        return table3_sweep(args)
    rec = run(wl.CONFIGS[args.config], args)
    if not args.no_others and args.config == "mixtral":
        # the other large configurations, outside the headline's timed region: fewer steps,
        # no oracle, no compression measurement
        import copy
        a2 = copy.copy(args)
        a2.no_sr = a2.no_cpu_baseline = True
        a2.graph, a2.chunks, a2.copy_calibration = False, 0, False
        a2.steps, a2.warmup = min(args.steps, 10), max(args.warmup, 5)
        rec["other_configs"] = {}
        for name in ("small", "finegrained", "train"):
            r = run(wl.CONFIGS[name], a2, with_ceilings=False)
            rec["other_configs"][name] = {
                "workload": r["config"]["workload"], "n_loc_rows": r["config"]["n_loc_rows"],
                "steps": a2.steps, "warmup": a2.warmup,
                "ms_per_step": r["ms_per_step"], "tokens_per_s": r["value"],
                "gate_up_frac_of_peak": r["grouped_gemm"]["frac_of_peak_gate_up"],
                "down_frac_of_peak": r["grouped_gemm"]["frac_of_peak_down"],
                "ffn_call_frac_of_peak": r["grouped_gemm"]["frac_of_peak_whole_call"],
                "dispatch_frac_of_hbm_peak": r["hbm"]["dispatch_frac"],
                "combine_frac_of_hbm_peak": r["hbm"]["combine_frac"],
                "call_ms": r["call_ms"],
                **({"ffn_bwd_frac_of_peak": r["grouped_gemm"]["frac_of_peak_bwd_call"],
                    "ffn_fwd_bwd_frac_of_peak": r["grouped_gemm"]["frac_of_peak_fwd_bwd"]}
                   if "frac_of_peak_bwd_call" in r["grouped_gemm"] else {}),
            }
    print(json.dumps(rec))
    return 0


def table3_sweep(args) -> int:
    """The paper's own layer shapes (Sec. 5.1, Table 3) on one GPU's share of an 8-rank layout:
    4 home experts + 4 fetched ones resident, two-matrix expert, forward + backward.  Every
    parameter is varied alone around the base shape; B*L is the number of tokens."""
    from dataclasses import replace
    import moe_workloads as wl
    base = wl.CONFIGS["paper_train"]
    shapes = [dict()]
    shapes += [dict(k=K) for K in (1, 4)]
    shapes += [dict(T=T) for T in (1024, 4096, 16384)]
    shapes += [dict(d=H) for H in (512, 768)]
    shapes += [dict(f=M) for M in (768, 1024, 1536, 2048, 3072)]
    args.no_sr = args.no_cpu_baseline = True
    args.graph, args.chunks, args.copy_calibration = False, 0, False
    rows = []
    for i, sh in enumerate(shapes):
        cfg = replace(base, name="table3", seed=base.seed + i, **sh)
        r = run(cfg, args)
        g, c = r["grouped_gemm"], r["call_ms"]
        rows.append({"K": cfg.k, "tokens": cfg.T, "H": cfg.d, "M": cfg.f,
                     "n_loc_rows": r["config"]["n_loc_rows"], "ms_per_step": r["ms_per_step"],
                     "tokens_per_s": r["value"], "first_gemm_tflops": g["gate_up_tflops"],
                     "second_gemm_tflops": g["down_tflops"], "call_ms": c})
        print(f"table3 K={cfg.k} tokens={cfg.T} H={cfg.d} M={cfg.f}: "
              f"{r['ms_per_step']:.3f} ms per step", file=sys.stderr, flush=True)
    print(json.dumps({"metric": "MoE-layer step time over the paper's Table 3 shapes (1 GPU, forward "
                                "+ backward, E=32, two-matrix expert)", "unit": "ms", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "dtype": "bf16",
                      "data": "synthetic", "rows": rows}))
    return 0


def run(cfg, args, with_ceilings: bool = True) -> dict:
    """One workload: warm-up, the timed steps, the breakdown pass and the extras; returns the
    record that main() prints."""
    import torch
    import moe_workloads as wl
    import paper_2510_19470_amd as moe
    from paper_2510_19470_amd.layer import layer_from_inputs, to_device

    t_gen = time.perf_counter()
    inp = wl.make_inputs(cfg, experts="resident")
    t_gen = time.perf_counter() - t_gen
    lay = layer_from_inputs(inp)
    dev = lay.device
    x = to_device(inp.x, cfg.dtype)
    dout = to_device(inp.dOut, cfg.dtype) if cfg.backward else None
    T, k, d, E, f, R = cfg.T, cfg.k, cfg.d, cfg.E, cfg.f, cfg.R
    S = T * k
    tdt = lay.ctx.torch_dtype
    elem = 2 if cfg.dtype == "bf16" else 4

    # caller-owned buffers, allocated once
    i32 = dict(dtype=torch.int32, device=dev)
    topk_idx = torch.empty((T, k), **i32)
    topk_w = torch.empty((T, k), dtype=torch.float32, device=dev)
    disp = moe.binding.DispatchOut()
    disp.x_packed = torch.empty((S, d), dtype=tdt, device=dev)
    disp.slot_to_row = torch.empty(S, **i32)
    disp.row_to_slot = torch.empty(S, **i32)
    disp.expert_counts = torch.empty(E, **i32)
    disp.expert_offsets = torch.empty(E, **i32)
    disp.rank_counts = torch.empty(R, **i32)
    disp.rank_offsets = torch.empty(R + 1, **i32)
    y_packed = torch.zeros((S, d), dtype=tdt, device=dev)      # remote rows: "received" zeros
    out = torch.empty((T, d), dtype=tdt, device=dev)
    G = U = dy = dw = dxp = dx = None
    dW1 = dW3 = dW2 = None
    if cfg.backward:
        G = torch.zeros((S, f), dtype=tdt, device=dev)
        U = torch.zeros((S, f), dtype=tdt, device=dev) if cfg.gated else None
        dy = torch.empty((S, d), dtype=tdt, device=dev)
        dw = torch.empty((T, k), dtype=torch.float32, device=dev)
        dxp = torch.zeros((S, d), dtype=tdt, device=dev)
        dx = torch.empty((T, d), dtype=tdt, device=dev)
        mk = lambda ws: [None if w is None else torch.empty(w.shape, dtype=torch.float32, device=dev)
                         for w in ws]
        dW1, dW3, dW2 = mk(lay.W1), (mk(lay.W3) if cfg.gated else None), mk(lay.W2)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    names = ["route", "dispatch", "expert_ffn", "combine"] + \
        (["combine_bwd", "expert_ffn_bwd", "dispatch_bwd"] if cfg.backward else [])

    def step(marks=None):
        def mark(i):
            if marks is not None:
                marks[i].record()
        mark(0)
        moe.moe_route(lay.ctx, x, lay.Wg, lay.bias, topk_idx=topk_idx, topk_w=topk_w)
        mark(1)
        moe.moe_dispatch_routed(lay.ctx, x, topk_idx, out=disp)   # the routing moe_route just wrote
        mark(2)
        moe.moe_expert_ffn(lay.ctx, disp.x_packed, disp.expert_counts, disp.expert_offsets,
                           lay.W1, lay.W3, lay.W2, y_packed=y_packed, G_save=G, U_save=U)
        mark(3)
        moe.moe_combine(lay.ctx, y_packed, disp.slot_to_row, topk_w, out=out)
        mark(4)
        if cfg.backward:
            moe.moe_combine_bwd(lay.ctx, dout, y_packed, disp.slot_to_row, topk_w, dy_packed=dy,
                                dtopk_w=dw)
            mark(5)
            moe.moe_expert_ffn_bwd(lay.ctx, dy, disp.x_packed, G, U, disp.expert_counts,
                                   disp.expert_offsets, lay.W1, lay.W3, lay.W2, dx_packed=dxp,
                                   dW1=dW1, dW3=dW3, dW2=dW2)
            mark(6)
            moe.moe_dispatch_bwd(lay.ctx, dxp, disp.slot_to_row, dx=dx)
            mark(7)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps.  The only instrumentation inside it is the pair
    # of HIP events that the library records on the launch stream around the dominant kernel
    # (the gate/up GEMM): every event record leaves the GPU idle for a few microseconds.
    moe.moe_profile_ffn_launches(lay.ctx, 0b010)
    moe.moe_profile_ffn(lay.ctx, args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    up_ms, n_rec = moe.moe_profile_ffn_read(lay.ctx)
    moe.moe_profile_ffn(lay.ctx, 0)

    # ---- breakdown pass (not part of `value`): the same steps again with an event after every
    # call and around every internal launch of moe_expert_ffn
    marks = [[ev() for _ in range(len(names) + 1)] for _ in range(args.steps)]
    moe.moe_profile_ffn_launches(lay.ctx, 0b111)
    moe.moe_profile_ffn(lay.ctx, args.steps)
    for s in range(args.steps):
        step(marks[s])
    torch.cuda.synchronize()
    ffn_ms, _ = moe.moe_profile_ffn_read(lay.ctx)
    moe.moe_profile_ffn(lay.ctx, 0)
    ffn_ms[1] = up_ms[1]          # the dominant kernel's duration comes from the timed region

    if args.copy_calibration:
        src = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)          # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = wall * 1e3 / args.steps
    call_ms = {n: float(np.mean([marks[s][i].elapsed_time(marks[s][i + 1])
                                 for s in range(args.steps)])) for i, n in enumerate(names)}
    step_ms = [marks[s][0].elapsed_time(marks[s][len(names)]) for s in range(args.steps)]

    # dispatch and combine once more, back to back on the same buffers ("warm": what fits the
    # 256 MB Infinity Cache stays there; inside a step the expert GEMMs run in between and the
    # two calls find their data in HBM, which is what the roofline fractions use)
    def warm(fn, reps=10):
        fn()
        a, b_ = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b_.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b_) / reps
    warm_dispatch_ms = warm(lambda: moe.moe_dispatch_routed(lay.ctx, x, topk_idx, out=disp))
    warm_combine_ms = warm(lambda: moe.moe_combine(lay.ctx, y_packed, disp.slot_to_row, topk_w, out=out))
    n_loc = int(disp.rank_counts[cfg.local_rank].item())
    n_res = len(wl.resident_experts(cfg))

    # ---- algorithmic work ------------------------------------------------------------
    n_up = 2 if cfg.gated else 1              # matrices in the first GEMM (gate and up / W1 only)
    flops_up = 2.0 * n_up * n_loc * d * f     # first GEMM over the compute region
    flops_down = 2.0 * n_loc * d * f
    bytes_dispatch = T * d * elem + S * d * elem + S * 4 + 2 * S * 4
    bytes_combine = S * d * elem + T * d * elem + S * 8
    mfma = cfg.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if mfma else PEAK_F32_TFLOPS
    ach_up = flops_up / (ffn_ms[1] * 1e-3) / 1e12 if ffn_ms[1] > 0 else 0.0
    ach_down = flops_down / (ffn_ms[2] * 1e-3) / 1e12 if ffn_ms[2] > 0 else 0.0
    ach_ffn = (flops_up + flops_down) / (call_ms["expert_ffn"] * 1e-3) / 1e12
    gbs = lambda b, ms: b / (ms * 1e-3) / 1e9

    rec = {
        "metric": "MoE-layer tokens/s (1 GPU); grouped-GEMM % MFMA peak; dispatch % HBM BW",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={T} d_model={d} E={E} top-{k} ffn_dim={f} "
                               f"R={R} resident={n_res} experts, seed {cfg.seed}",
                   "T": T, "d_model": d, "E": E, "k": k, "ffn_dim": f, "R": R,
                   "resident_experts": n_res, "n_loc_rows": n_loc,
                   "steps_in_path": names},
        "roofline": {
            "kernel": ("ffn_mfma_kernel<0, false> (MODE_UP: gate/up grouped GEMM + SwiGLU)" if cfg.gated
                       else "ffn_mfma_kernel<4, false> (MODE_UP1: first GEMM of the two-matrix expert + ReLU)") if mfma
                      else "ffn_gate_up_kernel<float>",
            "bound": "mfma" if mfma else "alu",
            "achieved": ach_up, "peak": peak, "unit": "TFLOP/s", "frac": ach_up / peak,
            "traffic": traffic_from_profile(cfg.name, "ffn_mfma_kernel<0") if mfma and cfg.gated else None,
            "algorithmic_bytes": (n_up * n_res * d * f + n_loc * d + n_loc * f) * elem,
            "avg_launch_ms": ffn_ms[1], "flops_per_launch": flops_up, "launches": n_rec,
        },
        "grouped_gemm": {
            "gate_up_tflops": ach_up, "down_tflops": ach_down, "down_ms": ffn_ms[2],
            "schedule_ms": ffn_ms[0], "whole_call_tflops": ach_ffn,
            "frac_of_peak_gate_up": ach_up / peak, "frac_of_peak_down": ach_down / peak,
            "frac_of_peak_whole_call": ach_ffn / peak,
        },
        "hbm": {
            "dispatch_gbs": gbs(bytes_dispatch, call_ms["dispatch"]),
            "dispatch_frac": gbs(bytes_dispatch, call_ms["dispatch"]) / PEAK_HBM_GBS,
            "combine_gbs": gbs(bytes_combine, call_ms["combine"]),
            "combine_frac": gbs(bytes_combine, call_ms["combine"]) / PEAK_HBM_GBS,
            "bytes_dispatch": bytes_dispatch, "bytes_combine": bytes_combine, "peak_gbs": PEAK_HBM_GBS,
            "dispatch_warm_gbs": gbs(bytes_dispatch, warm_dispatch_ms),
            "combine_warm_gbs": gbs(bytes_combine, warm_combine_ms),
            "note": "dispatch_gbs / combine_gbs: inside a step (data in HBM); *_warm_gbs: the same "
                    "call repeated back to back (whatever fits the 256 MB Infinity Cache stays there)",
        },
        "call_ms": call_ms,
        "breakdown_step_ms": {"median": float(np.median(step_ms)), "min": float(np.min(step_ms)),
                              "max": float(np.max(step_ms)),
                              "note": "steps of the breakdown pass (an event after every call)"},
        "input_generation_s": t_gen,
    }
    if cfg.backward:
        # 12 n_loc d f for the data and weight gradients (8 for the two-matrix expert)
        flops_bwd = (2.0 * (n_up + 1) * 2) * n_loc * d * f
        t_b = call_ms["expert_ffn_bwd"] * 1e-3
        g = rec["grouped_gemm"]
        g["bwd_call_tflops"] = flops_bwd / t_b / 1e12
        g["frac_of_peak_bwd_call"] = g["bwd_call_tflops"] / peak
        g["frac_of_peak_fwd_bwd"] = ((flops_up + flops_down + flops_bwd) /
                                     (t_b + call_ms["expert_ffn"] * 1e-3) / 1e12 / peak)
    if mfma and with_ceilings and not args.no_others:
        w0 = next(w for w in lay.W1 if w is not None)
        c = measure_ceilings(n_loc, d, f, disp.x_packed, w0)
        rec["ceilings"] = c
        rec["roofline"]["frac_of_measured"] = ach_up / c["mfma_issue_varied_operands_tflops"]
        rec["roofline"]["measured_ceiling"] = ("mfma_issue_varied_operands_tflops: the bare MFMA "
                                               "issue loop on varied bf16 operands, this run")
        rec["roofline"]["vs_library_gemm"] = ach_up / c["library_gemm_tflops"]
        rec["hbm"]["dispatch_frac_of_measured_copy"] = \
            rec["hbm"]["dispatch_gbs"] / c["copy_read1_write2_gbs"]
        rec["hbm"]["combine_frac_of_measured_copy"] = \
            rec["hbm"]["combine_gbs"] / c["copy_read1_write1_gbs"]
    if mfma and not args.no_sr:
        rec["sr_compression"] = sr_compression_bench(lay.ctx, f, d)
    if cfg.backward:
        # gate backward (not one of the steps the training configuration names): timed on its
        # own after the steps, on the last step's tensors
        def gate_bwd():
            moe.moe_route_bwd(lay.ctx, x, lay.Wg, topk_idx, topk_w, dw, dx=dx)
        gate_bwd()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            gate_bwd()
        e1.record()
        torch.cuda.synchronize()
        t_rb = e0.elapsed_time(e1) / 10
        by = (2 * T * d + E * d) * elem + T * d * elem + T * E * 4 * 3 + E * d * 4
        rec["route_bwd"] = {"ms": t_rb, "algorithmic_bytes": by,
                            "gbs": by / (t_rb * 1e-3) / 1e9,
                            "note": "dlogits, dWg and dx += dlogits Wg; x read once, dx read and "
                                    "written; not part of the timed step"}
    if args.graph:
        # the same step captured once into a HIP graph (the calls launch kernels only)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for _ in range(max(args.warmup, 1)):
            graph.replay()
        e0, e1 = ev(), ev()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        t_graph = e0.elapsed_time(e1) / args.steps
        rec["graph_replay"] = {"ms_per_step": t_graph, "tokens_per_s": T / (t_graph * 1e-3),
                               "eager_ms_per_step": ms_per_step}
    if args.chunks > 0:
        # chunked overlap schedule: the same forward, cut into chunks on several streams
        pipe = moe.MoEPipeline(T_max=T, d=d, E=E, k=k, f=f, R=R, local_rank=cfg.local_rank,
                               dtype=lay.ctx.cfg.dtype, n_chunks=args.chunks,
                               n_streams=args.chunk_streams)
        pipe.set_placement(inp.dest_rank)
        pb = pipe.alloc_outputs(T, dev)
        for _ in range(max(args.warmup, 1)):
            pipe.forward(x, lay.Wg, lay.bias, lay.W1, lay.W3, lay.W2, pb)
        e0, e1 = ev(), ev()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            pipe.forward(x, lay.Wg, lay.bias, lay.W1, lay.W3, lay.W2, pb)
        e1.record()
        torch.cuda.synchronize()
        t_pipe = e0.elapsed_time(e1) / args.steps
        t_seq = sum(call_ms[n] for n in ("route", "dispatch", "expert_ffn", "combine"))
        rec["chunked_overlap"] = {"n_chunks": args.chunks, "n_streams": args.chunk_streams,
                                  "ms_per_forward": t_pipe, "unchunked_forward_ms": t_seq,
                                  "speedup": t_seq / t_pipe,
                                  "tokens_per_s": T / (t_pipe * 1e-3)}
        pipe.close()
    if not args.no_cpu_baseline:
        flops_tok = 2.0 * (n_up + 1) * d * f * k * (3 if cfg.backward else 1) + 2.0 * d * E
        sample = args.cpu_sample_tokens or int(max(16, min(cfg.T, 8e12 / flops_tok)))
        rec["cpu_baseline"] = cpu_baseline(cfg, inp, sample)
    lay.close()
    return rec


if __name__ == "__main__":
    sys.exit(main())
