#!/usr/bin/env python3
"""Benchmark of the expert-group MoE layer on one MI355X.

A step is one moe_ep_forward (gate, partition, routed gate/up + down grouped GEMM, shared
experts, aggregation, all r chunks) over one batch of synthetic input that is already
resident where the context expects it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--r R] [--order O]
                    [--variant V] [--no-cpu-baseline]
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak
RIDGE_FLOP_PER_BYTE = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)   # below it a GEMM launch is HBM-bound
STAGE_LABEL = {"routed_gate_up_gemm": "routed gate/up projection", "routed_down_gemm": "routed down projection",
               "shared_gate_up_gemm": "shared-expert gate/up projection",
               "shared_down_gemm": "shared-expert down projection"}


def kernel_name(ctx, stage):
    """The kernel the last forward launched for a projection, as rocprofv3 names its template
    arguments (read from the library: moe_ep_last_tile_shape), or None."""
    sh = ctx.last_tile_shape(stage)
    if sh is None:
        return None
    swiglu = "true" if "gate_up" in stage else "false"
    ragged = "true" if stage.startswith("routed") else "false"
    # last argument: what the epilogue writes (MOE_EP_EXPERT_OUT, the routed down projection only)
    epi = {"f": 1, "s": 2}.get(os.environ.get("MOE_EP_EXPERT_OUT", " ")[0], 0) if stage == "routed_down_gemm" else 0
    # and whether the weights are read from a tile-order copy (moe_ep_prepare_weights)
    return (f"grouped_gemm_kernel<{sh['rows']}, {sh['cols']}, {sh['k_step']}, {sh['ring_slots']}, "
            f"{sh['waves_m']}, {sh['waves_n']}, {swiglu}, {ragged}, {epi}, {'true' if sh['tile_order'] else 'false'}, "
            f"{sh['mfma_rows']}>")


def measured_traffic(workload, r_chunks, stage, kernel):
    """HBM-side bytes of one launch from the committed counter summary profiles/hbm_traffic_<workload>.txt
    (lines "traffic <r_chunks> <stage> <kernel> <read bytes> <written bytes>"): returned only when
    the kernel the library launches now is the one that was measured, else None."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split("|")
        if len(f) == 6 and f[0].strip() == "traffic" and int(f[1]) == r_chunks and f[2].strip() == stage:
            if f[3].strip() == kernel:
                return float(f[4]) + float(f[5])
    return None


def cpu_baseline(wl, inp, budget_s=15.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload's tokens."""
    import numpy as np
    import oracle
    kw = dict(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts, local_begin=wl.local_begin,
              n_local=wl.n_local, n_shared=wl.n_shared, shared_inter=wl.shared_inter,
              top_k=wl.top_k)
    cores = oracle.threads()
    n = min(wl.n_tokens, 2 * cores)
    ids = np.arange(n, dtype=np.int32)
    t0 = time.perf_counter()
    oracle.forward_tokens(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"], ids, **kw)
    dt = time.perf_counter() - t0
    total_n, total_t = n, dt
    n2 = int(min(wl.n_tokens - n, max(0, (budget_s - dt) / max(dt / n, 1e-9))))
    n2 = (n2 // cores) * cores
    if n2 > 0:
        ids = np.arange(n, n + n2, dtype=np.int32)
        t0 = time.perf_counter()
        oracle.forward_tokens(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"], ids, **kw)
        total_t += time.perf_counter() - t0
        total_n += n2
    return {"value": total_n / total_t, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"first {total_n} tokens of the workload through oracle.forward_tokens "
                      f"(fp64, plain C) in {total_t:.1f} s"}


COMPUTE_STAGES = ("router", "partition", "routed_gate_up_gemm", "routed_down_gemm", "shared_gate_up_gemm",
                  "shared_down_gemm", "aggregation")


def fit_pipeline(ctx, tokens, logits, routed, shared, out, T, k, order, stream, r_sweep=(1, 2, 4, 8)):
    """Pinned-host contexts: fit the linear task models of Sec. 4.1 (10 warm-up + 20 timed forwards per
    point, the protocol of Sec. 5.2), give them to the context, let it choose r_2, and measure the sweep.

    First set (tasks alone): forwards of ONE chunk of m tokens, where nothing overlaps; the copy times
    are the measured stage times, the compute time is the rest of the forward's wall time, so the three
    add up to what a one-chunk forward takes.  Second set (tasks beside other tasks): on one GPU the
    copies and the kernels slow each other down and kernel boundaries wait for host-bound writes, so
    isolated task times under-price a pipeline; instead the closed form S(r, m) = t_in + t_e + t_out +
    (r - 1) Y of Sec. 4.2 is fitted to forwards of 2 and of 4 chunks of m tokens each:
    S(2, m) and S(4, m) are fitted as alpha + beta m; Y(m) = (S(4, m) - S(2, m)) / 2 is the step per
    extra chunk and becomes the compute model, S(2, m) - 2 Y(m) is what the two links add and is split
    over them."""
    import torch
    import paper_2512_21487_amd as pkg

    def run(n_tokens, r, stages):
        for _ in range(10):
            ctx.forward(tokens, logits, routed, shared, k, r, order, n_tokens=n_tokens, out=out, stream=stream)
        torch.cuda.synchronize()
        if stages:
            ctx.set_profiling_stages(["copy_in", "copy_out"])
            ctx.set_profiling(20)
        t1 = time.perf_counter()
        for _ in range(20):
            ctx.forward(tokens, logits, routed, shared, k, r, order, n_tokens=n_tokens, out=out, stream=stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t1) / 20 * 1e3
        st = None
        if stages:
            st = ctx.get_stage_ms()
            ctx.set_profiling(0)
            ctx.set_profiling_stages(None)
        return wall, st

    pts = sorted({max(64, T // d) for d in (64, 32, 16, 8, 4, 2, 1)})
    alone = {n: [] for n in ("copy_in", "copy_out", "compute")}
    for m_tok in pts:
        wall, st = run(m_tok, 1, True)
        alone["copy_in"].append(st["copy_in"])
        alone["copy_out"].append(st["copy_out"])
        alone["compute"].append(max(wall - st["copy_in"] - st["copy_out"], 0.0))
    fit_a = {n: pkg.fit_linear(pts, v) for n, v in alone.items()}
    coeff = [fit_a["copy_in"][0], fit_a["copy_in"][1], fit_a["compute"][0], fit_a["compute"][1],
             fit_a["copy_out"][0], fit_a["copy_out"][1]]
    model_paper = pkg.PipelineModel(*coeff)                 # independent resources, as the paper assumes
    xs2 = [m for m in pts if 2 * m <= T] if ctx.cfg.max_chunks >= 4 else []
    xs4 = [m for m in pts if 4 * m <= T] if ctx.cfg.max_chunks >= 4 else []
    fit_b = None
    if len(xs4) >= 2:
        f2 = pkg.fit_linear(xs2, [run(2 * m, 2, False)[0] for m in xs2])       # S(2, m) = alpha + beta m
        f4 = pkg.fit_linear(xs4, [run(4 * m, 4, False)[0] for m in xs4])       # S(4, m)
        fy = (max(0.5 * (f4[0] - f2[0]), 0.0), max(0.5 * (f4[1] - f2[1]), 0.0))  # Y = (S4 - S2) / 2
        fr = (max(f2[0] - 2.0 * fy[0], 0.0), max(f2[1] - 2.0 * fy[1], 0.0))      # t_in + t_out = S2 - 2 Y
        fit_b = {"two_chunks": f2, "four_chunks": f4, "step_per_chunk": (*fy, min(f2[2], f4[2])),
                 "links_together": (*fr, min(f2[2], f4[2]))}
        coeff += [0.5 * fr[0], 0.5 * fr[1], fy[0], fy[1], 0.5 * fr[0], 0.5 * fr[1]]
    model = pkg.PipelineModel(*coeff)
    chosen = pkg.choose_chunks(model, T, ctx.cfg.max_chunks)
    r_sweep = sorted({r for r in r_sweep if r <= ctx.cfg.max_chunks} | {chosen})
    measured = {r: run(T, r, False)[0] for r in r_sweep}
    ctx.set_pipeline_model(model)
    ctx.forward(tokens, logits, routed, shared, k, 0, order, n_tokens=T, out=out, stream=stream)
    torch.cuda.synchronize()
    fmt = lambda fit: {n: {"alpha_ms": f[0], "beta_ms_per_token": f[1], "r2": f[2]} for n, f in fit.items()}
    return {
        "tokens_per_point": pts,
        "alpha_beta_r2": fmt(fit_a),
        "alpha_beta_r2_beside_other_tasks": fmt(fit_b) if fit_b else None,
        "predicted_ms": {str(r): pkg.pipeline_makespan(model, T, r) for r in r_sweep},
        "predicted_ms_independent_resources": {str(r): pkg.pipeline_makespan(model_paper, T, r) for r in r_sweep},
        "measured_ms": {str(r): measured[r] for r in r_sweep},
        "chosen_r": ctx.last_chunks(), "measured_best_r": min(measured, key=measured.get),
        "chosen_r_independent_resources": pkg.choose_chunks(model_paper, T, ctx.cfg.max_chunks),
    }


def run_repeats(args) -> int:
    """The measurement in args.repeats fresh processes, one after the other; one JSON line whose value and
    ms_per_step are the means over the processes (Sec. 5.4), with the per-process figures beside them."""
    import subprocess
    argv = [a for a in sys.argv[1:]]
    for i, a in enumerate(argv):
        if a == "--repeats":
            del argv[i:i + 2]
            break
        if a.startswith("--repeats="):
            del argv[i]
            break
    lines = []
    for rep_i in range(args.repeats):
        extra = [] if rep_i == 0 else ["--no-cpu-baseline"]   # the oracle is timed once
        p = subprocess.run([sys.executable, os.path.abspath(__file__), *argv, *extra], capture_output=True, text=True)
        if p.returncode != 0:
            sys.stderr.write(p.stderr[-4000:])
            return p.returncode
        lines.append(json.loads(p.stdout.strip().splitlines()[-1]))
    line = lines[0]
    vals = [l["value"] for l in lines]
    line["repeats"] = {"processes": len(lines), "value_each": vals, "ms_per_step_each": [l["ms_per_step"] for l in lines],
                       "grouped_gemm_pct_each": [l["grouped_gemm_pct_of_bf16_mfma_peak"] for l in lines]}
    line["value"] = sum(vals) / len(vals)
    line["ms_per_step"] = sum(l["ms_per_step"] for l in lines) / len(lines)
    pcts = [l["grouped_gemm_pct_of_bf16_mfma_peak"] for l in lines if l["grouped_gemm_pct_of_bf16_mfma_peak"] is not None]
    if pcts:
        line["grouped_gemm_pct_of_bf16_mfma_peak"] = sum(pcts) / len(pcts)
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="dsv2_eg")
    ap.add_argument("--r", type=int, default=1, help="r_chunks")
    ap.add_argument("--order", type=int, default=0, help="0 shared first, 1 interleaved")
    ap.add_argument("--variant", type=int, default=None, help="GEMM tile variant (tuning)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=1,
                    help="run the whole measurement in this many fresh processes (Sec. 5.4: throughput is the "
                         "average of 3 runs) and print one line: value = mean over the processes")
    ap.add_argument("--no-device-probe", action="store_true",
                    help="skip the register-only MFMA loop and the streaming copy that follow the timed forwards")
    ap.add_argument("--zero-operands", action="store_true",
                    help="time the same launches on all-zero tokens and weights (the routing stays): the matrix "
                         "units then switch almost nothing and the clock stays at its maximum, which separates what "
                         "the package power limit costs from what the kernels cost (a diagnostic, not a result)")
    ap.add_argument("--no-prepare-weights", action="store_true",
                    help="read the weights in the caller's row-major layout (no tile-order copy)")
    ap.add_argument("--no-stage-timing", action="store_true",
                    help="time the K steps without per-stage HIP events (stage figures are then absent)")
    ap.add_argument("--fit-pipeline", action="store_true",
                    help="pinned-host workloads: fit the linear task models of Sec. 4.1 from r=1 forwards at "
                         "several token counts, choose r_2 from them and compare with measured r sweeps")
    ap.add_argument("--layers", type=int, default=1,
                    help="steady state over several layers: after the main measurement, time this many "
                         "forwards back to back per step, each with its own copy of the weights "
                         "(Sec. 4.2: the per-layer offset of the multi-layer timeline)")
    ap.add_argument("--io", choices=["device", "pinned"], default=None,
                    help="override where the workload keeps tokens / gate scores / output")
    ap.add_argument("--graph", action="store_true",
                    help="device I/O only: after the main measurement, capture one forward in a HIP graph and "
                         "time its replays (launch gaps removed)")
    ap.add_argument("--timeline", action="store_true",
                    help="after the main measurement, record one forward with events around every stage and "
                         "add its measured schedule (stage, begin ms, end ms per chunk) to the JSON line")
    ap.add_argument("--dep", default=None, metavar="R1,R2,ATTN_US",
                    help="also run the layer as the disaggregated schedule (moe_ep_forward_dep): r_1 micro-batches of "
                         "r_2 chunks, attention stand-ins of ATTN_US microseconds, both orders, against the replay model")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="after the timed forwards, time the vendor library's plain GEMM (torch.matmul) on the two "
                         "shared-expert projection shapes with the same operands, in turn (context, not the product)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy kernel: the known-size reference "
                         "that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build drives one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if args.variant is not None:
        os.environ["MOE_EP_GEMM_VARIANT"] = str(args.variant)
    if args.repeats > 1:
        return run_repeats(args)

    import numpy as np
    import torch

    import paper_2512_21487_amd as pkg
    from workloads import CONFIGS, make_inputs

    wl = CONFIGS[args.workload]
    torch.cuda.set_device(0)
    inp = make_inputs(wl)
    T, M, H, k = wl.n_tokens, wl.hidden, wl.inter, wl.top_k
    pinned = wl.pinned_io if args.io is None else args.io == "pinned"

    def put(a, host=False):
        a = a.view(np.int16) if a.dtype == np.uint16 else a
        t = torch.from_numpy(np.ascontiguousarray(a))
        if host:
            p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
            p.copy_(t)
            return p
        return t.cuda()

    tokens, logits = put(inp["tokens"], pinned), put(inp["gate_logits"], pinned)
    routed = put(inp["routed_w"])
    shared = put(inp["shared_w"]) if inp["shared_w"] is not None else None
    if args.zero_operands:
        tokens.zero_()
        routed.zero_()
        if shared is not None:
            shared.zero_()
    if pinned:
        out = torch.zeros((T, M), dtype=torch.int16, pin_memory=True)
    else:
        out = torch.zeros((T, M), dtype=torch.int16, device="cuda")
    dep = None
    if args.dep:
        f = args.dep.split(",")
        dep = (int(f[0]), int(f[1]), float(f[2]))
    dep_chunks = dep[0] * dep[1] if dep else 1
    ctx = pkg.MoeEp(hidden=M, inter=H, n_experts=wl.n_experts, local_begin=wl.local_begin,
                    n_local=wl.n_local, n_shared=wl.n_shared, shared_inter=wl.shared_inter,
                    max_tokens=T, max_top_k=k, max_chunks=max(args.r, 8 if pinned else 1, dep_chunks),
                    io_mode=pkg.IO_PINNED_HOST if pinned else pkg.IO_DEVICE)
    stream = torch.cuda.current_stream().cuda_stream
    # The weights of an expert do not change between calls: they are laid out in tile order once, before
    # any timed forward, in memory the context owns (moe_ep_prepare_weights; its time is reported apart).
    weights = {"layout": "caller's row-major"}
    if not args.no_prepare_weights:
        torch.cuda.synchronize()
        t_p = time.perf_counter()
        ctx.prepare_weights(routed, shared, stream=stream)
        torch.cuda.synchronize()
        weights = {"layout": "tile order (moe_ep_prepare_weights, once, outside the timed region)",
                   "prepare_ms": round((time.perf_counter() - t_p) * 1e3, 3),
                   "copy_bytes": ctx.prepared_weight_bytes(True, shared is not None)}

    def step():
        ctx.forward(tokens, logits, routed, shared, k, args.r, args.order, n_tokens=T, out=out,
                    stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Timed region: HIP events (on the stream the kernel runs on) bracket only the dominant kernel,
    # the routed gate/up projection, whose duration the roofline object needs; events between all
    # stages would cost 2 % of a dsv2_eg forward and 20 % of a 256-token one.
    # The kernel with the largest share of the forward: the shared experts' gate/up projection when
    # the workload has shared experts (42 % of a dsv2_eg forward), else the routed one.  The routed
    # gate/up projection is timed too: it carries the metric's "grouped GEMM % of peak".
    dominant = "shared_gate_up_gemm" if wl.n_shared > 0 else "routed_gate_up_gemm"
    timed_stages = sorted({dominant, "routed_gate_up_gemm", "routed_down_gemm"})
    if not args.no_stage_timing:
        ctx.set_profiling_stages(timed_stages + ["forward"])   # + one event pair around every forward
        ctx.set_profiling(min(args.steps, 256))   # the library keeps events of at most 256 forwards
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    t_enq = time.perf_counter() - t0       # host time spent enqueueing (the calls do not block)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if args.no_stage_timing:
        stages = {n: 0.0 for n in pkg.STAGES}
    else:
        # device time of each of the K forwards (Sec. 5.2 reports the timed trials of a point by one figure)
        per_forward_ms = [e - b for n, _, b, e in ctx.get_timeline() if n == "forward"]
        in_region = ctx.get_stage_ms()
        # Second pass, outside the timed region: the same forwards with events around every stage
        # (the per-stage breakdown; its "forward" is a little longer than ms_per_step for that reason).
        ctx.set_profiling_stages(None)
        ctx.set_profiling(min(args.steps, 256))   # the library keeps events of at most 256 forwards
        for _ in range(args.steps):
            step()
        stages = ctx.get_stage_ms()
        ctx.set_profiling(0)
        second_pass = {n: stages[n] for n in timed_stages}
        for n in timed_stages:
            stages[n] = in_region[n]

    routing = [ctx.get_routing(c) for c in range(args.r)]
    kept = sum(int(rt["offset"][-1]) for rt in routing)
    tokens_with_kept = sum(int((rt["pos"] >= 0).any(axis=1).sum()) for rt in routing)
    load = np.sum([rt["count"] for rt in routing], axis=0)   # realised rows per local expert
    ms_per_step = dt / args.steps * 1e3
    value = T * args.steps / dt

    def gemm_line(flop, nbytes, ms):
        """One projection: against the matrix peak, or, when its algorithmic flops per algorithmic byte
        (weights streamed once + activations in and out) lie below the ridge, against the HBM peak."""
        if ms <= 0:
            return None
        tf, gbs = flop / (ms * 1e-3) / 1e12, nbytes / (ms * 1e-3) / 1e9
        if flop / max(nbytes, 1.0) < RIDGE_FLOP_PER_BYTE:
            return {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                    "ms_per_step": ms, "tflops": tf, "flop_per_byte": flop / nbytes}
        return {"bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / PEAK_BF16_TFLOPS, "ms_per_step": ms, "flop_per_byte": flop / nbytes}

    def hbm_line(nbytes, ms):
        if ms <= 0:
            return None
        ach = nbytes / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "ms_per_step": ms}

    Ns, Hs = wl.n_shared, wl.shared_inter
    # algorithmic bytes of a projection launch: every chunk streams the weights of all local (or shared)
    # experts once, reads its input rows and writes its output rows (bf16)
    r = args.r
    kernels = {
        "routed_gate_up_gemm": gemm_line(4.0 * kept * M * H, r * wl.n_local * 4.0 * H * M + kept * 2.0 * (M + H),
                                         stages["routed_gate_up_gemm"]),
        "routed_down_gemm": gemm_line(2.0 * kept * M * H, r * wl.n_local * 2.0 * H * M + kept * 2.0 * (M + H),
                                      stages["routed_down_gemm"]),
        "shared_gate_up_gemm": gemm_line(4.0 * T * Ns * M * Hs, Ns * 4.0 * Hs * M + T * 2.0 * (M + Ns * Hs),
                                         stages["shared_gate_up_gemm"]),
        "shared_down_gemm": gemm_line(2.0 * T * Ns * M * Hs, Ns * 2.0 * Hs * M + T * 2.0 * (M + Ns * Hs),
                                      stages["shared_down_gemm"]),
        # partition: the routing arrays (masks, offsets, positions, row map); the token rows are
        # gathered by the gate/up projection's own tile loads unless MOE_EP_FUSED_GATHER=0, in which
        # case a grouped copy adds 2M bytes read + 2M written per kept row
        "partition": hbm_line((kept * 4.0 * M if os.environ.get("MOE_EP_FUSED_GATHER") == "0" else 0.0)
                              + T * k * 16.0, stages["partition"]),
        # aggregation: per kept row 2M bytes read; without shared experts every output row is written
        # (2M), with them only the rows of tokens that kept a slot are read and rewritten (4M)
        "aggregation": hbm_line(kept * 2.0 * M + (tokens_with_kept * 4.0 * M if Ns else T * 2.0 * M),
                                stages["aggregation"]),
        "router": hbm_line(T * (4.0 * wl.n_experts + 8.0 * k), stages["router"]),
    }
    routed_ms = stages["routed_gate_up_gemm"] + stages["routed_down_gemm"]
    routed_pct = 100.0 * 6.0 * kept * M * H / (routed_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS if routed_ms > 0 else None
    roof = dict(kernels[dominant] or {})
    roof.pop("ms_per_step", None)
    names = {st: kernel_name(ctx, st) for st in STAGE_LABEL}
    # HBM-side bytes of one launch of that kernel, from the committed counter summary, if it is of this kernel
    roof["traffic"] = measured_traffic(wl.name, args.r, dominant, names[dominant])
    roof["kernel"] = f"{names[dominant]} ({STAGE_LABEL[dominant]})"
    roof["launches_per_step"] = args.r if dominant.startswith("routed") or args.order == 1 else 1
    for st, line_ in kernels.items():
        if line_ is not None and st in names:
            line_["kernel"] = names[st]

    line = {
        "metric": "expert-layer tokens/sec at 1 GPU; grouped-GEMM % of bf16 MFMA peak",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic" if not args.zero_operands else "all-zero tokens and weights (power diagnostic, not a result)",
        "config": {"workload": f"{wl.name}: T={T} M={M} H={H} E={wl.n_experts} local={wl.n_local} "
                               f"top_k={k} shared={Ns}x{Hs} io={'pinned_host' if pinned else 'device'}",
                   "r_chunks": args.r, "order": args.order, "weights": weights, "kept_assignments": kept,
                   "expert_load": {"max": int(load.max()), "mean": float(load.mean()), "min": int(load.min()),
                                   "empty": int((load == 0).sum())}},
        "grouped_gemm_pct_of_bf16_mfma_peak": routed_pct,
        "roofline": roof,
        "kernels": kernels,
        "stage_ms": stages,
        "stage_ms_note": (", ".join(timed_stages) + ": HIP events inside the timed region; other stages: a "
                          "second pass of the same forwards with events around every stage"
                          + ("" if args.no_stage_timing else
                             " (there: " + ", ".join(f"{n} {second_pass[n]:.4f}" for n in timed_stages) + " ms)")),
        "host_enqueue_ms_per_step": t_enq / args.steps * 1e3,
    }
    if not args.no_stage_timing and per_forward_ms:
        med = float(np.median(per_forward_ms))
        line["ms_per_step_median"] = med                   # median device time of one forward over the K steps
        line["value_at_median"] = T / (med * 1e-3)
    if pinned:
        # Chunk pipeline against the closed form of Sec. 4.2 (layer 0, one slice): three resources
        # (inbound link, expert compute, outbound link), r chunks, steady-state step = the slowest
        # resource: makespan = t_in + t_e + t_out + (r - 1) * max(t_in, t_e, t_out).  The paper
        # takes t_in = t_out = t_a2e; here the inbound copy also carries the gate scores.
        r = args.r
        t_in, t_out = stages["copy_in"] / r, stages["copy_out"] / r
        t_e = sum(stages[n] for n in ("router", "partition", "routed_gate_up_gemm", "routed_down_gemm",
                                      "shared_gate_up_gemm", "shared_down_gemm", "aggregation")) / r
        line["pipeline"] = {
            "t_in_ms_per_chunk": t_in, "t_e_ms_per_chunk": t_e, "t_out_ms_per_chunk": t_out,
            "closed_form_ms": t_in + t_e + t_out + (r - 1) * max(t_in, t_e, t_out),
            "measured_ms": stages["forward"],
            "bytes_in_per_chunk": (T // r) * (2 * M + 4 * wl.n_experts), "bytes_out_per_chunk": (T // r) * 2 * M,
        }
    if pinned and args.fit_pipeline:
        line["pipeline_fit"] = fit_pipeline(ctx, tokens, logits, routed, shared, out, T, k, args.order, stream)
    if args.graph and not pinned:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            ctx.forward(tokens, logits, routed, shared, k, args.r, args.order, n_tokens=T, out=out,
                        stream=torch.cuda.current_stream().cuda_stream)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t1) / args.steps * 1e3
        line["graph_replay"] = {"ms_per_step": g_ms, "tokens_per_s": T / (g_ms * 1e-3), "eager_ms_per_step": ms_per_step}
    if args.timeline:
        ctx.set_profiling_stages(None)
        ctx.set_profiling(1)
        step()
        line["timeline"] = [{"stage": n, "begin_ms": round(b, 4), "end_ms": round(e, 4)}
                            for n, _, b, e in ctx.get_timeline() if n != "forward"]
        ctx.get_stage_ms()
        ctx.set_profiling(0)
    if dep:
        # Sec. 2.3 on one GPU: measured makespan of both attention-group orders, the task durations the
        # timeline shows, and what the earliest-start replay of Eq. limitation predicts from them
        r_1, r_2, attn_us = dep
        res = {"r_1": r_1, "r_2": r_2, "attn_us": attn_us, "io": "pinned" if pinned else "device",
               "measured_ms": {}, "model_ms": {}, "bounds_ms": {}, "tasks_ms": {}}
        # durations of the shared-expert and expert tasks running alone: one micro-batch through the
        # plain forward (shared experts first, then its r_2 chunks one after the other)
        T_mb = -(-T // r_1)
        ctx.set_profiling_stages(None)
        for _ in range(3):
            ctx.forward(tokens, logits, routed, shared, k, r_2, 0, n_tokens=T_mb, out=out, stream=stream)
        ctx.set_profiling(10)
        for _ in range(10):
            ctx.forward(tokens, logits, routed, shared, k, r_2, 0, n_tokens=T_mb, out=out, stream=stream)
        st_mb = ctx.get_stage_ms()
        ctx.set_profiling(0)
        alone_ms = {"shared": st_mb["shared_gate_up_gemm"] + st_mb["shared_down_gemm"],
                    "experts_per_chunk": sum(st_mb[n] for n in ("router", "partition", "routed_gate_up_gemm",
                                                                 "routed_down_gemm", "aggregation")) / r_2}
        res["tasks_alone_ms"] = alone_ms
        for name, order in (("ASAS", 0), ("AASS", 1)):
            def dep_step():
                ctx.forward_dep(tokens, logits, routed, shared, k, r_1, r_2, order, attn_us, n_tokens=T, out=out,
                                stream=stream)
            for _ in range(3):
                dep_step()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                dep_step()
            torch.cuda.synchronize()
            res["measured_ms"][name] = (time.perf_counter() - t1) / args.steps * 1e3
            ctx.set_profiling_stages(None)
            ctx.set_profiling(1)
            dep_step()
            by = {}
            for n, _, b, e in ctx.get_timeline():
                by.setdefault(n, []).append((b, e))
            ctx.get_stage_ms()
            ctx.set_profiling(0)
            mean = lambda xs: float(np.mean(xs)) if len(xs) else 0.0
            t_a = mean([e - b for b, e in by.get("attention", [])])
            t_s = mean([e2 - b1 for (b1, _), (_, e2) in zip(by.get("shared_gate_up_gemm", []), by.get("shared_down_gemm", []))])
            t_e = mean([e2 - b1 for (b1, _), (_, e2) in zip(by["router"], by["routed_down_gemm"])]) + \
                mean([e - b for b, e in by["aggregation"]])
            t_c = mean([e - b for b, e in by.get("copy_in", []) + by.get("copy_out", [])])
            res["tasks_ms"][name] = {"attention": t_a, "shared": t_s, "experts_per_chunk": t_e, "link_per_chunk": t_c}
            mod = pkg.DepModels(t_a, 0.0, t_s, 0.0, t_e, 0.0, t_c, 0.0)
            prob = pkg.DepProblem(ag=1, n_experts=wl.n_experts, top_k=k, seq_len=1, n_layers=1)
            res["model_ms"][name] = pkg.dep_replay(mod, prob, 1, r_1, r_2, order)[0]
            # the same rules plus "shared experts and experts share the compute units", fed with what
            # the tasks take alone (a plain forward over one micro-batch, chunk by chunk)
            # two-sided: the replay fed with what the tasks take alone is a lower bound when the groups are
            # taken as independent (the paper's case) and an upper bound under the extra rule "shared
            # experts and experts share the compute units and never overlap" (moe_ep_dep_replay_one_gpu);
            # on one GPU they do overlap, each slower, and the measured makespan lies between the two
            alone = pkg.DepModels(t_a, 0.0, alone_ms["shared"], 0.0, alone_ms["experts_per_chunk"], 0.0, t_c, 0.0)
            res["bounds_ms"][name] = {"independent_groups": pkg.dep_replay(alone, prob, 1, r_1, r_2, order)[0],
                                      "one_gpu_no_overlap": pkg.dep_replay(alone, prob, 1, r_1, r_2, order, one_gpu=True)[0]}
        line["dep_layer"] = res
    if args.layers > 1:
        # layer l > 0 uses a rolled copy of layer 0's weights: distinct memory, same distribution, so no
        # layer finds its weights in a cache the previous one filled
        L = args.layers
        routed_l = [routed] + [torch.roll(routed, 4099 * l) for l in range(1, L)]
        shared_l = [shared] + [None if shared is None else torch.roll(shared, 4099 * l) for l in range(1, L)]
        if not args.no_prepare_weights:
            for l in range(1, L):
                ctx.prepare_weights(routed_l[l], shared_l[l], stream=stream)

        def layer_step():
            for l in range(L):
                ctx.forward(tokens, logits, routed_l[l], shared_l[l], k, args.r, args.order, n_tokens=T, out=out,
                            stream=stream)
        for _ in range(3):
            layer_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            layer_step()
        torch.cuda.synchronize()
        per_layer_ms = (time.perf_counter() - t1) / (args.steps * L) * 1e3
        # the schedule model's per-layer term max(G, r_1 F) (Sec. 4.2), fed with this run's task times; it
        # assumes shared experts, links and routed experts on hardware of their own, here they share one GPU
        rr = args.r
        t_s = stages["shared_gate_up_gemm"] + stages["shared_down_gemm"]
        t_e = sum(stages[n] for n in ("router", "partition", "routed_gate_up_gemm", "routed_down_gemm", "aggregation")) / rr
        t_c = 0.5 * (stages["copy_in"] + stages["copy_out"]) / rr
        mod = pkg.DepModels(0.0, 0.0, t_s, 0.0, t_e, 0.0, t_c, 0.0)
        span = lambda n: pkg.dep_makespan(mod, pkg.DepProblem(ag=1, n_experts=wl.n_experts, top_k=k, seq_len=1,
                                                              n_layers=n), 1, 1, rr)
        line["multi_layer"] = {"layers": L, "ms_per_layer": per_layer_ms, "tokens_per_s": T / (per_layer_ms * 1e-3),
                               "single_layer_ms": ms_per_step,
                               "model_ms_per_layer": (span(L) - span(1)) / (L - 1),
                               "model_tasks_ms": {"shared": t_s, "experts_per_chunk": t_e, "link_per_chunk": t_c}}
    if not args.no_device_probe:
        # what this machine sustains, measured right after the timed forwards (outside the timed region):
        # a register-only MFMA loop on random bf16 operands and a streaming copy; the vendor peaks in
        # "roofline" assume the maximum clock, which the power limit does not grant real operands
        probe = pkg.probe_device(0)
        line["device_probe"] = {"mfma_tflops_random_operands": probe["mfma_tflops"], "mfma_ghz": probe["mfma_ghz"],
                                "copy_gbs_read_plus_write": probe["copy_gbs"]}
        if roof.get("bound") == "mfma" and probe["mfma_tflops"] > 0:
            line["roofline"]["frac_of_measured_ceiling"] = roof["achieved"] / probe["mfma_tflops"]
        if roof.get("bound") == "hbm" and probe["copy_gbs"] > 0:
            line["roofline"]["frac_of_measured_ceiling"] = roof["achieved"] / probe["copy_gbs"]
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, inp)
    if args.vendor_gemm and wl.n_shared > 0 and not pinned:
        # Context: the vendor library's GEMM on the shapes of the two shared-expert launches, same token rows and
        # weights, the two in turn as a forward runs them (no SwiGLU: its gate/up result is twice as wide).
        Hs, Ns = wl.shared_inter, wl.n_shared
        sw = shared.view(torch.bfloat16).reshape(Ns, 3 * Hs * M)
        w_gu = torch.cat([sw[i, :2 * Hs * M].reshape(2 * Hs, M) for i in range(Ns)], 0).contiguous()
        w_d = torch.cat([sw[i, 2 * Hs * M:].reshape(M, Hs) for i in range(Ns)], 1).contiguous()
        x = tokens.view(torch.bfloat16)
        act = (0.5 * torch.randn(T, Ns * Hs, device="cuda")).to(torch.bfloat16)
        n_pairs = 40
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(3 * n_pairs)]
        for i in range(n_pairs):
            evs[3 * i].record()
            _ = x @ w_gu.t()
            evs[3 * i + 1].record()
            _ = act @ w_d.t()
            evs[3 * i + 2].record()
        torch.cuda.synchronize()
        tail = range(n_pairs // 4, n_pairs)
        g_ms = sum(evs[3 * i].elapsed_time(evs[3 * i + 1]) for i in tail) / len(tail)
        d_ms = sum(evs[3 * i + 1].elapsed_time(evs[3 * i + 2]) for i in tail) / len(tail)
        line["vendor_gemm"] = {"what": "torch.matmul (hipBLASLt) on the shared-expert shapes, same operands, in turn",
                               "gate_up_ms": g_ms, "gate_up_tflops": 4.0 * T * M * Ns * Hs / (g_ms * 1e-3) / 1e12,
                               "down_ms": d_ms, "down_tflops": 2.0 * T * M * Ns * Hs / (d_ms * 1e-3) / 1e12,
                               "library_gate_up_ms": stages["shared_gate_up_gemm"],
                               "library_down_ms": stages["shared_down_gemm"]}
    if args.copy_probe:
        src = torch.ones(1 << 29, dtype=torch.int16, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
    ctx.destroy()
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
