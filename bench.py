#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X: `python bench.py [--gpus 1] [--steps K] [--warmup W]`.

One step = one pass of the whole path (gate logits -> top-k + slots -> encode -> expert FFN -> decode) over one batch
of seeded synthetic input that is already resident in HBM.  The bench line is the largest of the five workloads
(T=131072, M=4096, H=1024, E=128, top-8; `--config N` picks another).  Prints one JSON line:
  value      layer forward tokens/s (T / mean step time)
  roofline   the dominant kernel (grouped bf16 MFMA GEMM of the expert FFN): algorithmic FLOP per launch divided by
             its mean launch time, measured with HIP events recorded on the library's stream inside the timed loop
             (on every fifth timed step: the event records themselves cost stream time); `traffic` is read from the
             rocprofv3 counter summary of the same workload under profiles/ (null where none is recorded)
  stages     per-stage mean milliseconds and, for encode/decode, algorithmic HBM GB/s
  cpu_baseline  the CPU oracle timed on this machine's host cores on a bounded sample of the same workload
  fused_dispatch  the same step through moe_layer_forward_fused (the first expert GEMM gathers its rows from the tokens,
             no dispatch buffer), timed in a second loop of the same length; information only, `value` is the plain path
  other_workloads  the other four workloads measured the same way in the same run (not bench lines)
  hip_graph_ms_per_step  (workloads under 2 ms per step) the same step replayed from a captured HIP graph; information only
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VECTOR_PEAK_TFLOPS = 157.3
HEADLINE_CONFIG = 4


def to_device(a, dtype_code):
    import torch
    from paper_2206_03382_amd import synth
    if a is None:
        return None
    if dtype_code == synth.DT_BF16:
        return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def recorded_gemm_traffic(workload: str):
    """HBM bytes per grouped-GEMM launch from the rocprofv3 --pmc summary of this workload under profiles/, or None."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"^gemm_traffic_bytes_per_launch:\s*(\d+)", open(path).read(), flags=re.M)
    return int(m.group(1)) if m else None


def workload_name(cfg, C):
    return (f"{cfg.name}: T={cfg.T} M={cfg.M} H={cfg.H} E={cfg.E} top-{cfg.k} f={cfg.f} C={C} "
            f"act={('relu', 'gelu', 'silu')[cfg.act]}")


def measure(cfg, inp, steps: int, warmup: int, cold: bool = True):
    """Times `steps` passes of moe_layer_forward (and of the fused-dispatch variant) on one workload."""
    import torch
    from paper_2206_03382_amd import moe, synth

    d = cfg.dtype
    x = to_device(inp["x"], d)
    gate_bias = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).cuda()
    layer = moe.MoELayer(to_device(inp["Wg"], d), gate_bias, to_device(inp["W1"], d), to_device(inp["b1"], d),
                         to_device(inp["W2"], d), to_device(inp["b2"], d), T=cfg.T, k=cfg.k, f=cfg.f,
                         normalize=cfg.normalize, act=cfg.act, keep_routing=True)
    # Stage events are recorded on every `stride`-th timed step only: each of the seven records costs a few microseconds
    # of stream time, and the steps in between run exactly as a caller without instrumentation would run them.
    stride = 5 if steps >= 10 else 1
    sampled = [i for i in range(steps) if i % stride == 0]
    events = {i: moe.StageEvents() for i in sampled}

    for _ in range(warmup):
        layer.forward(x)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        layer.forward(x, events.get(i))
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    per_step = np.array([events[i].stage_ms() for i in sampled])     # [sampled steps, stages] from the library's own events
    stage_ms = np.mean(per_step, axis=0)

    for _ in range(warmup):
        layer.forward(x, fuse_dispatch=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        layer.forward(x, events.get(i), fuse_dispatch=True)
    torch.cuda.synchronize()
    fused_ms = (time.perf_counter() - t0) * 1e3 / steps
    fused_stage_ms = np.mean(np.array([events[i].stage_ms() for i in sampled]), axis=0)
    for e in events.values():
        e.close()

    # launch-bound workloads: the same step replayed from a HIP graph (the layer call allocates nothing, clears nothing by
    # memset and never synchronises, so it is captured as it stands); the eager figure above stays the reported one
    graph_ms = None
    if ms_per_step < 2.0:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            layer.forward(x)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
        del graph

    counts = layer.routing["counts"].cpu().numpy().astype(np.int64)
    C, T, M, H, E, k = layer.C, cfg.T, cfg.M, cfg.H, cfg.E, cfg.k
    es = 4 if d == synth.DT_F32 else 2
    R = int(np.minimum(counts, C).sum())                         # filled slots = kept (token, choice) pairs
    flop_per_gemm = 2.0 * R * M * H                              # GEMM1 [R,M]x[M,H] and GEMM2 [R,H]x[H,M]: same count
    gemm_ms = float(stage_ms[3] + stage_ms[4]) / 2.0
    bf16 = d == synth.DT_BF16
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else FP32_VECTOR_PEAK_TFLOPS
    achieved = flop_per_gemm / (gemm_ms * 1e-3) / 1e12
    # encode inside the layer: a token feeding several slots is read once and written to each (k >= 2); with one choice per
    # token the slots gather their rows (one read per slot); unfilled slots are left alone either way
    live_tokens = int((layer.routing["loc"] < C).any(dim=1).sum().item())
    enc_bytes = ((live_tokens if k >= 2 else R) + R) * M * es + 8 * T * k
    dec_bytes = (R + T) * M * es + 12 * T * k                    # read each kept expert-output row once, write [T,M]
    logit_bytes = T * M * es + M * E * es + 4 * T * E            # read every token row once, write the logits
    topk_bytes = 4 * T * E + 12 * T * k + 4 * E + 4 * E * C
    stages = {name: round(float(ms), 5) for name, ms in zip(moe.STAGE_NAMES, stage_ms)}
    stages["gate_logits_frac_hbm"] = round(logit_bytes / (stage_ms[0] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    stages["gate_topk_frac_hbm"] = round(topk_bytes / (stage_ms[1] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    stages["encode_GBps"] = round(enc_bytes / (stage_ms[2] * 1e-3) / 1e9, 1)
    stages["decode_GBps"] = round(dec_bytes / (stage_ms[5] * 1e-3) / 1e9, 1)
    stages["encode_frac_hbm"] = round(stages["encode_GBps"] / HBM_PEAK_GBS, 4)
    stages["decode_frac_hbm"] = round(stages["decode_GBps"] / HBM_PEAK_GBS, 4)
    stages["ffn_gemm1_TFLOPs"] = round(flop_per_gemm / (stage_ms[3] * 1e-3) / 1e12, 1)
    stages["ffn_gemm2_TFLOPs"] = round(flop_per_gemm / (stage_ms[4] * 1e-3) / 1e12, 1)

    # layer roofline: the stages run back to back on one stream, so their bounds add (HBM 8 TB/s for the data-movement
    # stages, 2.5 PFLOP/s for the two GEMMs); algorithmic bytes and flop only
    t_roof_ms = ((logit_bytes + topk_bytes + enc_bytes + dec_bytes) / (HBM_PEAK_GBS * 1e9) + 2 * flop_per_gemm / (peak * 1e12)) * 1e3
    step_from_events = per_step.sum(axis=1)

    # cold-cache variant: three separate sets of inputs, weights and workspaces used in rotation, so that no step finds
    # its operands in the 256 MB memory-side cache (the default loop reuses one set; caches are not flushed between steps)
    cold_ms = None
    if cold and E * (M * H * 2) * es + T * M * es < (2 << 30):
        sets = [(layer, x)]
        for _ in range(2):
            l2 = moe.MoELayer(layer.Wg.clone(), None if layer.gate_bias is None else layer.gate_bias.clone(), layer.W1.clone(),
                              None if layer.b1 is None else layer.b1.clone(), layer.W2.clone(),
                              None if layer.b2 is None else layer.b2.clone(), T=T, k=k, f=cfg.f, normalize=cfg.normalize,
                              act=cfg.act, keep_routing=False)
            sets.append((l2, x.clone()))
        for i in range(6):
            sets[i % 3][0].forward(sets[i % 3][1])
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for i in range(steps):
            sets[i % 3][0].forward(sets[i % 3][1])
        torch.cuda.synchronize()
        cold_ms = (time.perf_counter() - c0) * 1e3 / steps
        del sets

    res = {
        "workload": workload_name(cfg, C), "filled_slots": R, "slots": E * C,
        "ms_per_step": round(ms_per_step, 5), "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "roofline": {"bound": "mfma" if bf16 else "alu", "kernel": "grouped_gemm_mfma_kernel" if bf16 else "gemm_generic_kernel",
                     "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "flop_per_launch": flop_per_gemm, "avg_launch_ms": round(gemm_ms, 5),
                     "traffic": recorded_gemm_traffic(cfg.name)},
        "stages": stages,
        "layer_roofline": {"t_roofline_ms": round(t_roof_ms, 5), "frac": round(t_roof_ms / ms_per_step, 4),
                           "step_ms_median": round(float(np.median(step_from_events)), 5),
                           "step_ms_min": round(float(step_from_events.min()), 5),
                           "cold_cache_ms_per_step": None if cold_ms is None else round(cold_ms, 5),
                           "instrumented_steps": len(sampled)},
        "hip_graph_ms_per_step": None if graph_ms is None else round(graph_ms, 5),
        "fused_dispatch": {"ms_per_step": round(fused_ms, 5), "value": round(T / (fused_ms * 1e-3), 1), "unit": "tokens/s",
                           "stages": {name: round(float(ms), 5) for name, ms in zip(moe.STAGE_NAMES, fused_stage_ms)}},
    }
    return res, layer, x


def cpu_baseline(cfg, inp, budget_s: float = 12.0):
    """The oracle as it stands on this machine's host cores.  Workloads the oracle finishes in seconds run whole (repeated for
    about 10 s); the large ones run the gate and the routing in full and the expert-by-expert tier (dispatch, FFN,
    combine of one expert at a time) on the first experts until the budget is spent, scaled to all experts."""
    from oracle import moe_oracle as O
    from threadpoolctl import threadpool_info
    blas = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
    threads = max(blas) if blas else (os.cpu_count() or 1)     # the oracle's time is in numpy's BLAS matmuls
    T, E = cfg.T, cfg.E
    C = O.capacity(T, E, cfg.k, cfg.f)
    if 4.0 * min(T * cfg.k, E * C) * cfg.M * cfg.H < 2e12:       # a few seconds of fp64 BLAS per pass
        reps, c0 = 0, time.perf_counter()
        while reps == 0 or time.perf_counter() - c0 < 10.0:
            O.moe_layer(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                        cfg.k, cfg.f, cfg.normalize, cfg.act, tier="sparse")
            reps += 1
        cpu_s = time.perf_counter() - c0
        return {"value": round(T * reps / cpu_s, 1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
                "sample": f"the full workload {reps} times (all {T} tokens each, fp64 numpy, zero-skipping tier), {cpu_s:.1f} s"}
    c0 = time.perf_counter()
    logits = O.gate_logits(inp["x"], inp["Wg"], inp["gate_bias"])
    r = O.route(logits, cfg.k, C, cfg.normalize)
    gate_s = time.perf_counter() - c0
    out = np.zeros((T, cfg.M), dtype=np.float64)
    rows_done, experts_done, c1 = 0, 0, time.perf_counter()
    for e, tokens, w, Ze, Ye in O.expert_slabs(inp["x"], r["idx"], r["loc"], r["gate_w"], C, inp["W1"], inp["b1"], inp["W2"],
                                               inp["b2"], cfg.act):
        out[tokens] += w[:, None] * Ye
        rows_done += len(tokens)
        experts_done += 1
        if time.perf_counter() - c1 > budget_s:
            break
    expert_s = time.perf_counter() - c1
    rows_all = int(np.minimum(r["counts"], C).sum())
    est = gate_s + expert_s * rows_all / max(rows_done, 1)
    return {"value": round(T / est, 1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"gate logits and routing of all {T} tokens in full ({gate_s:.1f} s); dispatch, expert FFN and combine of the "
                      f"first {experts_done} of {E} experts ({rows_done} of {rows_all} filled slots, {expert_s:.1f} s, expert-by-expert "
                      f"tier, fp64 numpy) scaled to all filled slots: estimated {est:.0f} s per pass"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=HEADLINE_CONFIG,
                    help="index into the five workloads (default 4: T=131072, M=4096, H=1024, E=128, top-8, the largest)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the other four workloads (`other_workloads`)")
    ap.add_argument("--no-probe", action="store_true", help="skip the register-only MFMA probe (`mfma_only_sustained_TFLOPs`)")
    ap.add_argument("--backward", action="store_true",
                    help="also time the backward of encode and decode (moe_encode_backward, moe_decode_backward) on this "
                         "workload's routing and report their HBM GB/s as `backward_dispatch`")
    ap.add_argument("--bpr", action="store_true",
                    help="also time top-k + slot assignment with batch prioritized routing (moe_gate_topk_bpr) on this workload")
    ap.add_argument("--cosine", action="store_true",
                    help="also time the cosine router's logits (moe_gate_logits_cosine, D = 256) on this workload's tokens")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 256 MiB device copies first, so that a rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of "
                         "this command can be scaled by what the same counter reads for a copy of known size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU hot path only: run it with --gpus 1 "
              "(this build has no cross-GPU all-to-all: the experts' exchange is not part of it).", file=sys.stderr)
        return 2

    import torch
    from paper_2206_03382_amd import moe, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    moe.lib()
    cfg = synth.CONFIGS[args.config]
    inp = synth.make_inputs(cfg, seed=0)
    d = cfg.dtype
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    res, layer, x = measure(cfg, inp, args.steps, args.warmup)
    C, T, M, H, E, k = layer.C, cfg.T, cfg.M, cfg.H, cfg.E, cfg.k
    es = 4 if d == synth.DT_F32 else 2
    R = res["filled_slots"]
    flop_per_gemm = res["roofline"]["flop_per_launch"]
    bf16 = d == synth.DT_BF16
    stages = res["stages"]

    # an achievable streaming ceiling on this machine: a plain device copy of 256 MiB (read + write)
    csrc = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    cdst = torch.empty_like(csrc)
    for _ in range(3):
        cdst.copy_(csrc)
    ca, cb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ca.record()
    for _ in range(10):
        cdst.copy_(csrc)
    cb.record()
    torch.cuda.synchronize()
    copy_GBps = 2 * (256 << 20) * 10 / (ca.elapsed_time(cb) * 1e-3) / 1e9
    del csrc, cdst
    stages["copy_ceiling_GBps"] = round(copy_GBps, 1)
    stages["encode_frac_copy_ceiling"] = round(stages["encode_GBps"] / copy_GBps, 4)
    stages["decode_frac_copy_ceiling"] = round(stages["decode_GBps"] / copy_GBps, 4)
    res["layer_roofline"]["note"] = ("sum over stages of max(algorithmic bytes / 8 TB/s, flop / peak); median and min over the "
                                     "instrumented steps (every fifth timed step records the library's stage events; they cost "
                                     "stream time, so these are a little slower than ms_per_step); caches are not flushed between "
                                     "steps, the cold variant (workloads under 2 GiB of weights) rotates three sets of inputs, "
                                     "weights and workspaces")

    result = {
        "metric": "MoE layer fwd tokens/s on 1 MI355X",
        "value": res["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": res["workload"], "filled_slots": R, "slots": E * C},
        "roofline": res["roofline"],
        "stages": stages,
        "layer_roofline": res["layer_roofline"],
        "fused_dispatch": res["fused_dispatch"],
    }
    if res["hip_graph_ms_per_step"] is not None:
        result["hip_graph_ms_per_step"] = res["hip_graph_ms_per_step"]

    if bf16 and not args.no_probe:
        # what the matrix cores alone sustain at the board's power limit on random bf16 operands (about a second of
        # register-only MFMA launches): the practical ceiling of `achieved`
        from paper_2206_03382_amd import probe
        sustained = probe.mfma_sustained_tflops(True, seconds=1.0)
        result["roofline"]["mfma_only_sustained_TFLOPs"] = round(sustained, 1)
        result["roofline"]["frac_of_mfma_only_sustained"] = round(res["roofline"]["achieved"] / sustained, 4)

    if args.backward:
        r = layer.routing
        slot_src = moe.slot_sources(r["idx"], r["loc"], E, C)
        slabs = torch.randn((E, C, M), device="cuda").to(x.dtype)             # stands in for dZ and for the expert outputs
        d_out = torch.randn((T, M), device="cuda").to(x.dtype)

        def timed(fn):
            for _ in range(args.warmup):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(args.steps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / args.steps

        enc_b = timed(lambda: moe.encode_backward(slabs, r["idx"], r["loc"]))
        dec_b = timed(lambda: moe.decode_backward(d_out, slabs, r["idx"], r["loc"], r["gate_w"], slot_src))
        enc_b_bytes = (R + T) * M * es + 8 * T * k                 # read each kept slot row, write [T,M]
        dec_b_bytes = (R + E * C) * M * es + (R + T) * M * es + 24 * T * k   # dY: read kept d_out rows, write all slots; dgate_w: d_out rows + kept Y rows
        Zb = moe.encode(x, r["idx"], r["loc"], slot_src, E, C)
        ffn_f = timed(lambda: moe.expert_ffn_train(Zb, layer.W1, layer.b1, layer.W2, layer.b2, cfg.act, counts=r["counts"]))
        _, hidden, pre = moe.expert_ffn_train(Zb, layer.W1, layer.b1, layer.W2, layer.b2, cfg.act, counts=r["counts"])
        ffn_b = timed(lambda: moe.expert_ffn_backward(Zb, layer.W1, layer.b1, layer.W2, hidden, slabs, cfg.act, counts=r["counts"], pre=pre))
        ffn_b_re = timed(lambda: moe.expert_ffn_backward(Zb, layer.W1, layer.b1, layer.W2, hidden, slabs, cfg.act, counts=r["counts"]))
        result["backward_ffn"] = {"ms": round(ffn_b, 5), "algorithmic_TFLOPs": round(4 * flop_per_gemm / (ffn_b * 1e-3) / 1e12, 1),
                                  "ms_recomputing_pre_activations": round(ffn_b_re, 5),
                                  "training_forward_ffn_ms": round(ffn_f, 5),
                                  "note": "dZ, dW1, db1, dW2, db2 from the pre-activations the training forward kept; four "
                                          "GEMMs' worth of algorithmic flop (2*R*M*H each); the time also holds the bias "
                                          "gradients' column sums and torch's allocation of workspace and outputs"}
        dgw = torch.randn((T, k), device="cuda")
        dxb = torch.empty_like(x)
        gate_b = timed(lambda: moe.gate_backward(x, layer.Wg, r["logits"], r["idx"], dgw, cfg.normalize, dx=dxb))
        result["backward_gate_ms"] = round(gate_b, 5)
        result["backward_total_ms"] = round(gate_b + ffn_b + enc_b + dec_b, 5)
        # the whole training step through the two layer-level entry points (one state buffer, outputs preallocated)
        tl = moe.TrainLayer(layer.Wg, layer.gate_bias, layer.W1, layer.b1, layer.W2, layer.b2, T=T, k=k, f=cfg.f,
                            normalize=cfg.normalize, act=cfg.act)
        tl.forward(x)
        grads = tl.backward(x, d_out)
        fwd_t = timed(lambda: tl.forward(x))
        bwd_t = timed(lambda: tl.backward(x, d_out, grads))
        result["training_step"] = {"forward_ms": round(fwd_t, 5), "backward_ms": round(bwd_t, 5),
                                   "tokens_per_s": round(T / ((fwd_t + bwd_t) * 1e-3), 1),
                                   "note": "moe_layer_forward_train + moe_layer_backward, all parameter gradients and dx"}
        del tl, grads
        result["backward_dispatch"] = {
            "encode_backward_ms": round(enc_b, 5), "encode_backward_frac_hbm": round(enc_b_bytes / (enc_b * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "decode_backward_ms": round(dec_b, 5), "decode_backward_frac_hbm": round(dec_b_bytes / (dec_b * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "note": "torch allocates the outputs inside the timed calls; algorithmic bytes as for encode/decode"}

    if args.bpr:
        lg = layer.routing["logits"]

        def timed_gate(bpr):
            for _ in range(args.warmup):
                moe.gate_topk(lg, k, C, cfg.normalize, bpr=bpr)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(args.steps):
                moe.gate_topk(lg, k, C, cfg.normalize, bpr=bpr)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / args.steps

        result["batch_prioritized_routing"] = {"gate_topk_ms": round(timed_gate(False), 5), "gate_topk_bpr_ms": round(timed_gate(True), 5),
                                               "note": "standalone calls (torch allocates outputs and workspace inside)"}

    if args.cosine:
        D = 256
        Wp = (torch.randn((M, D), device="cuda") / M ** 0.5).to(x.dtype)
        Me = torch.randn((E, D), device="cuda")
        for _ in range(args.warmup):
            moe.gate_logits_cosine(x, Wp, Me, 0.07)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.steps):
            moe.gate_logits_cosine(x, Wp, Me, 0.07)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / args.steps
        result["cosine_router"] = {"ms": round(ms, 5), "D": D, "fp64_GFLOP": round(2.0 * T * M * D / 1e9, 2),
                                   "fp64_TFLOPs": round(2.0 * T * M * D / (ms * 1e-3) / 1e12, 1),
                                   "note": "projection on the fp64 matrix cores (peak 78.6 TFLOP/s) + fp64 cosine per (token, expert)"}

    del layer, x
    torch.cuda.empty_cache()

    if not args.no_others:
        # the other four workloads, measured the same way in this run: step time, tokens/s, GEMM fraction of the MFMA
        # peak, encode/decode fraction of the HBM peak
        others = {}
        for i, ocfg in enumerate(synth.CONFIGS):
            if i == args.config:
                continue
            oinp = synth.make_inputs(ocfg, seed=0)
            ores, olayer, ox = measure(ocfg, oinp, args.steps, args.warmup, cold=False)
            del olayer, ox, oinp
            torch.cuda.empty_cache()
            st = ores["stages"]
            others[ocfg.name] = {
                "workload": ores["workload"], "ms_per_step": ores["ms_per_step"], "tokens_per_s": ores["tokens_per_s"],
                "gemm_TFLOPs": ores["roofline"]["achieved"], "gemm_frac_of_peak": ores["roofline"]["frac"],
                "gemm_peak_TFLOPs": ores["roofline"]["peak"],
                "encode_frac_hbm": st["encode_frac_hbm"], "decode_frac_hbm": st["decode_frac_hbm"],
                "gate_logits_frac_hbm": st["gate_logits_frac_hbm"], "gate_topk_frac_hbm": st["gate_topk_frac_hbm"],
                "stage_ms": {name: st[name] for name in moe.STAGE_NAMES},
                "fused_dispatch_ms_per_step": ores["fused_dispatch"]["ms_per_step"],
                "hip_graph_ms_per_step": ores["hip_graph_ms_per_step"],
                "layer_roofline_frac": ores["layer_roofline"]["frac"],
                "gemm_traffic": ores["roofline"]["traffic"]}
        result["other_workloads"] = others

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, inp)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
