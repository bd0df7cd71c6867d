#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X: `python bench.py [--gpus 1] [--steps K] [--warmup W]`.

One step = one pass of the whole path (gate logits -> top-k + slots -> encode -> expert FFN -> decode) over one batch
of seeded synthetic input that is already resident in HBM.  Prints one JSON line:
  value      layer forward tokens/s (T / mean step time)
  roofline   the dominant kernel (grouped bf16 MFMA GEMM of the expert FFN): algorithmic FLOP per launch divided by
             its mean launch time, measured with HIP events recorded on the library's stream inside the timed loop
             (on every fifth timed step: the event records themselves cost stream time)
  stages     per-stage mean milliseconds and, for encode/decode, algorithmic HBM GB/s
  cpu_baseline  the CPU oracle timed on this machine's host cores on the same workload
  fused_dispatch  the same step through moe_layer_forward_fused (the first expert GEMM gathers its rows from the tokens,
             no dispatch buffer), timed in a second loop of the same length; information only, `value` is the plain path
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VECTOR_PEAK_TFLOPS = 157.3
# HBM bytes per grouped-GEMM launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see profiles/), keyed by
# workload name; None where no counter run has been recorded.
MEASURED_GEMM_TRAFFIC_BYTES = {"mid_bf16": 563_358_861}     # profiles/bench_mid_bf16_hbm_traffic.txt


def to_device(a, dtype_code):
    import torch
    from paper_2206_03382_amd import synth
    if a is None:
        return None
    if dtype_code == synth.DT_BF16:
        return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=1, help="index into the five workloads (default 1: T=16384, M=H=2048, E=8, top-2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    x = to_device(inp["x"], d)
    gate_bias = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).cuda()
    layer = moe.MoELayer(to_device(inp["Wg"], d), gate_bias, to_device(inp["W1"], d), to_device(inp["b1"], d),
                         to_device(inp["W2"], d), to_device(inp["b2"], d), T=cfg.T, k=cfg.k, f=cfg.f,
                         normalize=cfg.normalize, act=cfg.act, keep_routing=True)
    # Stage events are recorded on every `stride`-th timed step only: each of the seven records costs a few microseconds
    # of stream time, and the steps in between run exactly as a caller without instrumentation would run them.
    stride = 5 if args.steps >= 10 else 1
    sampled = [i for i in range(args.steps) if i % stride == 0]
    events = {i: moe.StageEvents() for i in sampled}
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        layer.forward(x)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        layer.forward(x, events.get(i))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed * 1e3 / args.steps
    per_step = np.array([events[i].stage_ms() for i in sampled])     # [sampled steps, stages] from the library's own events
    stage_ms = np.mean(per_step, axis=0)

    for _ in range(args.warmup):
        layer.forward(x, fuse_dispatch=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        layer.forward(x, events.get(i), fuse_dispatch=True)
    torch.cuda.synchronize()
    fused_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    fused_stage_ms = np.mean(np.array([events[i].stage_ms() for i in sampled]), axis=0)
    for e in events.values():
        e.close()
    counts = layer.routing["counts"].cpu().numpy().astype(np.int64)
    C, T, M, H, E, k = layer.C, cfg.T, cfg.M, cfg.H, cfg.E, cfg.k
    es = 4 if d == synth.DT_F32 else 2
    R = int(np.minimum(counts, C).sum())                         # filled slots = kept (token, choice) pairs
    flop_per_gemm = 2.0 * R * M * H                              # GEMM1 [R,M]x[M,H] and GEMM2 [R,H]x[H,M]: same count
    gemm_ms = float(stage_ms[3] + stage_ms[4]) / 2.0
    bf16 = d == synth.DT_BF16
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else FP32_VECTOR_PEAK_TFLOPS
    achieved = flop_per_gemm / (gemm_ms * 1e-3) / 1e12
    enc_bytes = 2 * R * M * es + 4 * E * C                       # read each kept row once, write it once (the layer leaves unfilled slots alone)
    dec_bytes = (R + T) * M * es + 12 * T * k                    # read each kept expert-output row once, write [T,M]
    stages = {name: round(float(ms), 5) for name, ms in zip(moe.STAGE_NAMES, stage_ms)}
    stages["encode_GBps"] = round(enc_bytes / (stage_ms[2] * 1e-3) / 1e9, 1)
    stages["decode_GBps"] = round(dec_bytes / (stage_ms[5] * 1e-3) / 1e9, 1)
    stages["encode_frac_hbm"] = round(stages["encode_GBps"] / HBM_PEAK_GBS, 4)
    stages["decode_frac_hbm"] = round(stages["decode_GBps"] / HBM_PEAK_GBS, 4)
    stages["ffn_TFLOPs_filled_rows"] = round(2 * flop_per_gemm / ((stage_ms[3] + stage_ms[4]) * 1e-3) / 1e12, 1)

    # layer roofline: the stages run back to back on one stream, so their bounds add (HBM 8 TB/s for the data-movement
    # stages, 2.5 PFLOP/s for the two GEMMs); algorithmic bytes and flop only
    gate_bytes = T * M * es + M * E * es + 4 * T * E + (4 * T * E + 12 * T * k + 4 * E + 4 * E * C)
    t_roof_ms = ((gate_bytes + enc_bytes + dec_bytes) / (HBM_PEAK_GBS * 1e9) + 2 * flop_per_gemm / (peak * 1e12)) * 1e3
    step_from_events = per_step.sum(axis=1)

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

    # cold-cache variant: three separate sets of inputs, weights and workspaces used in rotation, so that no step finds
    # its operands in the 256 MB memory-side cache (the default loop reuses one set; caches are not flushed between steps)
    cold_ms = None
    if E * (M * H * 2) * es + T * M * es < (2 << 30):
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
        for i in range(args.steps):
            sets[i % 3][0].forward(sets[i % 3][1])
        torch.cuda.synchronize()
        cold_ms = (time.perf_counter() - c0) * 1e3 / args.steps
        del sets

    result = {
        "metric": "MoE layer fwd tokens/s on 1 MI355X",
        "value": round(T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={T} M={M} H={H} E={E} top-{k} f={cfg.f} C={C} act={('relu', 'gelu', 'silu')[cfg.act]}",
                   "filled_slots": R, "slots": E * C},
        "roofline": {"bound": "mfma" if bf16 else "alu", "kernel": "grouped_gemm_mfma_kernel" if bf16 else "gemm_generic_kernel",
                     "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                     "flop_per_launch": flop_per_gemm, "avg_launch_ms": round(gemm_ms, 5),
                     "traffic": MEASURED_GEMM_TRAFFIC_BYTES.get(cfg.name)},
        "stages": stages,
        "layer_roofline": {"t_roofline_ms": round(t_roof_ms, 5), "frac": round(t_roof_ms / ms_per_step, 4),
                           "step_ms_median": round(float(np.median(step_from_events)), 5),
                           "step_ms_min": round(float(step_from_events.min()), 5),
                           "cold_cache_ms_per_step": None if cold_ms is None else round(cold_ms, 5),
                           "instrumented_steps": len(sampled),
                           "note": "sum over stages of max(algorithmic bytes / 8 TB/s, flop / peak); median and min over the "
                                   "instrumented steps (every fifth timed step records the library's stage events; they cost "
                                   "stream time, so these are a little slower than ms_per_step); caches are not flushed between "
                                   "steps, the cold variant rotates three sets of inputs, weights and workspaces"},
        "fused_dispatch": {"ms_per_step": round(fused_ms, 5), "value": round(T / (fused_ms * 1e-3), 1), "unit": "tokens/s",
                           "stages": {name: round(float(ms), 5) for name, ms in zip(moe.STAGE_NAMES, fused_stage_ms)}},
    }

    if bf16:
        # live clock probe of the dominant kernel (outside the timed loops): the GEMM runs at the board's power cap, so its
        # shader clock, not 2.4 GHz, is what the matrix pipes get
        r0 = layer.routing
        Zp = moe.encode(x, r0["idx"], r0["loc"], moe.slot_sources(r0["idx"], r0["loc"], E, C), E, C)
        try:
            for _ in range(3):
                probe = moe.expert_ffn_clock_probe(Zp, layer.W1, layer.b1, layer.W2, layer.b2, cfg.act, r0["counts"])
            ghz = float(np.mean([p[0] for p in probe]))
            cyc = float(np.mean([p[1] for p in probe]))
            result["roofline"]["main_loop_shader_clock_GHz"] = round(ghz, 3)
            result["roofline"]["main_loop_cycles_per_64k_step"] = round(cyc, 0)
            result["roofline"]["mfma_issue_cycles_per_64k_step"] = 2048
            result["roofline"]["peak_at_measured_clock"] = round(peak * ghz / 2.4, 1)
        except moe.MoEError:
            pass                                                     # shapes the matrix-core kernel does not take
        del Zp
        # what the matrix cores alone sustain at the board's power limit on random bf16 operands (about a second of
        # register-only MFMA launches): the practical ceiling of `achieved`
        sustained = moe.mfma_sustained_tflops(True, seconds=1.0)
        result["roofline"]["mfma_only_sustained_TFLOPs"] = round(sustained, 1)
        result["roofline"]["frac_of_mfma_only_sustained"] = round(achieved / sustained, 4)

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
                                               "note": "standalone calls (torch allocates outputs and workspace inside); the "
                                                       "prioritized order is found by exact O(T^2) counting"}

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

    if not args.no_cpu_baseline:
        from oracle import moe_oracle as O
        from threadpoolctl import threadpool_info
        blas = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
        threads = max(blas) if blas else (os.cpu_count() or 1)     # the oracle's time is in numpy's BLAS matmuls
        reps, c0 = 0, time.perf_counter()
        while reps == 0 or time.perf_counter() - c0 < 10.0:          # about 10 s of oracle work, whole passes only
            O.moe_layer(inp["x"], inp["Wg"], inp["gate_bias"], inp["W1"], inp["b1"], inp["W2"], inp["b2"],
                        cfg.k, cfg.f, cfg.normalize, cfg.act, tier="sparse")
            reps += 1
        cpu_s = time.perf_counter() - c0
        result["cpu_baseline"] = {"value": round(T * reps / cpu_s, 1), "unit": "tokens/s", "cores": int(threads),
                                  "kind": "oracle", "sample": f"the full workload {reps} times (all {T} tokens each, fp64 numpy, zero-skipping tier), {cpu_s:.1f} s"}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
