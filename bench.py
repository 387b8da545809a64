#!/usr/bin/env python3
"""Benchmark of the nested quantized linear hot path on one MI355X.

One step = one pass of the whole hot path over the Gemma-2-9B-shaped MLP of the workload list (d_model 3584,
ffn 14336, 8192 tokens, weights N(0, 0.015^2) with 0.1 % outliers, loss weights (0.1, 0.1, 1.0) of appendix B;
seeded synthetic tensors already resident in HBM): for each of the three linears (gate, up, down) quantize the
fp32 master weight to int8 codes, slice and pack the r = 4 and r = 2 planes (r = 2 also with the extra-precision
overflow list), run the fused r = 8/4/2 forward with the L2 reconstruction objective of the three outputs
against the output of the full-precision layer evaluated in its epilogue (losses and the gradients dY_r; the
outputs themselves are not stored, the training step has no other use for them) and the straight-through
backward (dX, dW), round alpha/z to bf16 and run the decode GEMV at B = 1, 4, 16 on the int4 and int2 planes.

`value` is the metric's first half: the fused r = 8/4/2 forward in TFLOP/s (6 M N K flops per linear over the
HIP-event time of the three forward calls of a step, averaged over the timed steps); `roofline` prices it
against the bf16 matrix-core peak per linear.  The metric's second half, the sliced int2 GEMV in GB/s against
the HBM peak, is `gemv_roofline` (7B decode shapes, cache-defeating copies).  `ms_per_step` is the wall time of
the whole step; `step_blended_TFLOPs` divides all matrix-core work of the step (forward 6 MNK + backward 8 MNK)
by it, so the bandwidth-bound operations count against that figure.
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
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM-side bytes per launch of the fused forward kernel on the headline workload, per linear, from the
# FETCH_SIZE / WRITE_SIZE counter passes summarised in profiles/ (scale factors stated there); None until taken.
FWD_TRAFFIC_BYTES = {3: {"gate": 2424021 * 1024, "up": 2424021 * 1024, "down": 1950779 * 1024},
                     2: {"gate": None, "up": None, "down": None}}
WORKLOADS = {
    3: "configs[2]: Gemma-2-9B-shaped MLP, d_model 3584, ffn 14336, 8192 tokens, outlier weights, lambda = (0.1, 0.1, 1.0)",
    2: "configs[1]: Gemma-2-2B-shaped MLP, d_model 2304, ffn 9216, 4096 tokens",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, choices=(2, 3),
                    help="workload of the step: 3 = the Gemma-2-9B-shaped MLP (headline), 2 = the 2B-shaped one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gemv-sweep", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the 27B-shaped forward block and the added operations")
    ap.add_argument("--no-probes", action="store_true", help="skip the measured-ceiling probes")
    ap.add_argument("--only-decode", action="store_true",
                    help="run only the decode GEMV sweeps and the read probe (for counter passes over the decode kernels); "
                         "prints their sections, not the bench line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 256 MiB device-to-device copies before the timed region: a kernel of "
                         "known traffic against which hardware byte counters of a profiling run are scaled")
    return ap.parse_args()


class Linear:
    """Device buffers of one linear of the MLP; everything is allocated before the timed region."""

    def __init__(self, mq, torch, synth, config, name, M, rs, lambdas):
        dev = "cuda"
        case = synth.linear_case(config, name, with_grads=False)
        self.name, self.M, self.N, self.K, self.rs, self.lambdas = name, M, case.N, case.K, rs, lambdas
        N, K = self.N, self.K
        self.W = case.W.to(dev)
        self.X = case.X.to(dev)
        # y' of the layer-wise reconstruction objective: the output of the full-precision layer (computed once,
        # outside the timed region, with the framework's bf16 matmul: an input of the step, not part of it)
        self.T = (self.X @ self.W.to(torch.bfloat16).t()).contiguous()
        self.dY = [torch.empty(M, N, dtype=torch.bfloat16, device=dev) for _ in rs]
        self.losses = torch.empty(len(rs), dtype=torch.float32, device=dev)
        self.Q = torch.empty(N, K, dtype=torch.uint8, device=dev)
        self.alpha = torch.empty(N, dtype=torch.float32, device=dev)
        self.zero = torch.empty(N, dtype=torch.float32, device=dev)
        self.alpha16 = torch.empty(N, dtype=torch.bfloat16, device=dev)
        self.zero16 = torch.empty(N, dtype=torch.bfloat16, device=dev)
        self.p4 = torch.empty(N, K // 2, dtype=torch.uint8, device=dev)
        self.p2 = torch.empty(N, K // 4, dtype=torch.uint8, device=dev)
        self.ovf2 = mq.Overflow(N, N * K // 8, dev)   # room for 12.5 % overflow
        self.dX = torch.empty(M, K, dtype=torch.bfloat16, device=dev)
        self.dW = torch.empty(N, K, dtype=torch.float32, device=dev)
        self.ws_f = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD_L2, M, N, K, len(rs)), dtype=torch.uint8, device=dev)
        self.ws_b = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD, M, N, K, len(rs)), dtype=torch.uint8, device=dev)
        self.xdec = {B: synth.activations(config, f"dec{B}:" + name, B, K).to(dev) for B in (1, 4, 16)}
        self.ydec = {B: torch.empty(B, N, dtype=torch.bfloat16, device=dev) for B in (1, 4, 16)}


def event_ms(torch, fn, reps):
    """Average HIP-event time of `reps` calls of fn on the current stream (after one untimed call)."""
    fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives are part of the hot path).", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2502_06786_amd as mq
    from paper_2502_06786_amd import synth

    mq.lib()  # fails loudly when libmq.so is missing
    torch.cuda.set_device(0)
    if args.only_decode:
        from paper_2502_06786_amd import bench_probes
        print(json.dumps({"only": "decode", "measured_peaks": measured_peaks(torch, bench_probes),
                          "gemv_roofline": gemv_sweep(torch, mq, synth), "extra_precision_gemv": ep_gemv(torch, mq, synth)}))
        return
    cfg = args.config
    rs, lambdas = (8, 4, 2), synth.LAMBDAS[cfg]
    _, M = synth.mlp_shapes(cfg)
    layers = [Linear(mq, torch, synth, cfg, name, M, rs, lambdas) for name in ("gate", "up", "down")]

    ops = ["quantize", "slice", "fwd", "bwd", "gemv"]
    records = {op: [] for op in ops}   # (linear, start event, end event) inside the timed region

    def timed(op, L, fn, rec):
        if not rec:
            fn()
            return
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        records[op].append((L.name, a, b))

    def step(rec):
        for L in layers:
            timed("quantize", L, lambda: mq.mq_quantize_int8(L.W, Q=L.Q, alpha=L.alpha, zero=L.zero), rec)

            def do_slice():
                mq.mq_slice_multi(L.Q, (4, 2), out=[L.p4, L.p2], ovf_r=2, ovf=L.ovf2)
                mq.mq_params_to_bf16(L.alpha, L.zero, L.alpha16, L.zero16)
            timed("slice", L, do_slice, rec)
            # forward for r = 8, 4, 2 with the L2 reconstruction losses against y' and the gradients the
            # backward consumes formed in its epilogue
            timed("fwd", L, lambda: mq.mq_linear_fwd_multi_l2(L.X, L.Q, L.alpha, L.zero, rs, L.T, None, lambdas,
                                                              dY=L.dY, losses=L.losses, ws=L.ws_f), rec)
            # (the dY_r of the objective already carry lambda_r: the backward takes them unweighted)
            timed("bwd", L, lambda: mq.mq_linear_bwd(L.X, L.Q, L.alpha, L.zero, L.dY, None, rs, dX=L.dX, dW=L.dW,
                                                     ws=L.ws_b), rec)

            def do_gemv():
                for B in (1, 4, 16):
                    mq.mq_gemv_sliced(L.xdec[B], L.p4, L.alpha16, L.zero16, 4, L.K, y=L.ydec[B])
                    mq.mq_gemv_sliced(L.xdec[B], L.p2, L.alpha16, L.zero16, 2, L.K, y=L.ydec[B])
            timed("gemv", L, do_gemv, rec)

    if args.copy_calibration:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    mnk = sum(L.M * L.N * L.K for L in layers)
    flops_fwd, flops_bwd = 6.0 * mnk, 8.0 * mnk

    def op_ms_of(op, name=None):   # ms per step spent in `op` (of linear `name`)
        return sum(a.elapsed_time(b) for n, a, b in records[op] if name is None or n == name) / args.steps

    op_ms = {op: op_ms_of(op) for op in ops}
    nk = sum(L.N * L.K for L in layers)
    gemv_bytes = sum(sum(L.N * L.K * r // 8 + 4 * L.N + 2 * B * L.K + 2 * B * L.N for r in (4, 2)) for B in (1, 4, 16)
                     for L in layers)
    fwd_tf = flops_fwd / (op_ms["fwd"] * 1e-3) / 1e12
    per_op = {
        "fwd_TFLOPs": fwd_tf,
        "bwd_TFLOPs": flops_bwd / (op_ms["bwd"] * 1e-3) / 1e12,
        "quantize_GBs": 5.0 * nk / (op_ms["quantize"] * 1e-3) / 1e9,
        "slice_GBs": (1.0 + 0.5 + 0.25) * nk / (op_ms["slice"] * 1e-3) / 1e9,   # codes read once, int4 and int2 planes written
        "gemv_GBs": gemv_bytes / (op_ms["gemv"] * 1e-3) / 1e9,
        "ms": {k: round(v, 4) for k, v in op_ms.items()},
    }

    # Roofline of the dominant kernel, the fused r = 8/4/2 forward (one launch per linear): events bracket the
    # mq_linear_fwd_multi_l2 call, i.e. the kernel plus its few-microsecond row-sum pre-pass and the
    # one-workgroup finish of the loss sums.  Per linear and over the three.
    per_linear = {}
    for L in layers:
        ms = op_ms_of("fwd", L.name)
        tf = 6.0 * L.M * L.N * L.K / (ms * 1e-3) / 1e12
        per_linear[L.name] = {"M": L.M, "N": L.N, "K": L.K, "avg_launch_ms": round(ms, 4), "achieved": round(tf, 2),
                              "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                              "algorithmic_bytes": L.N * L.K + 2 * L.M * L.K + 8 * L.M * L.N,
                              "traffic": FWD_TRAFFIC_BYTES[cfg][L.name]}
    traffics = [per_linear[L.name]["traffic"] for L in layers]
    roofline = {"bound": "mfma", "kernel": "mq::fwd_kernel<3, true, false, MB, true> (r = 8/4/2 with the objective in the epilogue)",
                "achieved": round(fwd_tf, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(fwd_tf / PEAK_BF16_TFLOPS, 4),
                "traffic": None if any(t is None for t in traffics) else int(sum(traffics) / len(traffics)),
                "algorithmic_bytes": int(sum(v["algorithmic_bytes"] for v in per_linear.values()) / len(layers)),
                "avg_launch_ms": round(op_ms["fwd"] / len(layers), 4), "per_linear": per_linear}

    # the same forward without the objective (outputs stored), and the two halves of the backward on their
    # own, outside the timed region
    plain, bwd_split = {}, {}
    for L in layers:
        Y = [torch.empty(L.M, L.N, dtype=torch.bfloat16, device="cuda") for _ in rs]
        ws = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD, L.M, L.N, L.K, len(rs)), dtype=torch.uint8, device="cuda")
        ms = event_ms(torch, lambda: mq.mq_linear_fwd_multi(L.X, L.Q, L.alpha, L.zero, rs, Y=Y, ws=ws), 5)
        tf = 6.0 * L.M * L.N * L.K / (ms * 1e-3) / 1e12
        plain[L.name] = {"avg_launch_ms": round(ms, 4), "achieved": round(tf, 2), "frac": round(tf / PEAK_BF16_TFLOPS, 4)}
        del Y, ws
        ms_dx = event_ms(torch, lambda: mq.mq_linear_bwd(L.X, L.Q, L.alpha, L.zero, L.dY, None, rs, dX=L.dX,
                                                         need_dW=False, ws=L.ws_b), 3)
        ms_dw = event_ms(torch, lambda: mq.mq_linear_bwd(L.X, L.Q, L.alpha, L.zero, L.dY, None, rs, need_dX=False,
                                                         dW=L.dW, ws=L.ws_b), 3)
        tdx, tdw = 6.0 * L.M * L.N * L.K / (ms_dx * 1e-3) / 1e12, 2.0 * L.M * L.N * L.K / (ms_dw * 1e-3) / 1e12
        bwd_split[L.name] = {"dX_call_ms": round(ms_dx, 4), "dX_TFLOPs": round(tdx, 1), "dX_frac": round(tdx / PEAK_BF16_TFLOPS, 4),
                             "dW_call_ms": round(ms_dw, 4), "dW_TFLOPs": round(tdw, 1), "dW_frac": round(tdw / PEAK_BF16_TFLOPS, 4)}
    plain_ms = sum(v["avg_launch_ms"] for v in plain.values())
    plain_tf = flops_fwd / (plain_ms * 1e-3) / 1e12
    roofline["plain_forward"] = {"kernel": "mq::fwd_kernel<3, true, false, MB, false> (mq_linear_fwd_multi: Y_r stored, no objective)",
                                 "achieved": round(plain_tf, 2), "frac": round(plain_tf / PEAK_BF16_TFLOPS, 4),
                                 "per_linear": plain}
    bwd_split["note"] = ("mq_linear_bwd with only dX (prep pass + code transpose + dx_kernel, 6 MNK flops) and with only dW "
                         "(prep pass + activation transpose + dw_kernel, 2 MNK flops); helper passes included in each time")

    out = {
        "metric": "fused r=8/4/2 quant-linear TFLOP/s (%MFMA peak); sliced int2 GEMV GB/s (%HBM)",
        "value": round(fwd_tf, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[cfg] + "; step = per linear (gate, up, down): quantize + slice/pack r=4, r=2 (+ overflow "
                               "list) + fused r=8/4/2 fwd with L2 objective + STE bwd (dX, dW) + decode GEMV B=1/4/16 (int4, int2)",
                   "tokens": M, "rs": list(rs), "lambdas": list(lambdas), "seed": synth.config_seed(cfg)},
        "value_note": "6 MNK flops of the three fused forward calls of a step over their HIP-event time inside the timed region",
        "step_blended_TFLOPs": round((flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12, 2),
        "per_op": per_op,
        "roofline": roofline,
        "backward": bwd_split,
    }
    if not args.no_probes:
        from paper_2502_06786_amd import bench_probes
        peaks = measured_peaks(torch, bench_probes)
        out["measured_peaks"] = peaks
        # against the probe with the kernel's own product shape and occupancy, and against the best any bf16
        # loop sustains on this GPU on such operands (16x16x32 products, two waves per SIMD)
        roofline["frac_of_measured"] = round(fwd_tf / peaks["mfma_bf16_normal_operands_TFLOPs"], 4)
        roofline["frac_of_best_measured"] = round(
            fwd_tf / max(peaks["mfma_bf16_normal_operands_TFLOPs"], peaks["mfma16_bf16_normal_operands_TFLOPs"]), 4)
    if not args.no_gemv_sweep:
        out["gemv_roofline"] = gemv_sweep(torch, mq, synth)
        out["extra_precision_gemv"] = ep_gemv(torch, mq, synth)
        # the int2 GEMV of the metric: best over the 7B shapes of configuration 4, the stacked gate/up planes and the
        # plain int2 plane of the 27B-shaped matrix of configuration 5
        best = out["gemv_roofline"]["best_int2"]
        for B in (1, 4, 16):
            e = out["extra_precision_gemv"][f"plain_int2_B{B}"]
            if e["GBs"] > best["achieved"]:
                best.update({"case": f"int2_36864x4608_B{B}", "achieved": e["GBs"], "frac": round(e["GBs"] / PEAK_HBM_GBS, 4)})
        if not args.no_probes:
            best["frac_of_measured_read"] = round(best["achieved"] / peaks["hbm_read_85MB_GBs"], 4)
    if not args.no_extras:
        out["mixnmatch_decode"] = mixnmatch_decode(torch, mq, synth)
        out["clip_factor_grads"] = clip_factor_grads(torch, mq, layers, rs, lambdas)
        out["omniquant_step"] = omniquant_step(torch, mq, layers, rs, lambdas)
        out["ffn_block_train"] = ffn_block_train(torch, mq, layers, rs)
        out["attention_projections"] = attention_projections(torch, mq, synth)
        del layers
        torch.cuda.empty_cache()
        out["config5_forward"] = config5_forward(torch, mq, synth)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, synth)
    print(json.dumps(out))


def config5_forward(torch, mq, synth):
    """configs[4]: the Gemma-2-27B-shaped linears (36864 x 4608 and 4608 x 36864, heavy-tailed weights, 4096 tokens):
    quantize, then the forward for r = 8/4/2 in one launch, for r = 2 alone and for r = 2 with extra precision
    (outputs stored; HIP events around 3 calls each)."""
    res = {"workload": "configs[4]: Gemma-2-27B-shaped MLP, d_model 4608, ffn 36864, 4096 tokens, W ~ Student-t(3) * 0.01"}
    for name in ("gate", "down"):
        case = synth.linear_case(5, name, with_grads=False)
        M, N, K = case.M, case.N, case.K
        W, X = case.W.cuda(), case.X.cuda()
        Q, alpha, zero = mq.mq_quantize_int8(W)
        del W
        entry = {"M": M, "N": N, "K": K}
        Y = [torch.empty(M, N, dtype=torch.bfloat16, device="cuda") for _ in range(3)]
        ws = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD, M, N, K, 3), dtype=torch.uint8, device="cuda")
        for label, rs_, ep in (("r842", (8, 4, 2), False), ("r2", (2,), False), ("r2_extra_precision", (2,), True)):
            ms = event_ms(torch, lambda: mq.mq_linear_fwd_multi(X, Q, alpha, zero, rs_, extra_precision=ep,
                                                                Y=Y[:len(rs_)], ws=ws), 3)
            tf = 2.0 * len(rs_) * M * N * K / (ms * 1e-3) / 1e12
            entry[label] = {"avg_launch_ms": round(ms, 4), "achieved": round(tf, 2), "frac": round(tf / PEAK_BF16_TFLOPS, 4)}
        res[name] = entry
        del Q, X, Y, ws
        torch.cuda.empty_cache()
    res["note"] = "TFLOP/s = 2 * (number of bit-widths) * M N K over the HIP-event time of one mq_linear_fwd_multi call; peak 2500"
    return res


def measured_peaks(torch, mq):
    """What this GPU sustains on kernels that only multiply or only read (library probes): the matrix-core
    loop fed with N(0,1) bf16 operands (the bit patterns set the power drawn, hence the clock) and with a
    constant, a 1 GiB read, and reads of decode-sized 85 MB buffers (eight copies in turn)."""
    def timed(fn, reps=3):
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            n = fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(n / (e0.elapsed_time(e1) * 1e-3))
        return sorted(ts)[len(ts) // 2]

    g = torch.Generator().manual_seed(1234)
    normal = torch.randn(32768, generator=g).to(torch.bfloat16).cuda()
    const = torch.full((32768,), 128.0, dtype=torch.bfloat16, device="cuda")
    sink = torch.empty(65536, dtype=torch.float32, device="cuda")
    mq.mq_probe_mfma(normal, 2000, sink)
    res = {
        "mfma_bf16_normal_operands_TFLOPs": round(timed(lambda: mq.mq_probe_mfma(normal, 30000, sink)) / 1e12, 1),
        "mfma_bf16_constant_operands_TFLOPs": round(timed(lambda: mq.mq_probe_mfma(const, 30000, sink)) / 1e12, 1),
    }
    sink16 = torch.empty(131072, dtype=torch.float32, device="cuda")
    mq.mq_probe_mfma16(normal, 2000, sink16)
    res["mfma16_bf16_normal_operands_TFLOPs"] = round(timed(lambda: mq.mq_probe_mfma16(normal, 30000, sink16)) / 1e12, 1)
    res["mfma16_bf16_constant_operands_TFLOPs"] = round(timed(lambda: mq.mq_probe_mfma16(const, 30000, sink16)) / 1e12, 1)
    big = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
    isink = torch.zeros(1, dtype=torch.int32, device="cuda")
    mq.mq_probe_read(big, isink)
    res["hbm_read_1GiB_GBs"] = round(timed(lambda: mq.mq_probe_read(big, isink)) / 1e9, 1)
    nb = 36864 * 2304
    parts = [big[i * (128 << 20): i * (128 << 20) + nb] for i in range(8)]

    def decode_sized():
        for p in parts:
            mq.mq_probe_read(p, isink)
        return 8 * nb
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        decode_sized()

    def replay():
        graph.replay()
        return 8 * nb
    replay()
    res["hbm_read_85MB_GBs"] = round(timed(replay, reps=5) / 1e9, 1)
    res["note"] = ("library probes mq_probe_mfma (32x32x16 products, 1024 waves, 12 accumulators each, ~10 ms: the "
                   "shape and occupancy of the fused kernels), mq_probe_mfma16 (16x16x32 products, 2048 waves, 24 "
                   "accumulators each) and mq_probe_read; published peaks: 2500 TFLOP/s, 8000 GB/s")
    return res


def gemv_sweep(torch, mq, synth):
    """Decode GEMV on the 7B-shaped matrices of configs[3]: each shape gets enough independent copies to
    exceed the 256 MB last-level cache, and one stream-ordered sweep over all copies is timed."""
    res = {}
    best, best4 = None, None
    # (the last two are the stacked gate/up planes that mq_ffn_mixnmatch reads: 7B- and 27B-shaped, int2 and int4)
    for (N, K) in list(synth.DECODE_SHAPES) + [(28672, 4096), (73728, 4608)]:
        g = torch.Generator().manual_seed(N * 7 + K)
        for r in ((2, 4, 3, 6) if (N, K) in synth.DECODE_SHAPES else (2, 4)):
            kb = K * r // 8
            copies = max(8, int(640e6 // (N * kb)) + 1)
            planes = [torch.randint(0, 256, (N, kb), generator=g, dtype=torch.int32).to(torch.uint8).cuda()
                      for _ in range(2)]
            planes = planes + [planes[i % 2].clone() for i in range(copies - 2)]
            a16 = (torch.rand(N, generator=g) * 1e-3 + 1e-4).to(torch.bfloat16).cuda()
            z16 = (torch.rand(N, generator=g) * 255).to(torch.bfloat16).cuda()
            for B in (1, 4, 16):
                x = synth.activations(4, f"x{B}:{N}x{K}", B, K).cuda()
                y = torch.empty(B, N, dtype=torch.bfloat16, device="cuda")
                nbytes = N * kb + 4 * N + 2 * B * K + 2 * B * N

                def measure(call):
                    for p in planes[:2]:
                        call(p)
                    torch.cuda.synchronize()
                    # A decode loop is launch-bound from Python (several microseconds per call), so the sweep
                    # is captured once into a HIP graph and replayed; the kernels and their order are the same.
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph):
                        for p in planes:
                            call(p)
                    graph.replay()
                    torch.cuda.synchronize()
                    times = []
                    for _ in range(5):
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record()
                        graph.replay()
                        e1.record()
                        torch.cuda.synchronize()
                        times.append(e0.elapsed_time(e1) / len(planes))
                    del graph
                    ms = sorted(times)[len(times) // 2]
                    gbs = nbytes / (ms * 1e-3) / 1e9
                    return gbs, {"us": round(ms * 1e3, 2), "GBs": round(gbs, 1), "frac": round(gbs / PEAK_HBM_GBS, 4)}

                gbs, res[f"int{r}_{N}x{K}_B{B}"] = measure(lambda p: mq.mq_gemv_sliced(x, p, a16, z16, r, K, y=y))
                ws_bytes = mq.mq_workspace_bytes(mq.MQ_OP_GEMV, B, N, K, r)
                if ws_bytes > 256:
                    # the entry point that may split K over workgroups (long rows, few of them)
                    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
                    gbs_ws, res[f"int{r}_{N}x{K}_B{B}_with_workspace"] = measure(
                        lambda p: mq.mq_gemv_sliced_ws(x, p, a16, z16, r, K, y=y, ws=ws))
                    gbs = max(gbs, gbs_ws)
                if r == 2 and (best is None or gbs > best[1]):
                    best = (f"int{r}_{N}x{K}_B{B}", gbs)
                if r == 4 and (best4 is None or gbs > best4[1]):
                    best4 = (f"int{r}_{N}x{K}_B{B}", gbs)
            del planes
    res["bound"] = "hbm"
    res["peak"] = PEAK_HBM_GBS
    res["unit"] = "GB/s"
    res["best_int2"] = {"case": best[0], "achieved": round(best[1], 1), "frac": round(best[1] / PEAK_HBM_GBS, 4)}
    res["best_int4"] = {"case": best4[0], "achieved": round(best4[1], 1), "frac": round(best4[1] / PEAK_HBM_GBS, 4)}
    res["note"] = ("time per call from a HIP-graph replay of one stream-ordered sweep over independent copies of the "
                   "matrix (more than the 256 MB last-level cache holds); gaps between kernels included")
    return res


def ep_gemv(torch, mq, synth):
    """Configuration 5: int2 decode GEMV on the 27B-shaped gate matrix (36864 x 4608) with codes planted at the
    paper's overflow density (about 5 % at r = 2, Table 7): the plain int2 plane, the plane plus the sparse
    overflow list, and the dense 3-bit extra-precision plane.  Seven copies of each plane in turn (more than
    the last-level cache holds), HIP-graph replay, time per call."""
    N, K, r = 36864, 4608, 2
    # codes from 256 - half up round to 2^r: the overflow bucket of the errata section
    q = synth.planted_codes(55, N, K, 256 - (1 << (8 - r)) // 2, 0.05).cuda()
    plain, ovf = mq.mq_slice(q, r, packed=True, extra_precision=True, capacity=N * K // 8)
    dense = mq.mq_slice(q, r, packed=True, extra_precision=True, dense_ep=True)
    torch.cuda.synchronize()
    nnz = int(ovf.nnz.item())
    f = nnz / (N * K)
    del q
    g = torch.Generator().manual_seed(5)
    a16 = (torch.rand(N, generator=g) * 1e-3 + 1e-4).to(torch.bfloat16).cuda()
    z16 = (torch.rand(N, generator=g) * 255).to(torch.bfloat16).cuda()
    plains = [plain] + [plain.clone() for _ in range(6)]
    denses = [dense] + [dense.clone() for _ in range(6)]
    res = {"shape": f"{N}x{K}", "overflow_fraction": round(f, 4), "avg_bits_paper_accounting": round(r + f, 3),
           "stored_bits_list": round(r + 16 * f + 32.0 / K, 3), "stored_bits_dense": 3.0}
    for B in (1, 4, 16):
        x = synth.activations(5, f"ep{B}", B, K).cuda()
        y = torch.empty(B, N, dtype=torch.bfloat16, device="cuda")
        variants = {
            "plain_int2": (lambda p: mq.mq_gemv_sliced(x, p, a16, z16, r, K, y=y), plains, N * K // 4),
            "int2_plus_list": (lambda p: mq.mq_gemv_sliced(x, p, a16, z16, r, K, y=y, ovf=ovf), plains,
                               N * K // 4 + 2 * nnz + 4 * (N + 1)),
            "dense_3bit": (lambda p: mq.mq_gemv_sliced_dense_ep(x, p, a16, z16, r, K, y=y), denses, N * K * 3 // 8),
        }
        for name, (fn, planes, wbytes) in variants.items():
            fn(planes[0])
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for p in planes:
                    fn(p)
            graph.replay()
            torch.cuda.synchronize()
            times = []
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                graph.replay()
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1) / len(planes))
            del graph
            ms = sorted(times)[1]
            nbytes = wbytes + 4 * N + 2 * B * K + 2 * B * N
            res[f"{name}_B{B}"] = {"us": round(ms * 1e3, 2), "GBs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                                   "frac": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
    return res


def clip_factor_grads(torch, mq, layers, rs, lambdas, reps=2):
    """mq_linear_bwd_clip on the three linears of the step (the gradients dY_r the step left behind): one
    dY_r^T X contraction per bit-width plus a row reduction each."""
    res = {}
    for L in layers:
        ws = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD_CLIP, L.M, L.N, L.K, len(rs)), dtype=torch.uint8, device="cuda")
        mq.mq_linear_bwd_clip(L.W, L.X, L.Q, L.alpha, L.zero, L.dY, lambdas, rs, ws=ws)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            mq.mq_linear_bwd_clip(L.W, L.X, L.Q, L.alpha, L.zero, L.dY, lambdas, rs, ws=ws)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / reps
        res[L.name] = {"ms": round(ms, 4), "TFLOPs": round(2.0 * len(rs) * L.M * L.N * L.K / (ms * 1e-3) / 1e12, 1)}
        del ws
    res["note"] = "flops = 2 MNK per bit-width (the three dY_r^T X contractions); the row reductions are HBM-bound"
    return res


def omniquant_step(torch, mq, layers, rs, lambdas, reps=2):
    """One calibration step of the OmniQuant base algorithm under the MatQuant objective on each linear of the
    workload: affine re-parameterisation of weight and input, quantizer with clip factors, forward for r = 8/4/2
    with bias and the L2 objective, straight-through backward, gradients of gamma, beta, delta, s."""
    res = {}
    for L in layers:
        g = torch.Generator().manual_seed(17)
        gamma = (torch.rand(L.N, generator=g) * 0.2 + 0.8).cuda()
        beta = (torch.rand(L.N, generator=g) * 0.2 + 0.8).cuda()
        s = (torch.rand(L.K, generator=g) + 0.5).cuda()
        delta = (torch.randn(L.K, generator=g) * 0.05).cuda()
        ws_f = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD_L2, L.M, L.N, L.K, len(rs)), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD, L.M, L.N, L.K, len(rs)), dtype=torch.uint8, device="cuda")
        ws_c = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD_CLIP, L.M, L.N, L.K, len(rs)), dtype=torch.uint8, device="cuda")
        ws_a = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_AFFINE_BWD, L.M, L.N, L.K, len(rs)), dtype=torch.uint8, device="cuda")
        Xt = torch.empty_like(L.X)

        def one():
            Ws, c = mq.mq_affine_weight(L.W, s, delta, None)
            mq.mq_affine_input(L.X, s, delta, Xt=Xt)
            Q, a, z = mq.mq_quantize_int8(Ws, gamma, beta, Q=L.Q, alpha=L.alpha, zero=L.zero)
            mq.mq_linear_fwd_multi_l2(Xt, Q, a, z, rs, L.T, None, lambdas, dY=L.dY, losses=L.losses, ws=ws_f, bias=c)
            dXt, dWs = mq.mq_linear_bwd(Xt, Q, a, z, L.dY, None, rs, dX=L.dX, dW=L.dW, ws=ws_b)
            mq.mq_linear_bwd_clip(Ws, Xt, Q, a, z, L.dY, None, rs, gamma, beta, ws=ws_c)
            mq.mq_affine_bwd(L.X, dXt, L.W, dWs, L.dY, None, s, delta, ws=ws_a)

        one()
        a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a_.record()
        for _ in range(reps):
            one()
        b_.record()
        torch.cuda.synchronize()
        ms = a_.elapsed_time(b_) / reps
        flops = (6.0 + 8.0 + 6.0) * L.M * L.N * L.K      # forward, backward, one more contraction per bit-width for the clip factors
        res[L.name] = {"ms": round(ms, 4), "TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1)}
        del ws_f, ws_b, ws_c, ws_a, Xt
    res["note"] = ("mq_affine_weight + mq_affine_input + mq_quantize_int8(gamma, beta) + mq_linear_fwd_multi_l2(bias) + mq_linear_bwd "
                   "+ mq_linear_bwd_clip + mq_affine_bwd; flops = 20 MNK (forward 6, backward 8, clip-factor contractions 6)")
    return res


def ffn_block_train(torch, mq, layers, rs, reps=2):
    """Forward and straight-through backward of the whole gated feed-forward block of the workload for r = 8/4/2,
    composed from the library's calls: one fused forward over the stacked gate/up weight (rows interleaved) with the gate
    in its epilogue, one down forward per bit-width; back through the three down layers (dW accumulated) and the stacked
    layer, whose backward forms the gradient of the gated unit in its first pass.  Timed next to it: the same block with
    the gate as stand-alone kernels (mq_gated_unit_fwd / _bwd between the layer calls)."""
    gate, up, down = layers
    M, d, F = gate.M, gate.K, gate.N
    Wgu = torch.empty(2 * F, d, dtype=torch.float32, device="cuda")
    Wgu[0::2], Wgu[1::2] = gate.W, up.W
    Qg, ag, zg = mq.mq_quantize_int8(Wgu)
    del Wgu
    Qd, ad, zd = down.Q, down.alpha, down.zero
    mq.mq_quantize_int8(down.W, Q=Qd, alpha=ad, zero=zd)
    X = gate.X
    bf = dict(dtype=torch.bfloat16, device="cuda")
    GU = [torch.empty(M, 2 * F, **bf) for _ in rs]
    A = [torch.empty(M, F, **bf) for _ in rs]
    Y = [torch.empty(M, d, **bf) for _ in rs]
    dY = [(torch.randn(M, d, generator=torch.Generator().manual_seed(5 + i)) * 1e-3).to(torch.bfloat16).cuda() for i in range(len(rs))]
    dA = [torch.empty(M, F, **bf) for _ in rs]
    dGU = [torch.empty(M, 2 * F, **bf) for _ in rs]
    dX = torch.empty(M, d, **bf)
    dWgu = torch.empty(2 * F, d, dtype=torch.float32, device="cuda")
    dWd = torch.empty(d, F, dtype=torch.float32, device="cuda")
    u8 = dict(dtype=torch.uint8, device="cuda")
    ws_fg = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD, M, 2 * F, d, len(rs)), **u8)
    ws_fd = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD, M, d, F, 1), **u8)
    ws_bg = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD, M, 2 * F, d, len(rs)), **u8)
    ws_bd = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD, M, d, F, 1), **u8)

    def down_layers():
        for i, r in enumerate(rs):
            mq.mq_linear_fwd_multi(A[i], Qd, ad, zd, (r,), Y=[Y[i]], ws=ws_fd)
        for i, r in enumerate(rs):
            mq.mq_linear_bwd(A[i], Qd, ad, zd, [dY[i]], None, (r,), dX=dA[i], dW=dWd, accumulate_dW=i > 0, ws=ws_bd)

    def fused():
        mq.mq_linear_fwd_multi_gated(X, Qg, ag, zg, rs, GU=GU, A=A, ws=ws_fg)
        down_layers()
        mq.mq_linear_bwd_gated(X, Qg, ag, zg, GU, dA, None, rs, dX=dX, dW=dWgu, ws=ws_bg)

    def separate():
        mq.mq_linear_fwd_multi(X, Qg, ag, zg, rs, Y=GU, ws=ws_fg)
        mq.mq_gated_unit_fwd(GU, A=A)
        down_layers()
        mq.mq_gated_unit_bwd(GU, dA, dGU=dGU)
        mq.mq_linear_bwd(X, Qg, ag, zg, dGU, None, rs, dX=dX, dW=dWgu, ws=ws_bg)

    n = len(rs)
    # stacked layer: forward 2 n, dX 2 n, dW 2 (pre-summed); down layers: forward 2, dX 2, dW 2 per bit-width
    flops = (4.0 * n + 2.0) * M * 2 * F * d + 6.0 * n * M * d * F
    ms_f, ms_s = event_ms(torch, fused, reps), event_ms(torch, separate, reps)
    parts = {
        "stacked_fwd_with_gate_ms": round(event_ms(torch, lambda: mq.mq_linear_fwd_multi_gated(X, Qg, ag, zg, rs, GU=GU, A=A, ws=ws_fg), reps), 4),
        "stacked_fwd_ms": round(event_ms(torch, lambda: mq.mq_linear_fwd_multi(X, Qg, ag, zg, rs, Y=GU, ws=ws_fg), reps), 4),
        "gate_fwd_kernel_ms": round(event_ms(torch, lambda: mq.mq_gated_unit_fwd(GU, A=A), reps), 4),
        "stacked_bwd_with_gate_ms": round(event_ms(torch, lambda: mq.mq_linear_bwd_gated(X, Qg, ag, zg, GU, dA, None, rs, dX=dX, dW=dWgu, ws=ws_bg), reps), 4),
        "stacked_bwd_ms": round(event_ms(torch, lambda: mq.mq_linear_bwd(X, Qg, ag, zg, dGU, None, rs, dX=dX, dW=dWgu, ws=ws_bg), reps), 4),
        "gate_bwd_kernel_ms": round(event_ms(torch, lambda: mq.mq_gated_unit_bwd(GU, dA, dGU=dGU), reps), 4),
    }
    return {"M": M, "d": d, "F": F, "ms": round(ms_f, 4), "TFLOPs": round(flops / (ms_f * 1e-3) / 1e12, 1),
            "ms_with_stand_alone_gate_kernels": round(ms_s, 4), "parts": parts,
            "note": "mq_linear_fwd_multi_gated (stacked gate/up, r = 8/4/2, gate in the epilogue) + 3 x mq_linear_fwd_multi (down) + "
                    "3 x mq_linear_bwd (down) + mq_linear_bwd_gated (stacked, gate gradient in the first pass)"}


def attention_projections(torch, mq, synth, reps=3):
    """The fused r = 8/4/2 forward and the straight-through backward on attention-projection shapes of the 9B-shaped model
    (the paper also quantizes attention weights, section 5 'FFN + Attention'): a square projection d -> d and a
    grouped-query key/value projection d -> d / 4, 8192 tokens, weights N(0, 0.015^2)."""
    d, M, rs = 3584, 8192, (8, 4, 2)
    res = {"tokens": M}
    for name, N in (("d_to_d", d), ("d_to_d_over_4", d // 4)):
        g = torch.Generator().manual_seed(N)
        W = (torch.randn(N, d, generator=g) * 0.015).cuda()
        X = torch.randn(M, d, generator=g).to(torch.bfloat16).cuda()
        dY = [(torch.randn(M, N, generator=g) * 1e-3).to(torch.bfloat16).cuda() for _ in rs]
        Q, a, z = mq.mq_quantize_int8(W)
        Y = [torch.empty(M, N, dtype=torch.bfloat16, device="cuda") for _ in rs]
        ws_f = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_FWD, M, N, d, 3), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_LINEAR_BWD, M, N, d, 3), dtype=torch.uint8, device="cuda")
        dX = torch.empty(M, d, dtype=torch.bfloat16, device="cuda")
        dW = torch.empty(N, d, dtype=torch.float32, device="cuda")
        ms_f = event_ms(torch, lambda: mq.mq_linear_fwd_multi(X, Q, a, z, rs, Y=Y, ws=ws_f), reps)
        ms_b = event_ms(torch, lambda: mq.mq_linear_bwd(X, Q, a, z, dY, None, rs, dX=dX, dW=dW, ws=ws_b), reps)
        tf, tb = 6.0 * M * N * d / (ms_f * 1e-3) / 1e12, 8.0 * M * N * d / (ms_b * 1e-3) / 1e12
        res[name] = {"N": N, "K": d, "fwd_ms": round(ms_f, 4), "fwd_TFLOPs": round(tf, 1), "fwd_frac": round(tf / PEAK_BF16_TFLOPS, 4),
                     "bwd_ms": round(ms_b, 4), "bwd_TFLOPs": round(tb, 1), "bwd_frac": round(tb / PEAK_BF16_TFLOPS, 4)}
    return res


def mixnmatch_decode(torch, mq, synth):
    """Layer-wise Mix'n'Match on the decode path: a stack of eight Mistral-7B-shaped gated feed-forward layers
    (d 4096, F 14336; stacked gate/up plane 28672 x 4096, down plane 4096 x 14336) served as a pyramid
    (int2 at both ends, int8 in the middle; 4 bits per feed-forward weight on average) and homogeneously at
    int2 and int4.  Planes hold uniform random codes (the time does not depend on the values); the stack is
    captured into a HIP graph and replayed; bytes = the packed planes + parameters + activations."""
    d, F = 4096, 14336
    stacks = {"pyramid_2-2-4-8-8-4-2-2": (2, 2, 4, 8, 8, 4, 2, 2), "int2_x8": (2,) * 8, "int4_x8": (4,) * 8}
    g = torch.Generator().manual_seed(11)
    a_gu = (torch.rand(2 * F, generator=g) * 1e-4 + 5e-5).to(torch.bfloat16).cuda()
    z_gu = (torch.rand(2 * F, generator=g) * 40 + 108).to(torch.bfloat16).cuda()
    a_dn = (torch.rand(d, generator=g) * 1e-4 + 5e-5).to(torch.bfloat16).cuda()
    z_dn = (torch.rand(d, generator=g) * 40 + 108).to(torch.bfloat16).cuda()
    res = {"d": d, "F": F, "layers": 8}
    for name, rs in stacks.items():
        layers, wbytes = [], 0
        for r in rs:
            gu = torch.randint(0, 256, (2 * F, d * r // 8), generator=g, dtype=torch.int32).to(torch.uint8).cuda()
            dn = torch.randint(0, 256, (d, F * r // 8), generator=g, dtype=torch.int32).to(torch.uint8).cuda()
            layers.append(dict(gate_up=gu, down=dn, alpha_gu=a_gu, zero_gu=z_gu, alpha_dn=a_dn, zero_dn=z_dn, r=r))
            wbytes += gu.numel() + dn.numel() + 4 * (2 * F + d)
        entry = {"bits_per_weight": round(sum(rs) / len(rs), 3), "weight_MB": round(wbytes / 1e6, 1)}
        for B in (1, 4, 16):
            x = synth.activations(4, f"mnm{B}", B, d).cuda()
            y = torch.empty(B, d, dtype=torch.bfloat16, device="cuda")
            ws = torch.empty(mq.mq_workspace_bytes(mq.MQ_OP_FFN_DECODE, B, F, d, 1), dtype=torch.uint8, device="cuda")
            mq.mq_ffn_mixnmatch(x, layers, F, residual=True, y=y, ws=ws)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                mq.mq_ffn_mixnmatch(x, layers, F, residual=True, y=y, ws=ws)
            graph.replay()
            torch.cuda.synchronize()
            times = []
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                graph.replay()
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            del graph
            ms = sorted(times)[2]
            nbytes = wbytes + len(rs) * B * 2 * (2 * d + 3 * F + 2 * F + 2 * d)   # states, g/u, gated product: written and read
            entry[f"B{B}"] = {"us_per_layer": round(ms * 1e3 / len(rs), 2), "GBs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                              "frac": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        res[name] = entry
        del layers
    res["note"] = ("one mq_ffn_mixnmatch call (two GEMV launches per layer: gate activation and residual add run in their epilogues) from a HIP-graph "
                   "replay; every stack exceeds the 256 MB last-level cache except int2_x8 (352 MB of planes: it does too)")
    return res


def cpu_baseline(torch, synth):
    """The CPU oracle as it stands, timed on the host cores of the box on a bounded sample of the same work:
    configuration 1 in full, the decode GEMVs of configuration 4 in full, quantize + slice + pack of one whole
    matrix (gate) of configurations 2, 3 and 5, and the fp64 contractions of the gate linear of configurations 2, 3, 5
    on a slab (forward: all tokens x 256 channels per bit-width; dX: 128 tokens x all channels; dW: 256 weight
    rows x all tokens), extrapolated linearly to the full layer.  `value` is the oracle's fused-forward rate
    on the headline workload (configuration 3 slab)."""
    import numpy as np
    import oracle

    def bits(t):
        return t.contiguous().view(torch.int16).numpy().view(np.uint16)

    def clock(fn):
        t0 = time.perf_counter()
        r = fn()
        return time.perf_counter() - t0, r

    rs = (8, 4, 2)
    res = {}
    # configuration 1, every operation of the path in full
    c1 = synth.linear_case(1)
    t_q, (q, a, z) = clock(lambda: oracle.quantize_int8(c1.W.numpy()))
    t_s, _ = clock(lambda: [oracle.pack(oracle.slice_codes(q, r), r) for r in (4, 2)])
    xb, dyb = bits(c1.X), [bits(d) for d in c1.dY]
    t_f, _ = clock(lambda: [oracle.linear_fwd(xb, q, a, z, r) for r in rs])
    t_b, _ = clock(lambda: (oracle.linear_bwd_dx(q, a, z, dyb, c1.lambdas, rs), oracle.linear_bwd_dw(xb, dyb, c1.lambdas)))
    res["config1_full"] = {"quantize_ms": round(t_q * 1e3, 3), "slice_pack_ms": round(t_s * 1e3, 3),
                           "fwd_r842_ms": round(t_f * 1e3, 3), "bwd_ms": round(t_b * 1e3, 3)}
    # configuration 4: the decode GEMVs in full (r = 4, 2; B = 1, 4, 16)
    gemv = {}
    for (N, K) in synth.DECODE_SHAPES:
        W = synth.weight(4, f"{N}x{K}", (N, K)).numpy()
        q, a, z = oracle.quantize_int8(W)
        a16 = bits(torch.from_numpy(a).to(torch.bfloat16))
        z16 = bits(torch.from_numpy(z).to(torch.bfloat16))
        for r in (4, 2):
            plane = oracle.pack(oracle.slice_codes(q, r), r)
            for B in (1, 4, 16):
                x = bits(synth.activations(4, f"x{B}:{N}x{K}", B, K))
                t, _ = clock(lambda: oracle.gemv_sliced(x, plane, a16, z16, r, K))
                nbytes = N * K * r // 8 + 4 * N + 2 * B * K + 2 * B * N
                gemv[f"int{r}_{N}x{K}_B{B}"] = {"ms": round(t * 1e3, 2), "GBs": round(nbytes / t / 1e9, 3)}
    res["config4_gemv_full"] = gemv
    # quantize + slice + pack of a whole matrix, and the contractions on a slab, per configuration
    SLAB, SLAB_DX = 256, 128
    value = None
    for cfg in (2, 3, 5):
        case = synth.linear_case(cfg, "gate", with_grads=False, M=None)
        M, N, K = case.M, case.N, case.K
        t_q, (q, a, z) = clock(lambda: oracle.quantize_int8(case.W.numpy()))
        t_s, _ = clock(lambda: [oracle.pack(oracle.slice_codes(q, r), r) for r in (4, 2)])
        entry = {"shape": f"gate {N}x{K}, {M} tokens", "quantize_full_s": round(t_q, 3), "slice_pack_r4_r2_full_s": round(t_s, 3),
                 "quantize_GBs": round(5.0 * N * K / t_q / 1e9, 2), "slice_pack_GBs": round(2.75 * N * K / t_s / 1e9, 3)}
        xb = bits(case.X)
        t_f, _ = clock(lambda: [oracle.linear_fwd(xb, q[:SLAB], a[:SLAB], z[:SLAB], r) for r in rs])
        lam = synth.LAMBDAS[cfg]
        dY = [(torch.randn(SLAB_DX, N, generator=torch.Generator().manual_seed(i)) * 1e-3).to(torch.bfloat16) for i in range(3)]
        t_dx, _ = clock(lambda: oracle.linear_bwd_dx(q, a, z, [bits(d) for d in dY], lam, rs))
        dYw = [(torch.randn(M, SLAB, generator=torch.Generator().manual_seed(7 + i)) * 1e-3).to(torch.bfloat16) for i in range(3)]
        t_dw, _ = clock(lambda: oracle.linear_bwd_dw(xb, [bits(d) for d in dYw], lam))
        f_fwd, f_dx, f_dw = 6.0 * M * SLAB * K, 6.0 * SLAB_DX * N * K, 2.0 * M * SLAB * K
        entry.update({
            "fwd_slab": f"all {M} tokens x {SLAB} of {N} channels, r = 8/4/2", "fwd_slab_s": round(t_f, 3),
            "fwd_TFLOPs": round(f_fwd / t_f / 1e12, 5), "fwd_full_layer_s_extrapolated": round(t_f * N / SLAB, 1),
            "dX_slab": f"{SLAB_DX} of {M} tokens x all channels", "dX_slab_s": round(t_dx, 3),
            "dX_full_layer_s_extrapolated": round(t_dx * M / SLAB_DX, 1),
            "dW_slab": f"{SLAB} of {N} weight rows x all tokens", "dW_slab_s": round(t_dw, 3),
            "dW_full_layer_s_extrapolated": round(t_dw * N / SLAB, 1),
            "bwd_TFLOPs": round((f_dx + f_dw) / (t_dx + t_dw) / 1e12, 5)})
        res[f"config{cfg}_gate"] = entry
        if cfg == 3:
            value = f_fwd / t_f / 1e12
        del case, q, xb
    return {"value": round(value, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "fused r=8/4/2 forward of the configs[2] gate linear (8192 tokens, 14336 x 3584) on a slab of 256 of its "
                      "14336 output channels (all tokens, fp64 accumulation); full-layer times in `detail` are linear "
                      "extrapolations of the slabs and labelled so; configuration 1 and the configuration-4 GEMVs ran in full, "
                      "quantize/slice/pack ran on a whole matrix of configurations 2, 3 and 5",
            "detail": res}


if __name__ == "__main__":
    main()
