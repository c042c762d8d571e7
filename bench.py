#!/usr/bin/env python3
"""Benchmark of the reversible-stack hot path on one MI355X.

One step = revnet_stack_fwd + revnet_stack_bwd (reconstructing backward) over
one synthetic batch that is already resident in HBM.  Default workload: the
9-block basic stack at N=128, C=32 (16+16), 32x32, fp32 ("c2_stack9").

Prints ONE JSON line: images/s, the roofline of the dominant kernel (per-launch
duration measured with HIP events on the launch stream, in a separate profiled
pass of the same steps), the CPU oracle timed beside it on a bounded sample,
peak activation bytes versus depth and reconstruction error versus depth.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks.
PEAK = {"hbm": (8000.0, "GB/s"), "mfma_f32": (157.3, "TFLOP/s"), "mfma_bf16": (2500.0, "TFLOP/s"),
        "alu_f32": (157.3, "TFLOP/s")}

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs (profiles/), keyed by (workload, kernel family); None = not measured.
MEASURED_TRAFFIC = {
    # conv_mfma_f32_k at c2_stack9: (FETCH_SIZE 7108.5 KiB x 2.0 + WRITE_SIZE 8448.0 KiB x 1.0) per dispatch,
    # averaged over forward and recompute launches (profiles/c2_stack9_hbm_traffic.txt)
    ("c2_stack9", "conv_fwd"): 23207351,
    # c4_bneck12: conv1x1_bf16_k (128->64), conv3x3_bf16_k, conv1x1_bf16_k (64->128), same averaging
    # (profiles/c4_bneck12_hbm_traffic.txt)
    ("c4_bneck12", "conv_fwd"): 183077628,
    # c5_stage3: the two conv1x1_bf16_k shapes and conv3x3_bf16_k + its splitk_reduce_k
    # (profiles/c5_stage3_hbm_traffic.txt)
    ("c5_stage3", "conv_fwd"): 52837304,
}


def bound_of(family: str, conv: str, flops: float, nbytes: float):
    """Which roof a kernel family is held against: a convolution family whose
    algorithmic flops per algorithmic byte (summed over its launches in this
    workload) lie above the ridge of its matrix unit is matrix-bound, every
    other kernel is bound by HBM."""
    if family in ("conv_fwd", "conv_dgrad", "conv_wgrad", "conv_dgrad_wgrad"):
        key = "mfma_bf16" if conv == "bf16" else "mfma_f32"
        ridge = PEAK[key][0] * 1e12 / (PEAK["hbm"][0] * 1e9)
        if nbytes > 0 and flops / nbytes >= ridge:
            return ("mfma", key)
    return ("hbm", "hbm")


def profiled_pass(rv, torch, step, steps, conv, workload):
    """Per-kernel durations with HIP events on the launch stream, and the
    roofline entry of the kernel family that takes the most time."""
    rv.revnet_profile_begin()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    stats = rv.revnet_profile_end()
    kern = {}
    for name, st in stats.items():
        avg_us = st["total_ms"] * 1e3 / st["launches"]
        kern[name] = dict(launches_per_step=st["launches"] / steps, avg_us=round(avg_us, 3),
                          ms_per_step=round(st["total_ms"] / steps, 4),
                          GBps=round(st["algorithmic_bytes"] / st["total_ms"] / 1e6, 1) if st["total_ms"] else None,
                          TFLOPs=round(st["flops"] / st["total_ms"] / 1e9, 2) if st["flops"] else None)
    dom = max(stats, key=lambda k: stats[k]["total_ms"])
    bound, peak_key = bound_of(dom, conv, stats[dom]["flops"], stats[dom]["algorithmic_bytes"])
    peak, unit = PEAK[peak_key]
    d = stats[dom]
    per_launch_s = d["total_ms"] * 1e-3 / d["launches"]
    quantity = (d["flops"] / 1e12 if bound != "hbm" else d["algorithmic_bytes"] / 1e9) / d["launches"]
    achieved = quantity / per_launch_s
    roofline = dict(bound=bound, kernel=dom, achieved=round(achieved, 2), peak=peak, unit=unit,
                    frac=round(achieved / peak, 4), avg_launch_us=round(per_launch_s * 1e6, 3),
                    traffic=MEASURED_TRAFFIC.get((workload, dom)))
    return kern, roofline


def timed_steps(torch, step, steps, warmup, stream):
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return max((t1 - t0) * 1e3 / steps, ev0.elapsed_time(ev1) / steps)


def bench_body(args) -> int:
    """A multi-stage body (reversible stages joined by subsampling blocks): one
    step = body forward, then body backward from the stage tops alone."""
    import numpy as np
    import torch
    import synth_inputs as S
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import BodyRunner, NetRunner, _dev
    is_net = args.workload in S.NETS
    torch.cuda.reset_peak_memory_stats()
    if is_net:
        seed = S.BASE_SEED + 200 + list(S.NETS).index(args.workload)
        cfg, x, stem, stages, downs, dy = S.draw_net(seed, **S.NETS[args.workload])   # x: the image batch
        cfg["frac_bits"] = args.frac_bits
        net = NetRunner(cfg, stem)
        r = net.body
        net.set_params(stages, downs)
    else:
        cfg = dict(S.BODIES[args.workload])
        seed = S.BASE_SEED + 100 + list(S.BODIES).index(args.workload)
        x, stages, downs, dy = S.draw_body(seed, **cfg)
        stem = None
        cfg["frac_bits"] = args.frac_bits
        r = BodyRunner(**cfg)
        r.set_params(stages, downs)
    n, conv = cfg["n"], cfg["conv"]
    base_alloc = torch.cuda.memory_allocated()
    X, DY = _dev(x, r.device), _dev(dy, r.device)
    stream = torch.cuda.current_stream()

    def step():
        if is_net:
            net.forward(X, stream)       # image -> stem -> top of every stage
        else:
            r.forward(X, stream)         # x -> top of every stage
        r.dtops[-1].copy_(DY)            # the derivative arriving at the last stage's top
        if is_net:
            net.backward(stream)         # ... down to the stem's filter gradient
        else:
            r.backward(stream=stream)    # tops reconstructed in place, dtops[0] = derivative at the input

    ms_per_step = timed_steps(torch, step, args.steps, args.warmup, stream)
    kern, roofline = profiled_pass(rv, torch, step, args.steps, conv, args.workload)
    if is_net:   # the body's input is the stem's output: compare the reconstruction with a fresh stem forward
        ref0 = torch.empty_like(r.tops[0])
        rv.revnet_stem_fwd(net.stem_desc, X, net.stem_w, net.conv_out, ref0, stream)
        torch.cuda.synchronize()
        x0 = ref0.cpu().numpy().astype(np.float64)
    else:
        x0 = x
    if args.frac_bits:   # codes of the reconstructed stage-0 input against the encoded input
        enc = torch.empty_like(r.tops[0])
        rv.revnet_fixed_from_float(_dev(x0, r.device), args.frac_bits, enc, stream)
        torch.cuda.synchronize()
        rec = "exact" if torch.equal(enc.view(torch.int32), r.tops[0].view(torch.int32)) else "NOT exact"
    else:
        rec = float(np.linalg.norm(r.tops[0].cpu().numpy().astype(np.float64) - x0) / np.linalg.norm(x0))
    act = net.activation_bytes() if is_net else r.activation_bytes()
    shallow = BodyRunner(**dict(cfg, depths=tuple(1 for _ in cfg["depths"]))).activation_bytes()
    cfg.pop("frac_bits")
    out = {
        "metric": "images/sec reversible fwd+bwd per stack on 1 MI355X; peak activation HBM bytes",
        "value": round(n / (ms_per_step * 1e-3), 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if conv == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "kind": cfg["kind"], "n": n, "h": cfg["h"], "w": cfg["w"],
                   "channels": list(cfg["channels"]), "depths": list(cfg["depths"]), "widths": list(cfg["widths"]),
                   "conv_operands": conv,
                   "residual_stream": f"fixed point, {args.frac_bits} fraction bits" if args.frac_bits else "fp32",
                   "stem": (f"{stem['w'].shape[2]}x{stem['w'].shape[2]} stride {stem['stride']} convolution of a 3-channel "
                            f"{x.shape[2]}x{x.shape[3]} image" + (", 3x3 stride-2 max-pooling" if stem["pool"] else "") + ", fp32")
                   if is_net else "not part of the body: it starts at the stem's output"},
        "roofline": roofline,
        "kernels": kern,
        "peak_activation_bytes": {"analytic": act, "same_body_one_block_per_stage": shallow,
                                  "torch_max_allocated_over_params_and_inputs": int(torch.cuda.max_memory_allocated() - base_alloc)},
        "body_input_reconstruction_rel_error": rec,
    }
    if not args.no_cpu_baseline:
        from oracle import revnet_oracle as O
        O.build()

        def oracle_pass(ns):
            with O.conv_operands(conv):
                t0 = time.perf_counter()
                xin = x[:ns]
                if is_net:
                    xin, kept_stem = O.stem_fwd(xin, stem)
                _, kept = O.body_fwd(xin, stages, downs, keep=True)
                d0, _, _ = O.body_bwd_stored(kept, stages, downs, dy[:ns])
                if is_net:
                    O.stem_bwd(kept_stem, stem, d0)
                return time.perf_counter() - t0

        ns = min(args.cpu_sample_n, n) if args.cpu_sample_n else min(2, n)
        secs, passes = 0.0, 0
        while passes == 0 or (secs < 10.0 and passes < 8):
            secs += oracle_pass(ns)
            passes += 1
        out["cpu_baseline"] = {"value": round(ns * passes / secs, 2), "unit": "images/s", "cores": O.num_threads(),
                               "kind": "oracle", "seconds": round(secs, 2),
                               "sample": f"first {ns} of {n} images, same stages, {passes} pass(es) of one forward + "
                                         "stored-activation backward in float64"}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_stack9")
    ap.add_argument("--frac-bits", type=int, default=0,
                    help="keep the residual stream in fixed point with this many fraction bits (exact reconstruction); "
                         "0 = floating-point stream, the benchmark configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-n", type=int, default=0,
                    help="batch of the oracle timing sample (0: the whole batch if one pass takes under ~30 s, "
                         "else the largest power-of-two fraction that does)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run a plain elementwise copy of this many MiB (read + write that many each), "
                         "the reference reading for rocprofv3 FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import synth_inputs as S
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    rv.load_library()  # fails loudly if the HIP library is missing
    if args.workload in S.BODIES or args.workload in S.NETS:
        return bench_body(args)

    cfg, x, params, dy = S.draw_named(args.workload)
    n, c, h, w, depth, conv = cfg["n"], cfg["c"], cfg["h"], cfg["w"], cfg["depth"], cfg["conv"]
    r = StackRunner(frac_bits=args.frac_bits, **cfg)
    r.set_params(params)
    torch.cuda.reset_peak_memory_stats()
    base_alloc = torch.cuda.memory_allocated()
    X, DY = r.new_stream_pair(x), r.new_pair(dy)     # inputs, read only in every step
    Y, DX = r.new_stream_pair(), r.new_pair()        # top activations (reconstructed in place), gradients
    stream = torch.cuda.current_stream()

    def step():
        r.forward(X, Y, stream)               # x -> y, nothing else kept
        r.backward(Y, DY, Y, DX, stream=stream)   # y -> x in place; dy -> dx

    ms_per_step = timed_steps(torch, step, args.steps, args.warmup, stream)
    peak_alloc = torch.cuda.max_memory_allocated() - base_alloc

    # ---- the two halves of a step on their own (Section 3.2 "Computational overhead": forward N,
    #      reversible backward 3N, i.e. 4N against the 3N of backprop from stored activations)
    ms_forward = timed_steps(torch, lambda: r.forward(X, Y, stream), args.steps, 1, stream)
    r.forward(X, Y, stream)

    def bwd_only():      # Y is reconstructed in place to x, so run forward untimed to restore it
        r.backward(Y, DY, Y, DX, stream=stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ms_backward = 0.0
    for _ in range(args.steps):
        ev[0].record(stream)
        bwd_only()
        ev[1].record(stream)
        r.forward(X, Y, stream)
        torch.cuda.synchronize()
        ms_backward += ev[0].elapsed_time(ev[1]) / args.steps

    kern, roofline = profiled_pass(rv, torch, step, args.steps, conv, args.workload)

    if args.copy_probe_mib:
        src = torch.empty(args.copy_probe_mib * (1 << 20) // 4, dtype=torch.float32, device=r.device).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)   # one elementwise kernel: reads and writes copy_probe_mib MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- the same totals against the rooflines, whole step
    fwd_cost, bwd_cost = rv.revnet_stack_cost(r.desc, depth, n, h, w)
    step_flops = fwd_cost["conv_flops"] + bwd_cost["conv_flops"]
    step_bytes = fwd_cost["algorithmic_bytes"] + bwd_cost["algorithmic_bytes"]

    # ---- reconstruction error versus depth (input of block k, top block first)
    drift = None
    if args.frac_bits:
        drift = "exact" if torch.equal(X[0], Y[0]) else "NOT exact"   # integer codes of the input against the reconstruction
    elif depth > 1:
        drift = []
        fwd_only = []
        cur = r.new_pair(x)
        nxt = r.new_pair()
        for k in range(depth):               # block inputs from a forward pass, one block at a time
            fwd_only.append(r.to_host(cur[0]).astype(np.float32))
            rv.revnet_block_fwd(r.desc, cur[1], cur[2], r.params[k], nxt[1], nxt[2], r.ws, stream)
            cur, nxt = nxt, cur
        G = r.new_pair(dy)
        for k in range(depth - 1, -1, -1):
            rv.revnet_block_bwd_reconstruct(r.desc, cur[1], cur[2], G[1], G[2], r.params[k], cur[1], cur[2],
                                            G[1], G[2], r.grads[k], 0, r.ws, stream)
            torch.cuda.synchronize()
            rec = r.to_host(cur[0])
            ref = fwd_only[k].astype(np.float64)
            drift.append(float(np.linalg.norm(rec - ref) / np.linalg.norm(ref)))

    # ---- activation memory versus depth (the workspace query has no depth argument)
    act = r.activation_bytes()
    act_vs_depth = {}
    esz = 2 if conv == "bf16" else 4
    per_block_stored = 2 * sum(n * h * w * cin * (4 + esz) for cin, _, _ in S.func_layers(cfg["kind"], c // 2, cfg["width"]))
    for dd in (1, 2, 4, 9, 18, 36):
        query = rv.revnet_fixed_workspace_bytes if args.frac_bits else rv.revnet_workspace_bytes
        assert query(r.desc, n, h, w) == (r.fwd_bytes, r.bwd_bytes)
        act_vs_depth[str(dd)] = {"reversible": act["total"],
                                 "stored_activation_backprop": 2 * act["stream"] + dd * per_block_stored}

    out = {
        "metric": "images/sec reversible fwd+bwd per stack on 1 MI355X; peak activation HBM bytes",
        "value": round(n / (ms_per_step * 1e-3), 1),
        "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_forward": round(ms_forward, 4), "ms_backward": round(ms_backward, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if conv == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload, "kind": cfg["kind"], "n": n, "c": c, "h": h, "w": w,
                   "depth": depth, "width": cfg["width"], "conv_operands": conv,
                   "residual_stream": f"fixed point, {args.frac_bits} fraction bits" if args.frac_bits else "fp32"},
        "roofline": roofline,
        "step_totals": {"note": "launch and byte totals are those of the fp32-stream path" if args.frac_bits else None,
                        "conv_TFLOP": round(step_flops / 1e12, 4), "algorithmic_GB": round(step_bytes / 1e9, 3),
                        "kernel_launches": fwd_cost["kernel_launches"] + bwd_cost["kernel_launches"],
                        "achieved_TFLOPs": round(step_flops / 1e12 / (ms_per_step * 1e-3), 2),
                        "achieved_GBps": round(step_bytes / 1e9 / (ms_per_step * 1e-3), 1)},
        "kernels": kern,
        "peak_activation_bytes": {"analytic": act, "torch_max_allocated_over_params": int(peak_alloc),
                                  "vs_depth": act_vs_depth},
        "reconstruction_rel_error_top_block_first": drift,
    }

    if not args.no_cpu_baseline:
        from oracle import revnet_oracle as O
        c2 = c // 2
        sp = lambda t: (np.ascontiguousarray(t[:, :c2]), np.ascontiguousarray(t[:, c2:]))
        O.build()

        def oracle_pass(ns):
            with O.conv_operands(conv):
                t0 = time.perf_counter()
                if args.frac_bits:
                    q1, q2 = (O.fixed_encode(t, args.frac_bits) for t in sp(x[:ns]))
                    _, _, stored = O.stack_fwd_fixed(q1, q2, params, args.frac_bits, keep=True)
                else:
                    _, _, _, stored = O.stack_fwd(*sp(x[:ns]), params, keep=True)
                O.stack_bwd_stored(stored, params, *sp(dy[:ns]))
                return time.perf_counter() - t0

        # Bounded sample: 10-30 s of oracle work.  Probe on 2 images, then take the
        # largest batch that one pass finishes in ~30 s and repeat it up to ~10 s.
        ns = min(args.cpu_sample_n, n) if args.cpu_sample_n else n
        if not args.cpu_sample_n:
            per_image = oracle_pass(min(2, n)) / min(2, n)
            while ns > 1 and per_image * ns > 30.0:
                ns //= 2
        secs, passes = 0.0, 0
        while passes == 0 or (secs < 10.0 and passes < 8):
            secs += oracle_pass(ns)
            passes += 1
        out["cpu_baseline"] = {"value": round(ns * passes / secs, 2), "unit": "images/s", "cores": O.num_threads(),
                               "kind": "oracle", "seconds": round(secs, 2),
                               "sample": f"first {ns} of {n} images, same C/H/W/depth, {passes} pass(es) of one "
                                         "forward + stored-activation backward in float64"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
