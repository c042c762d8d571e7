#!/usr/bin/env python3
"""Benchmark of the reversible hot path on one MI355X.

One step = forward + reconstructing backward (revnet_stack_fwd + revnet_stack_bwd,
or the body / whole-network equivalents) over one synthetic batch that is already
resident in HBM.  Default workload: the 12-block bottleneck stack at N=64, C=256
(128+128), inner width 64, 56x56, bf16 convolution operands with fp32
accumulation ("c4_bneck12"), the largest single-stack workload.

Prints ONE JSON line: images/s of the primary workload, the roofline of its
dominant kernel family (per-launch duration measured with HIP events on the
launch stream, in a separate profiled pass of the same steps), the CPU oracle
timed beside it on a bounded sample (stored-activation backprop, and the
literal Algorithm 1), peak activation bytes versus depth, reconstruction error
versus depth, and under "secondary" the same throughput / roofline figures for
the fp32 stack and the two multi-stage bodies.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "images/sec reversible fwd+bwd per stack on 1 MI355X; peak activation HBM bytes"

# MI355X published peaks.  alu_f32: 256 compute units x 64 lanes x 2 flop x 2.4 GHz; the 157.3 figure
# of the data sheet counts packed fp32 instructions, which this library is built without.
PEAK = {"hbm": (8000.0, "GB/s"), "mfma_f32": (157.3, "TFLOP/s"), "mfma_bf16": (2500.0, "TFLOP/s"),
        "alu_f32": (78.6, "TFLOP/s")}

SECONDARY = ("c2_stack9", "c3_body", "c5_body")


def measured_traffic(workload: str, family: str):
    """HBM bytes per launch of a kernel family from the rocprofv3 counter summary
    profiles/<workload>_hbm_traffic.txt (a line `family <name> <bytes per launch>`);
    None if that workload or family has not been measured."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                m = re.match(r"\s*family\s+(\S+)\s+(\d+)", line)
                if m and m.group(1) == family:
                    return int(m.group(2))
    except OSError:
        pass
    return None


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
                    algorithmic_bytes_per_launch=round(d["algorithmic_bytes"] / d["launches"]),
                    traffic=measured_traffic(workload, dom))
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


def tensor_bytes(*ts):
    return sum(t.numel() * t.element_size() for t in ts)


def params_bytes(tree):
    if hasattr(tree, "numel"):
        return tree.numel() * tree.element_size()
    if isinstance(tree, dict):
        return sum(params_bytes(v) for v in tree.values())
    if isinstance(tree, (list, tuple)):
        return sum(params_bytes(v) for v in tree)
    return 0


def dtype_label(conv):
    return "f32" if conv == "f32" else "bf16 operands, fp32 accumulate"


def oracle_sample(run_pass, n, sample_n, what):
    """Time `run_pass(ns)` on a bounded sample: the largest batch (halving from n)
    that one pass finishes in about 30 s, repeated up to about 10 s."""
    ns = min(sample_n, n) if sample_n else n
    if not sample_n:
        probe = min(2, n)
        per_image = run_pass(probe) / probe
        while ns > 1 and per_image * ns > 30.0:
            ns //= 2
    secs, passes = 0.0, 0
    while passes == 0 or (secs < 10.0 and passes < 8):
        secs += run_pass(ns)
        passes += 1
    return dict(value=round(ns * passes / secs, 2), unit="images/s", seconds=round(secs, 2),
                sample=f"first {ns} of {n} images, same shapes and depths, {passes} pass(es) of {what}")


def copy_probe(args, torch, device):
    """--copy-probe-mib M: one elementwise kernel that reads and writes M MiB, the known-size
    copy that the HBM counters of a rocprofv3 run are scaled by."""
    if not args.copy_probe_mib:
        return
    src = torch.empty(args.copy_probe_mib * (1 << 20) // 4, dtype=torch.float32, device=device).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()
    del src, dst


def bench_body(args, workload, primary) -> dict:
    """A multi-stage body or whole network (reversible stages joined by subsampling
    blocks, optionally behind the stem): one step = forward, then backward from
    the stage tops alone."""
    import numpy as np
    import torch
    import synth_inputs as S
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import BodyRunner, NetRunner, _dev
    is_net = workload in S.NETS
    frac_bits = args.frac_bits if primary else 0
    base0 = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    if is_net:
        seed = S.BASE_SEED + 200 + list(S.NETS).index(workload)
        cfg, x, stem, stages, downs, dy = S.draw_net(seed, **S.NETS[workload])   # x: the image batch
        cfg["frac_bits"] = frac_bits
        net = NetRunner(cfg, stem)
        r = net.body
        net.set_params(stages, downs)
    else:
        cfg = dict(S.BODIES[workload])
        seed = S.BASE_SEED + 100 + list(S.BODIES).index(workload)
        x, stages, downs, dy = S.draw_body(seed, **cfg)
        stem = None
        cfg["frac_bits"] = frac_bits
        r = BodyRunner(**cfg)
        r.set_params(stages, downs)
    n, conv = cfg["n"], cfg["conv"]
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
    peak = torch.cuda.max_memory_allocated() - base0
    kern, roofline = profiled_pass(rv, torch, step, args.steps, conv, workload)
    out = {"value": round(n / (ms_per_step * 1e-3), 1), "unit": "images/s", "ms_per_step": round(ms_per_step, 4),
           "dtype": dtype_label(conv), "roofline": roofline}
    if not primary:
        out["kernels_ms_per_step"] = {k: v["ms_per_step"] for k, v in kern.items()}
        return out

    copy_probe(args, torch, r.device)
    if is_net:   # the body's input is the stem's output: compare the reconstruction with a fresh stem forward
        ref0 = torch.empty_like(r.tops[0])
        rv.revnet_stem_fwd(net.stem_desc, X, net.stem_w, net.conv_out, ref0, stream)
        torch.cuda.synchronize()
        x0 = ref0.cpu().numpy().astype(np.float64)
    else:
        x0 = x
    if frac_bits:   # codes of the reconstructed stage-0 input against the encoded input
        enc = torch.empty_like(r.tops[0])
        rv.revnet_fixed_from_float(_dev(x0, r.device), frac_bits, enc, stream)
        torch.cuda.synchronize()
        rec = "exact" if torch.equal(enc.view(torch.int32), r.tops[0].view(torch.int32)) else "NOT exact"
    else:
        rec = float(np.linalg.norm(r.tops[0].cpu().numpy().astype(np.float64) - x0) / np.linalg.norm(x0))
    act = net.activation_bytes() if is_net else r.activation_bytes()
    shallow = BodyRunner(**dict(cfg, depths=tuple(1 for _ in cfg["depths"]))).activation_bytes()
    # what the step keeps on the device besides parameters, their gradients and the two source tensors
    # (the input batch and the upstream derivative): the stage tops, their derivatives, the workspace
    held = params_bytes([r.stage_params, r.down_params, r.stage_grads, r.down_grads]) + tensor_bytes(X, DY)
    if is_net:
        held += tensor_bytes(net.stem_w, net.stem_dw)
        act["stem_input_is_the_source_batch"] = tensor_bytes(X)
        act["total_without_source_batch"] = act["total"] - tensor_bytes(X)
    cfg.pop("frac_bits")
    out.update({
        "config": {"workload": workload, "kind": cfg["kind"], "n": n, "h": cfg["h"], "w": cfg["w"],
                   "channels": list(cfg["channels"]), "depths": list(cfg["depths"]), "widths": list(cfg["widths"]),
                   "conv_operands": conv,
                   "residual_stream": f"fixed point, {frac_bits} fraction bits" if frac_bits else "fp32",
                   "stem": (f"{stem['w'].shape[2]}x{stem['w'].shape[2]} stride {stem['stride']} convolution of a 3-channel "
                            f"{x.shape[2]}x{x.shape[3]} image" + (", 3x3 stride-2 max-pooling" if stem["pool"] else "") + ", fp32")
                   if is_net else "not part of the body: it starts at the stem's output"},
        "kernels": kern,
        "peak_activation_bytes": {"analytic": act, "same_body_one_block_per_stage": shallow,
                                  "measured_max_allocated_minus_parameters_and_sources": int(peak - held)},
        "body_input_reconstruction_rel_error": rec,
    })
    if not args.no_cpu_baseline:
        from oracle import revnet_oracle as O
        O.build()

        def stored_pass(ns):
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

        def reversible_pass(ns):
            with O.conv_operands(conv):
                t0 = time.perf_counter()
                xin = x[:ns]
                if is_net:
                    xin, kept_stem = O.stem_fwd(xin, stem)
                tops = O.body_fwd(xin, stages, downs)
                d0 = O.body_reverse(tops, stages, downs, dy[:ns])[0]
                if is_net:
                    O.stem_bwd(kept_stem, stem, d0)
                return time.perf_counter() - t0

        ns = args.cpu_sample_n or min(2, n)
        base = oracle_sample(stored_pass, n, ns, "one forward + stored-activation backward in float64")
        lit = oracle_sample(reversible_pass, n, ns, "one forward + the memory-saving backward pass (Algorithm 1 inside the stages) in float64")
        out["cpu_baseline"] = dict(base, cores=O.num_threads(), kind="oracle", algorithm1_literal=lit)
    return out


def bench_stack(args, workload, primary) -> dict:
    import numpy as np
    import torch
    import synth_inputs as S
    import paper_1707_04585_amd as rv
    from paper_1707_04585_amd.torch_harness import StackRunner

    frac_bits = args.frac_bits if primary else 0
    cfg, x, params, dy = S.draw_named(workload)
    n, c, h, w, depth, conv = cfg["n"], cfg["c"], cfg["h"], cfg["w"], cfg["depth"], cfg["conv"]
    base0 = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    r = StackRunner(frac_bits=frac_bits, **cfg)
    r.set_params(params)
    X, DY = r.new_stream_pair(x), r.new_pair(dy)     # the two source tensors, read only in every step
    Y, DX = r.new_stream_pair(), r.new_pair()        # top activations (reconstructed in place), gradients
    stream = torch.cuda.current_stream()

    def step():
        r.forward(X, Y, stream)               # x -> y, nothing else kept
        r.backward(Y, DY, Y, DX, stream=stream)   # y -> x in place; dy -> dx

    ms_per_step = timed_steps(torch, step, args.steps, args.warmup, stream)
    peak_alloc = torch.cuda.max_memory_allocated() - base0
    out = {"value": round(n / (ms_per_step * 1e-3), 1), "unit": "images/s", "ms_per_step": round(ms_per_step, 4),
           "dtype": dtype_label(conv)}

    # ---- the two halves of a step on their own (Section 3.2 "Computational overhead": forward N,
    #      reversible backward 3N, i.e. 4N against the 3N of backprop from stored activations)
    ms_forward = timed_steps(torch, lambda: r.forward(X, Y, stream), args.steps, 1, stream)
    r.forward(X, Y, stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ms_backward = 0.0
    for _ in range(args.steps):      # Y is reconstructed in place to x, so run forward untimed to restore it
        ev[0].record(stream)
        r.backward(Y, DY, Y, DX, stream=stream)
        ev[1].record(stream)
        r.forward(X, Y, stream)
        torch.cuda.synchronize()
        ms_backward += ev[0].elapsed_time(ev[1]) / args.steps
    out.update(ms_forward=round(ms_forward, 4), ms_backward=round(ms_backward, 4))

    kern, roofline = profiled_pass(rv, torch, step, args.steps, conv, workload)
    out["roofline"] = roofline
    if not primary:
        out["kernels_ms_per_step"] = {k: v["ms_per_step"] for k, v in kern.items()}
        return out

    copy_probe(args, torch, r.device)

    # ---- the same totals against the rooflines, whole step
    fwd_cost, bwd_cost = rv.revnet_stack_cost(r.desc, depth, n, h, w)
    step_flops = fwd_cost["conv_flops"] + bwd_cost["conv_flops"]
    step_bytes = fwd_cost["algorithmic_bytes"] + bwd_cost["algorithmic_bytes"]

    # ---- reconstruction error versus depth (input of block k, top block first)
    drift = None
    if frac_bits:
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
        del cur, nxt, G

    # ---- activation memory versus depth (the workspace query has no depth argument).
    #      Alive between the end of forward and the end of backward in this harness: the top pair Y, the
    #      upstream derivative DY and the derivative DX it is turned into (an in-place call lets DX be DY
    #      and needs one stream-sized tensor less), the backward workspace.  The measured figure is the
    #      peak device allocation minus parameters, their gradients and the input batch X.
    act = r.activation_bytes()
    s = act["stream"]
    analytic = dict(stream=s, upstream_derivative=s, derivative_out=s, workspace=r.bwd_bytes,
                    total=3 * s + max(r.fwd_bytes, r.bwd_bytes), total_with_derivatives_in_place=act["total"])
    measured = int(peak_alloc - params_bytes([r.params, r.grads]) - tensor_bytes(X[0]))
    act_vs_depth = {}
    esz = 2 if conv == "bf16" else 4
    per_block_stored = 2 * sum(n * h * w * cin * (4 + esz) for cin, _, _ in S.func_layers(cfg["kind"], c // 2, cfg["width"]))
    for dd in (1, 2, 4, 9, 18, 36):
        query = rv.revnet_fixed_workspace_bytes if frac_bits else rv.revnet_workspace_bytes
        assert query(r.desc, n, h, w) == (r.fwd_bytes, r.bwd_bytes)
        act_vs_depth[str(dd)] = {"reversible": act["total"],
                                 "stored_activation_backprop": 2 * act["stream"] + dd * per_block_stored}

    out.update({
        "config": {"workload": workload, "kind": cfg["kind"], "n": n, "c": c, "h": h, "w": w,
                   "depth": depth, "width": cfg["width"], "conv_operands": conv,
                   "residual_stream": f"fixed point, {frac_bits} fraction bits" if frac_bits else "fp32"},
        "step_totals": {"note": "launch and byte totals are those of the fp32-stream path" if frac_bits else None,
                        "conv_TFLOP": round(step_flops / 1e12, 4), "algorithmic_GB": round(step_bytes / 1e9, 3),
                        "kernel_launches": fwd_cost["kernel_launches"] + bwd_cost["kernel_launches"],
                        "achieved_TFLOPs": round(step_flops / 1e12 / (ms_per_step * 1e-3), 2),
                        "achieved_GBps": round(step_bytes / 1e9 / (ms_per_step * 1e-3), 1),
                        "frac_of_hbm_peak": round(step_bytes / 1e9 / (ms_per_step * 1e-3) / PEAK["hbm"][0], 4)},
        "kernels": kern,
        "peak_activation_bytes": {"analytic": analytic, "measured_max_allocated_minus_parameters_and_input": measured,
                                  "vs_depth": act_vs_depth},
        "reconstruction_rel_error_top_block_first": drift,
    })

    if not args.no_cpu_baseline:
        from oracle import revnet_oracle as O
        c2 = c // 2
        sp = lambda t: (np.ascontiguousarray(t[:, :c2]), np.ascontiguousarray(t[:, c2:]))
        O.build()

        def stored_pass(ns):
            with O.conv_operands(conv):
                t0 = time.perf_counter()
                if frac_bits:
                    q1, q2 = (O.fixed_encode(t, frac_bits) for t in sp(x[:ns]))
                    _, _, stored = O.stack_fwd_fixed(q1, q2, params, frac_bits, keep=True)
                else:
                    _, _, _, stored = O.stack_fwd(*sp(x[:ns]), params, keep=True)
                O.stack_bwd_stored(stored, params, *sp(dy[:ns]))
                return time.perf_counter() - t0

        def reversible_pass(ns):    # forward keeping nothing, then Algorithm 1 from the top pair
            with O.conv_operands(conv):
                t0 = time.perf_counter()
                if frac_bits:
                    q1, q2 = (O.fixed_encode(t, frac_bits) for t in sp(x[:ns]))
                    y1, y2 = O.stack_fwd_fixed(q1, q2, params, frac_bits)
                    O.stack_reverse_fixed(y1, y2, *sp(dy[:ns]), params, frac_bits)
                else:
                    y1, y2 = O.stack_fwd(*sp(x[:ns]), params)
                    O.stack_reverse(y1, y2, *sp(dy[:ns]), params)
                return time.perf_counter() - t0

        base = oracle_sample(stored_pass, n, args.cpu_sample_n, "one forward + stored-activation backward in float64")
        ns_used = int(base["sample"].split()[1])
        lit = oracle_sample(reversible_pass, n, ns_used, "one forward + Algorithm 1 (reconstructing backward) in float64")
        out["cpu_baseline"] = dict(base, cores=O.num_threads(), kind="oracle", algorithm1_literal=lit)
    return out


def run_workload(args, workload, primary):
    import gc
    import torch
    import synth_inputs as S
    fn = bench_body if (workload in S.BODIES or workload in S.NETS) else bench_stack
    out = fn(args, workload, primary)
    gc.collect()
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4_bneck12")
    ap.add_argument("--frac-bits", type=int, default=0,
                    help="keep the residual stream in fixed point with this many fraction bits (exact reconstruction); "
                         "0 = floating-point stream, the benchmark configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true", help="time the primary workload only")
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

    import torch
    import paper_1707_04585_amd as rv

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    rv.load_library()  # fails loudly if the HIP library is missing

    res = run_workload(args, args.workload, True)
    out = {"metric": METRIC, "value": res.pop("value"), "unit": res.pop("unit"), "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": res.pop("dtype"), "data": "synthetic"}
    out.update(res)
    if not args.no_secondary:
        out["secondary"] = {w: run_workload(args, w, False) for w in SECONDARY if w != args.workload}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
