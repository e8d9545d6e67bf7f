#!/usr/bin/env python3
"""Benchmark of the ZeroPP stage hot path on one MI355X.

A step is one pass of the whole hot path over one scheduling unit of synthetic input:
stage_materialize_params, U x stage_forward, U x stage_backward_input, then the weight-gradient tasks
of the unit as one grouped task that adds into G (stage_backward_weight_group), shard_adam_step (with
zero_grad), zpp_stage_end_unit.  Other orders of the same work: --group g (g micro-batches per
weight-gradient task; 1 = one by one), --backward fused (U x stage_backward_accumulate), --accumulate
separate (stage_backward + stage_accumulate_grads); the last three give identical bits, grouping
changes the summation order inside G.  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3_gpt_6p2b] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, vendor figure
PEAK_FP32_TFLOPS = 157.3    # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, vendor figure


def model_flops_per_unit(sh) -> float:
    """Algorithmic work only: GEMMs 2*T*h*(3h+h+2f) forward (LLaMA 2*T*h*(4h+3f)), causal attention
    2*b*s^2*h forward; backward = 2x forward; norms/activations not counted."""
    T, h, f = sh.tokens, sh.hidden, sh.ffn
    gemm = 2.0 * T * h * (4 * h + (2 * f if sh.arch == 0 else 3 * f))
    attn = 2.0 * sh.micro_batch * sh.seq * sh.seq * h
    return 3.0 * (gemm + attn) * sh.n_blocks * sh.unit_mbs


def cpu_baseline(sh, seconds_hint: float = 20.0):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the workload:
    one block of the stage, one micro-batch, full T/h/f (forward, backward, accumulate)."""
    import numpy as np
    import oracle
    import synth
    sample = sh.replace(n_blocks=1, unit_mbs=1)
    st = oracle.OracleStage(sample, "f32")
    synth.make_params(sample, st.layout(), out=st.P)
    x, dy = synth.make_x(sample, 0), synth.make_dy(sample, 0)
    t0 = time.perf_counter()
    st.materialize()
    st.forward(0, x)
    st.backward(0, dy)
    st.accumulate(0, 1.0)
    dt = time.perf_counter() - t0
    flops = model_flops_per_unit(sample)
    threads = oracle.num_threads()
    st.close()
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"1 of {sh.n_blocks} blocks x 1 of {sh.unit_mbs} micro-batches at full T={sh.tokens}, "
                      f"h={sh.hidden}, f={sh.ffn}: materialise + forward + backward + accumulate, fp32 oracle"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="cfg3_gpt_6p2b")
    ap.add_argument("--accumulate", choices=("in_place", "separate"), default="in_place",
                    help="in_place: stage_backward_accumulate (dW products add into G from their epilogues); "
                         "separate: stage_backward into the staging buffer, then stage_accumulate_grads")
    ap.add_argument("--backward", choices=("fused", "split"), default="split",
                    help="split: the input-gradient tasks of all micro-batches of the unit first, then their "
                         "weight-gradient tasks; fused: one backward call per micro-batch")
    ap.add_argument("--stages", type=int, default=1,
                    help="V > 1: the configuration's blocks as V stages on the device (zpp_device.h): breadth-first "
                         "over the stages, one gathered stage live at a time, the next one's gather on a second stream")
    ap.add_argument("--no-prefetch", action="store_true", help="with --stages: one working-copy slot, gathers in line")
    ap.add_argument("--adam", choices=("uniform", "decay_ranges"), default="uniform",
                    help="decay_ranges: shard_adam_step_ranges with weight decay on matrices only")
    ap.add_argument("--group", type=int, default=0,
                    help="with --backward split: weight-gradient tasks of this many micro-batches as one product "
                         "(stage_backward_weight_group); 0 = the whole unit, 1 = one by one (bit-identical to fused)")
    ap.add_argument("--recompute", action="store_true",
                    help="activation recomputation: keep only block inputs, run each block's forward again in backward")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-five-call-order", action="store_true",
                    help="skip the extra timing of the unit through the five named calls (keeps a profile to the default step)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the path; this build has no multi-GPU leg "
              "(run with --gpus 1).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    import paper_2402_03791_amd as zpp

    sh = synth.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    props = torch.cuda.get_device_properties(0)
    # how the peaks used below come about: CUs x clock x 4096 bf16 flop per clock and CU (dense MFMA)
    device_info = {"name": props.name, "compute_units": props.multi_processor_count,
                   "peak_bf16_TFLOPs_used": PEAK_BF16_TFLOPS, "peak_hbm_GBps_used": PEAK_HBM_GBS,
                   "peak_note": "vendor figures: 256 CUs x 2.4 GHz x 4096 bf16 flop/clk/CU = 2.52 PFLOP/s dense; HBM3E 8 TB/s"}
    V = args.stages
    if args.recompute:
        args.backward = "fused"       # recomputation serves both gradient tasks of a block from one re-run
    if args.backward != "split" or sh.compute_dtype != 1:
        args.group = 1
    elif args.group == 0:
        args.group = sh.unit_mbs
    if args.group > 1 and args.accumulate != "in_place":
        print("--group > 1 adds into G in place: not with --accumulate separate", file=sys.stderr)
        sys.exit(2)
    if V > 1:
        if sh.n_blocks % V or args.accumulate != "in_place":
            print("--stages needs a divisor of the block count and the default --accumulate", file=sys.stderr)
            sys.exit(2)
        full_layout = zpp.Stage(sh, allocate=False).layout()
        st = zpp.Device(sh.replace(n_blocks=sh.n_blocks // V), V, prefetch=not args.no_prefetch,
                        recompute=args.recompute, split_backward=args.group if args.backward == "split" else 0)
        st.N = st.N_total
    else:
        st = zpp.Stage(sh, device="cuda:0", split_backward=args.group if args.backward == "split" else 0,
                       recompute=args.recompute)
        full_layout = st.layout()
    act = st.act_dtype

    # ---- synthetic inputs, resident in HBM before anything is timed
    P0 = synth.make_params(sh, full_layout)
    st.P.copy_(torch.from_numpy(P0))
    del P0
    xs = [torch.from_numpy(synth.make_x(sh, m)).to(dev, act) for m in range(sh.unit_mbs)]
    dys = [torch.from_numpy(synth.make_dy(sh, m)).to(dev, act) for m in range(sh.unit_mbs)]
    y = torch.empty_like(xs[0])
    dx = torch.empty_like(xs[0])
    stream = torch.cuda.current_stream()
    adam = dict(synth.ADAM)

    if V > 1:
        # the stages are wired in a chain on this one GPU: y of stage v is x of stage v+1, dx of v is dy of v-1
        U = sh.unit_mbs
        side = torch.cuda.Stream()
        mid = [[torch.empty_like(xs[0]) for _ in range(U)] for _ in range(V)]
        gmid = [[torch.empty_like(xs[0]) for _ in range(U)] for _ in range(V)]
        x_list = [(xs[m] if v == 0 else mid[v - 1][m]) for v in range(V) for m in range(U)]
        y_list = [mid[v][m] for v in range(V) for m in range(U)]
        dy_list = [(dys[m] if v == V - 1 else gmid[v + 1][m]) for v in range(V) for m in range(U)]
        dx_list = [gmid[v][m] for v in range(V) for m in range(U)]

    def step(t: int):
        if V > 1:
            st.forward_unit(x_list, y_list, stream, side)
            st.backward_unit(dy_list, dx_list, 1.0, stream, side)
            st.adam_step(step=t, zero_grad=1, stream=stream, **adam)
            st.end_unit()
            return
        st.materialize_params(stream)
        for m in range(sh.unit_mbs):
            st.forward(m, xs[m], y, stream)
        if args.backward == "split":
            for m in range(sh.unit_mbs):
                st.backward_input(m, dys[m], dx, stream)
            for m in range(0, sh.unit_mbs, args.group):
                if args.group > 1:
                    st.backward_weight_group(m, min(args.group, sh.unit_mbs - m), 1.0, stream)
                    continue
                st.backward_weight(m, args.accumulate == "in_place", 1.0, stream)
                if args.accumulate != "in_place":
                    st.accumulate_grads(m, 1.0, stream)
        for m in range(sh.unit_mbs if args.backward == "fused" else 0):
            if args.accumulate == "in_place":
                st.backward_accumulate(m, dys[m], dx, 1.0, stream)
            else:
                st.backward(m, dys[m], dx, stream)
                st.accumulate_grads(m, 1.0, stream)
        if args.adam == "decay_ranges":
            st.adam_step_ranges(ranges, step=t, zero_grad=1, write_back=1, stream=stream, **adam)
        else:
            st.adam_step(step=t, zero_grad=1, write_back=1, stream=stream, **adam)
        st.end_unit()

    ranges = st.decay_ranges(adam["lr"], adam["weight_decay"]) if args.adam == "decay_ranges" and V == 1 else None
    t = 0
    for _ in range(args.warmup):
        t += 1
        step(t)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        t += 1
        step(t)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    flops = model_flops_per_unit(sh)
    value = flops / (ms_per_step * 1e-3) / 1e12

    # ---- one more step with HIP events around every kernel class (same stream), for the roofline
    zpp.profile_reset()
    zpp.profile_enable(True)
    t += 1
    step(t)
    torch.cuda.synchronize()
    prof = zpp.profile_read()
    zpp.profile_enable(False)
    zpp.profile_reset()

    # the standalone accumulate pass on the stage's own buffers, for the HBM figure of the metric, when the
    # timed step does not contain it (in-place accumulation has no such launch)
    acc_standalone = None
    if args.accumulate == "in_place":
        S = st.region("S") if V == 1 else torch.empty_like(st.G)
        reps = 4
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        zpp.op_flat_accumulate(st.G, S, 1.0, stream=stream)
        a0.record(stream)
        for _ in range(reps):
            zpp.op_flat_accumulate(st.G, S, 1.0, stream=stream)
        a1.record(stream)
        torch.cuda.synchronize()
        acc_standalone = (reps, a0.elapsed_time(a1), reps * 12.0 * st.N)

    def rate(cls, scale):
        if cls == "accumulate" and acc_standalone:
            return acc_standalone[2] / (acc_standalone[1] * 1e-3) / scale
        n, ms, work, _ = prof[cls]
        return (work / (ms * 1e-3) / scale) if ms > 0 else 0.0

    def measured_traffic():
        """HBM bytes per GEMM launch from the committed rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE,
        scaled by what the counters read on the flat passes of known size), if they cover this workload."""
        path = os.path.join(ROOT, "profiles", "cfg3_gemm_traffic.kv")
        if not os.path.exists(path):
            return None
        kv = dict(l.strip().split("=", 1) for l in open(path) if "=" in l and not l.startswith("#"))
        return float(kv["gemm_hbm_bytes_per_launch"]) if kv.get("workload") == sh.name else None

    # the GEMM family = forward and input-gradient products ("gemm") + weight-gradient products ("gemm_dw")
    fam = [prof["gemm"], prof["gemm_dw"]]
    n_gemm, ms_gemm, fl_gemm, by_gemm = (sum(c[i] for c in fam) for i in range(4))
    gemm_tflops = fl_gemm / (ms_gemm * 1e-3) / 1e12 if ms_gemm > 0 else 0.0
    bf16 = sh.compute_dtype == 1
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS
    roofline = {
        "kernel": "gemm_bf16_nt_h_kernel, gemm_bf16_nt_d_kernel (all bf16 GEMMs of the step)" if bf16 else "gemm_f32_kernel",
        "bound": "mfma" if bf16 else "alu",
        "achieved": round(gemm_tflops, 2), "peak": peak, "unit": "TFLOP/s",
        "frac": round(gemm_tflops / peak, 4),
        "launches": n_gemm, "avg_launch_ms": round(ms_gemm / max(n_gemm, 1), 4),
        "flops_per_launch": fl_gemm / max(n_gemm, 1),
        "algorithmic_bytes": by_gemm / max(n_gemm, 1),
        "traffic": measured_traffic(),
        # the same family by kind: the weight-gradient products carry the gradient accumulation in their
        # epilogue when the step accumulates in place (one extra fp32 read of their output)
        "by_kind": {k: {"launches": prof[c][0], "ms": round(prof[c][1], 3), "TFLOP/s": round(rate(c, 1e12), 1),
                        "frac": round(rate(c, 1e12) / peak, 4)}
                    for k, c in (("forward_and_input_gradient", "gemm"), ("weight_gradient", "gemm_dw"))},
    }
    fb_ms = sum(prof[c][1] for c in ("gemm", "gemm_dw", "attn_fwd", "attn_bwd", "other"))
    phases = {c: {"launches": prof[c][0], "ms": round(prof[c][1], 3)} for c in prof}
    phases["gemm"]["TFLOP/s"] = round(rate("gemm", 1e12), 1)
    phases["gemm_dw"]["TFLOP/s"] = round(rate("gemm_dw", 1e12), 1)
    phases["attn_fwd"]["TFLOP/s"] = round(rate("attn_fwd", 1e12), 1)
    phases["attn_bwd"]["TFLOP/s"] = round(rate("attn_bwd", 1e12), 1)
    for c in ("accumulate", "adam", "materialize"):
        phases[c]["GB/s"] = round(rate(c, 1e9), 1)
        phases[c]["frac_hbm_peak"] = round(rate(c, 1e9) / PEAK_HBM_GBS, 4)
    acc_ms, acc_bytes = (acc_standalone[1], acc_standalone[2]) if acc_standalone else prof["accumulate"][1:3]
    if acc_standalone:
        phases["accumulate"]["standalone"] = {"launches": acc_standalone[0], "ms": round(acc_standalone[1], 3),
                                              "note": "not part of the timed step: timed alone on the stage's G and "
                                                      "staging buffers"}
    hbm_pass = {
        "adam_GBps": phases["adam"]["GB/s"], "accumulate_GBps": phases["accumulate"]["GB/s"],
        "combined_GBps": round((prof["adam"][2] + acc_bytes) / max((prof["adam"][1] + acc_ms) * 1e-3, 1e-12) / 1e9, 1),
        "peak_GBps": PEAK_HBM_GBS,
    }
    hbm_pass["combined_frac"] = round(hbm_pass["combined_GBps"] / PEAK_HBM_GBS, 4)

    out = {
        "metric": "stage fwd+bwd TFLOP/s per GPU (% bf16 MFMA peak); Adam/accum HBM GB/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": sh.name, "arch": "gpt" if sh.arch == 0 else "llama", "n_blocks": sh.n_blocks,
                   "hidden": sh.hidden, "n_heads": sh.n_heads, "ffn": sh.ffn, "seq": sh.seq,
                   "micro_batch": sh.micro_batch, "unit_mbs": sh.unit_mbs, "params": st.N,
                   "accumulate": args.accumulate, "backward": args.backward, "weight_task_group": args.group, "recompute": args.recompute,
                   "adam": args.adam, "stages_on_device": V, "prefetch": V > 1 and not args.no_prefetch,
                   "workspace_GB": round(st.workspace_bytes / 1e9, 2)},
        "model_flops_per_step": flops,
        "frac_bf16_peak_whole_step": round(value / PEAK_BF16_TFLOPS, 4),
        "fwd_bwd_TFLOPs": round(flops / (fb_ms * 1e-3) / 1e12, 2) if fb_ms > 0 else None,
        "wall_s_timed": round(wall, 3),
        "device": device_info,
        "roofline": roofline,
        "hbm_pass": hbm_pass,
        "phases": phases,
    }
    # The same unit through the five calls the interface is named after, one after the other per micro-batch
    # (materialise, forward, backward into the staging buffer, accumulate pass, Adam), timed the same way,
    # for comparison with the default order of the work above.
    if V == 1 and not args.recompute and not args.no_five_call_order and \
            (args.backward, args.accumulate) != ("fused", "separate"):
        st2 = zpp.Stage(sh, device="cuda:0")
        st2.P.copy_(st.P)

        def step5(tt: int):
            st2.materialize_params(stream)
            for m in range(sh.unit_mbs):
                st2.forward(m, xs[m], y, stream)
            for m in range(sh.unit_mbs):
                st2.backward(m, dys[m], dx, stream)
                st2.accumulate_grads(m, 1.0, stream)
            st2.adam_step(step=tt, zero_grad=1, stream=stream, **adam)
            st2.end_unit()

        step5(1)
        torch.cuda.synchronize()
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        f0.record(stream)
        for i in range(args.steps):
            step5(2 + i)
        f1.record(stream)
        torch.cuda.synchronize()
        ms5 = f0.elapsed_time(f1) / args.steps
        out["five_call_order"] = {"calls": "stage_materialize_params, U x stage_forward, U x (stage_backward, "
                                           "stage_accumulate_grads), shard_adam_step",
                                  "ms_per_step": round(ms5, 3), "value": round(flops / (ms5 * 1e-3) / 1e12, 2),
                                  "unit": "TFLOP/s"}
        st2.close()
        del st2
    if not args.no_cpu_baseline:
        st.close()
        del st, xs, dys
        out["cpu_baseline"] = cpu_baseline(sh)
        out["gpu_over_cpu"] = round(value / out["cpu_baseline"]["value"], 1)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
