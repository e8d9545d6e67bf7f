#!/usr/bin/env python3
"""Benchmark of the ZeroPP stage hot path on one MI355X.

A step is one pass of the whole hot path over one scheduling unit of synthetic input:
stage_materialize_params, the U forward tasks and then the U input-gradient tasks a few micro-batches per call
(stage_forward_group, stage_backward_input_group; two, or default_mb_group() of them), the weight-gradient tasks of the unit as one grouped task
that adds into G (stage_backward_weight_group), shard_adam_step (with zero_grad; --zero-grad release: G is
released instead and the next unit's first addition into it writes), zpp_stage_end_unit.  Other
orders of the same work: --mb-group g (micro-batches per forward / input-gradient call; 1 = the
one-micro-batch calls), --group g (g micro-batches per weight-gradient task; 1 = one by one), --backward fused
(stage_backward_accumulate), --accumulate separate (stage_backward + stage_accumulate_grads); y and dx are the
same bits in all of them, grouping changes the summation order inside G.  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line.

After the timed region the same process adds, outside `value`: one event-instrumented step (roofline, phases),
the unit through the five named calls, the Adam / accumulate passes on the wide configuration's 6.4 GB shard,
two steps of each other bf16 configuration, and the CPU oracle on a bounded sample.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg3_gpt_6p2b] [--no-cpu-baseline]
                  [--no-five-call-order] [--no-large-shard] [--no-other-workloads]
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


def default_mb_group(sh) -> int:
    """Micro-batches per forward / input-gradient call in the default order of the work: the fewest (two, four or
    eight, a divisor of U) for which every product of a block over the group's rows is a grid the library runs
    with its 256 x 256 tile, i.e. a whole number of rounds of one tile per CU (256 CUs) or at least four rounds;
    two if none does.  The group is one matrix of g * T rows, so g only decides how the tile grids come out:
    T x h at T = 4096, h = 5120 is 2.5 rounds at g = 2 and 5 at g = 4."""
    if sh.compute_dtype != 1:
        return 1                  # the tiny fp32 configuration: one micro-batch at a time
    widths = (3 * sh.hidden, sh.hidden, sh.ffn * (2 if sh.arch == 1 else 1))

    def whole_rounds(rows):
        tiles = [((rows + 255) // 256) * ((n + 255) // 256) for n in widths]
        return all(t >= 256 and (t % 256 == 0 or t >= 1024) for t in tiles)

    for g in (2, 4, 8):
        if sh.unit_mbs % g == 0 and whole_rounds(g * sh.tokens):
            return g
    return 2 if sh.unit_mbs % 2 == 0 else 1


def model_flops_per_unit(sh) -> float:
    """Algorithmic work only: GEMMs 2*T*h*(3h+h+2f) forward (LLaMA 2*T*h*(4h+3f)), causal attention
    2*b*s^2*h forward; backward = 2x forward; norms/activations not counted."""
    T, h, f = sh.tokens, sh.hidden, sh.ffn
    gemm = 2.0 * T * h * (4 * h + (2 * f if sh.arch == 0 else 3 * f))
    attn = 2.0 * sh.micro_batch * sh.seq * sh.seq * h
    return 3.0 * (gemm + attn) * sh.n_blocks * sh.unit_mbs


def kernel_sources_sha256() -> str:
    """One hash over the library's kernel and launch-sequence sources, to tie counter summaries to the code."""
    import hashlib
    d = os.path.join(ROOT, "paper_2402_03791_amd", "csrc")
    hsh = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".cpp", ".h")):
            hsh.update(name.encode())
            hsh.update(open(os.path.join(d, name), "rb").read())
    return hsh.hexdigest()


def hbm_large_shard(zpp, torch, synth, stream):
    """The flat passes on the wide configuration's shard (1.61e9 elements, 6.44 GB per fp32 buffer: far beyond any
    cache): Adam with zero_grad (32 B per element) and the accumulate pass (12 B per element), each timed with
    events on the launching stream over several launches."""
    n = zpp.Stage(synth.CONFIGS["cfg5_wide_gpt"], allocate=False).N
    g = torch.Generator(device="cuda").manual_seed(5)
    P = torch.randn(n, device="cuda", generator=g) * 0.02
    G = torch.randn(n, device="cuda", generator=g) * 1e-3
    S = torch.randn(n, device="cuda", generator=g) * 1e-3
    M = torch.zeros(n, device="cuda")
    V = torch.zeros(n, device="cuda")
    hp = dict(synth.ADAM)
    out = {"workload": "cfg5_wide_gpt flat shard", "elements": n, "GB_per_buffer": round(n * 4 / 1e9, 2)}
    for name, reps, bytes_per, fn in (
            ("adam", 3, 32.0, lambda i: zpp.op_flat_adam(P, M, V, G, step=i + 1, zero_grad=1, stream=stream, **hp)),
            ("accumulate", 4, 12.0, lambda i: zpp.op_flat_accumulate(G, S, 1.0, stream=stream))):
        fn(0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(reps):
            fn(1 + i)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = bytes_per * n / (ms * 1e-3) / 1e9
        out[name] = {"ms": round(ms, 3), "GB/s": round(gbs, 1), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4),
                     "bytes_per_element": bytes_per}
    tot_b = 32.0 * n + 12.0 * n
    tot_ms = out["adam"]["ms"] + out["accumulate"]["ms"]
    out["combined_GBps"] = round(tot_b / (tot_ms * 1e-3) / 1e9, 1)
    out["combined_frac"] = round(out["combined_GBps"] / PEAK_HBM_GBS, 4)
    return out


def time_default_step(zpp, torch, synth, sh, steps, warmup, stream):
    """The default order of the work (materialise, forward and input-gradient tasks in groups of default_mb_group()
    micro-batches, the unit's weight-gradient tasks as one grouped task, Adam with zero_grad and write-back) on
    another workload; whole-step figures only."""
    U, T, g = sh.unit_mbs, sh.tokens, default_mb_group(sh)
    st = zpp.Stage(sh, device="cuda:0", split_backward=U, group_mbs=g)
    P0 = synth.make_params(sh, st.layout())
    st.P.copy_(torch.from_numpy(P0))
    del P0
    act = st.act_dtype
    X = torch.empty(U * T, sh.hidden, device="cuda:0", dtype=act)
    DY = torch.empty_like(X)
    for m in range(U):
        X[m * T:(m + 1) * T].copy_(torch.from_numpy(synth.make_x(sh, m)))
        DY[m * T:(m + 1) * T].copy_(torch.from_numpy(synth.make_dy(sh, m)))
    Y = torch.empty(g * T, sh.hidden, device="cuda:0", dtype=act)
    DX = torch.empty_like(Y)

    def step(t):
        st.materialize_params(stream)
        for f in range(0, U, g):
            c = min(g, U - f)
            st.forward_group(f, c, X[f * T:(f + c) * T], Y[:c * T], stream)
        for f in range(0, U, g):
            c = min(g, U - f)
            st.backward_input_group(f, c, DY[f * T:(f + c) * T], DX[:c * T], stream)
        st.backward_weight_group(0, U, 1.0, stream)
        st.adam_step(step=t, zero_grad=1, write_back=1, stream=stream, **synth.ADAM)
        st.end_unit()

    for t in range(warmup):
        step(t + 1)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for t in range(steps):
        step(warmup + t + 1)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    fl = model_flops_per_unit(sh)
    res = {"ms_per_step": round(ms, 3), "value": round(fl / (ms * 1e-3) / 1e12, 2), "unit": "TFLOP/s",
           "frac_bf16_peak_whole_step": round(fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "steps": steps,
           "params": st.N, "workspace_GB": round(st.workspace_bytes / 1e9, 2)}
    st.close()
    return res


def cpu_baseline(sh):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the workload.
    Forward, backward and accumulate: one block of the stage at full T/h/f over k = 2 micro-batches,
    timed separately and scaled by (blocks x U / k) - the work is exactly linear in blocks and
    micro-batches.  Adam and materialise: timed in full over the stage's whole N-element shard with the
    oracle's flat passes.  Plus the whole tiny fp32 configuration on one thread."""
    import numpy as np
    import oracle
    import synth
    k = min(2, sh.unit_mbs)
    sample = sh.replace(n_blocks=1, unit_mbs=k)
    st = oracle.OracleStage(sample, "f32")
    synth.make_params(sample, st.layout(), out=st.P)
    xs = [synth.make_x(sample, m) for m in range(k)]
    dys = [synth.make_dy(sample, m) for m in range(k)]
    st.materialize()
    t = {"forward": 0.0, "backward": 0.0, "accumulate": 0.0}
    for m in range(k):
        t0 = time.perf_counter()
        st.forward(m, xs[m])
        t["forward"] += time.perf_counter() - t0
    for m in range(k):
        t0 = time.perf_counter()
        st.backward(m, dys[m])
        t1 = time.perf_counter()
        st.accumulate(m, 1.0)
        t["backward"] += t1 - t0
        t["accumulate"] += time.perf_counter() - t1
    st.close()
    del st, xs, dys
    scale = sh.n_blocks * sh.unit_mbs / k
    # the flat passes over the whole shard
    N = oracle.param_count(sh)
    hp = {kk: float(np.float32(v)) for kk, v in synth.ADAM.items()}
    P = synth.normal_f32(1, 1, N, 0.0, 0.02)
    G = synth.normal_f32(1, 2, N, 0.0, 1e-3)
    M = np.zeros(N, np.float32)
    V = np.zeros(N, np.float32)
    M[:] = 0.0   # touch the pages before timing
    V[:] = 0.0
    t0 = time.perf_counter()
    oracle.flat_adam(P, M, V, G, step=1, zero_grad=1, **hp)
    t["adam_full"] = time.perf_counter() - t0
    del M, V, G
    if sh.compute_dtype == 1:
        t0 = time.perf_counter()
        oracle.flat_materialize_bits(P)
        t["materialize_full"] = time.perf_counter() - t0
    else:
        t["materialize_full"] = 0.0
    del P
    unit_s = (t["forward"] + t["backward"] + t["accumulate"]) * scale + t["adam_full"] + t["materialize_full"]
    threads = oracle.num_threads()
    # the tiny fp32 configuration, whole unit, on one thread
    tiny = synth.CONFIGS["cfg1_tiny_gpt_fp32"]
    oracle.set_num_threads(1)
    o1 = oracle.OracleStage(tiny, "f32")
    synth.make_params(tiny, o1.layout(), out=o1.P)
    t0 = time.perf_counter()
    o1.materialize()
    for m in range(tiny.unit_mbs):
        o1.forward(m, synth.make_x(tiny, m))
    for m in range(tiny.unit_mbs):
        o1.backward(m, synth.make_dy(tiny, m))
        o1.accumulate(m, 1.0)
    o1.adam(step=1, **{kk: float(np.float32(v)) for kk, v in synth.ADAM.items()})
    tiny_s = time.perf_counter() - t0
    o1.close()
    oracle.set_num_threads(threads)
    return {"value": model_flops_per_unit(sh) / unit_s / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "affinity_cores": len(os.sched_getaffinity(0)), "omp_max_threads": threads,
            "seconds_measured": round(sum(t.values()), 2),
            "seconds_per_unit_extrapolated": round(unit_s, 1),
            "seconds": {kk: round(v, 3) for kk, v in t.items()},
            "cfg1_whole_unit_one_thread_s": round(tiny_s, 3),
            "cfg1_one_thread_TFLOPs": round(model_flops_per_unit(tiny) / tiny_s / 1e12, 5),
            "sample": f"fp32 oracle; forward + backward + accumulate of 1 of {sh.n_blocks} blocks x {k} of "
                      f"{sh.unit_mbs} micro-batches at full T={sh.tokens}, h={sh.hidden}, f={sh.ffn}, scaled by "
                      f"{scale:g} (extrapolated from {k} of {sh.unit_mbs}); Adam and materialise timed in full over "
                      f"the {N}-element shard"}


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
    ap.add_argument("--recompute", nargs="?", const="full", default="none", choices=("none", "full", "selective"),
                    help="activation recomputation: full (keep only block inputs, run each block's forward again in "
                         "backward) or selective (rebuild only the norm and activation outputs)")
    ap.add_argument("--mb-group", type=int, default=0,
                    help="micro-batches per forward / input-gradient (or fused backward) call: stage_forward_group etc. "
                         "run every linear layer once over this many micro-batches; 0 = the fewest that give whole "
                         "rounds of 256 x 256 tiles (default_mb_group), one where the other options need one")
    ap.add_argument("--zero-grad", choices=("zero", "release"), default="zero",
                    help="what the Adam step does with G: zero it in the same pass (the pass the HBM figure of the "
                         "metric is stated on), or release it (zpp_adam.zero_grad = 2: the next unit's first addition "
                         "into G writes instead; 4 + 4 bytes per parameter less per step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-large-shard", action="store_true",
                    help="skip the Adam / accumulate bandwidth leg on the wide configuration's 1.61e9-element shard")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short whole-step timings of the other bf16 configurations")
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
    zg = 2 if args.zero_grad == "release" else 1
    args.recompute = {"none": 0, "full": 1, "selective": 2}[args.recompute]
    if args.recompute:
        args.backward = "fused"       # recomputation serves both gradient tasks of a block from one re-run
    auto_mb_group = args.mb_group == 0
    if auto_mb_group:
        args.mb_group = default_mb_group(sh) if V == 1 and args.accumulate == "in_place" else 1
    if sh.compute_dtype != 1:
        args.mb_group = 1             # the tiny fp32 configuration: one micro-batch at a time
    if args.backward != "split" or sh.compute_dtype != 1:
        args.group = 1
    elif args.group == 0:
        args.group = sh.unit_mbs
    if auto_mb_group and args.backward == "split" and args.group % args.mb_group:
        args.mb_group = 1
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
                       recompute=args.recompute, group_mbs=args.mb_group)
        full_layout = st.layout()
    act = st.act_dtype

    # ---- synthetic inputs, resident in HBM before anything is timed
    P0 = synth.make_params(sh, full_layout)
    st.P.copy_(torch.from_numpy(P0))
    del P0
    # the unit's micro-batches lie back to back, so that a group of them is one matrix
    T = sh.tokens
    X = torch.empty(sh.unit_mbs * T, sh.hidden, device=dev, dtype=act)
    DY = torch.empty_like(X)
    for m in range(sh.unit_mbs):
        X[m * T:(m + 1) * T].copy_(torch.from_numpy(synth.make_x(sh, m)))
        DY[m * T:(m + 1) * T].copy_(torch.from_numpy(synth.make_dy(sh, m)))
    xs = [X[m * T:(m + 1) * T] for m in range(sh.unit_mbs)]
    dys = [DY[m * T:(m + 1) * T] for m in range(sh.unit_mbs)]
    mg = args.mb_group
    if mg < 1 or mg > sh.unit_mbs or (mg > 1 and (V > 1 or args.accumulate != "in_place")) or \
            (args.backward == "split" and args.group % mg):
        print("--mb-group needs 1 <= g <= U, a single stage, the default --accumulate and a weight-task --group "
              "that is a multiple of it", file=sys.stderr)
        sys.exit(2)
    Y = torch.empty(mg * T, sh.hidden, device=dev, dtype=act)
    DX = torch.empty_like(Y)
    y, dx = Y[:T], DX[:T]
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
            st.adam_step(step=t, zero_grad=zg, stream=stream, **adam)
            st.end_unit()
            return
        st.materialize_params(stream)
        if mg > 1:
            for f in range(0, sh.unit_mbs, mg):
                c = min(mg, sh.unit_mbs - f)
                st.forward_group(f, c, X[f * T:(f + c) * T], Y[:c * T], stream)
            for f in range(0, sh.unit_mbs, mg):
                c = min(mg, sh.unit_mbs - f)
                if args.backward == "split":
                    st.backward_input_group(f, c, DY[f * T:(f + c) * T], DX[:c * T], stream)
                else:
                    st.backward_accumulate_group(f, c, DY[f * T:(f + c) * T], DX[:c * T], 1.0, stream)
        for m in range(sh.unit_mbs if mg == 1 else 0):
            st.forward(m, xs[m], y, stream)
        if args.backward == "split":
            for m in range(sh.unit_mbs if mg == 1 else 0):
                st.backward_input(m, dys[m], dx, stream)
            for m in range(0, sh.unit_mbs, args.group):
                if args.group > 1:
                    st.backward_weight_group(m, min(args.group, sh.unit_mbs - m), 1.0, stream)
                    continue
                st.backward_weight(m, args.accumulate == "in_place", 1.0, stream)
                if args.accumulate != "in_place":
                    st.accumulate_grads(m, 1.0, stream)
        for m in range(sh.unit_mbs if args.backward == "fused" and mg == 1 else 0):
            if args.accumulate == "in_place":
                st.backward_accumulate(m, dys[m], dx, 1.0, stream)
            else:
                st.backward(m, dys[m], dx, stream)
                st.accumulate_grads(m, 1.0, stream)
        if args.adam == "decay_ranges":
            st.adam_step_ranges(ranges, step=t, zero_grad=zg, write_back=1, stream=stream, **adam)
        else:
            st.adam_step(step=t, zero_grad=zg, write_back=1, stream=stream, **adam)
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

    # the gather as a pass of its own (the cast of the whole shard plus the transposed copies this shape needs):
    # in the timed step an Adam step with write-back has already produced the working copy
    mat_standalone = None
    if V == 1:
        reps = 4
        c0, b0 = st.counters()
        m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        st.params_changed()
        st.materialize_params(stream)
        m0.record(stream)
        for _ in range(reps):
            st.params_changed()
            st.materialize_params(stream)
        m1.record(stream)
        torch.cuda.synchronize()
        c1, b1 = st.counters()
        mat_standalone = (reps, m0.elapsed_time(m1), (b1 - b0) * reps / (c1 - c0))

    def rate(cls, scale):
        if cls == "materialize" and mat_standalone:
            return mat_standalone[2] / (mat_standalone[1] * 1e-3) / scale
        if cls == "accumulate" and acc_standalone:
            return acc_standalone[2] / (acc_standalone[1] * 1e-3) / scale
        n, ms, work, _ = prof[cls]
        return (work / (ms * 1e-3) / scale) if ms > 0 else 0.0

    def profile_kv():
        """Figures taken from the committed rocprofv3 --pmc summaries (HBM bytes per GEMM launch from
        FETCH_SIZE / WRITE_SIZE scaled by what the counters read on the flat passes of known size; matrix-core
        busy cycles): counters cannot be read from inside this process, so they come from profiles/ and are
        used only when they were taken on this workload, this default order of the work and these kernel
        sources (hash of the csrc/ files recorded with them); otherwise the fields are null."""
        path = os.path.join(ROOT, "profiles", f"{sh.name}_counters.kv")
        if not os.path.exists(path) or not default_order:
            return {}
        kv = dict(l.strip().split("=", 1) for l in open(path) if "=" in l and not l.startswith("#"))
        if kv.get("workload") != sh.name or kv.get("kernel_sources_sha256") != kernel_sources_sha256():
            return {}
        return kv

    # The share the target is stated on: all matrix-core work of the step, i.e. the bf16 GEMM family (forward and
    # input-gradient products "gemm" + weight-gradient products "gemm_dw") and the attention kernels.
    fam = [prof["gemm"], prof["gemm_dw"]]
    n_gemm, ms_gemm, fl_gemm, by_gemm = (sum(c[i] for c in fam) for i in range(4))
    gemm_tflops = fl_gemm / (ms_gemm * 1e-3) / 1e12 if ms_gemm > 0 else 0.0
    mc = fam + [prof["attn_fwd"], prof["attn_bwd"]]
    n_mc, ms_mc, fl_mc = (sum(c[i] for c in mc) for i in range(3))
    mc_tflops = fl_mc / (ms_mc * 1e-3) / 1e12 if ms_mc > 0 else 0.0
    bf16 = sh.compute_dtype == 1
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_FP32_TFLOPS
    default_order = (V == 1 and args.backward == "split" and args.group == sh.unit_mbs and not args.recompute
                     and mg == default_mb_group(sh)
                     and args.accumulate == "in_place" and args.adam == "uniform" and args.zero_grad == "zero")
    kv = profile_kv()

    def kind(c):
        return {"launches": prof[c][0], "ms": round(prof[c][1], 3), "TFLOP/s": round(rate(c, 1e12), 1),
                "frac": round(rate(c, 1e12) / peak, 4)}

    roofline = {
        "kernel": ("bf16 GEMM family (gemm_bf16_kernel: NT forward, NN input-gradient, K-major weight-gradient) + MFMA "
                   "attention kernels: the GEMM/attention share of the step") if bf16 else "gemm_f32_kernel + generic attention kernels",
        "bound": "mfma" if bf16 else "alu",
        # algorithmic flops of all those launches of one step / their summed durations (HIP events on the
        # launching stream around each launch)
        "achieved": round(mc_tflops, 2), "peak": peak, "unit": "TFLOP/s",
        "frac": round(mc_tflops / peak, 4),
        "launches": n_mc, "avg_launch_ms": round(ms_mc / max(n_mc, 1), 4),
        "flops_per_launch": fl_mc / max(n_mc, 1),
        # HBM bytes per GEMM launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled) and matrix-core busy cycles, from
        # profiles/<workload>_counters.kv when it matches this code and order of work, else null
        "traffic": float(kv["gemm_hbm_bytes_per_launch"]) if "gemm_hbm_bytes_per_launch" in kv else None,
        "traffic_source": kv.get("source"),
        "mfma_busy": ({"gemm_and_attention_pct": float(kv["mfma_busy_pct"]), "gemm_pct": float(kv["mfma_busy_gemm_pct"]),
                       "gemm_clock_GHz": float(kv["gemm_clock_ghz"]), "source": kv.get("mfma_source")}
                      if "mfma_busy_pct" in kv else None),
        # the GEMM family alone (the dominant kernels: about 80 % of the step), and by kind: the weight-gradient
        # products carry the gradient accumulation in their epilogue when the step accumulates in place
        "gemm_family": {"launches": n_gemm, "ms": round(ms_gemm, 3), "TFLOP/s": round(gemm_tflops, 1),
                        "frac": round(gemm_tflops / peak, 4), "avg_launch_ms": round(ms_gemm / max(n_gemm, 1), 4),
                        "flops_per_launch": fl_gemm / max(n_gemm, 1),
                        "algorithmic_bytes_per_launch": by_gemm / max(n_gemm, 1)},
        "by_kind": {"forward_and_input_gradient": kind("gemm"), "weight_gradient": kind("gemm_dw"),
                    "attention_forward": kind("attn_fwd"), "attention_backward": kind("attn_bwd")},
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
    if mat_standalone:
        phases["materialize"]["standalone"] = {"launches": mat_standalone[0], "ms": round(mat_standalone[1], 3),
                                               "bytes_per_launch": int(mat_standalone[2] / mat_standalone[0]),
                                               "note": "a gather that casts the whole shard from P, timed alone; in the "
                                                       "timed step the Adam write-back leaves it nothing to do unless "
                                                       "the shape needs transposed copies"}
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
                   "accumulate": args.accumulate, "backward": args.backward, "weight_task_group": args.group, "micro_batch_group": mg, "zero_grad": args.zero_grad,
                   "recompute": ["none", "full", "selective"][args.recompute],
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
            st2.adam_step(step=tt, zero_grad=zg, stream=stream, **adam)
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
                                  "unit": "TFLOP/s",
                                  "frac_bf16_peak_whole_step": round(flops / (ms5 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        st2.close()
        del st2
    st.close()
    del st, xs, dys, y, dx, X, DY, Y, DX
    torch.cuda.empty_cache()
    if not args.no_large_shard and bf16:
        out["hbm_pass_large_shard"] = hbm_large_shard(zpp, torch, synth, stream)
        torch.cuda.empty_cache()
    if not args.no_other_workloads and default_order and args.config == "cfg3_gpt_6p2b":
        # the other bf16 configurations through the same default order of the work, two steps each
        out["other_workloads"] = {}
        for name in ("cfg2_gpt_1p3b", "cfg4_llama_13b", "cfg5_wide_gpt"):
            out["other_workloads"][name] = time_default_step(zpp, torch, synth, synth.CONFIGS[name], 2, 1, stream)
            torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(sh)
        out["gpu_over_cpu"] = round(value / out["cpu_baseline"]["value"], 1)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
