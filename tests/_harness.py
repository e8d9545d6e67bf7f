"""Shared helpers of the GPU parity tests: run the same seeded scheduling unit through the HIP
library and through the CPU oracle, and compare tensor by tensor."""
from __future__ import annotations

import numpy as np

import oracle
import synth


def rel_err(a: np.ndarray, ref: np.ndarray) -> float:
    """max|a - ref| / max|ref| : the per-tensor measure used for activations and gradients."""
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.abs(ref).max()
    return float(np.abs(a - ref).max() / (den if den > 0 else 1.0))


def to_dev(arr: np.ndarray, act_dtype, device="cuda:0"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(arr)).to(device=device, dtype=act_dtype)


def to_np(t) -> np.ndarray:
    return t.detach().to("cpu").float().numpy()


def make_inputs(shape, n_mbs):
    xs = [synth.make_x(shape, m) for m in range(n_mbs)]
    dys = [synth.make_dy(shape, m) for m in range(n_mbs)]
    return xs, dys


def run_oracle_unit(shape, P0: np.ndarray, xs, dys, dtype="f64", keep_stage=False):
    st = oracle.OracleStage(shape, dtype)
    st.P[:] = P0
    st.G[:] = 0
    st.materialize()
    ys = [st.forward(m, x) for m, x in enumerate(xs)]
    dxs, Ss = [], []
    for m, dy in enumerate(dys):
        dxs.append(st.backward(m, dy))
        Ss.append(st.S.copy() if m == 0 else None)
        st.accumulate(m, 1.0)
    out = dict(ys=ys, dxs=dxs, G=st.G.copy(), S0=Ss[0], W=st.W.copy())
    if keep_stage:
        out["stage"] = st
    else:
        st.close()
    return out


def run_gpu_unit(shape, P0: np.ndarray, xs, dys, keep_stage=False, in_place=False, scale=1.0, split=None,
                 recompute=0):
    """One scheduling unit on the GPU.  in_place: stage_backward_accumulate instead of the pair
    stage_backward + stage_accumulate_grads (then there is no staging snapshot S0).
    split: None, or the order in which the weight-gradient tasks run after ALL input-gradient tasks
    ("ascending", "descending"), or "interleaved" (each weight-gradient task right after its own
    input-gradient task), or ("group", g): afterwards, g micro-batches per grouped weight-gradient task."""
    import torch
    import paper_2402_03791_amd as zpp
    group = split[1] if isinstance(split, tuple) else 0
    st = zpp.Stage(shape, split_backward=max(group, int(split is not None)), recompute=recompute)
    st.P.copy_(torch.from_numpy(P0))
    st.G.zero_()
    st.materialize_params()
    ys = [st.forward(m, to_dev(x, st.act_dtype)) for m, x in enumerate(xs)]
    dxs = []
    S0 = None
    def weight_task(m):
        nonlocal S0
        st.backward_weight(m, in_place=in_place, scale=scale)
        if not in_place:
            if m == 0:
                S0 = to_np(st.region("S"))
            st.accumulate_grads(m, scale)

    for m, dy in enumerate(dys):
        if split is not None:
            dxs.append(st.backward_input(m, to_dev(dy, st.act_dtype)))
            if split == "interleaved":
                weight_task(m)
            continue
        if in_place:
            dxs.append(st.backward_accumulate(m, to_dev(dy, st.act_dtype), scale=scale))
            continue
        dxs.append(st.backward(m, to_dev(dy, st.act_dtype)))
        if m == 0:
            S0 = to_np(st.region("S"))
        st.accumulate_grads(m, scale)
    if group:
        for first in range(0, len(dys), group):
            st.backward_weight_group(first, min(group, len(dys) - first), scale)
    if split in ("ascending", "descending"):
        order = range(len(dys)) if split == "ascending" else reversed(range(len(dys)))
        for m in order:
            weight_task(m)
    torch.cuda.synchronize()
    out = dict(ys=[to_np(y) for y in ys], dxs=[to_np(d) for d in dxs], G=to_np(st.G), S0=S0,
               W=to_np(st.region("W")))
    if keep_stage:
        out["stage"] = st
    else:
        st.close()
    return out


def run_gpu_unit_grouped(shape, P0: np.ndarray, xs, dys, g: int, fused: bool, scale=1.0, recompute=0,
                         weight_group=None):
    """One scheduling unit with g micro-batches per call: stage_forward_group, then either
    stage_backward_accumulate_group (fused) or stage_backward_input_group followed by weight-gradient tasks
    over weight_group micro-batches (default g).  Inputs of a group are stacked into one [g*T, h] matrix."""
    import torch
    import paper_2402_03791_amd as zpp
    U = len(xs)
    wg = weight_group or g
    st = zpp.Stage(shape, split_backward=0 if fused else max(wg, 1), group_mbs=g, recompute=recompute)
    st.P.copy_(torch.from_numpy(P0))
    st.G.zero_()
    st.materialize_params()
    stack = lambda arrs: to_dev(np.concatenate(arrs, axis=0), st.act_dtype)
    ys, dxs = [], []
    groups = [(f, min(g, U - f)) for f in range(0, U, g)]
    for f, c in groups:
        y = st.forward_group(f, c, stack(xs[f:f + c]))
        ys += list(y.view(c, -1, y.shape[-1]))
    for f, c in groups:
        dy = stack(dys[f:f + c])
        dx = st.backward_accumulate_group(f, c, dy, scale=scale) if fused else st.backward_input_group(f, c, dy)
        dxs += list(dx.view(c, -1, dx.shape[-1]))
    if not fused:
        for f in range(0, U, wg):
            st.backward_weight_group(f, min(wg, U - f), scale)
    torch.cuda.synchronize()
    out = dict(ys=[to_np(y) for y in ys], dxs=[to_np(d) for d in dxs], G=to_np(st.G), S0=None,
               W=to_np(st.region("W")))
    st.close()
    return out


def compare_units(shape, gpu, ref, layout, tol, tol_small=None):
    """Asserts the per-tensor relative error bound on y, dx and every gradient tensor."""
    worst = {}
    for m, (a, b) in enumerate(zip(gpu["ys"], ref["ys"])):
        worst[f"y[{m}]"] = rel_err(a, b)
    for m, (a, b) in enumerate(zip(gpu["dxs"], ref["dxs"])):
        worst[f"dx[{m}]"] = rel_err(a, b)
    for name, off, r, c in layout:
        worst[f"G.{name}"] = rel_err(gpu["G"][off:off + r * c], ref["G"][off:off + r * c])
        if gpu.get("S0") is not None:
            worst[f"S0.{name}"] = rel_err(gpu["S0"][off:off + r * c], ref["S0"][off:off + r * c])
    bad = {k: v for k, v in worst.items() if not (v <= tol)}
    assert not bad, f"{shape.name}: tolerance {tol} exceeded: {bad}"
    return worst
