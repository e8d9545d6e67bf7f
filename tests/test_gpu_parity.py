"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.

Tolerances: per tensor max|gpu - ref| / max|ref| <= 2e-2 for bf16 MFMA paths with fp32 accumulation,
<= 1e-4 for the all-fp32 configuration (summation order only), and element-wise <= 1e-6 relative for
the Adam update when both sides start from bit-identical fp32 inputs."""
import numpy as np
import pytest
import torch

import oracle
import synth
from synth import StageShape
import paper_2402_03791_amd as zpp
from _harness import (compare_units, make_inputs, rel_err, run_gpu_unit, run_gpu_unit_grouped, run_oracle_unit, to_dev,
                      to_np)

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_FP32 = 1e-4
TOL_ADAM = 1e-6


def f32hp():
    """Adam hyper-parameters as the float32 values the C struct carries, widened for the oracle."""
    return {k: float(np.float32(v)) for k, v in synth.ADAM.items()}


# ------------------------------------------------------------------ flat-buffer passes
@pytest.mark.parametrize("n", [4, 1000, 1579520, 8 * 1024 * 1024 + 4])
def test_flat_adam_matches_oracle(n):
    print(f"flat adam n={n}", flush=True)
    sh = StageShape("flat", 0, 1, 8, 1, 8, 8, 1, 1, 0, 0)  # a dummy stage; only its flat buffers are used
    rng = np.random.default_rng(n)
    p0 = rng.normal(0, 0.02, n).astype(np.float32)
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    g[::11] = 0
    m0 = rng.normal(0, 1e-4, n).astype(np.float32)
    v0 = (rng.normal(0, 1e-4, n).astype(np.float32)) ** 2
    hp = f32hp()
    P, M, V, G = (torch.from_numpy(a.copy()).cuda() for a in (p0, m0, v0, g))
    for step, kw in ((1, {}), (7, dict(decoupled_wd=0, grad_scale=0.5, zero_grad=1))):
        zpp.op_flat_adam(P, M, V, G, step=step, **synth.ADAM, **kw)
        torch.cuda.synchronize()
        # oracle on the same inputs (its buffers are larger than n; only [0, n) is used)
        big = oracle.OracleStage(sh.replace(hidden=64, ffn=64 * 1024, n_heads=1), "f32")
        assert big.N >= n
        big.P[:n], big.M[:n], big.V[:n], big.G[:n] = p0, m0, v0, g
        big.adam(0, n, step=step, decoupled_wd=kw.get("decoupled_wd", 1), grad_scale=kw.get("grad_scale", 1.0),
                 zero_grad=kw.get("zero_grad", 0), **hp)
        for name, a, b in (("p", P, big.P[:n]), ("m", M, big.M[:n]), ("v", V, big.V[:n])):
            a = a.cpu().numpy()
            err = np.abs(a - b) / np.maximum(np.abs(b), 1e-30)
            assert n == 0 or err.max() <= TOL_ADAM, (name, step, err.max())
        if kw.get("zero_grad"):
            assert torch.count_nonzero(G).item() == 0
        p0, m0, v0 = big.P[:n].copy(), big.M[:n].copy(), big.V[:n].copy()
        P.copy_(torch.from_numpy(p0)); M.copy_(torch.from_numpy(m0)); V.copy_(torch.from_numpy(v0))
        big.close()


def test_flat_materialize_is_bit_exact_rne():
    # every bf16 high half with boundary low halves, plus a random bulk with a ragged tail
    highs = np.arange(1 << 16, dtype=np.uint32)
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    pats = ((highs[:, None] << 16) | lows[None, :]).reshape(-1)
    rnd = np.random.default_rng(0).integers(0, 1 << 32, 1000003, dtype=np.uint64).astype(np.uint32)
    bits = np.concatenate([pats, rnd])
    vals = bits.view(np.float32)
    P = torch.from_numpy(vals.copy()).cuda()
    W = torch.empty(P.numel(), dtype=torch.bfloat16, device="cuda")
    zpp.op_flat_materialize(P, W)
    got = W.view(torch.int16).cpu().numpy().view(np.uint16)
    finite = ~np.isnan(vals)
    sample = np.concatenate([np.arange(0, pats.size, 97), pats.size + np.arange(0, rnd.size, 1009)])
    for i in sample:
        if finite[i]:
            assert got[i] == oracle.bf16_bits_rne(float(vals[i])), hex(int(bits[i]))
    # vectorised check of everything finite: RNE by integer arithmetic
    b = bits[finite].astype(np.uint64)
    exp = ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(got[finite], exp)
    nan_out = got[~finite]
    assert np.all((nan_out & 0x7F80) == 0x7F80) and np.all((nan_out & 0x7F) != 0)
    # fp32 mode is a plain copy
    Wf = torch.empty_like(P)
    zpp.op_flat_materialize(P, Wf)
    assert torch.equal(Wf.view(torch.int32), P.view(torch.int32))


@pytest.mark.parametrize("n", [5, 4099, 3 * 1024 * 1024])
def test_flat_accumulate(n):
    rng = np.random.default_rng(n)
    g, s = rng.normal(size=n).astype(np.float32), rng.normal(size=n).astype(np.float32)
    G, S = torch.from_numpy(g.copy()).cuda(), torch.from_numpy(s).cuda()
    zpp.op_flat_accumulate(G, S, 0.25)
    ref = g.astype(np.float64) + 0.25 * s.astype(np.float64)
    assert n == 0 or np.abs(G.cpu().numpy() - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("name", ["cfg1_tiny_gpt_fp32", "small_gpt_5_blocks"])
def test_ranged_adam_matches_oracle_per_range(name):
    """One launch over many ranges, each with its own lr and weight decay (none on gains, offsets and
    biases), against the oracle's Adam called range by range; elements outside the ranges stay untouched."""
    sh = synth.CONFIGS[name] if name in synth.CONFIGS else small(0, 1, n_blocks=5)
    st = zpp.Stage(sh)
    n = st.N
    rng = np.random.default_rng(5)
    p0 = rng.normal(0, 0.02, n).astype(np.float32)
    g0 = rng.normal(0, 1e-3, n).astype(np.float32)
    m0 = rng.normal(0, 1e-4, n).astype(np.float32)
    v0 = rng.normal(0, 1e-4, n).astype(np.float32) ** 2
    hp = f32hp()
    ranges = st.decay_ranges(hp["lr"], 0.1)
    assert len(ranges) > 32 or name.startswith("cfg1")      # the five-block case needs more than one launch
    # leave a hole: drop one range, and give another its own learning rate
    hole = ranges.pop(3)
    ranges[1] = (ranges[1][0], ranges[1][1], 3e-4, ranges[1][3])
    for t, a in ((st.P, p0), (st.M, m0), (st.V, v0), (st.G, g0)):
        t.copy_(torch.from_numpy(a))
    kw = {k: v for k, v in synth.ADAM.items()}
    st.adam_step_ranges(ranges, step=3, zero_grad=1, **kw)
    torch.cuda.synchronize()
    o = oracle.OracleStage(sh, "f32")
    o.P[:], o.M[:], o.V[:], o.G[:] = p0, m0, v0, g0
    ohp = {k: v for k, v in hp.items() if k not in ("lr", "weight_decay")}
    for off, cnt, lr, wd in ranges:
        o.adam(off, cnt, step=3, zero_grad=1, lr=float(np.float32(lr)), weight_decay=float(np.float32(wd)), **ohp)
    for nm, a, b in (("p", st.P, o.P), ("m", st.M, o.M), ("v", st.V, o.V)):
        a = a.cpu().numpy()
        assert (np.abs(a - b) / np.maximum(np.abs(b), 1e-30)).max() <= TOL_ADAM, nm
    g = st.G.cpu().numpy()
    h0, h1 = hole[0], hole[0] + hole[1]
    assert np.array_equal(g[h0:h1], g0[h0:h1]) and np.count_nonzero(g[:h0]) == 0 and np.count_nonzero(g[h1:]) == 0
    assert np.array_equal(st.P.cpu().numpy()[h0:h1], p0[h0:h1])
    # with the same settings in every range the ranged launch equals the plain one bit for bit
    for t, a in ((st.P, p0), (st.M, m0), (st.V, v0), (st.G, g0)):
        t.copy_(torch.from_numpy(a))
    st.adam_step_ranges([(r[0], r[1], synth.ADAM["lr"], synth.ADAM["weight_decay"]) for r in st.decay_ranges(0, 0)],
                        step=2, **kw)
    p_ranged = st.P.clone()
    for t, a in ((st.P, p0), (st.M, m0), (st.V, v0), (st.G, g0)):
        t.copy_(torch.from_numpy(a))
    st.adam_step(step=2, **kw)
    torch.cuda.synchronize()
    assert torch.equal(p_ranged.view(torch.int32), st.P.view(torch.int32))
    st.close()
    o.close()


@pytest.mark.parametrize("arch,dtype,ranged", [(0, 1, False), (1, 1, True), (0, 0, False), (0, 0, True)])
def test_adam_write_back_is_the_cast_materialise_would_do(arch, dtype, ranged):
    sh = small(arch, dtype)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, sh.unit_mbs)
    st = zpp.Stage(sh)
    st.P.copy_(torch.from_numpy(P0))
    st.G.copy_(torch.from_numpy(synth.normal_f32(3, 70, st.N, std=1e-3)))
    st.materialize_params()
    calls0, bytes0 = st.counters()
    if ranged:
        st.adam_step_ranges(st.decay_ranges(synth.ADAM["lr"], 0.1), step=1, write_back=1, **synth.ADAM)
    else:
        st.adam_step(step=1, write_back=1, **synth.ADAM)
    torch.cuda.synchronize()
    # the plain working copy now equals the cast of the new P, bit for bit
    expect = torch.empty(st.N, dtype=st.act_dtype, device="cuda")
    zpp.op_flat_materialize(st.P, expect)
    view = torch.int16 if dtype else torch.int32
    assert torch.equal(st.region("W").view(view), expect.view(view))
    # ... so the next materialise only refreshes the transposed copy (and reads less)
    st.materialize_params()
    calls1, bytes1 = st.counters()
    assert calls1 == calls0 + 1 and bytes1 - bytes0 < bytes0
    y = st.forward(0, to_dev(xs[0], st.act_dtype)).clone()
    dx = st.backward_accumulate(0, to_dev(dys[0], st.act_dtype)).clone()
    torch.cuda.synchronize()
    ref = zpp.Stage(sh)
    ref.P.copy_(st.P)
    ref.G.zero_()
    ref.materialize_params()
    y2 = ref.forward(0, to_dev(xs[0], ref.act_dtype))
    dx2 = ref.backward_accumulate(0, to_dev(dys[0], ref.act_dtype))
    torch.cuda.synchronize()
    assert torch.equal(y.view(view), y2.view(view)) and torch.equal(dx.view(view), dx2.view(view))
    # a step without write-back makes the copy stale again: the next materialise reads P in full
    st.end_unit()
    st.adam_step(step=2, **synth.ADAM)
    st.materialize_params()
    calls2, bytes2 = st.counters()
    assert bytes2 - bytes1 == bytes0
    # the caller rewrites P: (1) with no Adam step in between, the next gather casts from P by itself
    # (a write-back is consumed by the first gather after it); (2) right after a write-back step the
    # caller has to say so
    def w_is_cast_of_p():
        torch.cuda.synchronize()
        zpp.op_flat_materialize(st.P, expect)
        return torch.equal(st.region("W").view(view), expect.view(view))
    st.adam_step(step=3, write_back=1, **synth.ADAM)
    st.materialize_params()
    st.P.mul_(1.5)
    st.materialize_params()
    assert w_is_cast_of_p()
    st.adam_step(step=4, write_back=1, **synth.ADAM)
    st.P.mul_(0.5)
    st.params_changed()
    with pytest.raises(zpp.ZppError):       # the working copy counts as stale until the next gather
        st.forward(0, to_dev(xs[0], st.act_dtype))
    st.materialize_params()
    assert w_is_cast_of_p()
    st.close()
    ref.close()
    dev = zpp.Device(sh, 2)
    with pytest.raises(zpp.ZppError) as e:      # the stages of a device share their working-copy slots
        dev.adam_step(step=1, write_back=1, **synth.ADAM)
    assert e.value.status == -2
    dev.close()


# ------------------------------------------------------------------ whole unit, fp32 (configs[0])
def test_cfg1_tiny_gpt_fp32_full_unit_and_adam():
    sh = synth.CONFIGS["cfg1_tiny_gpt_fp32"]
    print(f"unit {sh.name}", flush=True)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout)
    xs, dys = make_inputs(sh, sh.unit_mbs)
    ref = run_oracle_unit(sh, P0, xs, dys, "f64")
    gpu = run_gpu_unit(sh, P0, xs, dys, keep_stage=True)
    assert np.array_equal(gpu["W"], P0)
    worst = compare_units(sh, gpu, ref, layout, TOL_FP32)
    print("worst rel err", max(worst.values()), flush=True)
    # Adam on bit-identical inputs: feed the GPU's own fp32 G to the oracle
    st = gpu["stage"]
    o = oracle.OracleStage(sh, "f32")
    o.P[:] = P0
    o.G[:] = gpu["G"]
    o.adam(step=1, **f32hp())
    st.adam_step(step=1, **synth.ADAM)
    torch.cuda.synchronize()
    for name, a, b in (("p", st.P, o.P), ("m", st.M, o.M), ("v", st.V, o.V)):
        a = a.cpu().numpy()
        assert (np.abs(a - b) / np.maximum(np.abs(b), 1e-30)).max() <= TOL_ADAM, name
    # the working copy is stale after the step
    with pytest.raises(zpp.ZppError) as e:
        st.end_unit()
        st.forward(0, to_dev(xs[0], st.act_dtype))
    assert e.value.status == -2
    st.close()


def small(arch, dtype, **kw):
    base = dict(name=f"small_a{arch}_d{dtype}", arch=arch, n_blocks=2, hidden=256, n_heads=2, ffn=512, seq=192,
                micro_batch=1, unit_mbs=2, compute_dtype=dtype, seed=11)
    base.update(kw)
    return StageShape(**base)


@pytest.mark.parametrize("arch,dtype,kw", [
    (0, 0, {}), (1, 0, {}), (0, 0, dict(gelu_mode=1, micro_batch=2, seq=96)),
    (0, 1, {}), (1, 1, {}), (0, 1, dict(micro_batch=2, seq=160, ffn=768, n_heads=4)),
    (1, 1, dict(micro_batch=2, seq=96, ffn=320)),
    (1, 0, dict(hidden=192, n_heads=16, ffn=320)), (1, 1, dict(hidden=192, n_heads=16, ffn=320)),  # head dim 12
])
def test_small_stage_units(arch, dtype, kw):
    sh = small(arch, dtype, **kw)
    print(f"unit {sh.name} {kw}", flush=True)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, sh.unit_mbs)
    ref = run_oracle_unit(sh, P0, xs, dys, "f64")
    gpu = run_gpu_unit(sh, P0, xs, dys)
    if dtype == 1:
        assert np.array_equal(gpu["W"], ref["W"])  # same RNE cast on both sides
    worst = compare_units(sh, gpu, ref, layout, TOL_BF16 if dtype == 1 else TOL_FP32)
    print("worst rel err", max(worst.values()), flush=True)


@pytest.mark.parametrize("arch,dtype,kw,scale", [
    (0, 0, {}, 1.0), (1, 0, dict(micro_batch=2, seq=96), 0.37), (0, 1, {}, 1.0), (1, 1, {}, 0.37),
    (0, 1, dict(micro_batch=2, seq=160, ffn=768, n_heads=4, unit_mbs=3), 0.37),
    (1, 1, dict(micro_batch=2, seq=96, ffn=320), 1.0),
])
def test_backward_accumulate_equals_backward_then_accumulate(arch, dtype, kw, scale):
    """The in-place path adds the same fp32 gradient with the same single fused multiply-add per element
    and micro-batch, so G and dx must be bit-identical to the two-call sequence."""
    sh = small(arch, dtype, **kw)
    print(f"in-place unit {sh.name} {kw} scale {scale}", flush=True)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, sh.unit_mbs)
    two = run_gpu_unit(sh, P0, xs, dys, scale=scale)
    one = run_gpu_unit(sh, P0, xs, dys, scale=scale, in_place=True)
    for a, b in zip(two["dxs"], one["dxs"]):
        assert np.array_equal(a, b)
    bad = [name for name, off, r, c in layout
           if not np.array_equal(two["G"][off:off + r * c].view(np.uint32), one["G"][off:off + r * c].view(np.uint32))]
    assert not bad, bad
    # and against the oracle (scaled sum of the micro-batch gradients)
    ref = run_oracle_unit(sh, P0, xs, dys, "f64")
    tol = TOL_BF16 if dtype == 1 else TOL_FP32
    for name, off, r, c in layout:
        assert rel_err(one["G"][off:off + r * c], scale * ref["G"][off:off + r * c]) <= tol, name


@pytest.mark.parametrize("arch,dtype,kw", [
    (0, 0, dict(unit_mbs=3)), (1, 0, dict(micro_batch=2, seq=96, unit_mbs=3)),
    (0, 1, dict(unit_mbs=3)), (1, 1, dict(unit_mbs=3)),
    (0, 1, dict(micro_batch=2, seq=160, ffn=768, n_heads=4, n_blocks=3, unit_mbs=3)),
])
def test_split_backward_tasks_equal_the_fused_call(arch, dtype, kw):
    """Input-gradient and weight-gradient tasks (Section 2.3) run apart from each other - all input-gradient
    tasks of the unit first, weight-gradient tasks later - must reproduce the fused backward bit for bit:
    same kernels, same operands."""
    sh = small(arch, dtype, **kw)
    print(f"split unit {sh.name} {kw}", flush=True)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, sh.unit_mbs)

    def same(a, b, what):
        for x, y in zip(a["dxs"], b["dxs"]):
            assert np.array_equal(x, y), what + " dx"
        bad = [n for n, off, r, c in layout
               if not np.array_equal(a["G"][off:off + r * c].view(np.uint32), b["G"][off:off + r * c].view(np.uint32))]
        assert not bad, (what, bad)

    fused = run_gpu_unit(sh, P0, xs, dys, scale=0.37)
    # staging path: weight-gradient tasks in ascending order, each followed by the accumulate pass
    asc = run_gpu_unit(sh, P0, xs, dys, scale=0.37, split="ascending")
    same(fused, asc, "ascending/staging")
    # the split tasks against the oracle directly (unit scale, so that G is the plain sum)
    ref = run_oracle_unit(sh, P0, xs, dys, "f64")
    compare_units(sh, run_gpu_unit(sh, P0, xs, dys, split="descending"), ref, layout,
                  TOL_BF16 if dtype == 1 else TOL_FP32)
    assert np.array_equal(fused["S0"].view(np.uint32), asc["S0"].view(np.uint32))
    # in-place path, deferred and interleaved
    same(fused, run_gpu_unit(sh, P0, xs, dys, scale=0.37, split="ascending", in_place=True), "ascending/in place")
    same(fused, run_gpu_unit(sh, P0, xs, dys, scale=0.37, split="interleaved", in_place=True), "interleaved")
    # another order of the weight-gradient tasks changes G by summation order only
    desc = run_gpu_unit(sh, P0, xs, dys, scale=0.37, split="descending", in_place=True)
    for x, y in zip(fused["dxs"], desc["dxs"]):
        assert np.array_equal(x, y)
    for n, off, r, c in layout:
        assert rel_err(desc["G"][off:off + r * c], fused["G"][off:off + r * c]) <= 1e-5, n


@pytest.mark.parametrize("arch,dtype,kw", [
    (0, 0, dict(unit_mbs=3)), (1, 0, dict(micro_batch=2, seq=96)), (0, 1, dict(unit_mbs=3)), (1, 1, {}),
    (0, 1, dict(micro_batch=2, seq=160, ffn=768, n_heads=4, n_blocks=3)),
    (1, 1, dict(micro_batch=2, seq=96, ffn=320, n_blocks=3)),
])
def test_activation_recomputation_reproduces_the_stashed_run(arch, dtype, kw):
    """Section 3.3: with recomputation the backward runs each block's forward again from the block input
    that was kept; same kernels, same inputs, so y, dx and G equal the stashed run bit for bit, and the
    oracle bound holds as before."""
    sh = small(arch, dtype, **kw)
    print(f"recompute unit {sh.name} {kw}", flush=True)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, sh.unit_mbs)
    plain = run_gpu_unit(sh, P0, xs, dys)
    for mode in (1, 2):                 # full, selective
        for in_place in (False, True):
            rc = run_gpu_unit(sh, P0, xs, dys, recompute=mode, in_place=in_place)
            for a, b in zip(plain["ys"] + plain["dxs"], rc["ys"] + rc["dxs"]):
                assert np.array_equal(a, b), (mode, in_place)
            assert np.array_equal(plain["G"].view(np.uint32), rc["G"].view(np.uint32)), (mode, in_place)
            if not in_place:
                assert np.array_equal(plain["S0"].view(np.uint32), rc["S0"].view(np.uint32))
        # the two backward tasks apart, each rebuilding for itself: weight-gradient tasks after all
        # input-gradient tasks, so the shared slot has been through every block of every micro-batch in between
        sp = run_gpu_unit(sh, P0, xs, dys, recompute=mode, in_place=True, split="descending")
        for a, b in zip(plain["ys"] + plain["dxs"], sp["ys"] + sp["dxs"]):
            assert np.array_equal(a, b), (mode, "split")
        for n, off, r, c in layout:
            assert rel_err(sp["G"][off:off + r * c], plain["G"][off:off + r * c]) <= 1e-5, (mode, n)
    ref = run_oracle_unit(sh, P0, xs, dys, "f64")
    rc["S0"] = plain["S0"]
    compare_units(sh, rc, ref, layout, TOL_BF16 if dtype == 1 else TOL_FP32)
    sp["S0"] = None
    compare_units(sh, sp, ref, layout, TOL_BF16 if dtype == 1 else TOL_FP32)


@pytest.mark.parametrize("arch,dtype,V,per,prefetch,grp", [
    (0, 1, 2, 2, True, 0), (0, 1, 2, 2, False, 0), (1, 1, 4, 1, True, 0), (0, 0, 2, 1, True, 0), (0, 1, 3, 1, True, 0),
    (1, 1, 3, 1, False, 0), (0, 1, 2, 2, True, 2), (1, 1, 2, 1, True, 3), (0, 0, 2, 1, True, 2), (0, 1, 2, 1, False, 1),
])
def test_device_of_V_stages_equals_one_stage_of_all_blocks(arch, dtype, V, per, prefetch, grp):
    """V stages that take turns in one or two working-copy slots (the next one gathered on a second stream
    while the current one computes) against a single stage holding all V * per blocks: two units with an
    Adam step after each, everything bit-identical (same kernels, same operands, same order per tensor)."""
    sh_all = small(arch, dtype, n_blocks=V * per, unit_mbs=3)
    sh_one = sh_all.replace(n_blocks=per)
    print(f"device {sh_all.name} V={V} per={per} prefetch={prefetch}", flush=True)
    U = sh_all.unit_mbs
    P0 = synth.make_params(sh_all, oracle.param_layout(sh_all), gain_jitter=0.1)
    xs, dys = make_inputs(sh_all, U)

    st = zpp.Stage(sh_all, split_backward=grp)
    st.P.copy_(torch.from_numpy(P0))
    st.G.zero_()
    ref = []
    for unit in range(2):
        st.materialize_params()
        ys = [st.forward(m, to_dev(xs[m], st.act_dtype)) for m in range(U)]
        if grp == 0:
            dxs = [st.backward_accumulate(m, to_dev(dys[m], st.act_dtype), scale=0.5) for m in range(U)]
        else:
            # input-gradient tasks, then weight-gradient tasks in groups of grp (one by one in fp32)
            dxs = [st.backward_input(m, to_dev(dys[m], st.act_dtype)) for m in range(U)]
            for first in range(0, U, grp):
                st.backward_weight_group(first, min(grp, U - first), 0.5)
        g = st.G.clone()
        st.adam_step(step=unit + 1, zero_grad=1, **synth.ADAM)
        st.end_unit()
        torch.cuda.synchronize()
        ref.append((ys, dxs, g, st.P.clone()))
    st.close()

    dev = zpp.Device(sh_one, V, prefetch=prefetch, split_backward=grp)
    assert dev.N_total == P0.size
    dev.P.copy_(torch.from_numpy(P0))
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    act = dev.act_dtype
    x_in = [to_dev(xs[m], act) for m in range(U)]
    dy_in = [to_dev(dys[m], act) for m in range(U)]
    # activations between the stages: y of stage v is x of stage v+1; dx of stage v is dy of stage v-1
    mid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
    gmid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
    x_list = [(x_in[m] if v == 0 else mid[v - 1][m]) for v in range(V) for m in range(U)]
    y_list = [mid[v][m] for v in range(V) for m in range(U)]
    dy_list = [(dy_in[m] if v == V - 1 else gmid[v + 1][m]) for v in range(V) for m in range(U)]
    dx_list = [gmid[v][m] for v in range(V) for m in range(U)]
    layout = oracle.param_layout(sh_all)
    ora = run_oracle_unit(sh_all, P0, xs, dys, "f64")   # the V stages are one stack of V * per blocks
    tol = TOL_BF16 if dtype == 1 else TOL_FP32
    for unit in range(2):
        dev.forward_unit(x_list, y_list, main, side)
        dev.backward_unit(dy_list, dx_list, 0.5, main, side)
        torch.cuda.synchronize()
        if unit == 0:
            # the device against the oracle directly: outputs of the last stage, input gradients of the
            # first, and the accumulated gradients of all stages (scale 0.5)
            for m in range(U):
                assert rel_err(to_np(mid[V - 1][m]), ora["ys"][m]) <= tol, ("y vs oracle", m)
                assert rel_err(to_np(gmid[0][m]), ora["dxs"][m]) <= tol, ("dx vs oracle", m)
            g_host = to_np(dev.G)
            for name, off, r, c in layout:
                assert rel_err(g_host[off:off + r * c], 0.5 * ora["G"][off:off + r * c]) <= tol, ("G vs oracle", name)
        ys, dxs, g, p = ref[unit]
        for m in range(U):
            assert torch.equal(mid[V - 1][m].view(torch.int16 if dtype else torch.int32),
                               ys[m].view(torch.int16 if dtype else torch.int32)), ("y", unit, m)
            assert torch.equal(gmid[0][m].view(torch.int16 if dtype else torch.int32),
                               dxs[m].view(torch.int16 if dtype else torch.int32)), ("dx", unit, m)
        assert torch.equal(dev.G.view(torch.int32), g.view(torch.int32)), ("G", unit)
        dev.adam_step(step=unit + 1, zero_grad=1, **synth.ADAM)
        dev.end_unit()
        torch.cuda.synchronize()
        assert torch.equal(dev.P.view(torch.int32), p.view(torch.int32)), ("P", unit)
    dev.close()


@pytest.mark.parametrize("arch,kw,g", [
    (0, dict(unit_mbs=4), 2), (0, dict(unit_mbs=5, n_blocks=3), 3), (1, dict(unit_mbs=4), 4),
    (0, dict(micro_batch=2, seq=128, ffn=768, n_heads=4, unit_mbs=3), 2),
])
def test_grouped_weight_gradient_tasks(arch, kw, g):
    """Weight-gradient tasks of g micro-batches as one product over K = g*T: the sum over the group is formed
    in the product's fp32 accumulator, so G matches the one-by-one result up to summation order, dx exactly."""
    sh = small(arch, 1, **kw)
    print(f"grouped W {sh.name} {kw} g={g}", flush=True)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, sh.unit_mbs)
    fused = run_gpu_unit(sh, P0, xs, dys, scale=0.37, in_place=True)
    grouped = run_gpu_unit(sh, P0, xs, dys, scale=0.37, in_place=True, split=("group", g))
    for x, y in zip(fused["dxs"], grouped["dxs"]):
        assert np.array_equal(x, y)
    ref = run_oracle_unit(sh, P0, xs, dys, "f64")
    for n, off, r, c in layout:
        assert rel_err(grouped["G"][off:off + r * c], fused["G"][off:off + r * c]) <= 1e-5, n
        assert rel_err(grouped["G"][off:off + r * c], 0.37 * ref["G"][off:off + r * c]) <= TOL_BF16, n
    # more micro-batches than the configuration allows, and a micro-batch without its input-gradient task
    st = zpp.Stage(sh, split_backward=g)
    st.materialize_params()
    x, dy = to_dev(xs[0], st.act_dtype), to_dev(dys[0], st.act_dtype)
    for m in range(sh.unit_mbs):
        st.forward(m, x)
    st.backward_input(0, dy)
    for first, count, status in ((0, g + 1, -2 if g + 1 <= sh.unit_mbs else -1), (0, 2, -2), (sh.unit_mbs - 1, 2, -1)):
        with pytest.raises(zpp.ZppError) as e:
            st.backward_weight_group(first, count)
        assert e.value.status == status, (first, count)
    st.backward_weight_group(0, 1)
    st.close()


@pytest.mark.parametrize("arch,dtype,kw,g", [
    (0, 1, dict(unit_mbs=4), 2), (1, 1, dict(unit_mbs=5, n_blocks=3), 3), (0, 0, dict(unit_mbs=4), 4),
    (1, 0, dict(micro_batch=2, seq=96, unit_mbs=3), 2), (0, 1, dict(micro_batch=2, seq=128, ffn=768, n_heads=4, unit_mbs=4), 4),
])
def test_grouped_calls_equal_the_one_by_one_calls(arch, dtype, kw, g):
    """g micro-batches per call as one [g*T, h] matrix (forward, input-gradient and fused backward tasks):
    row by row the same arithmetic, so y and dx equal the one-micro-batch calls bit for bit; the gradients
    of a group are summed inside the products, so G agrees up to summation order; and everything is held
    to the oracle bound directly."""
    sh = small(arch, dtype, **kw)
    print(f"grouped calls {sh.name} {kw} g={g}", flush=True)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, sh.unit_mbs)
    one = run_gpu_unit(sh, P0, xs, dys, in_place=True)
    ref = run_oracle_unit(sh, P0, xs, dys, "f64")
    tol = TOL_BF16 if dtype == 1 else TOL_FP32
    runs = dict(split=run_gpu_unit_grouped(sh, P0, xs, dys, g, fused=False),
                fused=run_gpu_unit_grouped(sh, P0, xs, dys, g, fused=True),
                split_wide=run_gpu_unit_grouped(sh, P0, xs, dys, max(g // 2, 1), fused=False, weight_group=g),
                fused_full_recompute=run_gpu_unit_grouped(sh, P0, xs, dys, g, fused=True, recompute=1),
                split_selective=run_gpu_unit_grouped(sh, P0, xs, dys, g, fused=False, recompute=2))
    for tag, grp in runs.items():
        for a, b in zip(one["ys"] + one["dxs"], grp["ys"] + grp["dxs"]):
            assert np.array_equal(a, b), tag
        for n, off, r, c in layout:
            assert rel_err(grp["G"][off:off + r * c], one["G"][off:off + r * c]) <= 2e-5, (tag, n)
        compare_units(sh, grp, ref, layout, tol)
    # a weight-gradient task must cover grouped input-gradient tasks whole
    st = zpp.Stage(sh, split_backward=g, group_mbs=g)
    st.materialize_params()
    x = to_dev(np.concatenate(xs[:2], axis=0), st.act_dtype)
    dy = to_dev(np.concatenate(dys[:2], axis=0), st.act_dtype)
    st.forward_group(0, 2, x)
    st.backward_input_group(0, 2, dy)
    with pytest.raises(zpp.ZppError) as e:
        st.backward_weight(0, in_place=True)
    assert e.value.status == -2
    st.backward_weight_group(0, 2)
    st.close()


@pytest.mark.parametrize("arch,dtype", [(0, 1), (1, 1), (0, 0)])
@pytest.mark.parametrize("order,scale", [("group", 1.0), ("group", 0.5), ("fused", 1.0), ("five", 1.0), ("five", 0.25)])
def test_released_gradient_buffer_gives_what_zeroing_gives(arch, dtype, order, scale):
    """Adam with zero_grad = 2 leaves the old gradients in G and the stage treats G as zero: the first call that
    adds into G afterwards writes instead.  Two units in a row, the Adam step between them zeroing G or releasing
    it: the second unit's G and the parameters after a second step are equal (as values: an exact zero may differ
    in sign), in every order of the work and with a scale other than 1."""
    sh = small(arch, dtype, unit_mbs=4)
    print(f"released G {sh.name} {order} scale {scale}", flush=True)
    U = sh.unit_mbs
    layout = oracle.param_layout(sh)
    P0 = torch.from_numpy(synth.make_params(sh, layout, gain_jitter=0.1))
    xs, dys = make_inputs(sh, U)

    def unit(st):
        st.materialize_params()
        xd = [to_dev(x, st.act_dtype) for x in xs]
        dyd = [to_dev(d, st.act_dtype) for d in dys]
        if order == "group":
            for f in range(0, U, 2):
                st.forward_group(f, 2, torch.cat(xd[f:f + 2]))
            for f in range(0, U, 2):
                st.backward_input_group(f, 2, torch.cat(dyd[f:f + 2]))
            st.backward_weight_group(0, 2, scale)
            st.backward_weight_group(2, 2, scale)
        else:
            for m in range(U):
                st.forward(m, xd[m])
            for m in range(U):
                if order == "fused":
                    st.backward_accumulate(m, dyd[m], scale=scale)
                else:
                    st.backward(m, dyd[m])
                    st.accumulate_grads(m, scale)
        st.end_unit()

    res = {}
    for zg in (1, 2):
        st = zpp.Stage(sh, split_backward=2 if order == "group" else 0, group_mbs=2)
        st.P.copy_(P0)
        st.G.zero_()
        unit(st)
        g1 = st.G.clone()
        st.adam_step(step=1, zero_grad=zg, write_back=1, **synth.ADAM)
        if zg == 1:
            assert float(st.G.abs().max()) == 0.0
        else:
            assert torch.equal(st.G, g1)          # nothing was written: the release is bookkeeping
        unit(st)
        g2 = st.G.clone()
        st.adam_step(step=2, zero_grad=zg, write_back=1, **synth.ADAM)
        torch.cuda.synchronize()
        res[zg] = (g2, st.P.clone(), st.M.clone(), st.V.clone())
        st.close()
    for a, b in zip(res[1], res[2]):
        assert bool(torch.isfinite(a).all()) and float(a.abs().max()) > 0
        assert torch.equal(a, b)
    # a release needs the whole shard, and only a stage can hold it
    st = zpp.Stage(sh)
    with pytest.raises(zpp.ZppError) as e:
        st.adam_step(offset=0, count=st.N - 4, step=1, zero_grad=2, **synth.ADAM)
    assert e.value.status == -1
    with pytest.raises(zpp.ZppError) as e:
        st.adam_step(step=1, zero_grad=3, **synth.ADAM)
    assert e.value.status == -1
    st.close()


@pytest.mark.parametrize("grp", [0, 2])
def test_device_with_released_gradient_buffers(grp):
    """Every stage of a device holds its own release: two units through V = 2 stages with the Adam step between
    them zeroing or releasing G give the same gradients and parameters (scale 1: the in-place tasks of the
    second unit write)."""
    sh = small(0, 1, n_blocks=1, unit_mbs=4)
    U, V = sh.unit_mbs, 2
    sh_all = sh.replace(n_blocks=V)
    print(f"device released G grp={grp}", flush=True)
    P0 = torch.from_numpy(synth.make_params(sh_all, oracle.param_layout(sh_all), gain_jitter=0.1))
    xs, dys = make_inputs(sh, U)
    res = {}
    for zg in (1, 2):
        dev = zpp.Device(sh, V, prefetch=True, split_backward=grp)
        dev.P.copy_(P0)
        main, side = torch.cuda.current_stream(), torch.cuda.Stream()
        x_in = [to_dev(xs[m], dev.act_dtype) for m in range(U)]
        dy_in = [to_dev(dys[m], dev.act_dtype) for m in range(U)]
        mid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
        gmid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
        x_list = [(x_in[m] if v == 0 else mid[v - 1][m]) for v in range(V) for m in range(U)]
        y_list = [mid[v][m] for v in range(V) for m in range(U)]
        dy_list = [(dy_in[m] if v == V - 1 else gmid[v + 1][m]) for v in range(V) for m in range(U)]
        dx_list = [gmid[v][m] for v in range(V) for m in range(U)]
        out = []
        for unit in range(2):
            dev.forward_unit(x_list, y_list, main, side)
            dev.backward_unit(dy_list, dx_list, 1.0, main, side)
            torch.cuda.synchronize()
            out.append(dev.G.clone())
            dev.adam_step(step=unit + 1, zero_grad=zg, **synth.ADAM)
            dev.end_unit()
            torch.cuda.synchronize()
            out.append(dev.P.clone())
            if unit == 0 and zg == 2:
                assert torch.equal(dev.G, out[0])      # released, not written
        res[zg] = out
        dev.close()
    for a, b in zip(res[1], res[2]):
        assert bool(torch.isfinite(a).all()) and float(a.abs().max()) > 0
        assert torch.equal(a, b)


def test_device_recomputes_every_stage_but_the_last():
    """Section 3.3: the stages mapped to a device recompute (one rebuild serves their two back-to-back gradient
    tasks) except the last one, whose tasks are scheduled apart and which keeps its activations.  Same kernels
    on the same operands as a device that keeps everything: identical y and dx, G up to summation order, and
    the oracle bound directly."""
    sh = small(0, 1, n_blocks=1, unit_mbs=4)
    U, V = sh.unit_mbs, 3
    sh_all = sh.replace(n_blocks=V)
    layout = oracle.param_layout(sh_all)
    P0 = synth.make_params(sh_all, layout, gain_jitter=0.1)
    xs, dys = make_inputs(sh, U)
    ora = run_oracle_unit(sh_all, P0, xs, dys, "f64")
    results = []
    for modes in ([0, 0, 0], [1, 1, 0], [2, 1, 0]):
        dev = zpp.Device(sh, V, prefetch=True, recompute=modes, split_backward=2)
        dev.P.copy_(torch.from_numpy(P0))
        main, side = torch.cuda.current_stream(), torch.cuda.Stream()
        x_in = [to_dev(xs[m], dev.act_dtype) for m in range(U)]
        dy_in = [to_dev(dys[m], dev.act_dtype) for m in range(U)]
        mid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
        gmid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
        dev.forward_unit([(x_in[m] if v == 0 else mid[v - 1][m]) for v in range(V) for m in range(U)],
                         [mid[v][m] for v in range(V) for m in range(U)], main, side)
        dev.backward_unit([(dy_in[m] if v == V - 1 else gmid[v + 1][m]) for v in range(V) for m in range(U)],
                          [gmid[v][m] for v in range(V) for m in range(U)], 1.0, main, side)
        torch.cuda.synchronize()
        results.append(dict(ys=[to_np(t) for t in mid[V - 1]], dxs=[to_np(t) for t in gmid[0]], G=to_np(dev.G),
                            stash=dev.memory_terms()["stash"]))
        dev.close()
    for r in results:
        compare_units(sh_all, r, ora, layout, TOL_BF16)
    for r in results[1:]:
        for a, b in zip(results[0]["ys"] + results[0]["dxs"], r["ys"] + r["dxs"]):
            assert np.array_equal(a, b)
        for n, off, rr, c in layout:
            assert rel_err(r["G"][off:off + rr * c], results[0]["G"][off:off + rr * c]) <= 2e-5, n
    assert results[1]["stash"] < 0.6 * results[0]["stash"]


def test_device_with_recomputation_matches_device_without():
    sh = small(1, 1, n_blocks=2, unit_mbs=3)
    U, V = sh.unit_mbs, 2
    P0 = synth.make_params(sh.replace(n_blocks=4), oracle.param_layout(sh.replace(n_blocks=4)), gain_jitter=0.1)
    xs, dys = make_inputs(sh, U)
    results = []
    for rc in (False, True):
        dev = zpp.Device(sh, V, prefetch=True, recompute=rc)
        dev.P.copy_(torch.from_numpy(P0))
        main, side = torch.cuda.current_stream(), torch.cuda.Stream()
        x_in = [to_dev(xs[m], dev.act_dtype) for m in range(U)]
        dy_in = [to_dev(dys[m], dev.act_dtype) for m in range(U)]
        mid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
        gmid = [[torch.empty_like(x_in[0]) for _ in range(U)] for _ in range(V)]
        dev.forward_unit([(x_in[m] if v == 0 else mid[v - 1][m]) for v in range(V) for m in range(U)],
                         [mid[v][m] for v in range(V) for m in range(U)], main, side)
        dev.backward_unit([(dy_in[m] if v == V - 1 else gmid[v + 1][m]) for v in range(V) for m in range(U)],
                          [gmid[v][m] for v in range(V) for m in range(U)], 1.0, main, side)
        torch.cuda.synchronize()
        results.append((dev.G.clone(), [t.clone() for t in gmid[0]], dev.memory_terms()["stash"]))
        dev.close()
    assert torch.equal(results[0][0].view(torch.int32), results[1][0].view(torch.int32))
    for a, b in zip(results[0][1], results[1][1]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert results[1][2] < results[0][2] / 3      # the stashes shrink to the block inputs


def test_split_backward_state_machine():
    sh = small(0, 1)
    st = zpp.Stage(sh, split_backward=True)
    st.P.copy_(torch.from_numpy(synth.make_params(sh, oracle.param_layout(sh))))
    st.G.zero_()
    st.materialize_params()
    xs, dys = make_inputs(sh, sh.unit_mbs)
    x, dy = to_dev(xs[0], st.act_dtype), to_dev(dys[0], st.act_dtype)

    def refused(fn):
        with pytest.raises(zpp.ZppError) as e:
            fn()
        assert e.value.status == -2

    refused(lambda: st.backward_input(0, dy))           # no forward yet
    st.forward(0, x)
    st.forward(1, x)
    refused(lambda: st.backward_weight(0))              # no input-gradient task yet
    st.backward_input(0, dy)
    refused(lambda: st.backward_input(0, dy))           # twice
    refused(lambda: st.backward(0, dy))                 # the fused call no longer applies
    refused(lambda: st.adam_step(step=1, **synth.ADAM))  # a weight-gradient task is due
    refused(lambda: st.end_unit())
    st.backward_input(1, dy)                            # another input-gradient task may come first
    st.backward_weight(1, in_place=False)
    refused(lambda: st.backward_weight(0, in_place=False))  # staging buffer holds micro-batch 1
    st.backward_weight(0, in_place=True, scale=1.0)     # in place does not need the staging buffer
    refused(lambda: st.backward_weight(0, in_place=True))
    st.accumulate_grads(1)
    st.adam_step(step=1, **synth.ADAM)
    st.end_unit()
    torch.cuda.synchronize()
    st.close()
    plain = zpp.Stage(sh)
    plain.materialize_params()
    plain.forward(0, x)
    refused(lambda: plain.backward_input(0, dy))        # created without split_backward
    plain.close()


def test_backward_accumulate_state_machine():
    sh = small(0, 1)
    st = zpp.Stage(sh)
    st.P.copy_(torch.from_numpy(synth.make_params(sh, oracle.param_layout(sh))))
    st.G.zero_()
    st.materialize_params()
    xs, dys = make_inputs(sh, sh.unit_mbs)
    x, dy = to_dev(xs[0], st.act_dtype), to_dev(dys[0], st.act_dtype)
    with pytest.raises(zpp.ZppError) as e:   # no forward yet
        st.backward_accumulate(0, dy)
    assert e.value.status == -2
    st.forward(0, x)
    st.forward(1, x)
    with pytest.raises(zpp.ZppError) as e:   # forward-done micro-batches would meet new weights in backward
        st.adam_step(step=1, **synth.ADAM)
    assert e.value.status == -2
    st.backward(1, dy)
    st.backward_accumulate(0, dy)            # does not use the staging buffer, which still holds micro-batch 1
    with pytest.raises(zpp.ZppError) as e:   # ... and still waits for its accumulate pass
        st.adam_step(step=1, **synth.ADAM)
    assert e.value.status == -2
    st.accumulate_grads(1)
    with pytest.raises(zpp.ZppError) as e:   # already accumulated
        st.accumulate_grads(0)
    assert e.value.status == -2
    with pytest.raises(zpp.ZppError) as e:
        st.backward_accumulate(0, dy)
    assert e.value.status == -2
    st.adam_step(step=1, **synth.ADAM)       # nothing pending
    torch.cuda.synchronize()
    st.close()


@pytest.mark.parametrize("arch,kw", [(0, {}), (1, dict(ffn=320)), (0, dict(hidden=512, n_heads=4, ffn=1024)),
                                     (0, dict(hidden=320, n_heads=4, ffn=640)), (1, dict(hidden=192, n_heads=2, ffn=448))])
def test_transposed_working_copy_is_the_transposed_cast(arch, kw):
    """The gather also writes transposed every matrix whose input-gradient product cannot read it as stored
    (in not a multiple of 256 or out not a multiple of 64): bit for bit the transposed round-to-nearest-even
    cast of P, the gate and up matrices of the LLaMA block as one [h, 2f].  The other matrices have no
    transposed copy (first and third case: none at all)."""
    sh = small(arch, 1, **kw)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout, gain_jitter=0.1)
    st = zpp.Stage(sh)
    st.P.copy_(torch.from_numpy(P0))
    st.materialize_params()
    torch.cuda.synchronize()
    wt = st.region("Wt").view(torch.int16).cpu().numpy().view(np.uint16)
    pos = 0
    for name, off, r, c in layout:
        if r <= 1 or name.endswith("mlp.wup"):
            continue
        if name.endswith("mlp.wgate"):
            r *= 2
        if c % 256 == 0 and r % 64 == 0 and off % 8 == 0:
            continue
        expect = oracle.flat_materialize_bits(P0[off:off + r * c]).reshape(r, c).T
        assert np.array_equal(wt[pos:pos + r * c].reshape(c, r), expect), name
        pos += r * c
    assert pos == wt.size
    st.close()


@pytest.mark.parametrize("dtype", [0, 1])
def test_gelu_far_from_zero(dtype):
    """Activations far out on both sides (MLP pre-activations of several tens): the tanh-form GeLU and its
    derivative, evaluated through exp2 and a reciprocal on the device, saturate to 0 / u and 0 / 1 and stay
    finite, in the forward epilogue, the backward epilogue and the element-wise rebuild."""
    sh = small(0, dtype, n_blocks=1, unit_mbs=1)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout)
    for name, off, r, c in layout:
        if name.endswith("mlp.w1"):
            P0[off:off + r * c] *= 60.0                      # pre-activations u of a few tens
    xs, dys = make_inputs(sh, 1)
    ref = run_oracle_unit(sh, P0, xs, dys, dtype="f64", keep_stage=True)
    u = np.array(ref["stage"].stash(0, 0, "u"))
    ref["stage"].close()
    assert np.abs(u).max() > 20.0 and u.min() < -20.0
    got = run_gpu_unit(sh, P0, xs, dys)
    assert all(np.isfinite(a).all() for k in ("ys", "dxs") for a in got[k]) and np.isfinite(got["G"]).all()
    compare_units(sh, got, ref, layout, TOL_BF16 if dtype == 1 else TOL_FP32)


def test_materialize_counters_and_idempotence():
    sh = small(0, 1)
    layout = oracle.param_layout(sh)
    P0 = synth.make_params(sh, layout)
    st = zpp.Stage(sh)
    st.P.copy_(torch.from_numpy(P0))
    st.materialize_params()
    w1 = st.region("W").clone()
    x = to_dev(synth.make_x(sh, 0), st.act_dtype)
    y1 = st.forward(0, x).clone()
    st.materialize_params()  # the paper's second gather before the backward phase: must not change anything
    assert torch.equal(w1.view(torch.int16), st.region("W").view(torch.int16))
    calls, nbytes = st.counters()
    assert calls == 2 and nbytes > 0
    st.end_unit()
    y2 = st.forward(0, x)
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))  # run-to-run identical
    st.close()


# ------------------------------------------------------------------ operators
@pytest.mark.parametrize("M,N,K,tile", [
    (256, 256, 64, "256x256"), (300, 520, 192, "256x256"), (300, 520, 192, "128x128"), (300, 520, 192, "256x128"),
    (300, 520, 192, "128x256"), (64, 96, 128, "auto"), (1, 1, 64, "128x128"), (1, 1, 64, "128x256"),
    (777, 129, 256, "auto"), (2048, 512, 1024, "auto"), (512, 2048, 64, "256x256"), (1000, 1000, 320, "256x256"),
    (1000, 1000, 320, "128x128"), (1000, 1000, 320, "256x128"), (512, 256, 768, "256x128"), (256, 512, 1024, "128x256"),
])
def test_gemm_bf16_nt_against_oracle(M, N, K, tile):
    print(f"gemm {M}x{N}x{K} tile {tile}", flush=True)
    a = synth.normal_f32(1, 50, M * K, bf16_exact=True).reshape(M, K)
    b = synth.normal_f32(1, 51, N * K, std=0.05, bf16_exact=True).reshape(N, K)
    bias = synth.normal_f32(1, 52, N, bf16_exact=True)
    res = synth.normal_f32(1, 53, M * N, bf16_exact=True).reshape(M, N)
    ref = oracle.Ops("f64").linear_fwd(a, b, bias) + res
    A, B, Bi, R = (to_dev(t, torch.bfloat16) for t in (a, b, bias, res))
    C = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    zpp.op_gemm_bf16_nt(A, B, C, bias=Bi, resid=R, tile=tile)
    assert rel_err(to_np(C), ref) <= 8e-3  # bf16 output rounding only (2^-9 relative)
    Cf = torch.empty(M, N, dtype=torch.float32, device="cuda")
    zpp.op_gemm_bf16_nt(A, B, Cf, tile=tile)
    ref2 = oracle.Ops("f64").linear_fwd(a, b)
    assert rel_err(to_np(Cf), ref2) <= 1e-5      # fp32 accumulation of exact bf16 products
    # accumulation in place: every element receives exactly one rounded add of the same fp32 product
    g0 = torch.from_numpy(synth.normal_f32(1, 54, M * N).reshape(M, N)).cuda()
    G = g0.clone()
    zpp.op_gemm_bf16_nt(A, B, G, tile=tile, accumulate=True)
    assert torch.equal(G, g0 + Cf)


@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (256, 512, 192), (768, 256, 1024), (1024, 2048, 512)])
def test_gemm_bf16_tt_against_oracle(M, N, K):
    """dW = dY^T . X straight from the token-major operands, with strided rows, written and accumulated."""
    print(f"gemm tt {M}x{N}x{K}", flush=True)
    dy = synth.normal_f32(4, 80, K * M, bf16_exact=True).reshape(K, M)
    x = synth.normal_f32(4, 81, K * N, bf16_exact=True).reshape(K, N)
    ref, _ = oracle.Ops("f64").linear_bwd_weight(dy, x)
    # operands as column slices of wider matrices, so the leading dimensions differ from M and N
    Aw = torch.zeros(K, M + 64, dtype=torch.bfloat16, device="cuda")
    Bw = torch.zeros(K, N + 128, dtype=torch.bfloat16, device="cuda")
    Aw[:, 64:] = to_dev(dy, torch.bfloat16)
    Bw[:, :N] = to_dev(x, torch.bfloat16)
    A, B = Aw[:, 64:], Bw[:, :N]
    C = torch.empty(M, N, dtype=torch.float32, device="cuda")
    zpp.op_gemm_bf16_tt(A, B, C)
    assert rel_err(to_np(C), ref) <= 1e-5
    Cb = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    zpp.op_gemm_bf16_tt(A, B, Cb)
    assert rel_err(to_np(Cb), ref) <= 8e-3
    g0 = torch.from_numpy(synth.normal_f32(1, 54, M * N).reshape(M, N)).cuda()
    G = g0.clone()
    zpp.op_gemm_bf16_tt(A, B, G, accumulate=True)
    assert torch.equal(G, g0 + C)
    with pytest.raises(zpp.ZppError) as e:      # shapes the K-major kernel does not take are refused, not mangled
        zpp.op_gemm_bf16_tt(A[:, :128], B, C[:128])
    assert e.value.status == -6


@pytest.mark.parametrize("shapes,K", [(((256, 256),), 128),
                                      (((768, 256), (256, 256), (1024, 256), (256, 1024)), 512),
                                      # 75 + 25 + 270 + 135 tiles: one product ends and the next begins inside a
                                      # round of one tile per CU, three times; no product's tile count is a multiple of 8
                                      (((3840, 1280), (1280, 1280), (6912, 2560), (1280, 6912)), 192),
                                      (((512, 256),) * 8, 64)])
def test_gemm_bf16_tt_group_equals_the_single_products(shapes, K):
    """Several K-major products as one grid: the first against the oracle, all of them bit for bit against one
    launch per product (written, accumulated, bf16 output), operands with their own leading dimensions."""
    print(f"gemm tt group {shapes} K={K}", flush=True)
    As, Bs = [], []
    for i, (M, N) in enumerate(shapes):
        Aw = torch.zeros(K, M + 8 * (i + 1), dtype=torch.bfloat16, device="cuda")
        Bw = torch.zeros(K, N + 64, dtype=torch.bfloat16, device="cuda")
        Aw[:, :M] = to_dev(synth.normal_f32(6, 90 + i, K * M, bf16_exact=True).reshape(K, M), torch.bfloat16)
        Bw[:, 64:] = to_dev(synth.normal_f32(6, 190 + i, K * N, bf16_exact=True).reshape(K, N), torch.bfloat16)
        As.append(Aw[:, :M])
        Bs.append(Bw[:, 64:])
    for dtype in (torch.float32, torch.bfloat16):
        Cs = [torch.full((M, N), 7.0, dtype=dtype, device="cuda") for M, N in shapes]
        zpp.op_gemm_bf16_tt_group(As, Bs, Cs)
        for A, B, C in zip(As, Bs, Cs):
            assert torch.equal(C, zpp.op_gemm_bf16_tt(A, B, torch.empty_like(C)))
    M0, N0 = shapes[0]
    ref, _ = oracle.Ops("f64").linear_bwd_weight(to_np(As[0]), to_np(Bs[0]))
    assert rel_err(to_np(Cs[0]), ref) <= 8e-3
    G0 = [torch.from_numpy(synth.normal_f32(6, 290 + i, M * N).reshape(M, N)).cuda() for i, (M, N) in enumerate(shapes)]
    G = [g.clone() for g in G0]
    zpp.op_gemm_bf16_tt_group(As, Bs, G, accumulate=True)
    for A, B, g, g0 in zip(As, Bs, G, G0):
        assert torch.equal(g, zpp.op_gemm_bf16_tt(A, B, g0.clone(), accumulate=True))
    with pytest.raises(zpp.ZppError) as e:      # a product the K-major kernel does not take refuses the whole group
        zpp.op_gemm_bf16_tt_group(As[:1] + [As[0][:, :128]], Bs[:1] + Bs[:1], [G[0], G[0][:128]])
    assert e.value.status == -6
    with pytest.raises(zpp.ZppError) as e:
        zpp.op_gemm_bf16_tt_group(As[:1] * 9, Bs[:1] * 9, G[:1] * 9)
    assert e.value.status == -1


@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (200, 512, 192), (1000, 256, 1024), (2048, 1024, 512),
                                   (4096, 4096, 256)])
def test_gemm_bf16_nn_against_oracle(M, N, K):
    """dX = dY . W from the weights as stored ([out, in] = [K, N]); ragged M, strided rows, both tile shapes."""
    print(f"gemm nn {M}x{N}x{K}", flush=True)
    dy = synth.normal_f32(5, 80, M * K, bf16_exact=True).reshape(M, K)
    w = synth.normal_f32(5, 81, K * N, bf16_exact=True).reshape(K, N)
    ref = oracle.Ops("f64").linear_bwd_input(dy, w)
    Aw = torch.zeros(M, K + 64, dtype=torch.bfloat16, device="cuda")
    Bw = torch.zeros(K, N + 128, dtype=torch.bfloat16, device="cuda")
    Aw[:, 64:] = to_dev(dy, torch.bfloat16)
    Bw[:, :N] = to_dev(w, torch.bfloat16)
    A, B = Aw[:, 64:], Bw[:, :N]
    C = torch.empty(M, N, dtype=torch.float32, device="cuda")
    zpp.op_gemm_bf16_nn(A, B, C)
    assert rel_err(to_np(C), ref) <= 1e-5
    Cb = torch.full((M + 3, N), 7.0, dtype=torch.bfloat16, device="cuda")
    zpp.op_gemm_bf16_nn(A, B, Cb[:M])
    assert rel_err(to_np(Cb[:M]), ref) <= 8e-3
    assert bool((Cb[M:] == 7.0).all())           # rows past M are not written
    with pytest.raises(zpp.ZppError) as e:
        zpp.op_gemm_bf16_nn(A, B[:, :128], C[:, :128])
    assert e.value.status == -6


@pytest.mark.parametrize("dtype,b,s,nh,d", [(torch.float32, 2, 70, 3, 32), (torch.bfloat16, 1, 130, 2, 128),
                                            (torch.float32, 1, 1, 1, 64)])
def test_generic_attention_against_oracle(dtype, b, s, nh, d):
    print(f"attention generic {dtype} b{b} s{s} nh{nh} d{d}", flush=True)
    h, T = nh * d, b * s
    qkv = synth.normal_f32(2, 60, T * 3 * h, bf16_exact=(dtype == torch.bfloat16)).reshape(T, 3 * h)
    da = synth.normal_f32(2, 61, T * h, bf16_exact=(dtype == torch.bfloat16)).reshape(T, h)
    ops = oracle.Ops("f64")
    split = lambda t: t.reshape(b, s, nh, d).transpose(0, 2, 1, 3)
    q, k, v = (split(qkv[:, i * h:(i + 1) * h]) for i in range(3))
    A, Pr = ops.attention_fwd(q, k, v)
    dq, dk, dv = ops.attention_bwd(q, k, v, Pr, split(da))
    merge = lambda t: t.transpose(0, 2, 1, 3).reshape(T, h)
    QKV, DA = to_dev(qkv, dtype), to_dev(da, dtype)
    AT = torch.empty(T, h, dtype=dtype, device="cuda")
    lse = torch.empty(b * nh * s, dtype=torch.float32, device="cuda")
    delta = torch.empty(2 * lse.numel(), dtype=torch.float32, device="cuda")
    DQKV = torch.empty_like(QKV)
    zpp.op_attention_fwd(QKV, AT, lse, b, s, nh, d, impl=0)
    zpp.op_attention_bwd(QKV, AT, DA, lse, delta, DQKV, b, s, nh, d, impl=0)
    tol = 1e-2 if dtype == torch.bfloat16 else 1e-5
    assert rel_err(to_np(AT), merge(A)) <= tol
    got = to_np(DQKV)
    for i, r in enumerate((dq, dk, dv)):
        assert rel_err(got[:, i * h:(i + 1) * h], merge(r)) <= tol
    S = np.einsum("bnid,bnjd->bnij", q, k) / np.sqrt(d)
    S = np.where(np.tril(np.ones((s, s), bool)), S, -np.inf)
    ref_lse = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(lse.cpu().numpy().reshape(b, nh, s) - ref_lse).max() <= 1e-3


@pytest.mark.parametrize("b,s,nh", [(1, 128, 1), (1, 256, 2), (2, 384, 3), (1, 512, 8), (2, 768, 4), (1, 1024, 2)])
def test_mfma_attention_against_oracle(b, s, nh):
    print(f"attention mfma b{b} s{s} nh{nh}", flush=True)
    d = 128
    h, T = nh * d, b * s
    qkv = synth.normal_f32(3, 70, T * 3 * h, bf16_exact=True).reshape(T, 3 * h)
    da = synth.normal_f32(3, 71, T * h, std=0.1, bf16_exact=True).reshape(T, h)
    ops = oracle.Ops("f64")
    split = lambda t: t.reshape(b, s, nh, d).transpose(0, 2, 1, 3)
    merge = lambda t: t.transpose(0, 2, 1, 3).reshape(T, h)
    q, k, v = (split(qkv[:, i * h:(i + 1) * h]) for i in range(3))
    A, Pr = ops.attention_fwd(q, k, v)
    dq, dk, dv = ops.attention_bwd(q, k, v, Pr, split(da))
    QKV, DA = to_dev(qkv, torch.bfloat16), to_dev(da, torch.bfloat16)
    AT = torch.empty(T, h, dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(b * nh * s, dtype=torch.float32, device="cuda")
    delta = torch.empty(2 * lse.numel(), dtype=torch.float32, device="cuda")
    DQKV = torch.empty_like(QKV)
    zpp.op_attention_fwd(QKV, AT, lse, b, s, nh, d, impl=1)
    torch.cuda.synchronize()
    assert rel_err(to_np(AT), merge(A)) <= 1e-2
    S = np.einsum("bnid,bnjd->bnij", q, k) / np.sqrt(d)
    S = np.where(np.tril(np.ones((s, s), bool)), S, -np.inf)
    ref_lse = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(lse.cpu().numpy().reshape(b, nh, s) - ref_lse).max() <= 2e-3
    zpp.op_attention_bwd(QKV, AT, DA, lse, delta, DQKV, b, s, nh, d, impl=1)
    torch.cuda.synchronize()
    got = to_np(DQKV)
    for i, r in enumerate((dq, dk, dv)):
        assert rel_err(got[:, i * h:(i + 1) * h], merge(r)) <= 1.5e-2, i

@pytest.mark.parametrize("b,bs,s,nh", [(6, 2, 2048, 32), (6, 1, 2048, 32), (6, 2, 2048, 24), (10, 2, 1024, 48),
                                       (10, 1, 1024, 48)])
def test_mfma_attention_one_launch_of_many_pairs_equals_smaller_launches(b, bs, s, nh):
    """What a launch computes for a sample does not depend on how many samples it holds.  Launches with more
    (sample, head) pairs than a chunk walk their work-groups chunk by chunk (whole chunks, or a shorter last one);
    which work-group computes what must not change any bit: the whole batch in one launch against launches of `bs`
    samples, which have no more pairs than a chunk (the plain heavy-first order that the oracle tests above
    cover)."""
    print(f"attention mfma chunked b{b} bs{bs} s{s} nh{nh}", flush=True)
    d = 128
    h, T = nh * d, b * s
    assert b % bs == 0 and nh * bs <= max(16, (1024 // (s // 128)) // 16 * 16) < nh * b
    g = torch.Generator(device="cuda").manual_seed(11)
    QKV = torch.randn(T, 3 * h, device="cuda", generator=g).to(torch.bfloat16)
    DA = (0.1 * torch.randn(T, h, device="cuda", generator=g)).to(torch.bfloat16)

    def run(q, da, nb):
        at = torch.empty(nb * s, h, dtype=torch.bfloat16, device="cuda")
        lse = torch.empty(nb * nh * s, dtype=torch.float32, device="cuda")
        delta = torch.empty(2 * lse.numel(), dtype=torch.float32, device="cuda")
        dq = torch.full_like(q, float("nan"))
        zpp.op_attention_fwd(q, at, lse, nb, s, nh, d, impl=1)
        zpp.op_attention_bwd(q, at, da, lse, delta, dq, nb, s, nh, d, impl=1)
        return at, lse, dq

    at, lse, dq = run(QKV, DA, b)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dq.float()).all())
    for i in range(0, b, bs):
        rows = slice(i * s, (i + bs) * s)
        a1, l1, d1 = run(QKV[rows].contiguous(), DA[rows].contiguous(), bs)
        torch.cuda.synchronize()
        assert torch.equal(at[rows].view(torch.int16), a1.view(torch.int16)), i
        assert torch.equal(lse[i * nh * s:(i + bs) * nh * s], l1), i
        assert torch.equal(dq[rows].view(torch.int16), d1.view(torch.int16)), i
