"""Pins for the CPU oracle: everything here checks the oracle against something other than itself.

Finite differences, closed forms, invariants, special cases that reduce to library routines
(torch CPU ops with autograd, scipy), brute force on tiny inputs, and the few constants the
paper prints (tests/golden/paper_constants.txt).  No GPU is used.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
import synth
from synth import StageShape

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def golden():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            k, *v = line.split()
            out[k] = [float(t) for t in v]
    return out


def tiny(arch, gelu_mode=0, **kw):
    base = dict(name="tiny", arch=arch, n_blocks=2, hidden=16, n_heads=2, ffn=32, seq=8, micro_batch=2,
                unit_mbs=2, compute_dtype=0, seed=7, gelu_mode=gelu_mode)
    base.update(kw)
    return StageShape(**base)


def make_stage(shape, dtype="f64", jitter=0.1):
    st = oracle.OracleStage(shape, dtype)
    p = synth.make_params(shape, st.layout(), gain_jitter=jitter)
    # larger weights than the benchmark recipe so every path carries signal in the FD check
    st.P[:] = p * (5.0 if jitter else 1.0)
    if jitter:
        for name, off, r, c in st.layout():
            if name.endswith(".gamma") or name.endswith(".beta"):
                st.P[off:off + r * c] = p[off:off + r * c]
    st.materialize()
    return st


def inputs(shape, dtype=np.float64):
    xs = [synth.normal_f64(shape.seed, 1, shape.tokens * shape.hidden, first=m * shape.tokens * shape.hidden)
          .reshape(shape.tokens, shape.hidden).astype(dtype) for m in range(shape.unit_mbs)]
    dys = [synth.normal_f64(shape.seed, 2, shape.tokens * shape.hidden, std=0.1,
                            first=m * shape.tokens * shape.hidden)
           .reshape(shape.tokens, shape.hidden).astype(dtype) for m in range(shape.unit_mbs)]
    return xs, dys


def run_unit(st, xs, dys):
    """forward all, backward all, accumulate; returns ys, dxs (G holds the sum)."""
    st.G[:] = 0
    ys = [st.forward(m, x) for m, x in enumerate(xs)]
    dxs = []
    for m, dy in enumerate(dys):
        dxs.append(st.backward(m, dy))
        st.accumulate(m, 1.0)
    return ys, dxs


# --------------------------------------------------------------------------- layout / paper constants
def test_param_counts_and_paper_block_size():
    g = golden()
    expect = {"cfg1_tiny_gpt_fp32": 1579520, "cfg2_gpt_1p3b": 201433088, "cfg3_gpt_6p2b": 805519360,
              "cfg4_llama_13b": 1268817920, "cfg5_wide_gpt": 1610825728}
    for k, sh in synth.CONFIGS.items():
        n = oracle.param_count(sh)
        assert n == expect[k]
        h, f, L = sh.hidden, sh.ffn, sh.n_blocks
        if sh.arch == 0:
            assert n == L * (4 * h * h + 2 * h * f + 9 * h + f)
            if h >= 2048:  # "around 12 h^2" (Section 4.1) once the small-order terms are negligible
                assert abs(n / (L * g["block_param_coeff"][0] * h * h) - 1) < 5e-3
        else:
            assert n == L * (4 * h * h + 3 * h * f + 2 * h)


def test_layout_is_contiguous_and_ordered():
    for sh in synth.CONFIGS.values():
        off = 0
        for name, o, r, c in oracle.param_layout(sh):
            assert o == off
            off += r * c
        assert off == oracle.param_count(sh)
    names = [n for n, *_ in oracle.param_layout(synth.CONFIGS["cfg1_tiny_gpt_fp32"])][:12]
    assert names == ["blk0." + s for s in ["ln1.gamma", "ln1.beta", "attn.wqkv", "attn.bqkv", "attn.wo",
                                            "attn.bo", "ln2.gamma", "ln2.beta", "mlp.w1", "mlp.b1",
                                            "mlp.w2", "mlp.b2"]]


def test_paper_comm_condition_on_configs():
    g = golden()
    a, b9 = g["comm_cond_lhs_coeff"][0], g["comm_cond_rhs_coeff"][0]
    holds = {k: a * sh.seq * sh.unit_mbs * sh.micro_batch > b9 * sh.hidden for k, sh in synth.CONFIGS.items()}
    assert holds == {"cfg1_tiny_gpt_fp32": False, "cfg2_gpt_1p3b": True, "cfg3_gpt_6p2b": True,
                     "cfg4_llama_13b": True, "cfg5_wide_gpt": True}
    # the condition is the ratio of the two printed volumes: 8Bbsh > 36Bh^2/U  <=>  2sUb > 9h
    assert g["comm_zeropp_coeff"][0] / g["comm_tp_coeff"][0] == b9 / a


def test_table3_model_sizes_from_block_estimate():
    g = golden()
    for key, billions in (("model_14p6b", 14.6), ("model_28p3b", 28.3)):
        L, _, h, _ = g[key]
        assert abs(g["block_param_coeff"][0] * h * h * L / 1e9 / billions - 1) < 0.05


# --------------------------------------------------------------------------- linear layer (Section 2.3)
def test_linear_backward_bruteforce():
    ops = oracle.Ops("f64")
    rng = np.random.default_rng(0)
    T, i, o = 5, 4, 3
    x, W, b, dy = rng.normal(size=(T, i)), rng.normal(size=(o, i)), rng.normal(size=o), rng.normal(size=(T, o))
    y = ops.linear_fwd(x, W, b)
    for t in range(T):
        for oo in range(o):
            assert abs(y[t, oo] - (sum(x[t, k] * W[oo, k] for k in range(i)) + b[oo])) < 1e-12
    dx = ops.linear_bwd_input(dy, W)
    dW, db = ops.linear_bwd_weight(dy, x)
    for t in range(T):
        for k in range(i):
            assert abs(dx[t, k] - sum(dy[t, oo] * W[oo, k] for oo in range(o))) < 1e-12
    for oo in range(o):
        assert abs(db[oo] - sum(dy[t, oo] for t in range(T))) < 1e-12
        for k in range(i):
            assert abs(dW[oo, k] - sum(dy[t, oo] * x[t, k] for t in range(T))) < 1e-12
    # a transposed-operand mistake would survive square shapes only; these are not square
    assert dx.shape == (T, i) and dW.shape == (o, i)


# --------------------------------------------------------------------------- finite differences
@pytest.mark.parametrize("arch,gelu_mode", [(0, 0), (0, 1), (1, 0)])
def test_finite_differences_whole_stage(arch, gelu_mode):
    sh = tiny(arch, gelu_mode)
    st = make_stage(sh)
    xs, dys = inputs(sh)
    ys, dxs = run_unit(st, xs, dys)
    G = st.G.copy()

    def phi(xs_):
        return sum(float(np.vdot(dy, st.forward(m, x))) for m, (x, dy) in enumerate(zip(xs_, dys)))

    rng = np.random.default_rng(1)
    eps = 1e-5
    worst = 0.0
    for name, off, r, c in st.layout():
        for j in rng.choice(r * c, size=min(4, r * c), replace=False):
            i = off + int(j)
            p0 = st.P[i]
            st.P[i] = p0 + eps; st.materialize(); fp = phi(xs)
            st.P[i] = p0 - eps; st.materialize(); fm = phi(xs)
            st.P[i] = p0
            fd = (fp - fm) / (2 * eps)
            err = abs(fd - G[i]) / max(abs(fd), abs(G[i]), 1e-3)
            worst = max(worst, err)
            assert err < 2e-6, (name, int(j), fd, G[i])
    st.materialize()
    # input gradients
    for m in range(sh.unit_mbs):
        for _ in range(6):
            t, k = rng.integers(sh.tokens), rng.integers(sh.hidden)
            x0 = xs[m][t, k]
            xs[m][t, k] = x0 + eps; fp = phi(xs)
            xs[m][t, k] = x0 - eps; fm = phi(xs)
            xs[m][t, k] = x0
            fd = (fp - fm) / (2 * eps)
            assert abs(fd - dxs[m][t, k]) / max(abs(fd), abs(dxs[m][t, k]), 1e-3) < 2e-6


# --------------------------------------------------------------------------- torch CPU (library ops + autograd)
def torch_stage(sh, P, xs, dys):
    """The stage written with torch library routines in fp64; gradients by autograd."""
    import torch.nn.functional as F
    P = torch.tensor(P, dtype=torch.float64, requires_grad=True)
    lay = {n: (o, r, c) for n, o, r, c in oracle.param_layout(sh)}

    def w(blk, nm):
        o, r, c = lay[f"blk{blk}.{nm}"]
        t = P[o:o + r * c]
        return t.view(r, c) if r > 1 else t

    h, nh, s, b = sh.hidden, sh.n_heads, sh.seq, sh.micro_batch
    d = h // nh

    def rope(u):  # [b, nh, s, d]
        i = torch.arange(d // 2, dtype=torch.float64)
        th = torch.arange(s, dtype=torch.float64)[:, None] * sh.rope_base ** (-2 * i / d)[None, :]
        z = torch.view_as_complex(u.reshape(b, nh, s, d // 2, 2).contiguous()) * torch.polar(torch.ones_like(th), th)
        return torch.view_as_real(z).reshape(b, nh, s, d)

    ys, xts = [], []
    for x in xs:
        xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
        xts.append(xt)
        cur = xt
        for blk in range(sh.n_blocks):
            if sh.arch == 0:
                n1 = F.layer_norm(cur, (h,), w(blk, "ln1.gamma"), w(blk, "ln1.beta"), sh.norm_eps)
                qkv = F.linear(n1, w(blk, "attn.wqkv"), w(blk, "attn.bqkv"))
            else:
                n1 = cur * torch.rsqrt(cur.pow(2).mean(-1, keepdim=True) + sh.norm_eps) * w(blk, "norm1.gamma")
                qkv = F.linear(n1, w(blk, "attn.wqkv"))
            q, k, v = [t.view(b, s, nh, d).transpose(1, 2) for t in qkv.split(h, dim=-1)]
            if sh.arch == 1:
                q, k = rope(q), rope(k)
            a = F.scaled_dot_product_attention(q, k, v, is_causal=True)
            a = a.transpose(1, 2).reshape(b * s, h)
            if sh.arch == 0:
                x1 = cur + F.linear(a, w(blk, "attn.wo"), w(blk, "attn.bo"))
                n2 = F.layer_norm(x1, (h,), w(blk, "ln2.gamma"), w(blk, "ln2.beta"), sh.norm_eps)
                u = F.linear(n2, w(blk, "mlp.w1"), w(blk, "mlp.b1"))
                g = F.gelu(u, approximate="tanh" if sh.gelu_mode == 0 else "none")
                cur = x1 + F.linear(g, w(blk, "mlp.w2"), w(blk, "mlp.b2"))
            else:
                x1 = cur + F.linear(a, w(blk, "attn.wo"))
                n2 = x1 * torch.rsqrt(x1.pow(2).mean(-1, keepdim=True) + sh.norm_eps) * w(blk, "norm2.gamma")
                act = F.silu(F.linear(n2, w(blk, "mlp.wgate"))) * F.linear(n2, w(blk, "mlp.wup"))
                cur = x1 + F.linear(act, w(blk, "mlp.wdown"))
        ys.append(cur)
    loss = sum((y * torch.tensor(dy)).sum() for y, dy in zip(ys, dys))
    loss.backward()
    return [y.detach().numpy() for y in ys], [x.grad.numpy() for x in xts], P.grad.numpy()


@pytest.mark.parametrize("arch,gelu_mode", [(0, 0), (0, 1), (1, 0)])
def test_whole_stage_against_torch_autograd(arch, gelu_mode):
    sh = tiny(arch, gelu_mode, hidden=32, n_heads=4, ffn=48, seq=12, micro_batch=2, unit_mbs=3, n_blocks=3)
    st = make_stage(sh)
    xs, dys = inputs(sh)
    ys, dxs = run_unit(st, xs, dys)
    tys, tdxs, tG = torch_stage(sh, st.P.copy(), xs, dys)
    for a, b in zip(ys, tys):
        assert np.abs(a - b).max() < 1e-10 * max(1, np.abs(b).max())
    for a, b in zip(dxs, tdxs):
        assert np.abs(a - b).max() < 1e-10 * max(1, np.abs(b).max())
    for name, off, r, c in st.layout():
        a, b = st.G[off:off + r * c], tG[off:off + r * c]
        assert np.abs(a - b).max() <= 1e-10 * max(1e-3, np.abs(b).max()), name


def test_f32_instantiation_tracks_f64():
    sh = tiny(0)
    a, b = make_stage(sh, "f64"), make_stage(sh, "f32")
    xs, dys = inputs(sh)
    ya, dxa = run_unit(a, xs, dys)
    yb, dxb = run_unit(b, [x.astype(np.float32) for x in xs], [d.astype(np.float32) for d in dys])
    assert np.abs(ya[0] - yb[0]).max() < 2e-5 * np.abs(ya[0]).max()
    assert np.abs(dxa[1] - dxb[1]).max() < 2e-5 * np.abs(dxa[1]).max()
    assert np.abs(a.G - b.G).max() < 2e-5 * np.abs(a.G).max()


# --------------------------------------------------------------------------- accumulation invariant
@pytest.mark.parametrize("arch", [0, 1])
def test_accumulated_grads_equal_concatenated_batch(arch):
    sh = tiny(arch, unit_mbs=3)
    st = make_stage(sh)
    xs, dys = inputs(sh)
    run_unit(st, xs, dys)
    big = sh.replace(micro_batch=sh.micro_batch * sh.unit_mbs, unit_mbs=1)
    st2 = make_stage(big)
    assert np.array_equal(st.P, st2.P)
    y2, dx2 = run_unit(st2, [np.concatenate(xs)], [np.concatenate(dys)])
    assert np.abs(st.G - st2.G).max() < 1e-12 * np.abs(st2.G).max()
    # order of micro-batches only matters at rounding level
    st3 = make_stage(sh)
    run_unit(st3, xs[::-1], dys[::-1])
    assert np.abs(st.G - st3.G).max() < 1e-12 * np.abs(st.G).max()


def test_accumulate_scale_and_staging():
    sh = tiny(0)
    st = make_stage(sh)
    xs, dys = inputs(sh)
    st.G[:] = 0
    st.forward(0, xs[0]); st.backward(0, dys[0])
    S = st.S.copy()
    st.accumulate(0, 0.5)
    assert np.allclose(st.G, 0.5 * S, rtol=0, atol=0)
    st.accumulate(0, 2.0)
    assert np.allclose(st.G, 2.5 * S, rtol=1e-15, atol=0)


# --------------------------------------------------------------------------- Adam
def test_adam_first_step_closed_form():
    sh = tiny(0)
    for dtype, tol in (("f64", 1e-13), ("f32", 3e-7)):
        st = oracle.OracleStage(sh, dtype)
        rng = np.random.default_rng(3)
        p0 = rng.normal(0, 0.02, st.N)
        g = rng.normal(0, 1e-3, st.N)
        g[::7] = 0.0
        st.P[:] = p0; st.G[:] = g; st.M[:] = 0; st.V[:] = 0
        p0, g = st.P.astype(np.float64), st.G.astype(np.float64)
        hp = synth.ADAM
        st.adam(step=1, **hp)
        # from m = v = 0: mhat = g, vhat = g^2, so the update direction is g/(|g|+eps)
        expect = p0 - hp["lr"] * (g / (np.abs(g) + hp["eps"]) + hp["weight_decay"] * p0)
        assert np.abs(st.P - expect).max() <= tol * np.abs(expect).max() + (1e-11 if dtype == "f32" else 0)
        zero = g == 0
        assert np.allclose(st.P[zero], p0[zero] * (1 - hp["lr"] * hp["weight_decay"]), rtol=tol * 4, atol=0)
        assert np.allclose(st.M, (1 - hp["beta1"]) * g, rtol=tol * 4, atol=0)
        assert np.allclose(st.V, (1 - hp["beta2"]) * g * g, rtol=tol * 4, atol=1e-30)
        big = np.abs(g) > 1e-5
        step = (st.P - p0 * (1 - hp["lr"] * hp["weight_decay"]))[big]
        assert np.allclose(np.abs(step), hp["lr"], rtol=2e-3)
        assert np.all(np.sign(step) == -np.sign(g[big]))


def test_adam_l2_form_subrange_and_zero_grad():
    sh = tiny(0)
    st = oracle.OracleStage(sh, "f64")
    rng = np.random.default_rng(4)
    p0, g = rng.normal(0, 0.02, st.N), rng.normal(0, 1e-3, st.N)
    st.P[:] = p0; st.G[:] = g
    hp = dict(synth.ADAM)
    off, cnt = 256, 1024
    st.adam(off, cnt, step=1, decoupled_wd=0, zero_grad=1, grad_scale=0.5, **hp)
    ge = 0.5 * g + hp["weight_decay"] * p0
    expect = p0 - hp["lr"] * ge / (np.abs(ge) + hp["eps"])
    sl = slice(off, off + cnt)
    assert np.allclose(st.P[sl], expect[sl], rtol=1e-13, atol=0)
    assert np.array_equal(st.P[:off], p0[:off]) and np.array_equal(st.P[off + cnt:], p0[off + cnt:])
    assert np.all(st.G[sl] == 0) and np.array_equal(st.G[:off], g[:off])
    assert np.all(st.M[:off] == 0) and np.all(st.V[off + cnt:] == 0)


def test_adam_multi_step_against_torch_adamw():
    sh = tiny(0)
    rng = np.random.default_rng(5)
    hp = synth.ADAM
    st64, st32 = oracle.OracleStage(sh, "f64"), oracle.OracleStage(sh, "f32")
    n = 4096
    p0 = rng.normal(0, 0.02, n).astype(np.float32)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                            weight_decay=hp["weight_decay"])
    for s in (st64, st32):
        s.P[:n] = p0
    for t in range(1, 6):
        g = rng.normal(0, 1e-3, n).astype(np.float32)
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        for s in (st64, st32):
            s.G[:n] = g
            s.adam(0, n, step=t, **hp)
    ref = tp.detach().numpy()
    # torch.optim.AdamW divides by (sqrt(v)/sqrt(1-b2^t) + eps): the same formula
    assert np.abs(st64.P[:n] - ref).max() <= 1e-12 * np.abs(ref).max()
    assert np.abs(st32.P[:n] - ref).max() <= 1e-6 * np.abs(ref).max()


def test_flat_array_passes_closed_forms():
    """The flat passes over caller-owned arrays (used slice by slice on shards too large for a host Stage):
    first Adam step in closed form, bf16 bits against torch's cast, accumulate against float64."""
    rng = np.random.default_rng(11)
    n = 10007
    hp = synth.ADAM
    p0 = rng.normal(0, 0.02, n).astype(np.float32)
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    g[::5] = 0.0
    P, M, V, G = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), g.copy()
    oracle.flat_adam(P, M, V, G, step=1, zero_grad=1, **hp)
    p64, g64 = p0.astype(np.float64), g.astype(np.float64)
    expect = p64 - hp["lr"] * (g64 / (np.abs(g64) + hp["eps"]) + hp["weight_decay"] * p64)
    assert np.abs(P - expect).max() <= 3e-7 * np.abs(expect).max() + 1e-11
    assert np.allclose(M, (1 - hp["beta1"]) * g64, rtol=2e-6, atol=0)
    assert np.allclose(V, (1 - hp["beta2"]) * g64 * g64, rtol=2e-6, atol=1e-30)
    assert not G.any()
    bits = oracle.flat_materialize_bits(p0)
    assert np.array_equal(bits, torch.from_numpy(p0).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    A, S = p0.copy(), g.copy()
    oracle.flat_accumulate(A, S, 0.5)
    assert np.abs(A - (p64 + 0.5 * g64)).max() <= 6e-8 * np.abs(p64).max()


# --------------------------------------------------------------------------- materialise (bf16 RNE)
def nearest_bf16_by_distance(v: np.float32) -> int:
    """Nearest 8-bit-significand value by exact distance (ties to even pattern)."""
    u = int(np.array(v, np.float32).view(np.uint32))
    lo = u & 0xFFFF0000
    hi = lo + 0x10000
    f = lambda b: float(np.array(b & 0xFFFFFFFF, np.uint32).view(np.float32))
    x = float(v)
    if math.isinf(f(hi)) and not math.isinf(x):
        # rounding up into infinity is what RNE does at the top of the range
        d_lo, d_hi = abs(x - f(lo)), abs(2.0 ** 128 * (1 if x > 0 else -1) - x)
    else:
        d_lo, d_hi = abs(x - f(lo)), abs(f(hi) - x)
    if d_lo < d_hi:
        return lo >> 16
    if d_hi < d_lo:
        return (hi >> 16) & 0xFFFF
    return (lo >> 16) if ((lo >> 16) & 1) == 0 else (hi >> 16) & 0xFFFF


def test_bf16_rounding_against_distance_definition_and_torch():
    rng = np.random.default_rng(6)
    highs = rng.integers(0, 1 << 16, 3000, dtype=np.uint32)
    highs = highs[((highs >> 7) & 0xFF) != 0xFF]  # finite
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000], dtype=np.uint32)
    pats = ((highs[:, None] << 16) | lows[None, :]).reshape(-1).astype(np.uint32)
    vals = pats.view(np.float32)
    tor = torch.tensor(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for v, t in zip(vals[::5], tor[::5]):
        got = oracle.bf16_bits_rne(float(v))
        assert got == int(t)
        assert got == nearest_bf16_by_distance(v)
    assert oracle.bf16_bits_rne(float("inf")) == 0x7F80 and oracle.bf16_bits_rne(float("-inf")) == 0xFF80
    nan = oracle.bf16_bits_rne(float("nan"))
    assert (nan & 0x7F80) == 0x7F80 and (nan & 0x7F) != 0
    # carry out of the significand and into infinity
    assert oracle.bf16_bits_rne(float(np.array(0x3FFFFFFF, np.uint32).view(np.float32))) == 0x4000
    assert oracle.bf16_bits_rne(float(np.array(0x7F7FFFFF, np.uint32).view(np.float32))) == 0x7F80


def test_materialize_modes():
    sh = tiny(0)
    st = oracle.OracleStage(sh, "f32")
    st.P[:] = synth.normal_f32(0, 5, st.N, 0, 0.02)
    st.materialize()
    assert np.array_equal(st.W, st.P)
    sb = oracle.OracleStage(sh.replace(compute_dtype=1), "f32")
    sb.P[:] = st.P
    sb.materialize()
    ref = torch.tensor(st.P.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(sb.W, ref)
    assert np.array_equal(sb.P, st.P)  # master untouched


# --------------------------------------------------------------------------- attention
def test_attention_invariants():
    ops = oracle.Ops("f64")
    rng = np.random.default_rng(8)
    b, nh, s, d = 2, 3, 9, 4
    q, k, v = (rng.normal(size=(b, nh, s, d)) for _ in range(3))
    A, Pr = ops.attention_fwd(q, k, v)
    assert np.allclose(Pr.sum(-1), 1.0, atol=1e-14)
    assert np.all(np.triu(Pr, 1) == 0)
    # library definition: scipy softmax of masked scores
    from scipy.special import softmax
    S = np.einsum("bnid,bnjd->bnij", q, k) / math.sqrt(d)
    S = np.where(np.tril(np.ones((s, s), bool)), S, -np.inf)
    assert np.allclose(Pr, softmax(S, axis=-1), atol=1e-14)
    assert np.allclose(A, np.einsum("bnij,bnjd->bnid", softmax(S, axis=-1), v), atol=1e-13)
    # s = 1 -> A = V
    A1, _ = ops.attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1])
    assert np.array_equal(A1, v[:, :, :1])
    # K = 0 -> uniform over the visible prefix
    A0, _ = ops.attention_fwd(q, np.zeros_like(k), v)
    pref = np.cumsum(v, axis=2) / np.arange(1, s + 1)[None, None, :, None]
    assert np.allclose(A0, pref, atol=1e-14)
    # causality: changing later positions leaves earlier rows bit-unchanged
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for t in (q2, k2, v2):
        t[:, :, 5:] += 1.0
    A2, _ = ops.attention_fwd(q2, k2, v2)
    assert np.array_equal(A2[:, :, :5], A[:, :, :5])
    # large logits do not overflow (row max subtracted)
    A3, P3 = ops.attention_fwd(q * 1e3, k * 1e3, v)
    assert np.isfinite(A3).all() and np.allclose(P3.sum(-1), 1.0)


def test_attention_backward_against_autograd():
    ops = oracle.Ops("f64")
    rng = np.random.default_rng(9)
    b, nh, s, d = 1, 2, 7, 6
    q, k, v, dA = (rng.normal(size=(b, nh, s, d)) for _ in range(4))
    A, Pr = ops.attention_fwd(q, k, v)
    dq, dk, dv = ops.attention_bwd(q, k, v, Pr, dA)
    tq, tk, tv = (torch.tensor(t, requires_grad=True) for t in (q, k, v))
    ta = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    ta.backward(torch.tensor(dA))
    assert np.allclose(A, ta.detach().numpy(), atol=1e-13)
    for a, t in ((dq, tq), (dk, tk), (dv, tv)):
        assert np.allclose(a, t.grad.numpy(), atol=1e-12)


# --------------------------------------------------------------------------- norms
def test_layernorm_invariants_and_library():
    ops = oracle.Ops("f64")
    rng = np.random.default_rng(10)
    T, h, eps = 6, 24, 1e-5
    x = rng.normal(1.5, 2.0, size=(T, h))
    n, xhat, rstd = ops.layernorm_fwd(x, np.ones(h), np.zeros(h), eps)
    var = x.var(-1)
    assert np.allclose(n.mean(-1), 0, atol=1e-14)
    assert np.allclose(n.var(-1), var / (var + eps), rtol=1e-12)
    gamma, beta, dn = rng.normal(1, 0.2, h), rng.normal(0, 0.2, h), rng.normal(size=(T, h))
    n, xhat, rstd = ops.layernorm_fwd(x, gamma, beta, eps)
    dx, dg, db = ops.layernorm_bwd(dn, xhat, rstd, gamma)
    assert np.allclose(dx.sum(-1), 0, atol=1e-12)
    # orthogonality to xhat is exact only as eps -> 0 (sum xhat^2 = h var/(var+eps))
    _, xh0, rs0 = ops.layernorm_fwd(x, gamma, beta, 1e-30)
    dx0, _, _ = ops.layernorm_bwd(dn, xh0, rs0, gamma)
    assert np.allclose((dx0 * xh0).sum(-1), 0, atol=1e-10)
    tx, tg, tb = (torch.tensor(t, requires_grad=True) for t in (x, gamma, beta))
    tn = torch.nn.functional.layer_norm(tx, (h,), tg, tb, eps)
    tn.backward(torch.tensor(dn))
    assert np.allclose(n, tn.detach().numpy(), atol=1e-13)
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-12)
    assert np.allclose(dg, tg.grad.numpy(), atol=1e-12)
    assert np.allclose(db, tb.grad.numpy(), atol=1e-12)


def test_rmsnorm_invariants_and_autograd():
    ops = oracle.Ops("f64")
    rng = np.random.default_rng(11)
    T, h = 5, 16
    x, gamma, dn = rng.normal(size=(T, h)), rng.normal(1, 0.2, h), rng.normal(size=(T, h))
    n0, _, _ = ops.rmsnorm_fwd(x, gamma, 1e-30)
    n1, _, _ = ops.rmsnorm_fwd(3.7 * x, gamma, 1e-30)
    assert np.allclose(n0, n1, rtol=1e-13)  # scale invariance as eps -> 0
    assert np.allclose((n0 / gamma) ** 2 @ np.ones(h) / h, 1.0, rtol=1e-12)
    n, xhat, rinv = ops.rmsnorm_fwd(x, gamma, 1e-5)
    dx, dg = ops.rmsnorm_bwd(dn, xhat, rinv, gamma)
    tx, tg = torch.tensor(x, requires_grad=True), torch.tensor(gamma, requires_grad=True)
    tn = tx * torch.rsqrt(tx.pow(2).mean(-1, keepdim=True) + 1e-5) * tg
    tn.backward(torch.tensor(dn))
    assert np.allclose(n, tn.detach().numpy(), atol=1e-13)
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-12)
    assert np.allclose(dg, tg.grad.numpy(), atol=1e-12)


# --------------------------------------------------------------------------- RoPE
def test_rope_properties():
    ops = oracle.Ops("f64")
    rng = np.random.default_rng(12)
    b, nh, s, d = 1, 2, 10, 8
    q, k = rng.normal(size=(b, nh, s, d)), rng.normal(size=(b, nh, s, d))
    rq, rk = ops.rope(q), ops.rope(k)
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    assert np.array_equal(rq[:, :, 0], q[:, :, 0])  # position 0 is the identity
    # <R_m q, R_n k> depends only on m - n: put the same vectors at every position
    qq = np.broadcast_to(q[:, :, :1], q.shape).copy()
    kk = np.broadcast_to(k[:, :, :1], k.shape).copy()
    S = np.einsum("bnid,bnjd->bnij", ops.rope(qq), ops.rope(kk))
    for off in range(-3, 4):
        diag = np.diagonal(S, offset=off, axis1=2, axis2=3)
        assert np.allclose(diag, diag[..., :1], atol=1e-12)
    # first pair rotates by exactly p radians (base^0 = 1), adjacent pairing
    p = 3
    assert np.allclose(rq[0, 0, p, 0], q[0, 0, p, 0] * math.cos(p) - q[0, 0, p, 1] * math.sin(p))
    assert np.allclose(rq[0, 0, p, 1], q[0, 0, p, 0] * math.sin(p) + q[0, 0, p, 1] * math.cos(p))
    th = p * 10000.0 ** (-2 * 2 / d)
    assert np.allclose(rq[0, 0, p, 4], q[0, 0, p, 4] * math.cos(th) - q[0, 0, p, 5] * math.sin(th))
    # backward is the inverse rotation
    assert np.allclose(ops.rope(rq, sign=-1), q, atol=1e-14)


# --------------------------------------------------------------------------- GeLU
def test_gelu_forms_and_derivative():
    ops = oracle.Ops("f64")
    u = np.linspace(-6, 6, 241)
    from scipy.special import erf
    g1, d1 = ops.gelu(u, 1)
    assert np.allclose(g1, 0.5 * u * (1 + erf(u / math.sqrt(2))), atol=1e-15)
    g0, d0 = ops.gelu(u, 0)
    t = torch.nn.functional.gelu(torch.tensor(u), approximate="tanh").numpy()
    assert np.allclose(g0, t, atol=1e-14)
    assert 1e-4 < np.abs(g0 - g1).max() < 1e-2  # the two forms differ measurably
    e = 1e-6
    for mode, dg in ((0, d0), (1, d1)):
        fd = (ops.gelu(u + e, mode)[0] - ops.gelu(u - e, mode)[0]) / (2 * e)
        assert np.allclose(dg, fd, atol=1e-8)


# --------------------------------------------------------------------------- block structure
@pytest.mark.parametrize("arch", [0, 1])
def test_zero_output_projections_make_identity(arch):
    sh = tiny(arch)
    st = make_stage(sh)
    for name, off, r, c in st.layout():
        if name.split(".", 1)[1] in ("attn.wo", "attn.bo", "mlp.w2", "mlp.b2", "mlp.wdown"):
            st.P[off:off + r * c] = 0
    st.materialize()
    xs, dys = inputs(sh)
    y = st.forward(0, xs[0])
    dx = st.backward(0, dys[0])
    assert np.array_equal(y, xs[0]) and np.array_equal(dx, dys[0])


def test_samples_do_not_attend_across_the_micro_batch():
    sh = tiny(0)
    st = make_stage(sh)
    xs, _ = inputs(sh)
    y = st.forward(0, xs[0])
    x2 = xs[0].copy()
    x2[sh.seq:] += 1.0  # second sample changed
    y2 = st.forward(0, x2)
    assert np.array_equal(y[:sh.seq], y2[:sh.seq])


# --------------------------------------------------------------------------- generator
def test_generator_is_counter_based_and_normal():
    a = synth.normal_f32(3, 9, 10000)
    b = synth.normal_f32(3, 9, 4000, first=6000)
    assert np.array_equal(a[6000:], b)
    assert abs(a.mean()) < 0.05 and abs(a.std() - 1) < 0.05
    c = synth.normal_f32(3, 9, 1000, bf16_exact=True)
    assert np.all(c.view(np.uint32) & 0xFFFF == 0)
    assert not np.array_equal(synth.normal_f32(3, 10, 100), a[:100])
