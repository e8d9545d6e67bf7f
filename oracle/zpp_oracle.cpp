// ---------------------------------------------------------------------------
// CPU ORACLE — TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// A plain, slow, obviously-correct implementation of what one GPU does under
// the ZeroPP schedule (Section 3.1 "ZeRO-compatible pipeline parallelism",
// Section 3.2 "ZeRO-3 + PP + DP"): a pipeline stage of contiguous transformer
// blocks whose parameters are gathered once per scheduling unit of U
// micro-batches, run forward and backward for each micro-batch of the unit,
// whose gradients are reduced once per unit, followed by the optimizer step on
// the local partition.  With one GPU the gather is a local copy and the
// reduce-scatter is a local accumulation.
//
// The schedule changes *when* things are communicated, never the numbers, so
// the oracle is the plain definition of mini-batch training of a stack of
// transformer blocks (Section 4.1 reasons about the standard transformer block of
// hidden size h with about 12h^2 parameters): forward, the chain
// rule, a sum over micro-batches, one Adam update.  For every linear layer the
// backward is exactly Section 2.3: input gradient = activation gradient times
// weights, weight gradient = activation gradient (transposed) times inputs.
//
// Everything is templated on the real type; the library exports an fp32 and an
// fp64 instantiation.  Loops are straightforward; sums run in ascending index
// order except where an `omp simd reduction` lets the compiler use vector
// partial sums.  No blocking, no fusion, no BLAS.
//
// Only tests, the smoke check and the benchmark's cpu_baseline leg may use
// this file.  It shares no code with the HIP path.
// ---------------------------------------------------------------------------
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

struct OCfg {
    int32_t arch;         // 0 GPT: pre-LN LayerNorm, biases, GeLU. 1 LLaMA: RMSNorm, RoPE, SwiGLU, no biases
    int32_t n_blocks;     // transformer blocks in the stage
    int32_t hidden;       // h
    int32_t n_heads;      // nh, head dim d = h / nh
    int32_t ffn;          // f
    int32_t seq;          // s
    int32_t micro_batch;  // b
    int32_t unit_mbs;     // U, micro-batches in one scheduling unit
    int32_t round_bf16;   // 1: the materialised working copy is rounded to bf16 (RNE) and widened again
    int32_t gelu_mode;    // 0 tanh form, 1 erf form
    double norm_eps;
    double rope_base;
};

struct LayoutEntry {
    std::string name;
    uint64_t offset, rows, cols;
};

// Flat layout of the stage's parameters; every matrix is [out_features, in_features] row-major
// so that y = x W^T + b.  Blocks are concatenated without padding.
std::vector<LayoutEntry> make_layout(const OCfg &c)
{
    std::vector<LayoutEntry> L;
    uint64_t off = 0;
    const uint64_t h = c.hidden, f = c.ffn;
    auto add = [&](int blk, const char *nm, uint64_t r, uint64_t cc) {
        L.push_back({"blk" + std::to_string(blk) + "." + nm, off, r, cc});
        off += r * cc;
    };
    for (int b = 0; b < c.n_blocks; ++b) {
        if (c.arch == 0) {
            add(b, "ln1.gamma", 1, h);
            add(b, "ln1.beta", 1, h);
            add(b, "attn.wqkv", 3 * h, h);
            add(b, "attn.bqkv", 1, 3 * h);
            add(b, "attn.wo", h, h);
            add(b, "attn.bo", 1, h);
            add(b, "ln2.gamma", 1, h);
            add(b, "ln2.beta", 1, h);
            add(b, "mlp.w1", f, h);
            add(b, "mlp.b1", 1, f);
            add(b, "mlp.w2", h, f);
            add(b, "mlp.b2", 1, h);
        } else {
            add(b, "norm1.gamma", 1, h);
            add(b, "attn.wqkv", 3 * h, h);
            add(b, "attn.wo", h, h);
            add(b, "norm2.gamma", 1, h);
            add(b, "mlp.wgate", f, h);
            add(b, "mlp.wup", f, h);
            add(b, "mlp.wdown", h, f);
        }
    }
    return L;
}

uint64_t layout_total(const std::vector<LayoutEntry> &L)
{
    return L.empty() ? 0 : L.back().offset + L.back().rows * L.back().cols;
}

// ---------------------------------------------------------------------------
// fp32 -> bf16 -> fp32, round to nearest, ties to even; NaN stays NaN, Inf stays Inf.
// ---------------------------------------------------------------------------
inline uint16_t bf16_bits_rne(float v)
{
    uint32_t u;
    std::memcpy(&u, &v, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0)
        return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN, keep sign
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

inline float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float v;
    std::memcpy(&v, &u, 4);
    return v;
}

// ---------------------------------------------------------------------------
// Operators.  T = number of tokens (rows).  All tensors row-major.
// ---------------------------------------------------------------------------

// LayerNorm over the last axis with biased variance:
//   mu = mean(x), var = mean((x-mu)^2), xhat = (x-mu)/sqrt(var+eps), n = gamma*xhat + beta
template <class R>
void layernorm_fwd(int64_t T, int64_t h, const R *x, const R *gamma, const R *beta, R eps, R *xhat,
                   R *rstd, R *n)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const R *xr = x + t * h;
        R mu = 0;
        for (int64_t i = 0; i < h; ++i) mu += xr[i];
        mu /= (R)h;
        R var = 0;
        for (int64_t i = 0; i < h; ++i) var += (xr[i] - mu) * (xr[i] - mu);
        var /= (R)h;
        R rs = (R)1 / std::sqrt(var + eps);
        rstd[t] = rs;
        for (int64_t i = 0; i < h; ++i) {
            R xh = (xr[i] - mu) * rs;
            xhat[t * h + i] = xh;
            n[t * h + i] = gamma[i] * xh + beta[i];
        }
    }
}

// With ghat = dn*gamma:  dx = (ghat - mean(ghat) - xhat*mean(ghat*xhat)) * rstd
//   dgamma = sum_t dn*xhat,  dbeta = sum_t dn
template <class R>
void layernorm_bwd(int64_t T, int64_t h, const R *dn, const R *xhat, const R *rstd, const R *gamma,
                   R *dx, R *dgamma, R *dbeta)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const R *d = dn + t * h, *xh = xhat + t * h;
        R m1 = 0, m2 = 0;
        for (int64_t i = 0; i < h; ++i) {
            R gh = d[i] * gamma[i];
            m1 += gh;
            m2 += gh * xh[i];
        }
        m1 /= (R)h;
        m2 /= (R)h;
        for (int64_t i = 0; i < h; ++i) {
            R gh = d[i] * gamma[i];
            dx[t * h + i] = (gh - m1 - xh[i] * m2) * rstd[t];
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < h; ++i) {
        R sg = 0, sb = 0;
        for (int64_t t = 0; t < T; ++t) {
            sg += dn[t * h + i] * xhat[t * h + i];
            sb += dn[t * h + i];
        }
        dgamma[i] = sg;
        if (dbeta) dbeta[i] = sb;
    }
}

// RMSNorm: r = sqrt(mean(x^2)+eps), xhat = x/r, n = gamma*xhat
template <class R>
void rmsnorm_fwd(int64_t T, int64_t h, const R *x, const R *gamma, R eps, R *xhat, R *rinv, R *n)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const R *xr = x + t * h;
        R ms = 0;
        for (int64_t i = 0; i < h; ++i) ms += xr[i] * xr[i];
        ms /= (R)h;
        R ri = (R)1 / std::sqrt(ms + eps);
        rinv[t] = ri;
        for (int64_t i = 0; i < h; ++i) {
            R xh = xr[i] * ri;
            xhat[t * h + i] = xh;
            n[t * h + i] = gamma[i] * xh;
        }
    }
}

// dx = (ghat - xhat*mean(ghat*xhat))/r,  dgamma = sum_t dn*xhat
template <class R>
void rmsnorm_bwd(int64_t T, int64_t h, const R *dn, const R *xhat, const R *rinv, const R *gamma,
                 R *dx, R *dgamma)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const R *d = dn + t * h, *xh = xhat + t * h;
        R m2 = 0;
        for (int64_t i = 0; i < h; ++i) m2 += d[i] * gamma[i] * xh[i];
        m2 /= (R)h;
        for (int64_t i = 0; i < h; ++i) dx[t * h + i] = (d[i] * gamma[i] - xh[i] * m2) * rinv[t];
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < h; ++i) {
        R sg = 0;
        for (int64_t t = 0; t < T; ++t) sg += dn[t * h + i] * xhat[t * h + i];
        dgamma[i] = sg;
    }
}

// y[t,o] = b[o] + sum_i x[t,i] * W[o,i]
template <class R>
void linear_fwd(int64_t T, int64_t in, int64_t out, const R *x, const R *W, const R *b, R *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const R *xr = x + t * in;
        for (int64_t o = 0; o < out; ++o) {
            const R *wr = W + o * in;
            R acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int64_t i = 0; i < in; ++i) acc += xr[i] * wr[i];
            y[t * out + o] = acc + (b ? b[o] : (R)0);
        }
    }
}

// Input gradient of a linear layer (Section 2.3): dX = dY . W
template <class R>
void linear_bwd_input(int64_t T, int64_t in, int64_t out, const R *dy, const R *W, R *dx)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        R *dr = dx + t * in;
        for (int64_t i = 0; i < in; ++i) dr[i] = 0;
        for (int64_t o = 0; o < out; ++o) {
            const R g = dy[t * out + o];
            const R *wr = W + o * in;
            for (int64_t i = 0; i < in; ++i) dr[i] += g * wr[i];
        }
    }
}

// Weight gradient of a linear layer (Section 2.3): dW = dY^T . X, db = column sums of dY
template <class R>
void linear_bwd_weight(int64_t T, int64_t in, int64_t out, const R *dy, const R *x, R *dW, R *db)
{
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < out; ++o) {
        R *wr = dW + o * in;
        for (int64_t i = 0; i < in; ++i) wr[i] = 0;
        R sb = 0;
        for (int64_t t = 0; t < T; ++t) {
            const R g = dy[t * out + o];
            const R *xr = x + t * in;
            for (int64_t i = 0; i < in; ++i) wr[i] += g * xr[i];
            sb += g;
        }
        if (db) db[o] = sb;
    }
}

// Rotary embedding on u[b, nh, s, d], adjacent pairs (2i, 2i+1), angle p * base^(-2i/d);
// sign = +1 forward, -1 rotates back (used for gradients).
template <class R>
void rope_apply(int64_t b, int64_t nh, int64_t s, int64_t d, R *u, double base, int sign)
{
#pragma omp parallel for schedule(static)
    for (int64_t bn = 0; bn < b * nh; ++bn) {
        for (int64_t p = 0; p < s; ++p) {
            R *r = u + (bn * s + p) * d;
            for (int64_t i = 0; i < d / 2; ++i) {
                double theta = (double)p * std::pow(base, -2.0 * (double)i / (double)d);
                R c = (R)std::cos(theta), sn = (R)(sign * std::sin(theta));
                R a = r[2 * i], bb = r[2 * i + 1];
                r[2 * i] = a * c - bb * sn;
                r[2 * i + 1] = a * sn + bb * c;
            }
        }
    }
}

// Causal softmax attention per (sample, head): S = Q K^T / sqrt(d); keys j > i masked;
// Pr = softmax_j(S) (row max subtracted); A = Pr V.  q,k,v,A: [b, nh, s, d]; Pr: [b, nh, s, s].
template <class R>
void attention_fwd(int64_t b, int64_t nh, int64_t s, int64_t d, const R *q, const R *k, const R *v,
                   R *Pr, R *A)
{
    const R scale = (R)1 / std::sqrt((R)d);
#pragma omp parallel for schedule(dynamic) collapse(2)
    for (int64_t bn = 0; bn < b * nh; ++bn) {
        for (int64_t i = 0; i < s; ++i) {
            const R *qi = q + (bn * s + i) * d;
            R *pr = Pr + (bn * s + i) * s;
            R mx = -INFINITY;
            for (int64_t j = 0; j <= i; ++j) {
                const R *kj = k + (bn * s + j) * d;
                R acc = 0;
                for (int64_t e = 0; e < d; ++e) acc += qi[e] * kj[e];
                pr[j] = acc * scale;
                if (pr[j] > mx) mx = pr[j];
            }
            R den = 0;
            for (int64_t j = 0; j <= i; ++j) {
                pr[j] = std::exp(pr[j] - mx);
                den += pr[j];
            }
            for (int64_t j = 0; j <= i; ++j) pr[j] /= den;
            for (int64_t j = i + 1; j < s; ++j) pr[j] = 0;
            R *ai = A + (bn * s + i) * d;
            for (int64_t e = 0; e < d; ++e) ai[e] = 0;
            for (int64_t j = 0; j <= i; ++j) {
                const R *vj = v + (bn * s + j) * d;
                for (int64_t e = 0; e < d; ++e) ai[e] += pr[j] * vj[e];
            }
        }
    }
}

// dV = Pr^T dA; dPr = dA V^T; dS = Pr o (dPr - rowsum(dPr o Pr)); dQ = dS K / sqrt(d); dK = dS^T Q / sqrt(d)
template <class R>
void attention_bwd(int64_t b, int64_t nh, int64_t s, int64_t d, const R *q, const R *k, const R *v,
                   const R *Pr, const R *dA, R *dq, R *dk, R *dv)
{
    const R scale = (R)1 / std::sqrt((R)d);
#pragma omp parallel for schedule(dynamic)
    for (int64_t bn = 0; bn < b * nh; ++bn) {
        std::vector<R> dS((size_t)s);
        R *dkb = dk + bn * s * d, *dvb = dv + bn * s * d;
        for (int64_t z = 0; z < s * d; ++z) dkb[z] = dvb[z] = 0;
        for (int64_t i = 0; i < s; ++i) {
            const R *pr = Pr + (bn * s + i) * s;
            const R *dai = dA + (bn * s + i) * d;
            const R *qi = q + (bn * s + i) * d;
            R rs = 0;
            for (int64_t j = 0; j <= i; ++j) {
                const R *vj = v + (bn * s + j) * d;
                R dp = 0;
                for (int64_t e = 0; e < d; ++e) dp += dai[e] * vj[e];
                dS[j] = dp;
                rs += dp * pr[j];
            }
            R *dqi = dq + (bn * s + i) * d;
            for (int64_t e = 0; e < d; ++e) dqi[e] = 0;
            for (int64_t j = 0; j <= i; ++j) {
                const R ds = pr[j] * (dS[j] - rs);
                const R *kj = k + (bn * s + j) * d;
                R *dkj = dkb + j * d, *dvj = dvb + j * d;
                for (int64_t e = 0; e < d; ++e) {
                    dqi[e] += ds * kj[e] * scale;
                    dkj[e] += ds * qi[e] * scale;
                    dvj[e] += pr[j] * dai[e];
                }
            }
        }
    }
}

template <class R>
inline R gelu_val(R u, int mode)
{
    if (mode == 1) return (R)0.5 * u * ((R)1 + std::erf(u * (R)0.70710678118654752440));
    const R c = (R)0.79788456080286535588;  // sqrt(2/pi)
    return (R)0.5 * u * ((R)1 + std::tanh(c * (u + (R)0.044715 * u * u * u)));
}

template <class R>
inline R gelu_grad(R u, int mode)
{
    if (mode == 1) {
        const R phi = std::exp(-(R)0.5 * u * u) * (R)0.39894228040143267794;  // 1/sqrt(2 pi)
        return (R)0.5 * ((R)1 + std::erf(u * (R)0.70710678118654752440)) + u * phi;
    }
    const R c = (R)0.79788456080286535588;
    const R th = std::tanh(c * (u + (R)0.044715 * u * u * u));
    return (R)0.5 * ((R)1 + th) + (R)0.5 * u * ((R)1 - th * th) * c * ((R)1 + (R)3 * (R)0.044715 * u * u);
}

template <class R>
inline R sigmoid_val(R z)
{
    return (R)1 / ((R)1 + std::exp(-z));
}

// ---------------------------------------------------------------------------
// Stage
// ---------------------------------------------------------------------------
template <class R>
struct Stash {
    // one (micro-batch, block) worth of saved tensors, keyed by name
    std::map<std::string, std::vector<R>> t;
    std::vector<R> &get(const std::string &n, size_t size)
    {
        auto &v = t[n];
        v.assign(size, (R)0);
        return v;
    }
    const std::vector<R> &at(const std::string &n) const { return t.at(n); }
};

template <class R>
struct Stage {
    OCfg c;
    std::vector<LayoutEntry> layout;
    uint64_t N;
    std::vector<R> P, G, M, V, W, S;
    std::vector<std::vector<Stash<R>>> stash;  // [U][n_blocks]

    explicit Stage(const OCfg &cfg) : c(cfg), layout(make_layout(cfg)), N(layout_total(layout))
    {
        P.assign(N, 0);
        G.assign(N, 0);
        M.assign(N, 0);
        V.assign(N, 0);
        W.assign(N, 0);
        S.assign(N, 0);
        stash.resize(c.unit_mbs);
        for (auto &s : stash) s.resize(c.n_blocks);
    }

    uint64_t off(int blk, const char *nm) const
    {
        std::string full = "blk" + std::to_string(blk) + "." + nm;
        for (auto &e : layout)
            if (e.name == full) return e.offset;
        std::fprintf(stderr, "oracle: no tensor %s\n", full.c_str());
        return 0;
    }

    // Stand-in for the per-unit parameter all-gather (Section 3.2): the working copy of the whole
    // stage is produced from the fp32 master shard.
    void materialize()
    {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < (int64_t)N; ++i) {
            if (c.round_bf16)
                W[i] = (R)bf16_bits_to_float(bf16_bits_rne((float)P[i]));
            else
                W[i] = P[i];
        }
    }

    // [T, 3h] -> q,k,v each [b, nh, s, d]; rows of Wqkv are all of Q (head-major), then K, then V.
    void split_heads(const R *qkv, R *q, R *k, R *v) const
    {
        const int64_t h = c.hidden, nh = c.n_heads, d = h / nh, s = c.seq, b = c.micro_batch;
        for (int64_t bi = 0; bi < b; ++bi)
            for (int64_t p = 0; p < s; ++p)
                for (int64_t n = 0; n < nh; ++n)
                    for (int64_t e = 0; e < d; ++e) {
                        const int64_t t = bi * s + p;
                        const int64_t dst = ((bi * nh + n) * s + p) * d + e;
                        q[dst] = qkv[t * 3 * h + n * d + e];
                        k[dst] = qkv[t * 3 * h + h + n * d + e];
                        v[dst] = qkv[t * 3 * h + 2 * h + n * d + e];
                    }
    }
    void merge_heads(const R *a, R *out) const  // [b,nh,s,d] -> [T,h]
    {
        const int64_t h = c.hidden, nh = c.n_heads, d = h / nh, s = c.seq, b = c.micro_batch;
        for (int64_t bi = 0; bi < b; ++bi)
            for (int64_t p = 0; p < s; ++p)
                for (int64_t n = 0; n < nh; ++n)
                    for (int64_t e = 0; e < d; ++e)
                        out[(bi * s + p) * h + n * d + e] = a[((bi * nh + n) * s + p) * d + e];
    }
    void unmerge_heads(const R *in, R *a) const  // [T,h] -> [b,nh,s,d]
    {
        const int64_t h = c.hidden, nh = c.n_heads, d = h / nh, s = c.seq, b = c.micro_batch;
        for (int64_t bi = 0; bi < b; ++bi)
            for (int64_t p = 0; p < s; ++p)
                for (int64_t n = 0; n < nh; ++n)
                    for (int64_t e = 0; e < d; ++e)
                        a[((bi * nh + n) * s + p) * d + e] = in[(bi * s + p) * h + n * d + e];
    }
    void join_qkv_grads(const R *dq, const R *dk, const R *dv, R *dqkv) const
    {
        const int64_t h = c.hidden, nh = c.n_heads, d = h / nh, s = c.seq, b = c.micro_batch;
        for (int64_t bi = 0; bi < b; ++bi)
            for (int64_t p = 0; p < s; ++p)
                for (int64_t n = 0; n < nh; ++n)
                    for (int64_t e = 0; e < d; ++e) {
                        const int64_t t = bi * s + p;
                        const int64_t src = ((bi * nh + n) * s + p) * d + e;
                        dqkv[t * 3 * h + n * d + e] = dq[src];
                        dqkv[t * 3 * h + h + n * d + e] = dk[src];
                        dqkv[t * 3 * h + 2 * h + n * d + e] = dv[src];
                    }
    }

    // One micro-batch through every block of the stage.  Per block:
    //   x1 = x + Attn(Norm1(x)) ; y = x1 + MLP(Norm2(x1))
    void forward(int mb, const R *xin, R *yout)
    {
        const int64_t h = c.hidden, f = c.ffn, nh = c.n_heads, d = h / nh, s = c.seq, b = c.micro_batch;
        const int64_t T = b * s;
        std::vector<R> cur(xin, xin + T * h);
        for (int blk = 0; blk < c.n_blocks; ++blk) {
            Stash<R> &st = stash[mb][blk];
            st.t.clear();
            auto &x = st.get("x", T * h);
            x = cur;
            auto &xhat1 = st.get("xhat1", T * h);
            auto &rstd1 = st.get("rstd1", T);
            auto &n1 = st.get("n1", T * h);
            if (c.arch == 0)
                layernorm_fwd<R>(T, h, x.data(), &W[off(blk, "ln1.gamma")], &W[off(blk, "ln1.beta")],
                                 (R)c.norm_eps, xhat1.data(), rstd1.data(), n1.data());
            else
                rmsnorm_fwd<R>(T, h, x.data(), &W[off(blk, "norm1.gamma")], (R)c.norm_eps, xhat1.data(),
                               rstd1.data(), n1.data());
            std::vector<R> qkv(T * 3 * h);
            linear_fwd<R>(T, h, 3 * h, n1.data(), &W[off(blk, "attn.wqkv")],
                          c.arch == 0 ? &W[off(blk, "attn.bqkv")] : nullptr, qkv.data());
            auto &q = st.get("q", T * h);
            auto &k = st.get("k", T * h);
            auto &v = st.get("v", T * h);
            split_heads(qkv.data(), q.data(), k.data(), v.data());
            if (c.arch == 1) {
                rope_apply<R>(b, nh, s, d, q.data(), c.rope_base, +1);
                rope_apply<R>(b, nh, s, d, k.data(), c.rope_base, +1);
            }
            auto &Pr = st.get("Pr", (size_t)b * nh * s * s);
            std::vector<R> Ah(T * h);
            attention_fwd<R>(b, nh, s, d, q.data(), k.data(), v.data(), Pr.data(), Ah.data());
            auto &A = st.get("A", T * h);
            merge_heads(Ah.data(), A.data());
            auto &x1 = st.get("x1", T * h);
            linear_fwd<R>(T, h, h, A.data(), &W[off(blk, "attn.wo")],
                          c.arch == 0 ? &W[off(blk, "attn.bo")] : nullptr, x1.data());
            for (int64_t i = 0; i < T * h; ++i) x1[i] += x[i];
            auto &xhat2 = st.get("xhat2", T * h);
            auto &rstd2 = st.get("rstd2", T);
            auto &n2 = st.get("n2", T * h);
            std::vector<R> y(T * h);
            if (c.arch == 0) {
                layernorm_fwd<R>(T, h, x1.data(), &W[off(blk, "ln2.gamma")], &W[off(blk, "ln2.beta")],
                                 (R)c.norm_eps, xhat2.data(), rstd2.data(), n2.data());
                auto &u = st.get("u", T * f);
                linear_fwd<R>(T, h, f, n2.data(), &W[off(blk, "mlp.w1")], &W[off(blk, "mlp.b1")], u.data());
                auto &g = st.get("g", T * f);
                for (int64_t i = 0; i < T * f; ++i) g[i] = gelu_val<R>(u[i], c.gelu_mode);
                linear_fwd<R>(T, f, h, g.data(), &W[off(blk, "mlp.w2")], &W[off(blk, "mlp.b2")], y.data());
            } else {
                rmsnorm_fwd<R>(T, h, x1.data(), &W[off(blk, "norm2.gamma")], (R)c.norm_eps, xhat2.data(),
                               rstd2.data(), n2.data());
                auto &gate = st.get("gate", T * f);
                auto &up = st.get("up", T * f);
                linear_fwd<R>(T, h, f, n2.data(), &W[off(blk, "mlp.wgate")], nullptr, gate.data());
                linear_fwd<R>(T, h, f, n2.data(), &W[off(blk, "mlp.wup")], nullptr, up.data());
                auto &act = st.get("act", T * f);
                for (int64_t i = 0; i < T * f; ++i) act[i] = gate[i] * sigmoid_val<R>(gate[i]) * up[i];
                linear_fwd<R>(T, f, h, act.data(), &W[off(blk, "mlp.wdown")], nullptr, y.data());
            }
            for (int64_t i = 0; i < T * h; ++i) y[i] += x1[i];
            auto &yst = st.get("y", T * h);
            yst = y;
            cur.swap(y);
        }
        std::memcpy(yout, cur.data(), sizeof(R) * T * h);
    }

    // Chain rule through the blocks in reverse; writes dx and this micro-batch's weight
    // gradients g_mb into the staging buffer S (same layout as P).
    void backward(int mb, const R *dyin, R *dxout)
    {
        const int64_t h = c.hidden, f = c.ffn, nh = c.n_heads, d = h / nh, s = c.seq, b = c.micro_batch;
        const int64_t T = b * s;
        std::vector<R> dcur(dyin, dyin + T * h);
        for (int blk = c.n_blocks - 1; blk >= 0; --blk) {
            const Stash<R> &st = stash[mb][blk];
            // ---- MLP branch:  y = x1 + MLP(n2)
            std::vector<R> dn2(T * h);
            if (c.arch == 0) {
                std::vector<R> dg(T * f);
                linear_bwd_weight<R>(T, f, h, dcur.data(), st.at("g").data(), &S[off(blk, "mlp.w2")],
                                     &S[off(blk, "mlp.b2")]);
                linear_bwd_input<R>(T, f, h, dcur.data(), &W[off(blk, "mlp.w2")], dg.data());
                const auto &u = st.at("u");
                for (int64_t i = 0; i < T * f; ++i) dg[i] *= gelu_grad<R>(u[i], c.gelu_mode);  // now du
                linear_bwd_weight<R>(T, h, f, dg.data(), st.at("n2").data(), &S[off(blk, "mlp.w1")],
                                     &S[off(blk, "mlp.b1")]);
                linear_bwd_input<R>(T, h, f, dg.data(), &W[off(blk, "mlp.w1")], dn2.data());
            } else {
                std::vector<R> dact(T * f), dgate(T * f), dup(T * f), tmp(T * h);
                linear_bwd_weight<R>(T, f, h, dcur.data(), st.at("act").data(), &S[off(blk, "mlp.wdown")],
                                     (R *)nullptr);
                linear_bwd_input<R>(T, f, h, dcur.data(), &W[off(blk, "mlp.wdown")], dact.data());
                const auto &gate = st.at("gate");
                const auto &up = st.at("up");
                for (int64_t i = 0; i < T * f; ++i) {
                    const R sg = sigmoid_val<R>(gate[i]);
                    dup[i] = dact[i] * gate[i] * sg;
                    dgate[i] = dact[i] * up[i] * (sg + gate[i] * sg * ((R)1 - sg));
                }
                linear_bwd_weight<R>(T, h, f, dgate.data(), st.at("n2").data(), &S[off(blk, "mlp.wgate")],
                                     (R *)nullptr);
                linear_bwd_weight<R>(T, h, f, dup.data(), st.at("n2").data(), &S[off(blk, "mlp.wup")],
                                     (R *)nullptr);
                linear_bwd_input<R>(T, h, f, dgate.data(), &W[off(blk, "mlp.wgate")], dn2.data());
                linear_bwd_input<R>(T, h, f, dup.data(), &W[off(blk, "mlp.wup")], tmp.data());
                for (int64_t i = 0; i < T * h; ++i) dn2[i] += tmp[i];
            }
            std::vector<R> dx1(T * h);
            if (c.arch == 0)
                layernorm_bwd<R>(T, h, dn2.data(), st.at("xhat2").data(), st.at("rstd2").data(),
                                 &W[off(blk, "ln2.gamma")], dx1.data(), &S[off(blk, "ln2.gamma")],
                                 &S[off(blk, "ln2.beta")]);
            else
                rmsnorm_bwd<R>(T, h, dn2.data(), st.at("xhat2").data(), st.at("rstd2").data(),
                               &W[off(blk, "norm2.gamma")], dx1.data(), &S[off(blk, "norm2.gamma")]);
            for (int64_t i = 0; i < T * h; ++i) dx1[i] += dcur[i];  // residual
            // ---- attention branch:  x1 = x + A Wo^T + bo
            std::vector<R> dA(T * h);
            linear_bwd_weight<R>(T, h, h, dx1.data(), st.at("A").data(), &S[off(blk, "attn.wo")],
                                 c.arch == 0 ? &S[off(blk, "attn.bo")] : (R *)nullptr);
            linear_bwd_input<R>(T, h, h, dx1.data(), &W[off(blk, "attn.wo")], dA.data());
            std::vector<R> dAh(T * h), dq(T * h), dk(T * h), dv(T * h);
            unmerge_heads(dA.data(), dAh.data());
            attention_bwd<R>(b, nh, s, d, st.at("q").data(), st.at("k").data(), st.at("v").data(),
                             st.at("Pr").data(), dAh.data(), dq.data(), dk.data(), dv.data());
            if (c.arch == 1) {
                rope_apply<R>(b, nh, s, d, dq.data(), c.rope_base, -1);
                rope_apply<R>(b, nh, s, d, dk.data(), c.rope_base, -1);
            }
            std::vector<R> dqkv(T * 3 * h);
            join_qkv_grads(dq.data(), dk.data(), dv.data(), dqkv.data());
            linear_bwd_weight<R>(T, h, 3 * h, dqkv.data(), st.at("n1").data(), &S[off(blk, "attn.wqkv")],
                                 c.arch == 0 ? &S[off(blk, "attn.bqkv")] : (R *)nullptr);
            std::vector<R> dn1(T * h), dx(T * h);
            linear_bwd_input<R>(T, h, 3 * h, dqkv.data(), &W[off(blk, "attn.wqkv")], dn1.data());
            if (c.arch == 0)
                layernorm_bwd<R>(T, h, dn1.data(), st.at("xhat1").data(), st.at("rstd1").data(),
                                 &W[off(blk, "ln1.gamma")], dx.data(), &S[off(blk, "ln1.gamma")],
                                 &S[off(blk, "ln1.beta")]);
            else
                rmsnorm_bwd<R>(T, h, dn1.data(), st.at("xhat1").data(), st.at("rstd1").data(),
                               &W[off(blk, "norm1.gamma")], dx.data(), &S[off(blk, "norm1.gamma")]);
            for (int64_t i = 0; i < T * h; ++i) dx[i] += dx1[i];  // residual
            dcur.swap(dx);
        }
        std::memcpy(dxout, dcur.data(), sizeof(R) * T * h);
    }

    // Stand-in for the per-unit gradient reduce-scatter: G <- G + scale * g_mb
    void accumulate(R scale)
    {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < (int64_t)N; ++i) G[i] = G[i] + scale * S[i];
    }

    // Adam on elements [offset, offset+count) of the flat shard; see adam_range below.
    void adam(uint64_t offset, uint64_t count, double lr, double beta1, double beta2, double eps,
              double wd, double grad_scale, int step, int decoupled, int zero_grad);
};

// Adam, t = step >= 1, ghat = grad_scale*G:
//   m <- b1 m + (1-b1) ghat ; v <- b2 v + (1-b2) ghat^2 ; mhat = m/(1-b1^t) ; vhat = v/(1-b2^t)
//   decoupled: p <- p - lr (mhat/(sqrt(vhat)+eps) + wd p_old) ; L2 form: ghat += wd p first.
// Every operation is rounded on its own (no fused multiply-add), so the result is the plain
// left-to-right evaluation of the formulas above in the working precision.
template <class R>
__attribute__((optimize("fp-contract=off"))) void adam_range(R *P, R *M, R *V, R *G, int64_t begin,
                                                             int64_t end, double lr, double beta1,
                                                             double beta2, double eps, double wd,
                                                             double grad_scale, int step, int decoupled,
                                                             int zero_grad)
{
    const R b1 = (R)beta1, b2 = (R)beta2;
    // 1-beta is formed in double from the given hyper-parameters, then rounded once
    const R omb1 = (R)(1.0 - beta1), omb2 = (R)(1.0 - beta2);
    const R c1 = (R)(1.0 - std::pow(beta1, (double)step));
    const R c2 = (R)(1.0 - std::pow(beta2, (double)step));
#pragma omp parallel for schedule(static)
    for (int64_t i = begin; i < end; ++i) {
        R g = (R)grad_scale * G[i];
        const R p = P[i];
        if (!decoupled) g = g + (R)wd * p;
        const R m = b1 * M[i] + omb1 * g;
        const R v = b2 * V[i] + (omb2 * g) * g;
        const R mhat = m / c1;
        const R vhat = v / c2;
        R upd = mhat / (std::sqrt(vhat) + (R)eps);
        if (decoupled) upd = upd + (R)wd * p;
        P[i] = p - (R)lr * upd;
        M[i] = m;
        V[i] = v;
        if (zero_grad) G[i] = 0;
    }
}

template <class R>
void Stage<R>::adam(uint64_t offset, uint64_t count, double lr, double beta1, double beta2, double eps,
                    double wd, double grad_scale, int step, int decoupled, int zero_grad)
{
    adam_range<R>(P.data(), M.data(), V.data(), G.data(), (int64_t)offset, (int64_t)(offset + count), lr,
                  beta1, beta2, eps, wd, grad_scale, step, decoupled, zero_grad);
}

template <class R>
R *buffer_ptr(Stage<R> *s, int which)
{
    switch (which) {
    case 0: return s->P.data();
    case 1: return s->G.data();
    case 2: return s->M.data();
    case 3: return s->V.data();
    case 4: return s->W.data();
    case 5: return s->S.data();
    }
    return nullptr;
}

}  // namespace

// ---------------------------------------------------------------------------
// C interface (used through ctypes by the tests)
// ---------------------------------------------------------------------------
extern "C" {

typedef OCfg oracle_cfg;

uint64_t oracle_stage_param_count(const oracle_cfg *c) { return layout_total(make_layout(*c)); }
int32_t oracle_stage_layout_size(const oracle_cfg *c) { return (int32_t)make_layout(*c).size(); }
int32_t oracle_stage_param_layout(const oracle_cfg *c, int32_t idx, char *name, int32_t name_cap,
                                  uint64_t *offset, uint64_t *rows, uint64_t *cols)
{
    auto L = make_layout(*c);
    if (idx < 0 || idx >= (int32_t)L.size()) return -1;
    std::snprintf(name, name_cap, "%s", L[idx].name.c_str());
    *offset = L[idx].offset;
    *rows = L[idx].rows;
    *cols = L[idx].cols;
    return 0;
}

int32_t oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
void oracle_set_num_threads(int32_t n)
{
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

uint16_t oracle_bf16_bits_rne(float v) { return bf16_bits_rne(v); }

// The three flat passes over caller-owned arrays, for shards too large to hold in a Stage on the host
// (a test walks the shard slice by slice).  Same element-wise definitions as Stage::materialize,
// Stage::accumulate and adam_range.
void oracle_flat_materialize_bits(const float *P, uint16_t *W, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) W[i] = bf16_bits_rne(P[i]);
}
void oracle_flat_accumulate_f32(float *G, const float *S, int64_t n, double scale)
{
    const float sc = (float)scale;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) G[i] = G[i] + sc * S[i];
}
void oracle_flat_adam_f32(float *P, float *M, float *V, float *G, int64_t n, double lr, double b1, double b2,
                          double eps, double wd, double grad_scale, int32_t step, int32_t decoupled,
                          int32_t zero_grad)
{
    adam_range<float>(P, M, V, G, 0, n, lr, b1, b2, eps, wd, grad_scale, step, decoupled, zero_grad);
}

#define ORACLE_API(SUF, R)                                                                               \
    void *oracle_stage_create_##SUF(const oracle_cfg *c) { return new Stage<R>(*c); }                    \
    void oracle_stage_destroy_##SUF(void *h) { delete (Stage<R> *)h; }                                   \
    R *oracle_stage_buffer_##SUF(void *h, int32_t which) { return buffer_ptr<R>((Stage<R> *)h, which); } \
    void oracle_stage_materialize_params_##SUF(void *h) { ((Stage<R> *)h)->materialize(); }              \
    void oracle_stage_forward_##SUF(void *h, int32_t mb, const R *x, R *y)                               \
    {                                                                                                    \
        ((Stage<R> *)h)->forward(mb, x, y);                                                              \
    }                                                                                                    \
    void oracle_stage_backward_##SUF(void *h, int32_t mb, const R *dy, R *dx)                            \
    {                                                                                                    \
        ((Stage<R> *)h)->backward(mb, dy, dx);                                                           \
    }                                                                                                    \
    void oracle_stage_accumulate_grads_##SUF(void *h, int32_t mb, double scale)                          \
    {                                                                                                    \
        (void)mb;                                                                                        \
        ((Stage<R> *)h)->accumulate((R)scale);                                                           \
    }                                                                                                    \
    void oracle_shard_adam_step_##SUF(void *h, uint64_t offset, uint64_t count, double lr, double b1,    \
                                      double b2, double eps, double wd, double grad_scale, int32_t step, \
                                      int32_t decoupled, int32_t zero_grad)                              \
    {                                                                                                    \
        ((Stage<R> *)h)->adam(offset, count, lr, b1, b2, eps, wd, grad_scale, step, decoupled,           \
                              zero_grad);                                                                \
    }                                                                                                    \
    void oracle_stage_release_stash_##SUF(void *h, int32_t mb)                                           \
    {                                                                                                    \
        for (auto &st : ((Stage<R> *)h)->stash[mb]) st.t.clear();                                        \
    }                                                                                                    \
    const R *oracle_stage_stash_##SUF(void *h, int32_t mb, int32_t blk, const char *name, uint64_t *n)   \
    {                                                                                                    \
        auto &m = ((Stage<R> *)h)->stash[mb][blk].t;                                                     \
        auto it = m.find(name);                                                                          \
        if (it == m.end()) {                                                                             \
            *n = 0;                                                                                      \
            return nullptr;                                                                              \
        }                                                                                                \
        *n = it->second.size();                                                                          \
        return it->second.data();                                                                        \
    }                                                                                                    \
    void oracle_layernorm_fwd_##SUF(int64_t T, int64_t h, const R *x, const R *g, const R *b, double eps, \
                                    R *xhat, R *rstd, R *n)                                              \
    {                                                                                                    \
        layernorm_fwd<R>(T, h, x, g, b, (R)eps, xhat, rstd, n);                                          \
    }                                                                                                    \
    void oracle_layernorm_bwd_##SUF(int64_t T, int64_t h, const R *dn, const R *xhat, const R *rstd,     \
                                    const R *g, R *dx, R *dg, R *db)                                     \
    {                                                                                                    \
        layernorm_bwd<R>(T, h, dn, xhat, rstd, g, dx, dg, db);                                           \
    }                                                                                                    \
    void oracle_rmsnorm_fwd_##SUF(int64_t T, int64_t h, const R *x, const R *g, double eps, R *xhat,     \
                                  R *rinv, R *n)                                                         \
    {                                                                                                    \
        rmsnorm_fwd<R>(T, h, x, g, (R)eps, xhat, rinv, n);                                               \
    }                                                                                                    \
    void oracle_rmsnorm_bwd_##SUF(int64_t T, int64_t h, const R *dn, const R *xhat, const R *rinv,       \
                                  const R *g, R *dx, R *dg)                                              \
    {                                                                                                    \
        rmsnorm_bwd<R>(T, h, dn, xhat, rinv, g, dx, dg);                                                 \
    }                                                                                                    \
    void oracle_linear_fwd_##SUF(int64_t T, int64_t in, int64_t out, const R *x, const R *W, const R *b, \
                                 R *y)                                                                   \
    {                                                                                                    \
        linear_fwd<R>(T, in, out, x, W, b, y);                                                           \
    }                                                                                                    \
    void oracle_linear_bwd_input_##SUF(int64_t T, int64_t in, int64_t out, const R *dy, const R *W,      \
                                       R *dx)                                                            \
    {                                                                                                    \
        linear_bwd_input<R>(T, in, out, dy, W, dx);                                                      \
    }                                                                                                    \
    void oracle_linear_bwd_weight_##SUF(int64_t T, int64_t in, int64_t out, const R *dy, const R *x,     \
                                        R *dW, R *db)                                                    \
    {                                                                                                    \
        linear_bwd_weight<R>(T, in, out, dy, x, dW, db);                                                 \
    }                                                                                                    \
    void oracle_rope_##SUF(int64_t b, int64_t nh, int64_t s, int64_t d, R *u, double base, int32_t sign) \
    {                                                                                                    \
        rope_apply<R>(b, nh, s, d, u, base, sign);                                                       \
    }                                                                                                    \
    void oracle_attention_fwd_##SUF(int64_t b, int64_t nh, int64_t s, int64_t d, const R *q, const R *k, \
                                    const R *v, R *Pr, R *A)                                             \
    {                                                                                                    \
        attention_fwd<R>(b, nh, s, d, q, k, v, Pr, A);                                                   \
    }                                                                                                    \
    void oracle_attention_bwd_##SUF(int64_t b, int64_t nh, int64_t s, int64_t d, const R *q, const R *k, \
                                    const R *v, const R *Pr, const R *dA, R *dq, R *dk, R *dv)           \
    {                                                                                                    \
        attention_bwd<R>(b, nh, s, d, q, k, v, Pr, dA, dq, dk, dv);                                      \
    }                                                                                                    \
    void oracle_gelu_##SUF(int64_t n, const R *u, int32_t mode, R *g, R *dg)                             \
    {                                                                                                    \
        for (int64_t i = 0; i < n; ++i) {                                                                \
            if (g) g[i] = gelu_val<R>(u[i], mode);                                                       \
            if (dg) dg[i] = gelu_grad<R>(u[i], mode);                                                    \
        }                                                                                                \
    }

ORACLE_API(f32, float)
ORACLE_API(f64, double)

}  // extern "C"
