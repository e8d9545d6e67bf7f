// Host side of the C ABI declared in include/zpp.h: configuration checks, the flat parameter
// layout, the carve-up of the caller's workspace, the per-unit state machine, and the sequence of
// kernel launches that make up materialise / forward / backward / accumulate / Adam for one
// pipeline stage (paper Sections 3.1 and 3.2).  No device memory is allocated here.
#include "../../include/zpp.h"
#include "../../include/zpp_ops.h"
#include "kernels.h"
#include "stage_internal.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

namespace zpp {
hipError_t launch_attn_simple_fwd(int dt, const void *qkv, void *attn, float *lse, int64_t b, int64_t seq,
                                  int64_t nh, int64_t d, hipStream_t s);
hipError_t launch_attn_simple_bwd(int dt, const void *qkv, const void *attn, const void *dattn,
                                  const float *lse, float *delta, void *dqkv, int64_t b, int64_t seq,
                                  int64_t nh, int64_t d, hipStream_t s);
}  // namespace zpp

using namespace zpp;

namespace {

thread_local char g_err[512] = "";
}

zpp_status zpp::set_error(zpp_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

namespace {

zpp_status fail(zpp_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool aligned(const void *p) { return ((uintptr_t)p % kAlign) == 0; }

struct Tensor {
    std::string name;
    uint64_t offset, rows, cols;
};

struct Region {
    uint64_t off = 0, elems = 0;
    int esz = 0;
};

enum MbState { MB_IDLE = 0, MB_FWD = 1, MB_BWD = 2, MB_ACC = 3, MB_BIN = 4 /* input gradient done, weight gradient due */ };

// ---- optional per-kernel-class timing with HIP events on the caller's stream -------------------
struct ProfRec {
    int cls;
    double work, bytes;
    hipEvent_t e0, e1;
};
// The switch and the records are process-wide and shared by all stages and streams; a mutex keeps host
// threads that drive different stages from corrupting them.
std::atomic<bool> g_prof_on{false};
std::mutex g_prof_mu;
std::vector<ProfRec> g_prof;
std::vector<hipEvent_t> g_event_pool;

hipEvent_t prof_event()
{
    {
        std::lock_guard<std::mutex> lock(g_prof_mu);
        if (!g_event_pool.empty()) {
            hipEvent_t e = g_event_pool.back();
            g_event_pool.pop_back();
            return e;
        }
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

// Brackets the launches of its scope with two events.  If an event cannot be created the scope is simply
// not recorded (timing is an optional extra; the launches themselves are unaffected).
struct ProfScope {
    bool on;
    ProfRec r;
    hipStream_t st;
    ProfScope(int cls, double work, hipStream_t s, double bytes = 0.0) : on(g_prof_on.load()), st(s)
    {
        if (!on) return;
        r = {cls, work, bytes, prof_event(), prof_event()};
        if (!r.e0 || !r.e1) {
            std::lock_guard<std::mutex> lock(g_prof_mu);
            if (r.e0) g_event_pool.push_back(r.e0);
            if (r.e1) g_event_pool.push_back(r.e1);
            on = false;
            return;
        }
        (void)hipEventRecord(r.e0, st);
    }
    ~ProfScope()
    {
        if (!on) return;
        (void)hipEventRecord(r.e1, st);
        std::lock_guard<std::mutex> lock(g_prof_mu);
        g_prof.push_back(r);
    }
};

}  // namespace

struct zpp_stage {
    zpp_stage_config c;
    int64_t T, h, f, f1, d, nh, L, U;
    int dt;
    size_t esz;
    std::vector<Tensor> layout;
    std::map<std::string, size_t> index;      // name -> layout idx
    struct WtEntry { uint64_t src_off, rows, cols, dst_off; };
    std::map<std::string, WtEntry> wt;        // matrix name -> its slot in the transposed working copy
    uint64_t N = 0, Nmat = 0;

    // workspace plan (byte offsets)
    Region rW, rWt, rS, rRope;
    // The stash of a unit is laid out [block][tensor][micro-batch]: the copies of one tensor for consecutive
    // micro-batches lie back to back, so a group of micro-batches is one [count * T, width] matrix.
    uint64_t stash_base = 0, stash_block_bytes = 0;
    std::map<std::string, Region> stash_t;    // kept per (micro-batch, block): off = start of the tensor's U copies
                                              // inside a block's area, elems = per micro-batch
    // With recomputation the tensors that are rebuilt in backward live in one slot instead, valid for the
    // block and the group of micro-batches (rc_first ...) it was rebuilt for last, laid out [tensor][micro-batch].
    uint64_t rc_base = 0;
    std::map<std::string, Region> rc_t;
    int rc_first = 0;
    int64_t gmax = 1;                         // most micro-batches a grouped call may take
    std::map<std::string, Region> tmp;        // shared temporaries
    uint64_t ws_bytes = 0;

    // bound memory
    float *P = nullptr, *G = nullptr, *M = nullptr, *V = nullptr;
    unsigned char *ws = nullptr;
    bool bound = false, materialized = false, rope_ready = false;
    bool w_fresh = false;        // the plain working copy already holds cast(P) (an Adam step wrote it back)
    bool shared_wcopy = false;   // the working-copy part is a slot shared with other stages (zpp_device)
    std::vector<int> mb_state;
    int pending_acc = -1;
    uint64_t n_materialize = 0, materialize_bytes = 0;

    // Second levels of the column reductions (bias and gain gradients) of one stage_backward call: each
    // first level writes its partial rows into its own slot of the "redpool" scratch and is listed here;
    // one launch at the end of the call finishes them all.
    std::vector<FinishItem> finish;
    // per input-gradient task (of one micro-batch or a group): the norm-gain reductions it started (two per
    // block, top block first), finished by the weight-gradient task that covers its micro-batches
    struct InputTask {
        int first, count;
        std::vector<FinishItem> items;
    };
    std::vector<InputTask> input_tasks;
    uint64_t red_floats = 0;  // floats per slot and micro-batch
    int cur_count = 1;        // micro-batches of the call in progress,
    int64_t Tc = 0, bc = 0;   // its tokens (cur_count * T) and samples (cur_count * micro_batch)
    void begin_call(int count)
    {
        cur_count = count;
        Tc = (int64_t)count * T;
        bc = (int64_t)count * c.micro_batch;
    }
    // whether the first MLP product stores its pre-activation (fp32 stages; selective recomputation) or the
    // activation's derivative in its place
    bool keeps_preactivation() const { return dt != DT_BF16 || c.recompute == ZPP_RECOMPUTE_SELECTIVE; }
    float *red_slot() const
    {
        return (float *)(ws + tmp.at("redpool").off) + finish.size() * red_floats * (uint64_t)cur_count;
    }
    FinishItem *defer()
    {
        finish.emplace_back();
        return &finish.back();
    }

    uint64_t off(int blk, const char *nm) const
    {
        return layout[index.at("blk" + std::to_string(blk) + "." + nm)].offset;
    }
    void *Wp(int blk, const char *nm) const { return ws + rW.off + off(blk, nm) * esz; }
    bool has_wt(int blk, const char *nm) const { return wt.count("blk" + std::to_string(blk) + "." + nm) != 0; }
    void *Wtp(int blk, const char *nm) const
    {
        return ws + rWt.off + wt.at("blk" + std::to_string(blk) + "." + nm).dst_off * 2;
    }
    // Where the gradient of a tensor goes during a backward call: its place in the staging buffer, or,
    // when the call accumulates in place (stage_backward_accumulate), its place in G.
    bool acc_in_place = false;
    float acc_scale = 1.0f;
    // An Adam step with zero_grad = 2 releases G instead of zeroing it: G counts as zero although its memory still
    // holds the old gradients, and the first task that adds into G afterwards writes instead (acc_write: the
    // weight-gradient products store their result, the column reductions store their sums - with scale 1 the bits
    // that adding onto zeros gives).
    bool g_released = false, acc_write = false;
    // weight-gradient products of the block in hand that wait for one launch together (K-major kernel only)
    std::vector<GemmProblem> dw_batch;
    double dw_batch_flops = 0.0, dw_batch_bytes = 0.0;
    float *Sp(int blk, const char *nm) const
    {
        return (acc_in_place ? G : (float *)(ws + rS.off)) + off(blk, nm);
    }
    // Address of a stashed tensor of micro-batch mb and block blk.
    uint64_t stash_off(int mb, int blk, const std::string &nm) const
    {
        auto it = stash_t.find(nm);
        if (it != stash_t.end())
            return stash_base + (uint64_t)blk * stash_block_bytes + it->second.off +
                   (uint64_t)mb * it->second.elems * it->second.esz;
        const Region &r = rc_t.at(nm);
        return rc_base + r.off + (uint64_t)(mb - rc_first) * r.elems * r.esz;
    }
    void *stash(int mb, int blk, const char *nm) const { return ws + stash_off(mb, blk, nm); }
    void *tp(const char *nm) const { return ws + tmp.at(nm).off; }
};

namespace {

void build_layout(zpp_stage *s)
{
    uint64_t off = 0;
    const uint64_t h = s->h, f = s->f;
    auto add = [&](int blk, const char *nm, uint64_t r, uint64_t c) {
        Tensor t{"blk" + std::to_string(blk) + "." + nm, off, r, c};
        s->index[t.name] = s->layout.size();
        s->layout.push_back(t);
        off += r * c;
    };
    for (int b = 0; b < s->L; ++b) {
        if (s->c.arch == ZPP_ARCH_GPT) {
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
    s->N = off;
    // Transposed working copy (bf16 mode): one [cols, rows] slot for every matrix whose input-gradient product
    // cannot read it as stored (the NN kernel takes W[out, in] in place when `in` is a multiple of 256 and `out`
    // of 64; the stages that are timed keep no transposed copy at all).  wgate and wup are adjacent and are used
    // as one [2f, h] matrix, so they share one [h, 2f] slot.
    uint64_t woff = 0;
    for (auto &t : s->layout) {
        if (t.rows <= 1) continue;
        const std::string leaf = t.name.substr(t.name.find('.') + 1);
        if (leaf == "mlp.wup") continue;
        const uint64_t rows = leaf == "mlp.wgate" ? 2 * t.rows : t.rows;
        if (t.offset % 8 == 0 && gemm_bf16_nn_supported(1, (int64_t)t.cols, (int64_t)rows, (int64_t)rows, (int64_t)t.cols))
            continue;
        s->wt[t.name] = {t.offset, rows, t.cols, woff};
        woff += rows * t.cols;
    }
    s->Nmat = woff;
}

constexpr uint64_t kRedPerBlock = 6;  // four bias gradients and two norm-gain gradients per block at most

// The workspace has three parts, each planned from its own base offset so that several stages on one
// device can share what only one of them uses at a time:
//   working copy  W, transposed copies where needed, the rotary table   (one gathered stage, Section 4.2)
//   scratch       the fp32 staging gradients and per-call temporaries
//   stash         the activations of the unit's micro-batches     (private to a stage)
// Returns the sizes of the three parts.
struct PartSizes {
    uint64_t wcopy, scratch, stash;
};

PartSizes plan_workspace(zpp_stage *s, uint64_t wcopy_off, uint64_t scratch_off, uint64_t stash_off)
{
    uint64_t cur = wcopy_off;
    auto carve = [&](uint64_t elems, int esz) {
        Region r;
        r.off = cur;
        r.elems = elems;
        r.esz = esz;
        cur = align_up(cur + elems * esz);
        return r;
    };
    const int e = (int)s->esz;
    const uint64_t T = s->T, h = s->h, f = s->f, f1 = s->f1;
    PartSizes sz;
    // ---- working copy
    s->rW = carve(s->N, e);
    if (s->dt == DT_BF16) s->rWt = carve(s->Nmat, 2);
    if (s->c.arch == ZPP_ARCH_LLAMA) s->rRope = carve((uint64_t)s->c.seq * (s->d / 2) * 2, 4);
    sz.wcopy = cur - wcopy_off;
    // ---- activation stash, [block][tensor][micro-batch]
    cur = stash_off;
    s->stash_t.clear();
    s->rc_t.clear();
    s->gmax = std::max<int64_t>({1, (int64_t)s->c.split_backward, (int64_t)s->c.group_mbs});
    {
        // recompute = 1 (full): only the block inputs stay per micro-batch; 2 (selective): everything but the
        // outputs of the norms and of the activation function, which backward rebuilds element-wise
        auto rebuilt = [&](const std::string &nm) {
            if (s->c.recompute == ZPP_RECOMPUTE_FULL)
                return nm == "mean1" || nm == "rstd1" || nm == "n1" || nm == "qkv" || nm == "attn" || nm == "lse" ||
                       nm == "x1" || nm == "mean2" || nm == "rstd2" || nm == "n2" || nm == "u" || nm == "g";
            if (s->c.recompute == ZPP_RECOMPUTE_SELECTIVE) return nm == "n1" || nm == "n2" || nm == "g";
            return false;
        };
        uint64_t rel = 0, rc_rel = 0;
        auto sc = [&](const char *nm, uint64_t elems, int esz) {
            Region r;
            r.elems = elems;
            r.esz = esz;
            if (rebuilt(nm)) {
                r.off = rc_rel;
                rc_rel = align_up(rc_rel + elems * esz * (uint64_t)s->gmax);
                s->rc_t[nm] = r;
            } else {
                r.off = rel;
                rel = align_up(rel + elems * esz * (uint64_t)s->U);
                s->stash_t[nm] = r;
            }
        };
        sc("x", T * h, e);
        sc("mean1", T, 4);
        sc("rstd1", T, 4);
        sc("n1", T * h, e);
        sc("qkv", T * 3 * h, e);
        sc("attn", T * h, e);
        sc("lse", (uint64_t)s->c.micro_batch * s->nh * s->c.seq, 4);
        sc("x1", T * h, e);
        sc("mean2", T, 4);
        sc("rstd2", T, 4);
        sc("n2", T * h, e);
        sc("u", T * f1, e);
        sc("g", T * f, e);
        if (s->c.split_backward) {
            // what the weight-gradient task of a micro-batch needs from its input-gradient task: the dY of
            // the four linear layers and the first-level partial sums of the two norm-gain reductions
            sc("d_y", T * h, e);
            sc("d_u", T * f1, e);
            sc("d_x1", T * h, e);
            sc("d_qkv", T * 3 * h, e);
            sc("red_n2", colreduce_scratch_floats((int64_t)T, (int64_t)h), 4);
            sc("red_n1", colreduce_scratch_floats((int64_t)T, (int64_t)h), 4);
        }
        s->stash_block_bytes = rel;
        s->stash_base = cur;
        cur = align_up(cur + (uint64_t)s->L * rel);
        s->rc_base = cur;
        cur = align_up(cur + rc_rel);
    }
    sz.stash = cur - stash_off;
    // ---- scratch
    cur = scratch_off;
    s->rS = carve(s->N, 4);
    s->tmp.clear();
    auto tmp = [&](const char *nm, uint64_t elems, int esz) { s->tmp[nm] = carve(elems, esz); };
    // grouped calls work on up to gmax micro-batches at once: every temporary holds that many
    const uint64_t gmax = (uint64_t)s->gmax;
    tmp("gA", T * h * gmax, e);
    tmp("gB", T * h * gmax, e);
    tmp("dn", T * h * gmax, e);
    tmp("dx1", T * h * gmax, e);
    tmp("dattn", T * h * gmax, e);
    tmp("dqkv", T * 3 * h * gmax, e);
    tmp("du", T * f1 * gmax, e);
    if (s->c.arch == ZPP_ARCH_LLAMA) tmp("dact", T * f * gmax, e);
    tmp("delta", 2 * (uint64_t)s->c.micro_batch * s->nh * s->c.seq * gmax, 4);  // per query: delta and a scaled log-sum-exp
    const uint64_t widest = std::max<uint64_t>(3 * h, f1);
    if (s->dt == DT_BF16) {
        // K-contiguous copies of the operands of a weight-gradient product over K = gmax * T tokens
        tmp("tA", widest * T * gmax, 2);
        tmp("tB", std::max<uint64_t>(h, f) * T * gmax, 2);
    }
    // reductions over count * T rows need at most count times the partial rows of one micro-batch
    s->red_floats = std::max(colreduce_scratch_floats((int64_t)T, (int64_t)widest),
                             transpose_colsum_scratch_floats((int64_t)T, (int64_t)widest));
    tmp("redpool", s->red_floats * kRedPerBlock * s->L * gmax, 4);  // one slot per column reduction of a backward call
    s->finish.reserve(kRedPerBlock * s->L);
    sz.scratch = cur - scratch_off;
    return sz;
}

#define ZPP_OTHER(expr)                                   \
    do {                                                  \
        ProfScope _prof(ZPP_PROF_OTHER, 0.0, st);         \
        ZPP_TRY(expr);                                    \
    } while (0)

#define ZPP_TRY(expr)                                                                                    \
    do {                                                                                                 \
        hipError_t _e = (expr);                                                                          \
        if (_e != hipSuccess)                                                                            \
            return fail(ZPP_ERR_DEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), __FILE__, \
                        __LINE__);                                                                       \
    } while (0)

// y[T,out] = epilogue(x[T,in] . W[out,in]^T)
hipError_t linear_fwd(zpp_stage *s, const void *x, int blk, const char *w, int64_t in, int64_t out, void *y,
                      GemmEpi epi, hipStream_t st)
{
    ProfScope prof(ZPP_PROF_GEMM, 2.0 * s->Tc * in * out, st,
                   (double)s->esz * ((double)s->Tc * in + (double)in * out + (double)s->Tc * out));
    if (s->dt == DT_BF16)
        return launch_gemm_bf16_nt(s->Tc, out, in, x, in, s->Wp(blk, w), in, y, out, epi, st);
    return launch_gemm_f32(s->Tc, out, in, (const float *)x, in, 1, (const float *)s->Wp(blk, w), in, 1,
                           (float *)y, out, epi, st);
}

// Input gradient (Section 2.3): dx[T,in] = epilogue(dy[T,out] . W[out,in])
hipError_t linear_dx(zpp_stage *s, const void *dy, int blk, const char *w, int64_t in, int64_t out, void *dx,
                     GemmEpi epi, hipStream_t st)
{
    ProfScope prof(ZPP_PROF_GEMM, 2.0 * s->Tc * in * out, st,
                   (double)s->esz * ((double)s->Tc * in + (double)in * out + (double)s->Tc * out));
    if (s->dt == DT_BF16) {
        // W[out, in] as stored is the K-major operand of the NN kernel; matrices of other shapes have a
        // transposed copy W^T[in, out], with which both operands are K-contiguous
        if (!s->has_wt(blk, w)) return launch_gemm_bf16_nn(s->Tc, in, out, dy, out, s->Wp(blk, w), in, dx, in, epi, st);
        return launch_gemm_bf16_nt(s->Tc, in, out, dy, out, s->Wtp(blk, w), out, dx, in, epi, st);
    }
    return launch_gemm_f32(s->Tc, in, out, (const float *)dy, out, 1, (const float *)s->Wp(blk, w), 1, in,
                           (float *)dx, in, epi, st);
}

// Weight gradient (Section 2.3): dW[out,in] = dy[T,out]^T . x[T,in]  (fp32, into the staging buffer),
// and optionally db[out] = column sums of dy.
// The K-major weight-gradient products collected since the last flush, as one launch.  Their operands (the
// block's stash slots and gradient buffers) must still hold what they held when linear_dw saw them: the callers
// flush before they leave a block.
hipError_t flush_dw_batch(zpp_stage *s, hipStream_t st)
{
    if (s->dw_batch.empty()) return hipSuccess;
    GemmEpi epi;
    epi.out_f32 = s->acc_in_place && !s->acc_write ? 2 : 1;
    epi.accum_scale = s->acc_scale;
    hipError_t e;
    {
        ProfScope prof(ZPP_PROF_GEMM_DW, s->dw_batch_flops, st, s->dw_batch_bytes);
        if (s->dw_batch.size() == 1) {
            const GemmProblem &q = s->dw_batch[0];
            e = launch_gemm_bf16_tt(q.M, q.N, s->Tc, q.A, q.lda, q.B, q.ldb, q.C, q.ldc, epi, st);
        } else {
            e = launch_gemm_bf16_tt_group(s->dw_batch.data(), (int)s->dw_batch.size(), s->Tc, epi, st);
        }
    }
    s->dw_batch.clear();
    s->dw_batch_flops = s->dw_batch_bytes = 0.0;
    return e;
}

hipError_t linear_dw(zpp_stage *s, const void *dy, const void *x, int blk, const char *w, const char *bias,
                     int64_t in, int64_t out, hipStream_t st)
{
    GemmEpi epi;
    epi.out_f32 = s->acc_in_place && !s->acc_write ? 2 : 1;
    epi.accum_scale = s->acc_scale;
    hipError_t e;
    if (s->dt == DT_BF16) {
        // Both operands are stored token-major.  The K-major kernel reads them in place (the bias gradient is
        // then a column-sum pass over dY); for shapes it does not take they are transposed into scratch first
        // so that the NT kernel sees K-contiguous operands, and the bias gradient comes out of the pass that
        // transposes dY.
        if (gemm_bf16_tt_supported(out, in, s->Tc, out, in)) {
            // K-major product: dY and X are read where they lie; the bias gradient needs its own pass over dY
            if (bias) {
                ProfScope prof(ZPP_PROF_OTHER, 0.0, st);
                float *slot = s->red_slot();
                e = launch_colreduce(DT_BF16, COLRED_SUM, dy, nullptr, nullptr, nullptr, s->Tc, out, out, s->Sp(blk, bias),
                                     nullptr, slot, st, s->defer());
                if (e != hipSuccess) return e;
            }
            // the product itself waits for the other products of its block: they go out as one grid
            s->dw_batch.push_back({out, in, dy, out, x, in, s->Sp(blk, w), in});
            s->dw_batch_flops += 2.0 * s->Tc * in * out;
            s->dw_batch_bytes += 2.0 * ((double)s->Tc * in + (double)s->Tc * out) + (s->acc_in_place && !s->acc_write ? 8.0 : 4.0) * in * out;
            if ((int)s->dw_batch.size() == kGemmGroupMax) return flush_dw_batch(s, st);
            return hipSuccess;
        }
        void *tA = s->tp("tA"), *tB = s->tp("tB");
        {
            ProfScope prof(ZPP_PROF_OTHER, 0.0, st);
            if (s->Tc % 64 == 0 && in % 64 == 0 && out % 64 == 0) {  // both transposes in one launch
                float *slot = bias ? s->red_slot() : nullptr;
                e = launch_transpose_pair(dy, s->Tc, out, out, tA, s->Tc, bias ? s->Sp(blk, bias) : nullptr, slot,
                                          bias ? s->defer() : nullptr, x, s->Tc, in, in, tB, s->Tc, st);
                if (e != hipSuccess) return e;
            } else {
                // ragged sizes: element-wise transposes and a separate column reduction for the bias gradient
                if ((e = launch_transpose(DT_BF16, dy, s->Tc, out, out, tA, s->Tc, st)) != hipSuccess) return e;
                if ((e = launch_transpose(DT_BF16, x, s->Tc, in, in, tB, s->Tc, st)) != hipSuccess) return e;
                if (bias) {
                    float *slot = s->red_slot();
                    e = launch_colreduce(DT_BF16, COLRED_SUM, dy, nullptr, nullptr, nullptr, s->Tc, out, out,
                                         s->Sp(blk, bias), nullptr, slot, st, s->defer());
                    if (e != hipSuccess) return e;
                }
            }
        }
        ProfScope prof(ZPP_PROF_GEMM_DW, 2.0 * s->Tc * in * out, st,
                       2.0 * ((double)s->Tc * in + (double)s->Tc * out) + (s->acc_in_place && !s->acc_write ? 8.0 : 4.0) * in * out);
        e = launch_gemm_bf16_nt(out, in, s->Tc, tA, s->Tc, tB, s->Tc, s->Sp(blk, w), in, epi, st);
        return e;
    } else {
        ProfScope prof(ZPP_PROF_GEMM_DW, 2.0 * s->Tc * in * out, st,
                       4.0 * ((double)s->Tc * in + (double)s->Tc * out + (double)in * out));
        e = launch_gemm_f32(out, in, s->Tc, (const float *)dy, 1, out, (const float *)x, 1, in, s->Sp(blk, w),
                            in, epi, st);
    }
    if (e != hipSuccess) return e;
    ProfScope prof2(ZPP_PROF_OTHER, 0.0, st);
    if (bias) {
        float *slot = s->red_slot();
        e = launch_colreduce(s->dt, COLRED_SUM, dy, nullptr, nullptr, nullptr, s->Tc, out, out, s->Sp(blk, bias),
                             nullptr, slot, st, s->defer());
    }
    return e;
}

// The attention kernels of a grouped call take the whole group in one launch (up to this many micro-batches):
// their work-group order walks the (sample, head) pairs in chunks, so locality in the L2s does not depend on
// the size of the launch, and the ramp and tail of a launch are paid once per group (forward at 32 heads x
// 2048: 51 us per micro-batch at two, 41 at eight; backward 168 and 154).
constexpr int kAttnMicroBatches = 64;

hipError_t attention_fwd(zpp_stage *s, const void *qkv, void *attn, float *lse, hipStream_t st)
{
    const int64_t b = s->c.micro_batch, T = s->T, h = s->h;
    for (int m = 0; m < s->cur_count; m += kAttnMicroBatches) {
        const int64_t nb = std::min<int64_t>(kAttnMicroBatches, s->cur_count - m) * b;
        const void *q = (const unsigned char *)qkv + (size_t)m * T * 3 * h * s->esz;
        void *o = (unsigned char *)attn + (size_t)m * T * h * s->esz;
        float *l = lse + (size_t)m * b * s->nh * s->c.seq;
        // causal convention: two matmuls over the lower triangle, 2*b*s^2*h flops
        ProfScope prof(ZPP_PROF_ATTN_FWD, 2.0 * nb * (double)s->c.seq * s->c.seq * h, st);
        hipError_t e;
        if (s->dt == DT_BF16 && attn_mfma_supported(s->c.seq, s->d))
            e = launch_attn_fwd(s->dt, q, o, l, nb, s->c.seq, s->nh, s->d, st);
        else
            e = launch_attn_simple_fwd(s->dt, q, o, l, nb, s->c.seq, s->nh, s->d, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t attention_bwd(zpp_stage *s, const void *qkv, const void *attn, const void *dattn, const float *lse,
                         void *dqkv, hipStream_t st)
{
    const int64_t b = s->c.micro_batch, T = s->T, h = s->h;
    for (int m = 0; m < s->cur_count; m += kAttnMicroBatches) {
        const int64_t nb = std::min<int64_t>(kAttnMicroBatches, s->cur_count - m) * b;
        const size_t row = (size_t)m * T * s->esz, stat = (size_t)m * b * s->nh * s->c.seq;
        const void *q = (const unsigned char *)qkv + row * 3 * h, *o = (const unsigned char *)attn + row * h;
        const void *dO = (const unsigned char *)dattn + row * h;
        void *dq = (unsigned char *)dqkv + row * 3 * h;
        float *delta = (float *)s->tp("delta") + 2 * stat;
        ProfScope prof(ZPP_PROF_ATTN_BWD, 4.0 * nb * (double)s->c.seq * s->c.seq * h, st);
        hipError_t e;
        if (s->dt == DT_BF16 && attn_mfma_supported(s->c.seq, s->d))
            e = launch_attn_bwd(s->dt, q, o, dO, lse + stat, delta, dq, nb, s->c.seq, s->nh, s->d, st);
        else
            e = launch_attn_simple_bwd(s->dt, q, o, dO, lse + stat, delta, dq, nb, s->c.seq, s->nh, s->d, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

zpp_status check_stage(const zpp_stage *s, bool need_bound)
{
    if (!s) return fail(ZPP_ERR_ARG, "stage is NULL");
    if (need_bound && !s->bound) return fail(ZPP_ERR_STATE, "stage has no bound memory (call zpp_stage_bind)");
    return ZPP_OK;
}

}  // namespace

extern "C" {

const char *zpp_last_error(void) { return g_err; }
const char *zpp_version(void) { return "zpp-stage 0.1 (gfx950)"; }

zpp_status zpp_stage_create(const zpp_stage_config *cfg, zpp_stage **out)
{
    if (!cfg || !out) return fail(ZPP_ERR_ARG, "cfg/out is NULL");
    *out = nullptr;
    const zpp_stage_config &c = *cfg;
    if (c.arch != ZPP_ARCH_GPT && c.arch != ZPP_ARCH_LLAMA) return fail(ZPP_ERR_ARG, "arch must be 0 or 1");
    if (c.compute_dtype != ZPP_DTYPE_FP32 && c.compute_dtype != ZPP_DTYPE_BF16)
        return fail(ZPP_ERR_ARG, "compute_dtype must be 0 or 1");
    if (c.gelu_mode != ZPP_GELU_TANH && c.gelu_mode != ZPP_GELU_ERF)
        return fail(ZPP_ERR_ARG, "gelu_mode must be 0 or 1");
    if (c.n_blocks <= 0 || c.hidden <= 0 || c.n_heads <= 0 || c.ffn <= 0 || c.seq <= 0 || c.micro_batch <= 0 ||
        c.unit_mbs <= 0)
        return fail(ZPP_ERR_ARG, "all sizes must be positive");
    if (c.hidden % c.n_heads) return fail(ZPP_ERR_ARG, "hidden (%d) not divisible by n_heads (%d)", c.hidden, c.n_heads);
    if (!(c.norm_eps > 0.0f)) return fail(ZPP_ERR_ARG, "norm_eps must be > 0");
    if (c.split_backward < 0 || c.split_backward > c.unit_mbs)
        return fail(ZPP_ERR_ARG, "split_backward must lie in [0, unit_mbs]");
    if (c.recompute != ZPP_RECOMPUTE_NONE && c.recompute != ZPP_RECOMPUTE_FULL && c.recompute != ZPP_RECOMPUTE_SELECTIVE)
        return fail(ZPP_ERR_ARG, "recompute must be 0 (none), 1 (full) or 2 (selective)");
    if (c.group_mbs < 0 || c.group_mbs > c.unit_mbs) return fail(ZPP_ERR_ARG, "group_mbs must lie in [0, unit_mbs]");
    const int64_t d = c.hidden / c.n_heads;
    if (c.arch == ZPP_ARCH_LLAMA && (d % 2)) return fail(ZPP_ERR_ARG, "rotary embedding needs an even head dim");
    if (c.arch == ZPP_ARCH_LLAMA && !(c.rope_base > 0.0f)) return fail(ZPP_ERR_ARG, "rope_base must be > 0");
    const int vec = c.compute_dtype == ZPP_DTYPE_BF16 ? 8 : 4;
    if (c.hidden % vec || c.ffn % vec)
        return fail(ZPP_ERR_UNSUPPORTED, "hidden and ffn must be multiples of %d elements (16-byte vectors)", vec);
    const int64_t T = (int64_t)c.micro_batch * c.seq;
    if (c.compute_dtype == ZPP_DTYPE_BF16) {
        if (c.hidden % 64 || c.ffn % 64 || T % 64)
            return fail(ZPP_ERR_UNSUPPORTED,
                        "bf16 MFMA GEMMs need hidden, ffn and micro_batch*seq to be multiples of 64");
    }
    if ((2 * d + 2 * (int64_t)c.seq) * 4 > 64 * 1024 &&
        !(c.compute_dtype == ZPP_DTYPE_BF16 && attn_mfma_supported(c.seq, d)))
        return fail(ZPP_ERR_UNSUPPORTED, "sequence too long for the generic attention kernel");
    if (c.micro_batch > 65535 || c.n_heads > 65535) return fail(ZPP_ERR_UNSUPPORTED, "micro_batch/n_heads too large");

    zpp_stage *s = new (std::nothrow) zpp_stage();
    if (!s) return fail(ZPP_ERR_ARG, "out of host memory");
    s->c = c;
    s->T = T;
    s->h = c.hidden;
    s->f = c.ffn;
    s->f1 = c.arch == ZPP_ARCH_LLAMA ? 2 * (int64_t)c.ffn : c.ffn;
    s->d = d;
    s->nh = c.n_heads;
    s->L = c.n_blocks;
    s->U = c.unit_mbs;
    s->dt = c.compute_dtype == ZPP_DTYPE_BF16 ? DT_BF16 : DT_F32;
    s->esz = dt_size(s->dt);
    build_layout(s);
    {
        // a stage on its own: the three parts one after the other
        const PartSizes sz = plan_workspace(s, 0, 0, 0);
        plan_workspace(s, 0, sz.wcopy, sz.wcopy + sz.scratch);
        s->ws_bytes = sz.wcopy + sz.scratch + sz.stash;
    }
    s->mb_state.assign(s->U, MB_IDLE);
    s->input_tasks.clear();
    *out = s;
    return ZPP_OK;
}

void zpp_stage_destroy(zpp_stage *s) { delete s; }

uint64_t zpp_stage_param_count(const zpp_stage *s) { return s ? s->N : 0; }
uint64_t zpp_stage_workspace_bytes(const zpp_stage *s) { return s ? s->ws_bytes : 0; }
int32_t zpp_stage_layout_size(const zpp_stage *s) { return s ? (int32_t)s->layout.size() : 0; }

zpp_status zpp_stage_param_layout(const zpp_stage *s, int32_t idx, const char **name, uint64_t *offset,
                                  uint64_t *rows, uint64_t *cols)
{
    if (check_stage(s, false)) return ZPP_ERR_ARG;
    if (idx < 0 || idx >= (int32_t)s->layout.size()) return fail(ZPP_ERR_ARG, "layout index %d out of range", idx);
    const Tensor &t = s->layout[idx];
    if (name) *name = t.name.c_str();
    if (offset) *offset = t.offset;
    if (rows) *rows = t.rows;
    if (cols) *cols = t.cols;
    return ZPP_OK;
}

namespace {

void attach(zpp_stage *s, float *P, float *G, float *M, float *V, void *base)
{
    s->P = P;
    s->G = G;
    s->M = M;
    s->V = V;
    s->ws = (unsigned char *)base;
    s->bound = true;
    s->materialized = false;
    s->rope_ready = false;
    s->w_fresh = false;
    s->g_released = false;
    s->pending_acc = -1;
    s->mb_state.assign(s->U, MB_IDLE);
    s->input_tasks.clear();
}

}  // namespace

zpp_status zpp_stage_bind(zpp_stage *s, float *P, float *G, float *M, float *V, void *workspace,
                          uint64_t workspace_bytes)
{
    if (check_stage(s, false)) return ZPP_ERR_ARG;
    if (!P || !G || !M || !V || !workspace) return fail(ZPP_ERR_ARG, "P, G, M, V and workspace must be non-NULL");
    if (!aligned(P) || !aligned(G) || !aligned(M) || !aligned(V) || !aligned(workspace))
        return fail(ZPP_ERR_ALIGN, "P, G, M, V and workspace must be 256-byte aligned");
    if (workspace_bytes < s->ws_bytes)
        return fail(ZPP_ERR_WORKSPACE, "workspace has %llu bytes, %llu needed", (unsigned long long)workspace_bytes,
                    (unsigned long long)s->ws_bytes);
    const PartSizes sz = plan_workspace(s, 0, 0, 0);
    plan_workspace(s, 0, sz.wcopy, sz.wcopy + sz.scratch);
    attach(s, P, G, M, V, workspace);
    s->shared_wcopy = false;
    return ZPP_OK;
}

extern "C++" {

StageParts zpp::stage_parts(const zpp_stage *s)
{
    zpp_stage probe = *s;  // planning writes the region tables
    const PartSizes sz = plan_workspace(&probe, 0, 0, 0);
    return {sz.wcopy, sz.scratch, sz.stash};
}

zpp_status zpp::stage_bind_parts(zpp_stage *s, float *P, float *G, float *M, float *V, void *base,
                                 uint64_t wcopy_off, uint64_t scratch_off, uint64_t stash_off)
{
    if (check_stage(s, false)) return ZPP_ERR_ARG;
    if (!P || !G || !M || !V || !base) return fail(ZPP_ERR_ARG, "P, G, M, V and workspace must be non-NULL");
    if (!aligned(P) || !aligned(G) || !aligned(M) || !aligned(V) || !aligned(base) || wcopy_off % kAlign ||
        scratch_off % kAlign || stash_off % kAlign)
        return fail(ZPP_ERR_ALIGN, "P, G, M, V, the workspace and its parts must be 256-byte aligned");
    plan_workspace(s, wcopy_off, scratch_off, stash_off);
    attach(s, P, G, M, V, base);
    s->shared_wcopy = true;
    return ZPP_OK;
}

void zpp::stage_drop_working_copy(zpp_stage *s) { s->materialized = false; }
bool zpp::stage_has_working_copy(const zpp_stage *s) { return s->materialized; }

}  // extern "C++"

zpp_status stage_materialize_params(zpp_stage *s, void *hip_stream)
{
    if (zpp_status e = check_stage(s, true)) return e;
    hipStream_t st = (hipStream_t)hip_stream;
    // an Adam step that wrote the new parameters back has already produced the plain copy
    const bool plain = !s->w_fresh;
    uint64_t bytes = plain ? s->N * (4 + s->esz) : 0;
    if (s->dt == DT_BF16) bytes += s->Nmat * 6;
    ProfScope prof(ZPP_PROF_MATERIALIZE, (double)bytes, st);
    if (plain) ZPP_TRY(launch_materialize(s->P, s->ws + s->rW.off, s->N, s->dt, st));
    if (s->dt == DT_BF16) {
        // the transposed copies: matrices of streaming-friendly shape batched into as few launches as the
        // table allows, the others one by one
        TransposeCastTable tab{};
        auto flush = [&]() -> hipError_t {
            const hipError_t e = launch_transpose_cast_many(s->P, s->ws + s->rWt.off, tab, st);
            tab.n = 0;
            return e;
        };
        for (auto &kv : s->wt) {
            const auto &w = kv.second;
            if (w.rows % 128 == 0 && w.cols % 64 == 0 && w.src_off % 4 == 0 && w.dst_off % 8 == 0) {
                tab.src[tab.n] = w.src_off;
                tab.dst[tab.n] = w.dst_off;
                tab.rows[tab.n] = w.rows;
                tab.cols[tab.n] = w.cols;
                if (++tab.n == kTransposeCastMax) ZPP_TRY(flush());
            } else {
                ZPP_TRY(launch_transpose_cast(s->P + w.src_off, s->ws + s->rWt.off + w.dst_off * 2, w.rows, w.cols, st));
            }
        }
        ZPP_TRY(flush());
    }
    if (s->c.arch == ZPP_ARCH_LLAMA && !s->rope_ready) {
        ZPP_TRY(launch_rope_table((float *)(s->ws + s->rRope.off), s->c.seq, s->d, (double)s->c.rope_base, st));
        s->rope_ready = true;
    }
    s->materialized = true;
    // a write-back is good for one gather: later ones cast from P again, so that parameters the caller
    // has rewritten since (zpp_stage_params_changed covers the gather right after an Adam step) are seen
    s->w_fresh = false;
    s->n_materialize++;
    s->materialize_bytes += bytes;
    return ZPP_OK;
}

zpp_status zpp_stage_params_changed(zpp_stage *s)
{
    if (zpp_status e = check_stage(s, true)) return e;
    s->w_fresh = false;
    s->materialized = false;
    return ZPP_OK;
}

namespace {

// Rebuilds what selective recomputation dropped in forward: the outputs of the two norms (from the kept
// block input / attention residual) and of the activation function (from the kept pre-activation), with
// the kernels that produced them in forward on the values forward stored, so the bits are the same.
zpp_status rebuild_elementwise(zpp_stage *s, int32_t mb, int blk, hipStream_t st)
{
    const bool gpt = s->c.arch == ZPP_ARCH_GPT;
    const int kind = gpt ? NORM_LAYER : NORM_RMS;
    const int64_t T = s->Tc, h = s->h, f = s->f;
    ZPP_OTHER(launch_norm_fwd(s->dt, kind, s->stash(mb, blk, "x"), s->Wp(blk, gpt ? "ln1.gamma" : "norm1.gamma"),
                            gpt ? s->Wp(blk, "ln1.beta") : nullptr, T, h, s->c.norm_eps, s->stash(mb, blk, "n1"),
                            (float *)s->stash(mb, blk, "mean1"), (float *)s->stash(mb, blk, "rstd1"), nullptr, st));
    ZPP_OTHER(launch_norm_fwd(s->dt, kind, s->stash(mb, blk, "x1"), s->Wp(blk, gpt ? "ln2.gamma" : "norm2.gamma"),
                            gpt ? s->Wp(blk, "ln2.beta") : nullptr, T, h, s->c.norm_eps, s->stash(mb, blk, "n2"),
                            (float *)s->stash(mb, blk, "mean2"), (float *)s->stash(mb, blk, "rstd2"), nullptr, st));
    if (gpt)
        ZPP_OTHER(launch_gelu_fwd(s->dt, s->stash(mb, blk, "u"), s->stash(mb, blk, "g"), T * f, s->c.gelu_mode, st));
    else
        ZPP_OTHER(launch_swiglu_fwd(s->dt, s->stash(mb, blk, "u"), s->stash(mb, blk, "g"), T, f, st));
    return ZPP_OK;
}

// Forward of one block for the micro-batches [mb, mb + cur_count) as one [Tc, h] matrix (the stash keeps the
// copies of a tensor for consecutive micro-batches back to back): x1 = xin + Attn(Norm1(xin));
// out = x1 + MLP(Norm2(x1)), everything backward needs written to the stash.  keep_x: also copy xin into the
// block's "x" slot (first block, whose input is the caller's).  out == nullptr: the recomputation before the
// block's backward, which needs the stashed tensors but not the block output, so the last linear layer is
// skipped.
zpp_status forward_block(zpp_stage *s, int32_t mb, int blk, const void *xin, bool keep_x, void *out, hipStream_t st)
{
    const bool gpt = s->c.arch == ZPP_ARCH_GPT;
    const int kind = gpt ? NORM_LAYER : NORM_RMS;
    const int64_t T = s->Tc, h = s->h, f = s->f, f1 = s->f1;
    s->rc_first = mb;
    void *xs = s->stash(mb, blk, "x");
    float *mean1 = (float *)s->stash(mb, blk, "mean1"), *rstd1 = (float *)s->stash(mb, blk, "rstd1");
    float *mean2 = (float *)s->stash(mb, blk, "mean2"), *rstd2 = (float *)s->stash(mb, blk, "rstd2");
    void *n1 = s->stash(mb, blk, "n1"), *qkv = s->stash(mb, blk, "qkv"), *attn = s->stash(mb, blk, "attn");
    void *x1 = s->stash(mb, blk, "x1"), *n2 = s->stash(mb, blk, "n2"), *u = s->stash(mb, blk, "u");
    void *g = s->stash(mb, blk, "g");
    float *lse = (float *)s->stash(mb, blk, "lse");

    ZPP_OTHER(launch_norm_fwd(s->dt, kind, xin, s->Wp(blk, gpt ? "ln1.gamma" : "norm1.gamma"),
                            gpt ? s->Wp(blk, "ln1.beta") : nullptr, T, h, s->c.norm_eps, n1, mean1, rstd1,
                            keep_x ? xs : nullptr, st));
    GemmEpi e_qkv;
    if (gpt) e_qkv.bias = s->Wp(blk, "attn.bqkv");
    ZPP_TRY(linear_fwd(s, n1, blk, "attn.wqkv", h, 3 * h, qkv, e_qkv, st));
    if (!gpt)
        ZPP_OTHER(launch_rope(s->dt, qkv, (const float *)(s->ws + s->rRope.off), T, s->c.seq, s->nh, s->d, +1, st));
    ZPP_TRY(attention_fwd(s, qkv, attn, lse, st));
    GemmEpi e_o;
    if (gpt) e_o.bias = s->Wp(blk, "attn.bo");
    e_o.resid = xs;
    ZPP_TRY(linear_fwd(s, attn, blk, "attn.wo", h, h, x1, e_o, st));
    ZPP_OTHER(launch_norm_fwd(s->dt, kind, x1, s->Wp(blk, gpt ? "ln2.gamma" : "norm2.gamma"),
                            gpt ? s->Wp(blk, "ln2.beta") : nullptr, T, h, s->c.norm_eps, n2, mean2, rstd2,
                            nullptr, st));
    GemmEpi e_2;
    e_2.resid = x1;
    if (gpt) {
        GemmEpi e_1;
        e_1.bias = s->Wp(blk, "mlp.b1");
        // bf16: the slot "u" of the stash receives gelu'(u) instead of u, which nothing but the derivative needs -
        // unless selective recomputation is to rebuild the activation's output from u
        e_1.act = s->keeps_preactivation() ? ACT_GELU_DUAL : ACT_GELU_GRAD_DUAL;
        e_1.out2 = g;
        e_1.gelu_mode = s->c.gelu_mode;
        ZPP_TRY(linear_fwd(s, n2, blk, "mlp.w1", h, f, u, e_1, st));
        e_2.bias = s->Wp(blk, "mlp.b2");
        if (out) ZPP_TRY(linear_fwd(s, g, blk, "mlp.w2", f, h, out, e_2, st));
    } else {
        // wgate and wup are adjacent in the layout: one GEMM against the [2f, h] matrix gives [gate | up]
        ZPP_TRY(linear_fwd(s, n2, blk, "mlp.wgate", h, f1, u, GemmEpi(), st));
        ZPP_OTHER(launch_swiglu_fwd(s->dt, u, g, T, f, st));
        if (out) ZPP_TRY(linear_fwd(s, g, blk, "mlp.wdown", f, h, out, e_2, st));
    }
    return ZPP_OK;
}

zpp_status check_group(const zpp_stage *s, int32_t first, int32_t count)
{
    if (count < 1 || first < 0 || first > s->U - count)
        return fail(ZPP_ERR_ARG, "micro-batches [%d, %d) outside [0,%d)", first, first + count, (int)s->U);
    if (count > s->gmax)
        return fail(ZPP_ERR_STATE, "the stage was created for groups of at most %d micro-batches (group_mbs, "
                                   "split_backward)", (int)s->gmax);
    return ZPP_OK;
}

zpp_status forward_group(zpp_stage *s, int32_t first, int32_t count, const void *x, void *y, void *hip_stream)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (zpp_status e = check_group(s, first, count)) return e;
    if (!x || !y) return fail(ZPP_ERR_ARG, "x/y is NULL");
    if (!aligned(x) || !aligned(y)) return fail(ZPP_ERR_ALIGN, "x and y must be 256-byte aligned");
    if (!s->materialized) return fail(ZPP_ERR_STATE, "stage_forward before stage_materialize_params");
    for (int m = first; m < first + count; ++m)
        if (s->mb_state[m] != MB_IDLE) return fail(ZPP_ERR_STATE, "stage_forward(%d) called twice in this unit", m);
    hipStream_t st = (hipStream_t)hip_stream;
    s->begin_call(count);
    for (int blk = 0; blk < s->L; ++blk) {
        const void *xin = blk == 0 ? x : s->stash(first, blk, "x");
        void *out = blk == s->L - 1 ? y : s->stash(first, blk + 1, "x");
        if (zpp_status e = forward_block(s, first, blk, xin, blk == 0, out, st)) return e;
    }
    for (int m = first; m < first + count; ++m) s->mb_state[m] = MB_FWD;
    return ZPP_OK;
}

}  // namespace

zpp_status stage_forward(zpp_stage *s, int32_t mb, const void *x, void *y, void *hip_stream)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (mb < 0 || mb >= s->U) return fail(ZPP_ERR_ARG, "micro_batch %d outside [0,%d)", mb, (int)s->U);
    return forward_group(s, mb, 1, x, y, hip_stream);
}

zpp_status stage_forward_group(zpp_stage *s, int32_t first, int32_t count, const void *x, void *y, void *hip_stream)
{
    return forward_group(s, first, count, x, y, hip_stream);
}

namespace {

// The backward sequence of the micro-batches [first, first + count) as one [count * T, h] matrix, whole or
// one of its two tasks (Section 2.3, Section 3.1.1):
//   BWD_INPUT  the input-gradient task: dX through every layer; with BWD_WEIGHT absent, each linear
//              layer's dY and the partial sums of the norm-gain reductions are parked in the stash;
//   BWD_WEIGHT the weight-gradient task: dW = dY^T . X, bias and gain gradients; with BWD_INPUT absent
//              it reads what the input-gradient tasks of its micro-batches parked.
// With in_place the gradients are added into G (scaled) as they are produced, otherwise they are written
// to the staging buffer.  Both orders of evaluation launch the same kernels on the same operands, so the
// split tasks reproduce the fused call bit for bit.  A weight-gradient task over several micro-batches
// forms their sum inside each product (K = count * T), which is the same value in another summation order.
enum { BWD_INPUT = 1, BWD_WEIGHT = 2 };

zpp_status backward_sequence(zpp_stage *s, int32_t mb, int32_t count, int tasks, const void *dy, void *dx,
                             bool in_place, float scale, void *hip_stream)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (count == 1 && (mb < 0 || mb >= s->U)) return fail(ZPP_ERR_ARG, "micro_batch %d outside [0,%d)", mb, (int)s->U);
    if (zpp_status e = check_group(s, mb, count)) return e;
    const bool do_in = tasks & BWD_INPUT, do_w = tasks & BWD_WEIGHT, split = !(do_in && do_w);
    if (split && !s->c.split_backward)
        return fail(ZPP_ERR_STATE, "the stage was created without split_backward (no stash room for dY)");
    if (do_in) {
        if (!dy || !dx) return fail(ZPP_ERR_ARG, "dy/dx is NULL");
        if (!aligned(dy) || !aligned(dx)) return fail(ZPP_ERR_ALIGN, "dy and dx must be 256-byte aligned");
    }
    if (count > 1 && do_w && !in_place)
        return fail(ZPP_ERR_ARG, "the staging buffer holds one micro-batch: a group adds into G in place");
    if (!s->materialized) return fail(ZPP_ERR_STATE, "working copy is stale: call stage_materialize_params");
    for (int m = mb; m < mb + count; ++m) {
        if (do_in && s->mb_state[m] != MB_FWD)
            return fail(ZPP_ERR_STATE, "backward of micro-batch %d needs exactly one stage_forward(%d) before it", m, m);
        if (!do_in && s->mb_state[m] != MB_BIN)
            return fail(ZPP_ERR_STATE, "the weight-gradient task of micro-batch %d needs exactly one "
                                       "stage_backward_input before it", m);
    }
    if (do_w && !in_place && s->pending_acc >= 0)
        return fail(ZPP_ERR_STATE, "staging buffer still holds micro-batch %d: call stage_accumulate_grads first",
                    s->pending_acc);
    // A lone weight-gradient task finishes the norm-gain reductions its input-gradient tasks started, so it
    // has to cover those tasks whole (their partial sums mix the micro-batches of a task).
    std::vector<size_t> parked_tasks;
    if (!do_in) {
        int covered = 0;
        for (size_t i = 0; i < s->input_tasks.size(); ++i) {
            const auto &t = s->input_tasks[i];
            if (t.first + t.count <= mb || t.first >= mb + count) continue;
            if (t.first < mb || t.first + t.count > mb + count)
                return fail(ZPP_ERR_STATE, "micro-batches [%d, %d) cut through the input-gradient task of [%d, %d)", mb,
                            mb + count, t.first, t.first + t.count);
            parked_tasks.push_back(i);
            covered += t.count;
        }
        if (covered != count) return fail(ZPP_ERR_STATE, "no input-gradient task on record for micro-batches [%d, %d)", mb, mb + count);
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const bool gpt = s->c.arch == ZPP_ARCH_GPT;
    const int kind = gpt ? NORM_LAYER : NORM_RMS;
    s->begin_call(count);
    const int64_t T = s->Tc, h = s->h, f = s->f, f1 = s->f1;
    void *gbuf[2] = {s->tp("gA"), s->tp("gB")};
    void *dn = s->tp("dn"), *dattn = s->tp("dattn");
    s->finish.clear();
    s->acc_in_place = in_place;
    s->acc_scale = scale;
    s->acc_write = false;
    if (do_w && in_place && s->g_released) {
        // first addition into a released G: write instead of add; a scale other than 1 takes the plain way
        // (zero G, then add)
        if (scale == 1.0f)
            s->acc_write = true;
        else
            ZPP_OTHER(launch_fill_zero(s->G, s->N, st));
        s->g_released = false;
    }
    s->dw_batch.clear();  // (left over only if an earlier call failed half-way)
    s->dw_batch_flops = s->dw_batch_bytes = 0.0;
    zpp_stage::InputTask *rec = nullptr;
    if (do_in && split) {
        s->input_tasks.push_back({mb, count, {}});
        rec = &s->input_tasks.back();
        // the weight-gradient task of the top block needs the caller's dy after this call has returned
        ZPP_OTHER(hipMemcpyAsync(s->stash(mb, (int)s->L - 1, "d_y"), dy, (size_t)(T * h) * s->esz,
                                 hipMemcpyDeviceToDevice, st));
    }
    // the norm-gain reductions of further parked input-gradient tasks, each finished by a launch of its own
    // (they add into the same elements of G)
    std::vector<std::vector<FinishItem>> more_finish(parked_tasks.size() > 1 ? parked_tasks.size() - 1 : 0);
    const void *dcur = dy;
    for (int blk = (int)s->L - 1; blk >= 0; --blk) {
        // gradient buffers: temporaries in the fused call, stash slots when the tasks are split
        void *dout = blk == 0 ? dx : (split ? s->stash(mb, blk - 1, "d_y") : gbuf[blk & 1]);
        void *dx1 = split ? s->stash(mb, blk, "d_x1") : s->tp("dx1");
        void *dqkv = split ? s->stash(mb, blk, "d_qkv") : s->tp("dqkv");
        void *du = split ? s->stash(mb, blk, "d_u") : s->tp("du");
        if (split) dcur = s->stash(mb, blk, "d_y");
        // activation recomputation (Section 3.3): full - only the block input was kept, run the block forward
        // again; selective - rebuild the norm and activation outputs
        if (s->c.recompute == ZPP_RECOMPUTE_FULL) {
            if (zpp_status e = forward_block(s, mb, blk, s->stash(mb, blk, "x"), false, nullptr, st)) return e;
        } else if (s->c.recompute == ZPP_RECOMPUTE_SELECTIVE) {
            s->rc_first = mb;
            if (zpp_status e = rebuild_elementwise(s, mb, blk, st)) return e;
        }
        const void *xs = s->stash(mb, blk, "x"), *n1 = s->stash(mb, blk, "n1"), *qkv = s->stash(mb, blk, "qkv");
        const void *attn = s->stash(mb, blk, "attn"), *x1 = s->stash(mb, blk, "x1"), *n2 = s->stash(mb, blk, "n2");
        const void *u = s->stash(mb, blk, "u"), *g = s->stash(mb, blk, "g");
        const float *mean1 = (const float *)s->stash(mb, blk, "mean1"), *rstd1 = (const float *)s->stash(mb, blk, "rstd1");
        const float *mean2 = (const float *)s->stash(mb, blk, "mean2"), *rstd2 = (const float *)s->stash(mb, blk, "rstd2");
        const float *lse = (const float *)s->stash(mb, blk, "lse");
        const char *g2 = gpt ? "ln2.gamma" : "norm2.gamma", *g1 = gpt ? "ln1.gamma" : "norm1.gamma";
        // Norm backward: dx together with the first level of the gain-gradient reduction.  The fused call
        // finishes the reduction at its end; a lone input-gradient task parks the partial sums instead.
        auto norm_bwd = [&](const char *gname, const char *bname, const char *red, const void *x, const float *mean,
                            const float *rstd, const void *resid, void *out) -> zpp_status {
            float *slot = split ? (float *)s->stash(mb, blk, red) : s->red_slot();
            FinishItem *item = s->defer();
            ZPP_OTHER(launch_norm_bwd_colreduce(s->dt, kind, dn, x, mean, rstd, s->Wp(blk, gname), resid, out, T, h,
                                                s->Sp(blk, gname), gpt ? s->Sp(blk, bname) : nullptr, slot, item, st));
            if (split) {
                rec->items.push_back(*item);
                s->finish.pop_back();
            }
            return ZPP_OK;
        };
        // the parked items of this block, with their destinations set for this call (staging buffer or G)
        auto parked = [&](int which, const char *gname, const char *bname) {
            for (size_t i = 0; i < parked_tasks.size(); ++i) {
                FinishItem it = s->input_tasks[parked_tasks[i]].items[(size_t)((int)s->L - 1 - blk) * 2 + which];
                it.out0 = s->Sp(blk, gname);
                it.out1 = gpt ? s->Sp(blk, bname) : nullptr;
                if (i == 0)
                    *s->defer() = it;
                else
                    more_finish[i - 1].push_back(it);
            }
        };
        // ---- MLP branch
        if (gpt) {
            if (do_w) ZPP_TRY(linear_dw(s, dcur, g, blk, "mlp.w2", "mlp.b2", f, h, st));
            if (do_in) {
                GemmEpi e;
                e.act = s->keeps_preactivation() ? ACT_DGELU_MUL : ACT_MUL_AUX;
                e.aux = u;
                e.gelu_mode = s->c.gelu_mode;
                ZPP_TRY(linear_dx(s, dcur, blk, "mlp.w2", f, h, du, e, st));
            }
            if (do_w) ZPP_TRY(linear_dw(s, du, n2, blk, "mlp.w1", "mlp.b1", h, f, st));
            if (do_in) ZPP_TRY(linear_dx(s, du, blk, "mlp.w1", h, f, dn, GemmEpi(), st));
        } else {
            if (do_w) ZPP_TRY(linear_dw(s, dcur, g, blk, "mlp.wdown", nullptr, f, h, st));
            if (do_in) {
                void *dact = s->tp("dact");
                ZPP_TRY(linear_dx(s, dcur, blk, "mlp.wdown", f, h, dact, GemmEpi(), st));
                ZPP_OTHER(launch_swiglu_bwd(s->dt, u, dact, du, T, f, st));
            }
            if (do_w) ZPP_TRY(linear_dw(s, du, n2, blk, "mlp.wgate", nullptr, h, f1, st));
            if (do_in) ZPP_TRY(linear_dx(s, du, blk, "mlp.wgate", h, f1, dn, GemmEpi(), st));
        }
        if (do_in) {
            if (zpp_status e = norm_bwd(g2, "ln2.beta", "red_n2", x1, mean2, rstd2, dcur, dx1)) return e;
        } else {
            parked(0, g2, "ln2.beta");
        }
        // ---- attention branch
        if (do_w) ZPP_TRY(linear_dw(s, dx1, attn, blk, "attn.wo", gpt ? "attn.bo" : nullptr, h, h, st));
        if (do_in) {
            ZPP_TRY(linear_dx(s, dx1, blk, "attn.wo", h, h, dattn, GemmEpi(), st));
            ZPP_TRY(attention_bwd(s, qkv, attn, dattn, lse, dqkv, st));
            if (!gpt)
                ZPP_OTHER(launch_rope(s->dt, dqkv, (const float *)(s->ws + s->rRope.off), T, s->c.seq, s->nh, s->d, -1, st));
        }
        if (do_w) ZPP_TRY(linear_dw(s, dqkv, n1, blk, "attn.wqkv", gpt ? "attn.bqkv" : nullptr, h, 3 * h, st));
        if (do_in) {
            ZPP_TRY(linear_dx(s, dqkv, blk, "attn.wqkv", h, 3 * h, dn, GemmEpi(), st));
            if (zpp_status e = norm_bwd(g1, "ln1.beta", "red_n1", xs, mean1, rstd1, dx1, dout)) return e;
        } else {
            parked(1, g1, "ln1.beta");
        }
        if (do_w) ZPP_TRY(flush_dw_batch(s, st));
        dcur = dout;
    }
    // second level of every column reduction of this call, in one launch
    if (do_w) {
        ZPP_OTHER(launch_finish_columns(s->finish.data(), (int)s->finish.size(), st, in_place && !s->acc_write, scale));
        for (auto &items : more_finish)
            ZPP_OTHER(launch_finish_columns(items.data(), (int)items.size(), st, in_place, scale));
    }
    s->finish.clear();
    s->acc_in_place = false;
    s->acc_write = false;
    if (!do_in)  // the parked records are used up (erase from the back so the indices stay valid)
        for (size_t i = parked_tasks.size(); i-- > 0;) s->input_tasks.erase(s->input_tasks.begin() + (long)parked_tasks[i]);
    for (int m = mb; m < mb + count; ++m) {
        if (do_w)
            s->mb_state[m] = in_place ? MB_ACC : MB_BWD;
        else
            s->mb_state[m] = MB_BIN;
    }
    if (do_w && !in_place) s->pending_acc = mb;  // in place leaves the staging buffer (and who holds it) alone
    return ZPP_OK;
}

}  // namespace

zpp_status stage_backward(zpp_stage *s, int32_t mb, const void *dy, void *dx, void *hip_stream)
{
    return backward_sequence(s, mb, 1, BWD_INPUT | BWD_WEIGHT, dy, dx, false, 1.0f, hip_stream);
}

zpp_status stage_backward_accumulate(zpp_stage *s, int32_t mb, const void *dy, void *dx, float scale,
                                     void *hip_stream)
{
    return backward_sequence(s, mb, 1, BWD_INPUT | BWD_WEIGHT, dy, dx, true, scale, hip_stream);
}

zpp_status stage_backward_accumulate_group(zpp_stage *s, int32_t first, int32_t count, const void *dy, void *dx,
                                           float scale, void *hip_stream)
{
    return backward_sequence(s, first, count, BWD_INPUT | BWD_WEIGHT, dy, dx, true, scale, hip_stream);
}

zpp_status stage_backward_input(zpp_stage *s, int32_t mb, const void *dy, void *dx, void *hip_stream)
{
    return backward_sequence(s, mb, 1, BWD_INPUT, dy, dx, false, 1.0f, hip_stream);
}

zpp_status stage_backward_input_group(zpp_stage *s, int32_t first, int32_t count, const void *dy, void *dx,
                                      void *hip_stream)
{
    return backward_sequence(s, first, count, BWD_INPUT, dy, dx, false, 1.0f, hip_stream);
}

zpp_status stage_backward_weight(zpp_stage *s, int32_t mb, int32_t in_place, float scale, void *hip_stream)
{
    return backward_sequence(s, mb, 1, BWD_WEIGHT, nullptr, nullptr, in_place != 0, scale, hip_stream);
}

zpp_status stage_backward_weight_group(zpp_stage *s, int32_t first, int32_t count, float scale, void *hip_stream)
{
    return backward_sequence(s, first, count, BWD_WEIGHT, nullptr, nullptr, true, scale, hip_stream);
}

zpp_status stage_accumulate_grads(zpp_stage *s, int32_t mb, float scale, void *hip_stream)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (mb < 0 || mb >= s->U) return fail(ZPP_ERR_ARG, "micro_batch %d outside [0,%d)", mb, (int)s->U);
    if (s->mb_state[mb] != MB_BWD || s->pending_acc != mb)
        return fail(ZPP_ERR_STATE, "stage_accumulate_grads(%d) needs stage_backward(%d) right before it", mb, mb);
    {
        ProfScope prof(ZPP_PROF_ACCUMULATE, (s->g_released ? 8.0 : 12.0) * s->N, (hipStream_t)hip_stream);
        ZPP_TRY(launch_accumulate(s->G, (const float *)(s->ws + s->rS.off), s->N, scale, (hipStream_t)hip_stream,
                                  s->g_released));
        s->g_released = false;
    }
    s->mb_state[mb] = MB_ACC;
    s->pending_acc = -1;
    return ZPP_OK;
}

namespace {

// Host-side checks shared by the Adam entry points, and the kernel's argument block (lr and weight decay
// from hp; the ranged entry point overrides them per range).
zpp_status adam_args(zpp_stage *s, const zpp_adam *hp, AdamArgs *a)
{
    if (!hp) return fail(ZPP_ERR_ARG, "hyper-parameters are NULL");
    if (hp->step < 1) return fail(ZPP_ERR_ARG, "step must be >= 1");
    if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f && hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
        return fail(ZPP_ERR_ARG, "betas must lie in [0,1)");
    if (s->pending_acc >= 0)
        return fail(ZPP_ERR_STATE, "micro-batch %d is backward-done but not accumulated", s->pending_acc);
    for (int64_t m = 0; m < s->U; ++m) {
        if (s->mb_state[m] == MB_BIN)
            return fail(ZPP_ERR_STATE, "micro-batch %d has its input gradient but not its weight gradient", (int)m);
        // a stash computed with the old parameters must not meet a backward that runs with the new ones
        if (s->mb_state[m] == MB_FWD)
            return fail(ZPP_ERR_STATE, "micro-batch %d is forward-done but has no backward yet", (int)m);
    }
    a->lr = hp->lr;
    a->beta1 = hp->beta1;
    a->beta2 = hp->beta2;
    a->eps = hp->eps;
    a->wd = hp->weight_decay;
    a->grad_scale = hp->grad_scale;
    a->omb1 = (float)(1.0 - (double)hp->beta1);
    a->omb2 = (float)(1.0 - (double)hp->beta2);
    a->c1 = (float)(1.0 - std::pow((double)hp->beta1, (double)hp->step));
    a->c2 = (float)(1.0 - std::pow((double)hp->beta2, (double)hp->step));
    a->decoupled = hp->decoupled_wd ? 1 : 0;
    if (hp->zero_grad < 0 || hp->zero_grad > 2) return fail(ZPP_ERR_ARG, "zero_grad must be 0, 1 or 2");
    a->zero_grad = hp->zero_grad == 1 ? 1 : 0;
    a->wb = nullptr;
    a->wb_bf16 = s->dt == DT_BF16;
    if (hp->write_back) {
        if (s->shared_wcopy)
            return fail(ZPP_ERR_STATE, "write_back needs a working copy of the stage's own (stages of a zpp_device "
                                       "share theirs)");
        a->wb = s->ws + s->rW.off;
    }
    return ZPP_OK;
}

}  // namespace

zpp_status shard_adam_step(zpp_stage *s, uint64_t offset, uint64_t count, const zpp_adam *hp, void *hip_stream)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (!hp) return fail(ZPP_ERR_ARG, "hyper-parameters are NULL");
    if (offset > s->N || count > s->N - offset)
        return fail(ZPP_ERR_ARG, "range [%llu, +%llu) outside the shard of %llu elements", (unsigned long long)offset,
                    (unsigned long long)count, (unsigned long long)s->N);
    if (offset % 4 || (count % 4 && offset + count != s->N))
        return fail(ZPP_ERR_ALIGN, "offset and count must be multiples of 4 elements");
    if (hp->zero_grad == 2 && (offset != 0 || count != s->N))
        return fail(ZPP_ERR_ARG, "zero_grad = 2 releases the whole of G: it needs the step over the whole shard");
    AdamArgs a;
    if (zpp_status e = adam_args(s, hp, &a)) return e;
    if (a.wb) a.wb = (unsigned char *)a.wb + offset * s->esz;  // the kernel indexes from `offset`
    {
        ProfScope prof(ZPP_PROF_ADAM, ((a.zero_grad ? 32.0 : 28.0) + (a.wb ? (double)s->esz : 0.0)) * count,
                       (hipStream_t)hip_stream);
        ZPP_TRY(launch_adam(s->P + offset, s->M + offset, s->V + offset, s->G + offset, count, a,
                            (hipStream_t)hip_stream));
    }
    if (count) {
        s->materialized = false;
        // the plain working copy is current only if this call rewrote all of it (or kept up an already
        // current copy); a step without write-back leaves it behind P
        s->w_fresh = a.wb && (s->w_fresh || (offset == 0 && count == s->N));
    }
    if (hp->zero_grad == 2) s->g_released = true;
    return ZPP_OK;
}

zpp_status shard_adam_step_ranges(zpp_stage *s, const zpp_adam_range *ranges, int32_t n_ranges, const zpp_adam *hp,
                                  void *hip_stream)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (n_ranges < 0 || (n_ranges > 0 && !ranges)) return fail(ZPP_ERR_ARG, "ranges is NULL or n_ranges negative");
    uint64_t end = 0, total = 0;
    for (int32_t i = 0; i < n_ranges; ++i) {
        const zpp_adam_range &r = ranges[i];
        if (r.offset > s->N || r.count > s->N - r.offset)
            return fail(ZPP_ERR_ARG, "range %d [%llu, +%llu) outside the shard of %llu elements", i,
                        (unsigned long long)r.offset, (unsigned long long)r.count, (unsigned long long)s->N);
        if (r.offset < end) return fail(ZPP_ERR_ARG, "range %d overlaps its predecessor or is out of order", i);
        if (r.offset % 4 || r.count % 4) return fail(ZPP_ERR_ALIGN, "range %d: offset and count must be multiples of 4", i);
        end = r.offset + r.count;
        total += r.count;
    }
    if (hp && hp->zero_grad == 2 && total != s->N)
        return fail(ZPP_ERR_ARG, "zero_grad = 2 releases the whole of G: the ranges must cover the whole shard");
    AdamArgs a;
    if (zpp_status e = adam_args(s, hp, &a)) return e;
    ProfScope prof(ZPP_PROF_ADAM, ((a.zero_grad ? 32.0 : 28.0) + (a.wb ? (double)s->esz : 0.0)) * total,
                   (hipStream_t)hip_stream);
    for (int32_t base = 0; base < n_ranges; base += kAdamRanges) {
        AdamRanges tab{};
        tab.n = std::min<int32_t>(kAdamRanges, n_ranges - base);
        for (int32_t i = 0; i < tab.n; ++i) {
            tab.offset[i] = ranges[base + i].offset;
            tab.count[i] = ranges[base + i].count;
            tab.lr[i] = ranges[base + i].lr;
            tab.wd[i] = ranges[base + i].weight_decay;
        }
        ZPP_TRY(launch_adam_ranges(s->P, s->M, s->V, s->G, tab, a, (hipStream_t)hip_stream));
    }
    if (total) {
        s->materialized = false;
        s->w_fresh = a.wb && (s->w_fresh || total == s->N);  // disjoint ranges of N elements cover the shard
    }
    if (hp->zero_grad == 2) s->g_released = true;
    return ZPP_OK;
}

int32_t zpp_stage_decay_ranges(const zpp_stage *s, float lr, float weight_decay, zpp_adam_range *out, int32_t capacity)
{
    if (!s) return 0;
    int32_t n = 0;
    float last_wd = 0.0f;
    uint64_t last_end = 0;
    for (const Tensor &t : s->layout) {
        const float wd = t.rows > 1 ? weight_decay : 0.0f;  // matrices decay; gains, offsets and biases do not
        const uint64_t cnt = t.rows * t.cols;
        if (n > 0 && last_wd == wd && last_end == t.offset) {
            if (out && n <= capacity) out[n - 1].count += cnt;
        } else {
            if (out && n < capacity) out[n] = zpp_adam_range{t.offset, cnt, lr, wd};
            ++n;
        }
        last_wd = wd;
        last_end = t.offset + cnt;
    }
    return n;
}

zpp_status zpp_stage_end_unit(zpp_stage *s)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (s->pending_acc >= 0)
        return fail(ZPP_ERR_STATE, "micro-batch %d is backward-done but not accumulated", s->pending_acc);
    for (int64_t m = 0; m < s->U; ++m)
        if (s->mb_state[m] == MB_BIN)
            return fail(ZPP_ERR_STATE, "micro-batch %d has its input gradient but not its weight gradient", (int)m);
    s->mb_state.assign(s->U, MB_IDLE);
    s->input_tasks.clear();
    return ZPP_OK;
}

void zpp_stage_counters(const zpp_stage *s, uint64_t *calls, uint64_t *bytes)
{
    if (calls) *calls = s ? s->n_materialize : 0;
    if (bytes) *bytes = s ? s->materialize_bytes : 0;
}

zpp_status zpp_stage_region(const zpp_stage *s, const char *name, int32_t mb, int32_t blk, void **ptr,
                            uint64_t *elems, int32_t *elem_bytes)
{
    if (zpp_status e = check_stage(s, true)) return e;
    if (!name || !ptr) return fail(ZPP_ERR_ARG, "name/ptr is NULL");
    Region r;
    uint64_t base = 0;
    std::string n(name);
    if (n == "W") r = s->rW;
    else if (n == "S") r = s->rS;
    else if (n == "Wt" && s->dt == DT_BF16) r = s->rWt;
    else if (s->stash_t.count(n) || s->rc_t.count(n)) {
        if (mb < 0 || mb >= s->U || blk < 0 || blk >= s->L) return fail(ZPP_ERR_ARG, "(mb, block) out of range");
        const bool kept = s->stash_t.count(n) != 0;
        if (!kept && (mb < s->rc_first || mb >= s->rc_first + s->gmax))
            return fail(ZPP_ERR_STATE, "'%s' is rebuilt in backward and not held for micro-batch %d now", name, mb);
        r = kept ? s->stash_t.at(n) : s->rc_t.at(n);
        base = s->stash_off(mb, blk, n);
        r.off = 0;
    } else if (s->tmp.count(n)) r = s->tmp.at(n);
    else return fail(ZPP_ERR_ARG, "unknown region '%s'", name);
    *ptr = s->ws + base + r.off;
    if (elems) *elems = r.elems;
    if (elem_bytes) *elem_bytes = r.esz;
    return ZPP_OK;
}

zpp_status zpp_profile_enable(int32_t on)
{
    g_prof_on.store(on != 0);
    return ZPP_OK;
}

void zpp_profile_reset(void)
{
    std::lock_guard<std::mutex> lock(g_prof_mu);
    for (auto &r : g_prof) {
        g_event_pool.push_back(r.e0);
        g_event_pool.push_back(r.e1);
    }
    g_prof.clear();
}

zpp_status zpp_profile_read(int32_t cls, uint64_t *launches, double *total_ms, double *work, double *bytes)
{
    if (cls < 0 || cls >= ZPP_PROF_CLASSES) return fail(ZPP_ERR_ARG, "profile class %d out of range", cls);
    uint64_t n = 0;
    double ms = 0.0, w = 0.0, b = 0.0;
    std::lock_guard<std::mutex> lock(g_prof_mu);
    for (auto &r : g_prof) {
        if (r.cls != cls) continue;
        if (hipEventSynchronize(r.e1) != hipSuccess) return fail(ZPP_ERR_DEVICE, "event synchronize failed");
        float t = 0.0f;
        if (hipEventElapsedTime(&t, r.e0, r.e1) != hipSuccess) return fail(ZPP_ERR_DEVICE, "event elapsed failed");
        ms += t;
        w += r.work;
        b += r.bytes;
        ++n;
    }
    if (launches) *launches = n;
    if (total_ms) *total_ms = ms;
    if (work) *work = w;
    if (bytes) *bytes = b;
    return ZPP_OK;
}

// ---- operator-level entry points (include/zpp_ops.h) ---------------------------------------------
#define ZPP_OP_TRY(expr)                                                                     \
    do {                                                                                     \
        hipError_t _e = (expr);                                                              \
        if (_e != hipSuccess) return fail(ZPP_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(_e)); \
    } while (0)

zpp_status zpp_op_gemm_bf16_nt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, const void *bias, const void *resid,
                               int32_t out_f32, int32_t tile, void *hip_stream)
{
    if (!A || !B || !C) return fail(ZPP_ERR_ARG, "A/B/C is NULL");
    if (M < 0 || N < 0 || K <= 0) return fail(ZPP_ERR_ARG, "bad sizes");
    if (K % 64 || lda % 8 || ldb % 8 || lda < K || ldb < K || ldc < N)
        return fail(ZPP_ERR_UNSUPPORTED, "need K %% 64 == 0, lda/ldb multiples of 8 and >= K, ldc >= N");
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) % 16) return fail(ZPP_ERR_ALIGN, "16-byte alignment required");
    if (tile < GEMM_TILE_AUTO || tile > GEMM_TILE_LAST) return fail(ZPP_ERR_ARG, "tile must be -1..%d", GEMM_TILE_LAST);
    GemmEpi e;
    e.bias = bias;
    e.resid = resid;
    e.out_f32 = out_f32 == 2 ? 2 : (out_f32 != 0);
    hipError_t err = launch_gemm_bf16_nt(M, N, K, A, lda, B, ldb, C, ldc, e, (hipStream_t)hip_stream, tile);
    if (err != hipSuccess) return fail(ZPP_ERR_DEVICE, "gemm launch: %s", hipGetErrorString(err));
    return ZPP_OK;
}

zpp_status zpp_op_gemm_bf16_tt(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, int32_t out_f32, void *hip_stream)
{
    if (!A || !B || !C) return fail(ZPP_ERR_ARG, "A/B/C is NULL");
    if (M <= 0 || N <= 0 || K <= 0 || lda < M || ldb < N || ldc < N) return fail(ZPP_ERR_ARG, "bad sizes");
    if (!gemm_bf16_tt_supported(M, N, K, lda, ldb))
        return fail(ZPP_ERR_UNSUPPORTED, "need M, N multiples of 256, K a multiple of 64, lda/ldb multiples of 8");
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) % 16) return fail(ZPP_ERR_ALIGN, "16-byte alignment required");
    GemmEpi e;
    e.out_f32 = out_f32 == 2 ? 2 : (out_f32 != 0);
    hipError_t err = launch_gemm_bf16_tt(M, N, K, A, lda, B, ldb, C, ldc, e, (hipStream_t)hip_stream);
    if (err != hipSuccess) return fail(ZPP_ERR_DEVICE, "gemm launch: %s", hipGetErrorString(err));
    return ZPP_OK;
}

zpp_status zpp_op_gemm_bf16_tt_group(int32_t n, const int64_t *M, const int64_t *N, int64_t K, const void *const *A,
                                     const int64_t *lda, const void *const *B, const int64_t *ldb, void *const *C,
                                     const int64_t *ldc, int32_t out_f32, void *hip_stream)
{
    if (n < 1 || n > kGemmGroupMax) return fail(ZPP_ERR_ARG, "a group holds 1..%d products", kGemmGroupMax);
    if (!M || !N || !A || !lda || !B || !ldb || !C || !ldc) return fail(ZPP_ERR_ARG, "an argument array is NULL");
    GemmProblem q[kGemmGroupMax];
    for (int i = 0; i < n; ++i) {
        if (!A[i] || !B[i] || !C[i]) return fail(ZPP_ERR_ARG, "A/B/C of product %d is NULL", i);
        if (M[i] <= 0 || N[i] <= 0 || K <= 0 || lda[i] < M[i] || ldb[i] < N[i] || ldc[i] < N[i])
            return fail(ZPP_ERR_ARG, "bad sizes in product %d", i);
        if (!gemm_bf16_tt_supported(M[i], N[i], K, lda[i], ldb[i]))
            return fail(ZPP_ERR_UNSUPPORTED, "product %d: need M, N multiples of 256, K a multiple of 64, lda/ldb "
                                             "multiples of 8", i);
        if (((uintptr_t)A[i] | (uintptr_t)B[i] | (uintptr_t)C[i]) % 16)
            return fail(ZPP_ERR_ALIGN, "16-byte alignment required (product %d)", i);
        q[i] = {M[i], N[i], A[i], lda[i], B[i], ldb[i], C[i], ldc[i]};
    }
    GemmEpi e;
    e.out_f32 = out_f32 == 2 ? 2 : (out_f32 != 0);
    hipError_t err = launch_gemm_bf16_tt_group(q, n, K, e, (hipStream_t)hip_stream);
    if (err != hipSuccess) return fail(ZPP_ERR_DEVICE, "gemm launch: %s", hipGetErrorString(err));
    return ZPP_OK;
}

zpp_status zpp_op_gemm_bf16_nn(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                               int64_t ldb, void *C, int64_t ldc, int32_t out_f32, void *hip_stream)
{
    if (!A || !B || !C) return fail(ZPP_ERR_ARG, "A/B/C is NULL");
    if (M <= 0 || N <= 0 || K <= 0 || lda < K || ldb < N || ldc < N) return fail(ZPP_ERR_ARG, "bad sizes");
    if (!gemm_bf16_nn_supported(M, N, K, lda, ldb))
        return fail(ZPP_ERR_UNSUPPORTED, "need N a multiple of 256, K a multiple of 64, lda/ldb multiples of 8");
    if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) % 16) return fail(ZPP_ERR_ALIGN, "16-byte alignment required");
    GemmEpi e;
    e.out_f32 = out_f32 == 2 ? 2 : (out_f32 != 0);
    hipError_t err = launch_gemm_bf16_nn(M, N, K, A, lda, B, ldb, C, ldc, e, (hipStream_t)hip_stream);
    if (err != hipSuccess) return fail(ZPP_ERR_DEVICE, "gemm launch: %s", hipGetErrorString(err));
    return ZPP_OK;
}

zpp_status zpp_op_attention_fwd(int32_t dtype, int32_t impl, const void *qkv, void *attn, float *lse, int64_t b,
                                int64_t seq, int64_t nh, int64_t d, void *hip_stream)
{
    if (!qkv || !attn || !lse) return fail(ZPP_ERR_ARG, "NULL pointer");
    if (b <= 0 || seq <= 0 || nh <= 0 || d <= 0 || b > 65535 || nh > 65535) return fail(ZPP_ERR_ARG, "bad sizes");
    hipStream_t st = (hipStream_t)hip_stream;
    if (impl == 1) {
        if (dtype != ZPP_DTYPE_BF16 || !attn_mfma_supported(seq, d))
            return fail(ZPP_ERR_UNSUPPORTED, "MFMA attention needs bf16, d = 128 and seq %% 128 == 0");
        ZPP_OP_TRY(launch_attn_fwd(DT_BF16, qkv, attn, lse, b, seq, nh, d, st));
    } else {
        if ((d + seq) * 4 > 64 * 1024) return fail(ZPP_ERR_UNSUPPORTED, "sequence too long");
        ZPP_OP_TRY(launch_attn_simple_fwd(dtype == ZPP_DTYPE_BF16 ? DT_BF16 : DT_F32, qkv, attn, lse, b, seq, nh, d, st));
    }
    return ZPP_OK;
}

zpp_status zpp_op_attention_bwd(int32_t dtype, int32_t impl, const void *qkv, const void *attn, const void *dattn,
                                const float *lse, float *delta, void *dqkv, int64_t b, int64_t seq, int64_t nh,
                                int64_t d, void *hip_stream)
{
    if (!qkv || !attn || !dattn || !lse || !delta || !dqkv) return fail(ZPP_ERR_ARG, "NULL pointer");
    if (b <= 0 || seq <= 0 || nh <= 0 || d <= 0 || b > 65535 || nh > 65535) return fail(ZPP_ERR_ARG, "bad sizes");
    hipStream_t st = (hipStream_t)hip_stream;
    if (impl == 1) {
        if (dtype != ZPP_DTYPE_BF16 || !attn_mfma_supported(seq, d))
            return fail(ZPP_ERR_UNSUPPORTED, "MFMA attention needs bf16, d = 128 and seq %% 128 == 0");
        ZPP_OP_TRY(launch_attn_bwd(DT_BF16, qkv, attn, dattn, lse, delta, dqkv, b, seq, nh, d, st));
    } else {
        if ((2 * d + 2 * seq) * 4 > 64 * 1024) return fail(ZPP_ERR_UNSUPPORTED, "sequence too long");
        ZPP_OP_TRY(launch_attn_simple_bwd(dtype == ZPP_DTYPE_BF16 ? DT_BF16 : DT_F32, qkv, attn, dattn, lse, delta,
                                          dqkv, b, seq, nh, d, st));
    }
    return ZPP_OK;
}

zpp_status zpp_op_flat_adam(float *P, float *M, float *V, float *G, uint64_t n, const zpp_adam *hp, void *hip_stream)
{
    if (!P || !M || !V || !G || !hp) return fail(ZPP_ERR_ARG, "NULL pointer");
    if (((uintptr_t)P | (uintptr_t)M | (uintptr_t)V | (uintptr_t)G) % 16) return fail(ZPP_ERR_ALIGN, "16-byte alignment");
    if (hp->step < 1) return fail(ZPP_ERR_ARG, "step must be >= 1");
    if (hp->zero_grad != 0 && hp->zero_grad != 1) return fail(ZPP_ERR_ARG, "zero_grad must be 0 or 1 here (no stage to hold a released G)");
    AdamArgs a;
    a.lr = hp->lr; a.beta1 = hp->beta1; a.beta2 = hp->beta2; a.eps = hp->eps; a.wd = hp->weight_decay;
    a.grad_scale = hp->grad_scale;
    a.omb1 = (float)(1.0 - (double)hp->beta1);
    a.omb2 = (float)(1.0 - (double)hp->beta2);
    a.c1 = (float)(1.0 - std::pow((double)hp->beta1, (double)hp->step));
    a.c2 = (float)(1.0 - std::pow((double)hp->beta2, (double)hp->step));
    a.decoupled = hp->decoupled_wd ? 1 : 0;
    a.zero_grad = hp->zero_grad ? 1 : 0;
    ZPP_OP_TRY(launch_adam(P, M, V, G, n, a, (hipStream_t)hip_stream));
    return ZPP_OK;
}

zpp_status zpp_op_flat_accumulate(float *G, const float *S, uint64_t n, float scale, void *hip_stream)
{
    if (!G || !S) return fail(ZPP_ERR_ARG, "NULL pointer");
    if (((uintptr_t)G | (uintptr_t)S) % 16) return fail(ZPP_ERR_ALIGN, "16-byte alignment");
    ZPP_OP_TRY(launch_accumulate(G, S, n, scale, (hipStream_t)hip_stream));
    return ZPP_OK;
}

zpp_status zpp_op_flat_materialize(const float *P, void *W, uint64_t n, int32_t dtype, void *hip_stream)
{
    if (!P || !W) return fail(ZPP_ERR_ARG, "NULL pointer");
    if (((uintptr_t)P | (uintptr_t)W) % 16) return fail(ZPP_ERR_ALIGN, "16-byte alignment");
    ZPP_OP_TRY(launch_materialize(P, W, n, dtype == ZPP_DTYPE_BF16 ? DT_BF16 : DT_F32, (hipStream_t)hip_stream));
    return ZPP_OK;
}

}  // extern "C"
