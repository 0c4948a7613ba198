// C-ABI of libzo (see include/zo.h): argument checks, workspace layout, and the host-side
// schedule of one ZO-SGD step -- DistZO2 App. A, Alg. 1 (literal order), Alg. 2 (per-module
// dual forward with the deferred update) and Alg. 3 (upload / compute / offload overlap).
#include "../../include/zo.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "zo_kernels.h"
#include "zo_types.hip.h"

using namespace zo;

// ------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
#define ZO_HIP(expr)                                                                                   \
    do {                                                                                               \
        hipError_t e__ = (expr);                                                                       \
        if (e__ != hipSuccess) return fail(ZO_EHIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
    } while (0)
#define ZO_TRY(expr)                 \
    do {                             \
        int r__ = (expr);            \
        if (r__ != ZO_OK) return r__; \
    } while (0)

extern "C" const char *zo_last_error(void) { return g_err; }

// ------------------------------------------------------------------ model
namespace {

constexpr int kPerBlock = 16;
enum { K_LINEAR = ZO_K_LINEAR, K_ATTN = ZO_K_ATTENTION, K_STAGE = ZO_K_STAGE, K_UPDATE = ZO_K_UPDATE, K_NORM = ZO_K_NORM, K_CE = ZO_K_CE, K_OTHER = ZO_K_OTHER };
enum { T_LN1G, T_LN1B, T_WQ, T_BQ, T_WK, T_BK, T_WV, T_BV, T_WO, T_BO, T_LN2G, T_LN2B, T_W1, T_B1, T_W2, T_B2 };
enum SlotState { SLOT_EMPTY, SLOT_UPLOADED, SLOT_COMPUTED };

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Element offsets of the 16 tensors inside a block as stored (canonical order), and of the
// staged (q|k|v fused, weights next to each other) copies the forward reads.  A linear weight is stored
// [out, in], which is the K-contiguous layout the GEMMs take, so staging moves no element out of its row.
struct BlockLayout {
    size_t src_off[kPerBlock];   // in elements, canonical storage order
    uint32_t rows[kPerBlock], cols[kPerBlock];
    size_t total;                // elements per block
    // staged layout (elements): ln1_g, ln1_b, wqkv[3d,d], bqkv[3d], wo[d,d], bo, ln2_g, ln2_b, w1[F,d], b1, w2[d,F], b2
    size_t st_ln1g, st_ln1b, st_wqkv, st_bqkv, st_wo, st_bo, st_ln2g, st_ln2b, st_w1, st_b1, st_w2, st_b2;
};

BlockLayout make_layout(int d, int f)
{
    BlockLayout L{};
    const uint32_t r[kPerBlock] = {1, 1, (uint32_t)d, 1, (uint32_t)d, 1, (uint32_t)d, 1, (uint32_t)d, 1, 1, 1, (uint32_t)f, 1, (uint32_t)d, 1};
    const uint32_t c[kPerBlock] = {(uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)d,
                                   (uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)d, (uint32_t)f, (uint32_t)f, (uint32_t)d};
    size_t off = 0;
    for (int i = 0; i < kPerBlock; ++i) {
        L.rows[i] = r[i]; L.cols[i] = c[i]; L.src_off[i] = off; off += (size_t)r[i] * c[i];
    }
    L.total = off;
    size_t o = 0;
    const size_t D = d, F = f;
    L.st_ln1g = o; o += D; L.st_ln1b = o; o += D;
    L.st_wqkv = o; o += 3 * D * D; L.st_bqkv = o; o += 3 * D;
    L.st_wo = o; o += D * D; L.st_bo = o; o += D;
    L.st_ln2g = o; o += D; L.st_ln2b = o; o += D;
    L.st_w1 = o; o += D * F; L.st_b1 = o; o += F;
    L.st_w2 = o; o += F * D; L.st_b2 = o; o += D;
    return L;
}

struct Workspace {           // byte offsets into the caller's workspace
    size_t descs, resid, xbuf, qkv, att, mid, logits, stage[2], e_pm[2], pos_pm[2], lnf_pm[2], target, row_loss, scalars,
        slot[2], total;
    int logits_rows;
};

int check_cfg(const zo_config *c)
{
    if (!c) return fail(ZO_EINVAL, "cfg is NULL");
    if (c->n_layers < 1 || c->d_model < 8 || c->n_heads < 1 || c->d_ffn < 8 || c->vocab < 2 || c->max_pos < 1)
        return fail(ZO_EINVAL, "non-positive model dimension");
    if (c->d_model % c->n_heads) return fail(ZO_EINVAL, "d_model %d is not a multiple of n_heads %d", c->d_model, c->n_heads);
    if (c->d_model % 8 || c->d_ffn % 8) return fail(ZO_EINVAL, "d_model and d_ffn must be multiples of 8");
    if (c->d_model / c->n_heads > 128) return fail(ZO_EINVAL, "head size above 128 is not supported");
    if (c->dtype < 0 || c->dtype > 2) return fail(ZO_EINVAL, "dtype %d unknown", c->dtype);
    if (c->residency != ZO_RESIDENT && c->residency != ZO_STREAMED) return fail(ZO_EINVAL, "residency %d unknown", c->residency);
    if (!(c->ln_eps > 0.0f)) return fail(ZO_EINVAL, "ln_eps must be positive");
    return ZO_OK;
}

// Bytes the LM head needs in its scratch region: a chunk of fp32 (fp64) logits, or the fused path's
// (max, sum-exp) pairs and target logits for all rows, whichever is larger.
size_t lmhead_region_bytes(int dtype, size_t rows, int vocab)
{
    const size_t lr = rows < 2048 ? rows : 2048;
    const size_t chunk = lr * (size_t)vocab * acc_bytes(dtype);
    const size_t fused = rows * ((size_t)(2 * ((vocab + 127) / 128)) * 8 + 4) + 256;
    return chunk > fused ? chunk : fused;
}

Workspace plan_workspace(const zo_config &c, int batch, int seq)
{
    Workspace w{};
    const size_t e = elem_bytes(c.dtype), ab = act_bytes(c.dtype), rb = resid_bytes(c.dtype), cb = acc_bytes(c.dtype);
    const size_t rows = 2 * (size_t)batch * seq, d = c.d_model, f = c.d_ffn;
    const BlockLayout L = make_layout(c.d_model, c.d_ffn);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    w.descs = take(sizeof(TensorDesc) * (4 + (size_t)kPerBlock * c.n_layers));
    w.resid = take(rows * d * rb);
    w.xbuf = take(rows * d * ab);
    w.qkv = take(rows * 3 * d * ab);
    w.att = take(rows * d * ab);
    w.mid = take(rows * f * ab);
    size_t lr = rows < 2048 ? rows : 2048;       // logits are produced and reduced in row chunks
    w.logits_rows = (int)lr;
    w.logits = take(lmhead_region_bytes(c.dtype, rows, c.vocab));
    for (int s = 0; s < 2; ++s) w.stage[s] = take(L.total * e);
    for (int s = 0; s < 2; ++s) w.e_pm[s] = take((size_t)c.vocab * d * e);
    for (int s = 0; s < 2; ++s) w.pos_pm[s] = take((size_t)c.max_pos * d * e);
    for (int s = 0; s < 2; ++s) w.lnf_pm[s] = take(2 * d * e);
    w.target = take(rows * sizeof(int32_t));
    w.row_loss = take(rows * sizeof(double));
    w.scalars = take(256);
    if (c.residency == ZO_STREAMED)
        for (int s = 0; s < 2; ++s) w.slot[s] = take(L.total * e);
    w.total = o;
    return w;
}

}  // namespace

constexpr int kMaxPending = kMaxUpdates;   // longest write-back interval of a streamed model

struct zo_model {
    zo_config cfg;
    int n_tensors, max_batch, max_seq;
    BlockLayout lay;
    Workspace wsp;
    char *ws;
    std::vector<void *> tptr;
    std::vector<TensorDesc> descs;     // host copy; device copy at ws + wsp.descs
    uint64_t total_chunks;
    hipStream_t compute, upload, download;
    bool own_download;
    bool use_mfma;
    // device scalars
    double *loss_pm, *g;
    float *s_cur, *s_pend;             // update scalars on the device: this step's (resident model), the pending steps' (streamed)
    uint32_t *flags;
    // streamed state
    // A streamed model keeps every block where its pointers say: pinned host memory (uploaded for each visit, Alg. 3)
    // or device memory (as many blocks as HBM has room for stay there and cost no transfer).  blk_dev[l]: block l is
    // in device memory; blk_slot[l]: upload slot of a host block (its number among the host blocks, mod 2).
    std::vector<char> blk_dev;
    std::vector<int> blk_slot;
    int up_next;                       // zo_step / zo_flush_pending: first block whose upload has not been enqueued yet
    hipEvent_t ev_uploaded[2], ev_staged[2], ev_written[2];
    // How far the host may run ahead of the device in streamed steps: ev_step[j % 2] marks the end of step j's kernels;
    // with lookahead 1 the call that enqueues step j first waits for step j - 2, with 0 every step returns drained.
    hipEvent_t ev_step[2];
    uint64_t n_steps;
    int lookahead;
    int slot_block[2];
    SlotState slot_state[2];
    bool slot_dirty[2];
    // Streamed model: the steps whose update the host copies of the blocks do not hold yet, oldest first.  Each
    // block takes them, in order, right after its next upload; the blocks are written back in the step that finds
    // wb_interval of them (1 = Alg. 3 as printed: every step), after which the list starts again.  The tensors that
    // stay in HBM only ever lack the newest one.
    int wb_interval, pend_n;
    uint64_t pend_seed[kMaxPending];
    bool resident_pending;
    int update_rounding;               // ZO_ROUND_*: how the update of Eq. 2 goes into a 16-bit type
    // Resident model with deferred updates (Alg. 2's order on one GPU): a fused-mode step leaves its update pending
    // (pend_n = 1, pend_seed[0], s_pend[0], rounded as pend_round says) and the next staging pass over theta
    // applies it on the way.
    bool deferred;
    int pend_round;
    bool step_open;
    int next_block;
    uint64_t step_seed;
    float step_eps;
    int step_batch, step_seq;
    // per-launch timing (zo_profile_begin / zo_profile_end)
    bool prof_on;
    int prof_n;
    std::vector<hipEvent_t> prof_ev;      // 2 per record
    std::vector<int> prof_cls;
    std::vector<double> prof_work;
    // streamed models, while profiling: one record per upload, per block's kernels and per write-back
    struct Span { int kind, block; hipEvent_t t0, t1; };      // kind: ZO_SPAN_*
    std::vector<Span> spans;
};

namespace {

template <typename T> T *wsp_ptr(zo_model *m, size_t off) { return (T *)(m->ws + off); }

// Brackets one kernel launch with events on the compute stream while profiling is on.
struct ProfScope {
    zo_model *m;
    bool live;
    ProfScope(zo_model *m_, int cls, double work) : m(m_), live(false)
    {
        if (!m->prof_on || 2 * (m->prof_n + 1) > (int)m->prof_ev.size()) return;
        if (hipEventRecord(m->prof_ev[2 * m->prof_n], m->compute) != hipSuccess) return;
        m->prof_cls[m->prof_n] = cls;
        m->prof_work[m->prof_n] = work;
        live = true;
    }
    ~ProfScope()
    {
        if (live && hipEventRecord(m->prof_ev[2 * m->prof_n + 1], m->compute) == hipSuccess) ++m->prof_n;
    }
};
// Brackets one copy or one block's kernels of a streamed step with events on `s` while profiling is on.
struct SpanScope {
    zo_model *m;
    hipStream_t s;
    zo_model::Span sp;
    bool live;
    SpanScope(zo_model *m_, int kind, int block, hipStream_t s_) : m(m_), s(s_), sp{kind, block, nullptr, nullptr}, live(false)
    {
        if (!m->prof_on || m->spans.size() >= 4096) return;
        if (hipEventCreate(&sp.t0) != hipSuccess) return;
        if (hipEventCreate(&sp.t1) != hipSuccess) { (void)hipEventDestroy(sp.t0); return; }
        live = hipEventRecord(sp.t0, s) == hipSuccess;
        if (!live) { (void)hipEventDestroy(sp.t0); (void)hipEventDestroy(sp.t1); }
    }
    ~SpanScope()
    {
        if (!live) return;
        if (hipEventRecord(sp.t1, s) == hipSuccess) m->spans.push_back(sp);
        else { (void)hipEventDestroy(sp.t0); (void)hipEventDestroy(sp.t1); }
    }
};
#define ZO_PROF(m, cls, work, expr)       \
    do {                                  \
        ProfScope scope__(m, cls, work);  \
        ZO_HIP(expr);                     \
    } while (0)

size_t tensor_numel(const zo_config &c, const BlockLayout &L, int t)
{
    const int last = 2 + kPerBlock * c.n_layers;
    if (t == 0) return (size_t)c.vocab * c.d_model;
    if (t == 1) return (size_t)c.max_pos * c.d_model;
    if (t >= last) return (size_t)c.d_model;
    const int k = (t - 2) % kPerBlock;
    return (size_t)L.rows[k] * L.cols[k];
}

bool is_block_tensor(const zo_model *m, int t) { return t >= 2 && t < 2 + kPerBlock * m->cfg.n_layers; }

int check_batch(const zo_model *m, const int32_t *tokens, int batch, int seq)
{
    if (!tokens) return fail(ZO_EINVAL, "tokens is NULL");
    if (batch < 1 || seq < 2) return fail(ZO_EINVAL, "need batch >= 1 and seq >= 2 (got %d x %d)", batch, seq);
    if (seq > m->cfg.max_pos) return fail(ZO_EINVAL, "seq %d exceeds max_pos %d", seq, m->cfg.max_pos);
    if ((size_t)batch * seq > (size_t)m->max_batch * m->max_seq)
        return fail(ZO_EINVAL, "batch %d x seq %d exceeds the %d x %d the workspace was sized for", batch, seq, m->max_batch, m->max_seq);
    return ZO_OK;
}

// in-place theta <- rn(fma(scale, z, theta)) over tensors [first, first + n); `update` marks the update of
// Eq. 2, which alone follows the model's rounding mode (a perturbation is always rounded to nearest)
int axpy_range(zo_model *m, int first, int n, uint64_t seed, float scale, const float *dev_scale, bool update = false)
{
    if (n <= 0) return ZO_OK;
    const uint64_t c0 = m->descs[first].first_chunk;
    const uint64_t c1 = first + n < m->n_tensors ? m->descs[first + n].first_chunk : m->total_chunks;
    double bytes = 0;
    for (int t = first; t < first + n; ++t) bytes += 2.0 * (double)m->descs[t].numel * elem_bytes(m->cfg.dtype);
    ZO_PROF(m, K_UPDATE, bytes, launch_axpy_multi(wsp_ptr<TensorDesc>(m, m->wsp.descs) + first, n, c0, c1 - c0, m->cfg.dtype, seed, scale,
                                                  dev_scale, update && m->update_rounding == ZO_ROUND_STOCHASTIC, m->compute));
    return ZO_OK;
}

struct BlockPtrs {   // staged parameter pointers of one block, per sign
    const char *base[2];
};

// Stage the embeddings and the final LayerNorm: W+- copies (fused) or nothing (literal reads theta itself).
// upd_mode != 0: a pending update (seed m->pend_seed[0], scalar m->s_pend[0]) is applied to these tensors on the way.
// Only the first `seq` position rows are staged, so the position table takes its update in a pass of its own.
int stage_globals(zo_model *m, int seq, uint64_t seed, float eps, int upd_mode)
{
    const zo_config &c = m->cfg;
    StageBatch b{}, bpos{};
    const int lnf = 2 + kPerBlock * c.n_layers;
    const size_t e = elem_bytes(c.dtype);
    stage_batch_add(b, m->tptr[0], m->ws + m->wsp.e_pm[0], m->ws + m->wsp.e_pm[1], c.vocab, c.d_model, 0, false);
    stage_batch_add(upd_mode ? bpos : b, m->tptr[1], m->ws + m->wsp.pos_pm[0], m->ws + m->wsp.pos_pm[1], seq, c.d_model, 1, false);
    stage_batch_add(b, m->tptr[lnf], m->ws + m->wsp.lnf_pm[0], m->ws + m->wsp.lnf_pm[1], 1, c.d_model, lnf, false);
    stage_batch_add(b, m->tptr[lnf + 1], m->ws + m->wsp.lnf_pm[0] + c.d_model * e, m->ws + m->wsp.lnf_pm[1] + c.d_model * e, 1,
                    c.d_model, lnf + 1, false);
    const double n_rest = (double)c.vocab * c.d_model + 2.0 * c.d_model, n_pos = (double)seq * c.d_model;
    if (upd_mode) {
        const int keep = m->update_rounding;           // the rounding the pending step asked for
        m->update_rounding = m->pend_round;
        const int rc = axpy_range(m, 1, 1, m->pend_seed[0], 0.0f, m->s_pend, true);
        m->update_rounding = keep;
        ZO_TRY(rc);
        ZO_PROF(m, K_STAGE, 4.0 * e * n_rest, launch_stage(b, c.dtype, seed, eps, false, m->compute, upd_mode, m->pend_seed[0], m->s_pend));
        ZO_PROF(m, K_STAGE, 3.0 * e * n_pos, launch_stage(bpos, c.dtype, seed, eps, false, m->compute));
    } else {
        ZO_PROF(m, K_STAGE, 3.0 * e * (n_rest + n_pos), launch_stage(b, c.dtype, seed, eps, false, m->compute));
    }
    return ZO_OK;
}

// Stage one block into the per-sign scratch.  `slot_base` == nullptr: the block's 16 tensors are read
// where the caller keeps them (resident model, separately allocated); otherwise from a device copy of
// the block laid out contiguously in canonical order (streamed model).
int stage_block(zo_model *m, int layer, const char *slot_base, uint64_t seed, float eps, bool single, int upd_mode = 0, int pend = 0)
{
    const zo_config &c = m->cfg;
    const BlockLayout &L = m->lay;
    const size_t e = elem_bytes(c.dtype), D = c.d_model;
    char *sp = m->ws + m->wsp.stage[0], *sm = m->ws + m->wsp.stage[1];
    const int t0 = 2 + kPerBlock * layer;
    StageBatch b{};
    auto add = [&](int k, size_t dst_off) {
        const void *src = slot_base ? (const void *)(slot_base + L.src_off[k] * e) : (const void *)m->tptr[t0 + k];
        stage_batch_add(b, src, sp + dst_off * e, sm + dst_off * e, L.rows[k], L.cols[k], t0 + k, false);
    };
    add(T_LN1G, L.st_ln1g); add(T_LN1B, L.st_ln1b);
    add(T_WQ, L.st_wqkv); add(T_WK, L.st_wqkv + D * D); add(T_WV, L.st_wqkv + 2 * D * D);
    add(T_BQ, L.st_bqkv); add(T_BK, L.st_bqkv + D); add(T_BV, L.st_bqkv + 2 * D);
    add(T_WO, L.st_wo); add(T_BO, L.st_bo);
    add(T_LN2G, L.st_ln2g); add(T_LN2B, L.st_ln2b);
    add(T_W1, L.st_w1); add(T_B1, L.st_b1);
    add(T_W2, L.st_w2); add(T_B2, L.st_b2);
    ZO_PROF(m, K_STAGE, (single ? 2.0 : upd_mode ? 4.0 : 3.0) * e * (double)L.total,
            launch_stage(b, c.dtype, seed, eps, single, m->compute, upd_mode, m->pend_seed[pend], m->s_pend + pend));
    return ZO_OK;
}

// One decoder block on the staged parameters; activations in the workspace.
int block_forward(zo_model *m, int n_sign, int batch, int seq)
{
    const zo_config &c = m->cfg;
    const BlockLayout &L = m->lay;
    const size_t e = elem_bytes(c.dtype);
    const int m_half = batch * seq, d = c.d_model, f = c.d_ffn, dt = c.dtype;
    const char *P = m->ws + m->wsp.stage[0], *M = m->ws + m->wsp.stage[1];
    void *resid = m->ws + m->wsp.resid, *x = m->ws + m->wsp.xbuf, *qkv = m->ws + m->wsp.qkv, *att = m->ws + m->wsp.att,
         *mid = m->ws + m->wsp.mid;
    hipStream_t s = m->compute;
    auto at = [&](const char *base, size_t off) { return (const void *)(base + off * e); };
    const double rows = (double)n_sign * m_half;
    const double ln_bytes = rows * d * (resid_bytes(dt) + act_bytes(dt));
    const double attn_flops = 2.0 * (double)n_sign * batch * c.n_heads * ((double)seq * (seq + 1)) * (d / c.n_heads);
    ZO_PROF(m, K_NORM, ln_bytes, launch_layernorm(resid, at(P, L.st_ln1g), at(M, L.st_ln1g), at(P, L.st_ln1b), at(M, L.st_ln1b), x, dt,
                                                  n_sign, m_half, d, c.ln_eps, s));
    ZO_PROF(m, K_LINEAR, 2.0 * rows * 3 * d * d, launch_linear(x, at(P, L.st_wqkv), at(M, L.st_wqkv), at(P, L.st_bqkv), at(M, L.st_bqkv),
                                                               qkv, dt, n_sign, m_half, 3 * d, d, 0, m->use_mfma, s));
    ZO_PROF(m, K_ATTN, attn_flops, launch_attention(qkv, att, dt, n_sign * batch, seq, c.n_heads, d / c.n_heads, m->use_mfma, s));
    ZO_PROF(m, K_LINEAR, 2.0 * rows * d * d, launch_linear(att, at(P, L.st_wo), at(M, L.st_wo), at(P, L.st_bo), at(M, L.st_bo), resid, dt,
                                                           n_sign, m_half, d, d, 2, m->use_mfma, s));
    ZO_PROF(m, K_NORM, ln_bytes, launch_layernorm(resid, at(P, L.st_ln2g), at(M, L.st_ln2g), at(P, L.st_ln2b), at(M, L.st_ln2b), x, dt,
                                                  n_sign, m_half, d, c.ln_eps, s));
    ZO_PROF(m, K_LINEAR, 2.0 * rows * d * f, launch_linear(x, at(P, L.st_w1), at(M, L.st_w1), at(P, L.st_b1), at(M, L.st_b1), mid, dt,
                                                           n_sign, m_half, f, d, 1, m->use_mfma, s));
    ZO_PROF(m, K_LINEAR, 2.0 * rows * d * f, launch_linear(mid, at(P, L.st_w2), at(M, L.st_w2), at(P, L.st_b2), at(M, L.st_b2), resid, dt,
                                                           n_sign, m_half, d, f, 2, m->use_mfma, s));
    return ZO_OK;
}

// LM head (tied) + cross entropy over row chunks.  x: final-LayerNormed activations [n_sign*m_half, d].
int lmhead_ce(zo_model *prof, hipStream_t s, const void *x, const void *e_p, const void *e_m, const int32_t *target, double *row_loss,
              void *logits, int logits_rows, int dtype, int n_sign, int m_half, int d, int vocab, bool use_mfma)
{
    const size_t ab = act_bytes(dtype);
    if (use_mfma && dtype != kFP32 && mfma_linear_supported(m_half, vocab, d)) {
        // fused: one sign-batched launch over all rows, no logits in memory
        const int rows = n_sign * m_half, np = mfma_ce_partials(n_sign, m_half, vocab, d);
        float *tlogit = (float *)((char *)logits + align_up((size_t)rows * np * 8));
        const double flops = 2.0 * rows * (double)vocab * d;
        if (prof) {
            ZO_PROF(prof, K_LINEAR, flops, launch_linear_mfma(x, e_p, e_m, target, tlogit, logits, dtype, n_sign, m_half, vocab, d, 4, s));
            ZO_PROF(prof, K_CE, (double)rows * np * 8, launch_ce_finish(logits, np, tlogit, target, row_loss, rows, s));
        } else {
            ZO_HIP(launch_linear_mfma(x, e_p, e_m, target, tlogit, logits, dtype, n_sign, m_half, vocab, d, 4, s));
            ZO_HIP(launch_ce_finish(logits, np, tlogit, target, row_loss, rows, s));
        }
        return ZO_OK;
    }
    for (int sign = 0; sign < n_sign; ++sign) {
        const void *wt = sign ? e_m : e_p;
        for (int r0 = 0; r0 < m_half; r0 += logits_rows) {
            const int nr = m_half - r0 < logits_rows ? m_half - r0 : logits_rows;
            const size_t row = (size_t)sign * m_half + r0;
            const char *xa = (const char *)x + row * d * ab;
            if (prof) {
                ZO_PROF(prof, K_LINEAR, 2.0 * nr * (double)vocab * d, launch_linear(xa, wt, wt, nullptr, nullptr, logits, dtype, 1, nr, vocab, d, 3, use_mfma, s));
                ZO_PROF(prof, K_CE, (double)nr * vocab * acc_bytes(dtype), launch_ce_rows(logits, target + row, row_loss + row, dtype, nr, vocab, s));
            } else {
                ZO_HIP(launch_linear(xa, wt, wt, nullptr, nullptr, logits, dtype, 1, nr, vocab, d, 3, use_mfma, s));
                ZO_HIP(launch_ce_rows(logits, target + row, row_loss + row, dtype, nr, vocab, s));
            }
        }
    }
    return ZO_OK;
}

int head_and_loss(zo_model *m, int n_sign, int batch, int seq, const void *e_p, const void *e_m, const void *lnf_p,
                  const void *lnf_m, double *loss_out)
{
    const zo_config &c = m->cfg;
    const size_t e = elem_bytes(c.dtype);
    const int m_half = batch * seq, d = c.d_model;
    void *resid = m->ws + m->wsp.resid, *x = m->ws + m->wsp.xbuf;
    int32_t *target = wsp_ptr<int32_t>(m, m->wsp.target);
    double *row_loss = wsp_ptr<double>(m, m->wsp.row_loss);
    ZO_PROF(m, K_NORM, (double)n_sign * m_half * d * (resid_bytes(c.dtype) + act_bytes(c.dtype)),
            launch_layernorm(resid, lnf_p, lnf_m, (const char *)lnf_p + d * e, (const char *)lnf_m + d * e, x, c.dtype, n_sign, m_half, d,
                             c.ln_eps, m->compute));
    ZO_TRY(lmhead_ce(m, m->compute, x, e_p, e_m, target, row_loss, m->ws + m->wsp.logits, m->wsp.logits_rows, c.dtype, n_sign, m_half, d,
                     c.vocab, m->use_mfma));
    ZO_PROF(m, K_OTHER, 8.0 * n_sign * m_half, launch_loss_reduce(row_loss, n_sign, m_half, batch * (seq - 1), loss_out, m->compute));
    return ZO_OK;
}

int embed(zo_model *m, const int32_t *tokens, int n_sign, int batch, int seq, const void *e_p, const void *e_m, const void *pos_p,
          const void *pos_m)
{
    ZO_PROF(m, K_OTHER, (double)n_sign * batch * seq * m->cfg.d_model * (2.0 * elem_bytes(m->cfg.dtype) + resid_bytes(m->cfg.dtype)),
            launch_embed(tokens, e_p, e_m, pos_p, pos_m, m->ws + m->wsp.resid, wsp_ptr<int32_t>(m, m->wsp.target), m->flags, m->cfg.dtype,
                         n_sign, batch, seq, m->cfg.d_model, m->cfg.vocab, m->compute));
    return ZO_OK;
}

// Both signs in one batched pass over staged W+-; theta untouched.
int forward_fused_resident(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed, float eps)
{
    const zo_config &c = m->cfg;
    // a pending update (deferred mode) rides on this step's staging passes: every parameter is read here anyway
    const int upd_mode = m->pend_n > 0 ? (m->pend_round == ZO_ROUND_STOCHASTIC ? 2 : 1) : 0;
    ZO_TRY(stage_globals(m, seq, seed, eps, upd_mode));
    const char *ep = m->ws + m->wsp.e_pm[0], *em = m->ws + m->wsp.e_pm[1];
    ZO_TRY(embed(m, tokens, 2, batch, seq, ep, em, m->ws + m->wsp.pos_pm[0], m->ws + m->wsp.pos_pm[1]));
    for (int l = 0; l < c.n_layers; ++l) {
        ZO_TRY(stage_block(m, l, nullptr, seed, eps, false, upd_mode));
        ZO_TRY(block_forward(m, 2, batch, seq));
    }
    m->pend_n = 0;
    return head_and_loss(m, 2, batch, seq, ep, em, m->ws + m->wsp.lnf_pm[0], m->ws + m->wsp.lnf_pm[1], m->loss_pm);
}

// One forward of theta as it stands (literal mode), loss into loss_pm[slot].
int forward_single(zo_model *m, const int32_t *tokens, int batch, int seq, int slot)
{
    const zo_config &c = m->cfg;
    const int lnf = 2 + kPerBlock * c.n_layers;
    const size_t e = elem_bytes(c.dtype);
    // the final LayerNorm's gain and bias are separate tensors: gather them side by side
    StageBatch b{};
    stage_batch_add(b, m->tptr[lnf], m->ws + m->wsp.lnf_pm[0], nullptr, 1, c.d_model, lnf, false);
    stage_batch_add(b, m->tptr[lnf + 1], m->ws + m->wsp.lnf_pm[0] + c.d_model * e, nullptr, 1, c.d_model, lnf + 1, false);
    ZO_HIP(launch_stage(b, c.dtype, 0, 0.0f, true, m->compute));
    ZO_TRY(embed(m, tokens, 1, batch, seq, m->tptr[0], m->tptr[0], m->tptr[1], m->tptr[1]));
    for (int l = 0; l < c.n_layers; ++l) {
        ZO_TRY(stage_block(m, l, nullptr, 0, 0.0f, true));
        ZO_TRY(block_forward(m, 1, batch, seq));
    }
    return head_and_loss(m, 1, batch, seq, m->tptr[0], m->tptr[0], m->ws + m->wsp.lnf_pm[0], m->ws + m->wsp.lnf_pm[0],
                         m->loss_pm + slot);
}

int read_back(zo_model *m, double *host_g, double *host_loss_pm)
{
    if (!host_g && !host_loss_pm) return ZO_OK;
    double tmp[3];
    ZO_HIP(hipMemcpyAsync(tmp, m->loss_pm, 3 * sizeof(double), hipMemcpyDeviceToHost, m->compute));   // loss_pm[2], g adjacent
    ZO_HIP(hipStreamSynchronize(m->compute));
    if (host_loss_pm) { host_loss_pm[0] = tmp[0]; host_loss_pm[1] = tmp[1]; }
    if (host_g) *host_g = tmp[2];
    return ZO_OK;
}

// ---- streamed model: Alg. 3's three operations on a block ----
int stream_prefetch(zo_model *m, int block)
{
    if (m->blk_dev[block]) return ZO_OK;                  // lives in HBM: nothing to upload
    const int slot = m->blk_slot[block];
    if (m->slot_state[slot] == SLOT_UPLOADED)
        return fail(ZO_ESTATE, "slot %d still holds block %d awaiting COMPUTE", slot, m->slot_block[slot]);
    if (m->slot_state[slot] == SLOT_COMPUTED && m->slot_dirty[slot])
        return fail(ZO_ESTATE, "block %d was updated in slot %d and has not been written back", m->slot_block[slot], slot);
    const size_t bytes = m->lay.total * elem_bytes(m->cfg.dtype);
    // the slot is free once its previous occupant was staged (and, if updated, written back)
    ZO_HIP(hipStreamWaitEvent(m->upload, m->ev_staged[slot], 0));
    ZO_HIP(hipStreamWaitEvent(m->upload, m->ev_written[slot], 0));
    {
        SpanScope span(m, ZO_SPAN_UPLOAD, block, m->upload);
        ZO_HIP(hipMemcpyAsync(m->ws + m->wsp.slot[slot], m->tptr[2 + kPerBlock * block], bytes, hipMemcpyHostToDevice, m->upload));
    }
    ZO_HIP(hipEventRecord(m->ev_uploaded[slot], m->upload));
    m->slot_block[slot] = block;
    m->slot_state[slot] = SLOT_UPLOADED;
    m->slot_dirty[slot] = false;
    return ZO_OK;
}

// wait for the upload, apply the updates the host copy lacks, optionally stage + forward
int stream_compute(zo_model *m, int block, bool forward, bool force_writeback = false)
{
    if (m->blk_dev[block]) {
        // a block that stays in HBM is visited once per step and only ever lacks the newest update (Alg. 2: a
        // module takes last step's update at its visit)
        SpanScope span(m, ZO_SPAN_COMPUTE, block, m->compute);
        const int sr_mode = m->update_rounding == ZO_ROUND_STOCHASTIC ? 2 : 1;
        if (m->pend_n > 0 && !forward)
            ZO_TRY(axpy_range(m, 2 + kPerBlock * block, kPerBlock, m->pend_seed[m->pend_n - 1], 0.0f, m->s_pend + (m->pend_n - 1), true));
        if (forward) {
            // the pending update rides on the staging pass, which reads theta anyway
            ZO_TRY(stage_block(m, block, nullptr, m->step_seed, m->step_eps, false, m->pend_n > 0 ? sr_mode : 0, m->pend_n > 0 ? m->pend_n - 1 : 0));
            ZO_TRY(block_forward(m, 2, m->step_batch, m->step_seq));
        }
        return ZO_OK;
    }
    const int slot = m->blk_slot[block];
    if (m->slot_state[slot] != SLOT_UPLOADED || m->slot_block[slot] != block)
        return fail(ZO_ESTATE, "block %d was not prefetched", block);
    ZO_HIP(hipStreamWaitEvent(m->compute, m->ev_uploaded[slot], 0));
    SpanScope span(m, ZO_SPAN_COMPUTE, block, m->compute);      // from here on: the block's kernels, not the wait for its upload
    const bool fold = forward && m->pend_n == 1;     // a single pending update rides on the staging pass
    if (m->pend_n == 1 && !fold) {
        ZO_TRY(axpy_range(m, 2 + kPerBlock * block, kPerBlock, m->pend_seed[0], 0.0f, m->s_pend, true));
    } else if (m->pend_n > 1) {      // all of them in one pass over the block
        const int first = 2 + kPerBlock * block;
        UpdateSeeds upd{};
        upd.n = m->pend_n;
        double bytes = 0;
        for (int j = 0; j < m->pend_n; ++j) upd.seed[j] = m->pend_seed[j];
        for (int t = first; t < first + kPerBlock; ++t) bytes += 2.0 * (double)m->descs[t].numel * elem_bytes(m->cfg.dtype);
        const uint64_t c0 = m->descs[first].first_chunk;
        const uint64_t c1 = first + kPerBlock < m->n_tensors ? m->descs[first + kPerBlock].first_chunk : m->total_chunks;
        ZO_PROF(m, K_UPDATE, bytes * m->pend_n,
                launch_axpy_updates(wsp_ptr<TensorDesc>(m, m->wsp.descs) + first, kPerBlock, c0, c1 - c0, m->cfg.dtype, upd, m->s_pend,
                                    m->update_rounding == ZO_ROUND_STOCHASTIC, m->compute));
    }
    // the updated copy goes back to the host only in the step that closes a write-back interval (or at a flush);
    // otherwise it is dropped after use and the host copy stays pend_n steps behind
    m->slot_dirty[slot] = m->pend_n > 0 && (m->pend_n >= m->wb_interval || force_writeback);
    if (forward)
        ZO_TRY(stage_block(m, block, m->ws + m->wsp.slot[slot], m->step_seed, m->step_eps, false,
                           fold ? (m->update_rounding == ZO_ROUND_STOCHASTIC ? 2 : 1) : 0, 0));
    ZO_HIP(hipEventRecord(m->ev_staged[slot], m->compute));
    if (forward) ZO_TRY(block_forward(m, 2, m->step_batch, m->step_seq));
    m->slot_state[slot] = SLOT_COMPUTED;
    return ZO_OK;
}

int stream_writeback(zo_model *m, int block)
{
    if (m->blk_dev[block]) return ZO_OK;
    const int slot = m->blk_slot[block];
    if (m->slot_state[slot] != SLOT_COMPUTED || m->slot_block[slot] != block)
        return fail(ZO_ESTATE, "block %d is not computed in slot %d", block, slot);
    if (m->slot_dirty[slot]) {
        const size_t bytes = m->lay.total * elem_bytes(m->cfg.dtype);
        ZO_HIP(hipStreamWaitEvent(m->download, m->ev_staged[slot], 0));
        {
            SpanScope span(m, ZO_SPAN_WRITEBACK, block, m->download);
            ZO_HIP(hipMemcpyAsync(m->tptr[2 + kPerBlock * block], m->ws + m->wsp.slot[slot], bytes, hipMemcpyDeviceToHost, m->download));
        }
        ZO_HIP(hipEventRecord(m->ev_written[slot], m->download));
        m->slot_dirty[slot] = false;
    }
    return ZO_OK;
}

// Enqueue the uploads of the next host blocks for as long as a slot is free for them (one is while its previous
// occupant has been computed and, if it was updated, written back).  With two slots the upload of the block after
// next starts as soon as the one before it has been staged, whatever number of HBM-resident blocks lie in between.
int stream_fill(zo_model *m)
{
    for (int b = m->up_next; b < m->cfg.n_layers; ++b) {
        if (m->blk_dev[b]) continue;
        const int slot = m->blk_slot[b];
        if (m->slot_state[slot] == SLOT_UPLOADED || (m->slot_state[slot] == SLOT_COMPUTED && m->slot_dirty[slot])) break;
        ZO_TRY(stream_prefetch(m, b));
        m->up_next = b + 1;
    }
    return ZO_OK;
}

int stream_begin(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed, float eps)
{
    if (m->step_open) return fail(ZO_ESTATE, "a streamed step is already open");
    const zo_config &c = m->cfg;
    const int lnf = 2 + kPerBlock * c.n_layers;
    m->step_seed = seed; m->step_eps = eps; m->step_batch = batch; m->step_seq = seq;
    if (m->resident_pending) {   // Alg. 2: the resident modules take last step's update at their visit
        ZO_TRY(axpy_range(m, 0, 2, m->pend_seed[m->pend_n - 1], 0.0f, m->s_pend + (m->pend_n - 1), true));
        ZO_TRY(axpy_range(m, lnf, 2, m->pend_seed[m->pend_n - 1], 0.0f, m->s_pend + (m->pend_n - 1), true));
        m->resident_pending = false;
    }
    ZO_TRY(stage_globals(m, seq, seed, eps, 0));
    ZO_TRY(embed(m, tokens, 2, batch, seq, m->ws + m->wsp.e_pm[0], m->ws + m->wsp.e_pm[1], m->ws + m->wsp.pos_pm[0],
                 m->ws + m->wsp.pos_pm[1]));
    m->step_open = true;
    m->next_block = 0;
    return ZO_OK;
}

int stream_end(zo_model *m, float lr)
{
    if (!m->step_open) return fail(ZO_ESTATE, "no streamed step is open");
    if (m->next_block != m->cfg.n_layers) return fail(ZO_ESTATE, "only %d of %d blocks were computed", m->next_block, m->cfg.n_layers);
    ZO_TRY(head_and_loss(m, 2, m->step_batch, m->step_seq, m->ws + m->wsp.e_pm[0], m->ws + m->wsp.e_pm[1], m->ws + m->wsp.lnf_pm[0],
                         m->ws + m->wsp.lnf_pm[1], m->loss_pm));
    if (m->pend_n >= m->wb_interval) m->pend_n = 0;       // this step's uploads took them all and were written back
    ZO_HIP(launch_g_scalar(m->loss_pm, m->step_eps, lr, m->g, m->s_pend + m->pend_n, m->flags, m->compute));
    m->pend_seed[m->pend_n++] = m->step_seed;
    m->resident_pending = true;
    m->step_open = false;
    return ZO_OK;
}

}  // namespace

// ------------------------------------------------------------------ exported calls
extern "C" size_t zo_workspace_bytes(const zo_config *cfg, int batch, int seq)
{
    if (check_cfg(cfg) != ZO_OK || batch < 1 || seq < 2 || seq > cfg->max_pos) return 0;
    return plan_workspace(*cfg, batch, seq).total;
}

extern "C" int zo_init_model(const zo_config *cfg, void *const *tensor_ptrs, int n_tensors, void *workspace, size_t workspace_bytes,
                             int batch, int seq, void *compute_stream, void *copy_stream, zo_model **out)
{
    ZO_TRY(check_cfg(cfg));
    if (!tensor_ptrs || !workspace || !out) return fail(ZO_EINVAL, "NULL argument");
    if (n_tensors != 4 + kPerBlock * cfg->n_layers)
        return fail(ZO_EINVAL, "expected %d tensors for %d layers, got %d", 4 + kPerBlock * cfg->n_layers, cfg->n_layers, n_tensors);
    if (batch < 1 || seq < 2 || seq > cfg->max_pos) return fail(ZO_EINVAL, "bad batch %d x seq %d (max_pos %d)", batch, seq, cfg->max_pos);
    if ((uintptr_t)workspace % 256) return fail(ZO_EINVAL, "workspace must be 256-byte aligned");
    const Workspace wsp = plan_workspace(*cfg, batch, seq);
    if (workspace_bytes < wsp.total) return fail(ZO_ENOMEM, "workspace of %zu bytes given, %zu needed", workspace_bytes, wsp.total);
    for (int i = 0; i < n_tensors; ++i) {
        if (!tensor_ptrs[i]) return fail(ZO_EINVAL, "tensor %d is NULL", i);
        if ((uintptr_t)tensor_ptrs[i] % 16) return fail(ZO_EINVAL, "tensor %d is not 16-byte aligned", i);
    }
    if (cfg->residency == ZO_STREAMED && (!copy_stream || copy_stream == compute_stream))
        return fail(ZO_EINVAL, "a streamed model needs a copy stream distinct from the compute stream");

    zo_model *m = new (std::nothrow) zo_model();
    if (!m) return fail(ZO_ENOMEM, "host allocation failed");
    m->cfg = *cfg; m->n_tensors = n_tensors; m->max_batch = batch; m->max_seq = seq;
    m->lay = make_layout(cfg->d_model, cfg->d_ffn);
    m->wsp = wsp; m->ws = (char *)workspace;
    m->tptr.assign(tensor_ptrs, tensor_ptrs + n_tensors);
    m->compute = (hipStream_t)compute_stream; m->upload = (hipStream_t)copy_stream; m->download = nullptr; m->own_download = false;
    m->use_mfma = true;
    const size_t e = elem_bytes(cfg->dtype);
    m->blk_dev.assign(cfg->n_layers, cfg->residency == ZO_STREAMED ? 0 : 1);
    m->blk_slot.assign(cfg->n_layers, 0);
    m->up_next = 0;
    if (cfg->residency == ZO_STREAMED) {
        int n_host = 0;
        for (int l = 0; l < cfg->n_layers; ++l) {
            int n_dev = 0;
            for (int k = 0; k < kPerBlock; ++k) {
                hipPointerAttribute_t attr;
                if (hipPointerGetAttributes(&attr, m->tptr[2 + kPerBlock * l + k]) != hipSuccess) {
                    (void)hipGetLastError();                      // plain host memory on runtimes that report it as an error
                    continue;
                }
                if (attr.type == hipMemoryTypeDevice) ++n_dev;
            }
            if (n_dev != 0 && n_dev != kPerBlock) {
                delete m;
                return fail(ZO_EINVAL, "streamed model: block %d lies partly in device and partly in host memory", l);
            }
            m->blk_dev[l] = n_dev == kPerBlock;
            if (m->blk_dev[l]) continue;
            m->blk_slot[l] = n_host++ & 1;
            for (int k = 1; k < kPerBlock; ++k)
                if ((char *)m->tptr[2 + kPerBlock * l + k] != (char *)m->tptr[2 + kPerBlock * l] + m->lay.src_off[k] * e) {
                    delete m;
                    return fail(ZO_EINVAL, "streamed model: tensors of block %d are not adjacent in canonical order", l);
                }
        }
    }
    // descriptor table for the in-place passes; streamed block tensors are addressed in their device slot
    m->descs.resize(n_tensors);
    uint64_t chunk = 0;
    for (int t = 0; t < n_tensors; ++t) {
        TensorDesc &d = m->descs[t];
        void *p = m->tptr[t];
        if (is_block_tensor(m, t) && !m->blk_dev[(t - 2) / kPerBlock]) {
            const int l = (t - 2) / kPerBlock, k = (t - 2) % kPerBlock;
            p = m->ws + wsp.slot[m->blk_slot[l]] + m->lay.src_off[k] * e;
        }
        d.src = p; d.dst = p; d.numel = tensor_numel(*cfg, m->lay, t); d.first_chunk = chunk; d.tid = (uint32_t)t; d.pad = 0;
        chunk += (d.numel + kAxpyChunk - 1) / kAxpyChunk;
    }
    m->total_chunks = chunk;
    char *sc = m->ws + wsp.scalars;
    m->loss_pm = (double *)sc; m->g = (double *)(sc + 16); m->s_cur = (float *)(sc + 24);
    m->flags = (uint32_t *)(sc + 32);
    m->s_pend = (float *)(sc + 64);                     // kMaxPending floats
    hipError_t err = hipMemcpy(m->ws + wsp.descs, m->descs.data(), sizeof(TensorDesc) * n_tensors, hipMemcpyHostToDevice);
    if (err == hipSuccess) err = hipMemset(sc, 0, 256);
    if (err != hipSuccess) { delete m; return fail(ZO_EHIP, "initialising the workspace failed: %s", hipGetErrorString(err)); }
    m->wb_interval = 1; m->pend_n = 0; m->resident_pending = false; m->deferred = false; m->pend_round = ZO_ROUND_NEAREST; m->step_open = false; m->next_block = 0; m->prof_on = false; m->prof_n = 0;
    for (int s = 0; s < 2; ++s) {
        m->slot_block[s] = -1; m->slot_state[s] = SLOT_EMPTY; m->slot_dirty[s] = false;
        m->ev_uploaded[s] = m->ev_staged[s] = m->ev_written[s] = nullptr;
        m->ev_step[s] = nullptr;
    }
    m->n_steps = 0; m->lookahead = 0;
    if (cfg->residency == ZO_STREAMED) {
        err = hipStreamCreateWithFlags(&m->download, hipStreamNonBlocking);
        m->own_download = err == hipSuccess;
        for (int s = 0; s < 2 && err == hipSuccess; ++s) {
            err = hipEventCreateWithFlags(&m->ev_uploaded[s], hipEventDisableTiming);
            if (err == hipSuccess) err = hipEventCreateWithFlags(&m->ev_staged[s], hipEventDisableTiming);
            if (err == hipSuccess) err = hipEventCreateWithFlags(&m->ev_written[s], hipEventDisableTiming);
            if (err == hipSuccess) err = hipEventCreateWithFlags(&m->ev_step[s], hipEventDisableTiming);
        }
        if (err != hipSuccess) { zo_free(m); return fail(ZO_EHIP, "creating streams/events failed: %s", hipGetErrorString(err)); }
    }
    *out = m;
    return ZO_OK;
}

extern "C" int zo_free(zo_model *m)
{
    if (!m) return ZO_OK;
    if (m->cfg.residency == ZO_STREAMED) {
        if (m->upload) (void)hipStreamSynchronize(m->upload);
        if (m->download) (void)hipStreamSynchronize(m->download);
    }
    (void)hipStreamSynchronize(m->compute);
    for (int s = 0; s < 2; ++s) {
        if (m->ev_uploaded[s]) (void)hipEventDestroy(m->ev_uploaded[s]);
        if (m->ev_staged[s]) (void)hipEventDestroy(m->ev_staged[s]);
        if (m->ev_written[s]) (void)hipEventDestroy(m->ev_written[s]);
        if (m->ev_step[s]) (void)hipEventDestroy(m->ev_step[s]);
    }
    if (m->own_download) (void)hipStreamDestroy(m->download);
    for (hipEvent_t ev : m->prof_ev) (void)hipEventDestroy(ev);
    for (auto &sp : m->spans) { (void)hipEventDestroy(sp.t0); (void)hipEventDestroy(sp.t1); }
    delete m;
    return ZO_OK;
}

namespace {
// Resident model, deferred mode: bring theta up to date with the plain update pass (anything that reads or writes
// theta outside the fused staging calls this first).
int apply_pending_resident(zo_model *m)
{
    if (m->cfg.residency != ZO_RESIDENT || m->pend_n == 0) return ZO_OK;
    const int keep = m->update_rounding;
    m->update_rounding = m->pend_round;
    const int rc = axpy_range(m, 0, m->n_tensors, m->pend_seed[0], 0.0f, m->s_pend, true);
    m->update_rounding = keep;
    if (rc == ZO_OK) m->pend_n = 0;
    return rc;
}
}

namespace {
// Alg. 3: U(W_{i+1}) is in flight while C(W_i) runs; O(W_i) follows as soon as W_i is staged.
int streamed_step(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed, float eps, float lr)
{
    ZO_TRY(stream_begin(m, tokens, batch, seq, seed, eps));
    m->up_next = 0;
    ZO_TRY(stream_fill(m));
    for (int l = 0; l < m->cfg.n_layers; ++l) {
        ZO_TRY(stream_compute(m, l, true));
        m->next_block = l + 1;
        ZO_TRY(stream_writeback(m, l));
        ZO_TRY(stream_fill(m));
    }
    return stream_end(m, lr);
}

// A streamed step that failed half way (a HIP call returned an error): let what was enqueued finish, close the step and
// empty the upload slots, so that later calls are not refused with ZO_ESTATE for ever.  What the failed step had
// already written (updates applied to the blocks it reached) stays: theta is then neither the old nor the new iterate,
// as after any interrupted in-place pass, and the caller has to restore it from its own copy.
void stream_abort(zo_model *m)
{
    (void)hipStreamSynchronize(m->upload);
    (void)hipStreamSynchronize(m->compute);
    if (m->download) (void)hipStreamSynchronize(m->download);
    (void)hipGetLastError();
    m->step_open = false;
    m->next_block = 0;
    m->up_next = 0;
    for (int s = 0; s < 2; ++s) { m->slot_block[s] = -1; m->slot_state[s] = SLOT_EMPTY; m->slot_dirty[s] = false; }
}
}  // namespace

extern "C" int zo_perturb(zo_model *m, uint64_t seed, float scale, int first_tensor, int n_tensors)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (first_tensor < 0 || n_tensors < 0 || first_tensor + n_tensors > m->n_tensors)
        return fail(ZO_EINVAL, "tensor range [%d, %d) outside [0, %d)", first_tensor, first_tensor + n_tensors, m->n_tensors);
    if (m->cfg.residency == ZO_STREAMED)
        for (int t = first_tensor; t < first_tensor + n_tensors; ++t)
            if (is_block_tensor(m, t) && !m->blk_dev[(t - 2) / kPerBlock])
                return fail(ZO_ESTATE, "tensor %d lives in host memory; use the streamed step", t);
    ZO_TRY(apply_pending_resident(m));
    return axpy_range(m, first_tensor, n_tensors, seed, scale, nullptr);
}

extern "C" int zo_dual_forward(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed, float eps, int mode,
                               double *dev_loss_pm, double *host_loss_pm)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    ZO_TRY(check_batch(m, tokens, batch, seq));
    if (mode != ZO_MODE_FUSED && mode != ZO_MODE_LITERAL) return fail(ZO_EINVAL, "mode %d unknown", mode);
    if (!(eps > 0.0f)) return fail(ZO_EINVAL, "eps must be positive");
    if (m->cfg.residency == ZO_STREAMED) return fail(ZO_ESTATE, "a streamed model runs its forward inside zo_step / zo_stream_*");
    if (mode == ZO_MODE_FUSED) {
        ZO_TRY(forward_fused_resident(m, tokens, batch, seq, seed, eps));
    } else {
        ZO_TRY(apply_pending_resident(m));
        ZO_TRY(axpy_range(m, 0, m->n_tensors, seed, eps, nullptr));
        ZO_TRY(forward_single(m, tokens, batch, seq, 0));
        ZO_TRY(axpy_range(m, 0, m->n_tensors, seed, -2.0f * eps, nullptr));
        ZO_TRY(forward_single(m, tokens, batch, seq, 1));
        ZO_TRY(axpy_range(m, 0, m->n_tensors, seed, eps, nullptr));
    }
    if (dev_loss_pm) ZO_HIP(hipMemcpyAsync(dev_loss_pm, m->loss_pm, 2 * sizeof(double), hipMemcpyDeviceToDevice, m->compute));
    if (host_loss_pm) {
        ZO_HIP(hipMemcpyAsync(host_loss_pm, m->loss_pm, 2 * sizeof(double), hipMemcpyDeviceToHost, m->compute));
        ZO_HIP(hipStreamSynchronize(m->compute));
    }
    return ZO_OK;
}

extern "C" int zo_step(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed, float eps, float lr, int mode,
                       double *host_g, double *host_loss_pm)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    ZO_TRY(check_batch(m, tokens, batch, seq));
    if (!(eps > 0.0f)) return fail(ZO_EINVAL, "eps must be positive");
    if (m->cfg.residency == ZO_RESIDENT) {
        ZO_TRY(zo_dual_forward(m, tokens, batch, seq, seed, eps, mode, nullptr, nullptr));
        if (m->deferred && mode == ZO_MODE_FUSED) {       // Alg. 2: the update waits for the next pass over theta
            ZO_HIP(launch_g_scalar(m->loss_pm, eps, lr, m->g, m->s_pend, m->flags, m->compute));
            m->pend_seed[0] = seed;
            m->pend_round = m->update_rounding;
            m->pend_n = 1;
        } else {
            ZO_HIP(launch_g_scalar(m->loss_pm, eps, lr, m->g, m->s_cur, m->flags, m->compute));
            ZO_TRY(axpy_range(m, 0, m->n_tensors, seed, 0.0f, m->s_cur, true));
        }
        return read_back(m, host_g, host_loss_pm);
    }
    if (mode != ZO_MODE_FUSED) return fail(ZO_EINVAL, "a streamed model supports ZO_MODE_FUSED only");
    // The host runs at most `lookahead` steps ahead of the device.  Unbounded, a caller that does not ask for g queues
    // hundreds of copies, waits and thousands of launches over three streams, and the device no longer starts them in
    // the order Alg. 3 gives them; bounded to one step, the next step's uploads and launches are queued while this
    // step still runs and nothing idles between steps.
    if (m->lookahead >= 1 && m->n_steps >= 2) ZO_HIP(hipEventSynchronize(m->ev_step[m->n_steps & 1]));
    const int rc = streamed_step(m, tokens, batch, seq, seed, eps, lr);
    if (rc != ZO_OK) {
        stream_abort(m);
        return rc;
    }
    ZO_HIP(hipEventRecord(m->ev_step[m->n_steps & 1], m->compute));
    ++m->n_steps;
    if (m->lookahead < 1) ZO_HIP(hipStreamSynchronize(m->compute));
    return read_back(m, host_g, host_loss_pm);
}

extern "C" int zo_stream_begin(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed, float eps)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (m->cfg.residency != ZO_STREAMED) return fail(ZO_ESTATE, "not a streamed model");
    ZO_TRY(check_batch(m, tokens, batch, seq));
    if (!(eps > 0.0f)) return fail(ZO_EINVAL, "eps must be positive");
    return stream_begin(m, tokens, batch, seq, seed, eps);
}

extern "C" int zo_stream_block(zo_model *m, int block, int phase_flags)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (m->cfg.residency != ZO_STREAMED) return fail(ZO_ESTATE, "not a streamed model");
    if (block < 0 || block >= m->cfg.n_layers) return fail(ZO_EINVAL, "block %d outside [0, %d)", block, m->cfg.n_layers);
    if (!phase_flags || (phase_flags & ~7)) return fail(ZO_EINVAL, "phase_flags %d invalid", phase_flags);
    if (!m->step_open) return fail(ZO_ESTATE, "no streamed step is open (call zo_stream_begin)");
    if (phase_flags & ZO_PHASE_PREFETCH) ZO_TRY(stream_prefetch(m, block));
    if (phase_flags & ZO_PHASE_COMPUTE) {
        if (block != m->next_block) return fail(ZO_ESTATE, "blocks must be computed in order: expected %d, got %d", m->next_block, block);
        ZO_TRY(stream_compute(m, block, true));
        m->next_block = block + 1;
    }
    if (phase_flags & ZO_PHASE_WRITEBACK) ZO_TRY(stream_writeback(m, block));
    return ZO_OK;
}

extern "C" int zo_stream_end(zo_model *m, float lr, double *host_g, double *host_loss_pm)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (m->cfg.residency != ZO_STREAMED) return fail(ZO_ESTATE, "not a streamed model");
    ZO_TRY(stream_end(m, lr));
    return read_back(m, host_g, host_loss_pm);
}

extern "C" int zo_set_update_rounding(zo_model *m, int mode)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (mode != ZO_ROUND_NEAREST && mode != ZO_ROUND_STOCHASTIC) return fail(ZO_EINVAL, "unknown rounding mode %d", mode);
    if (mode == ZO_ROUND_STOCHASTIC && m->cfg.dtype == ZO_FP32)
        return fail(ZO_EINVAL, "stochastic rounding is for ZO_BF16 / ZO_FP16 storage");
    m->update_rounding = mode;
    return ZO_OK;
}

extern "C" int zo_set_deferred_update(zo_model *m, int on)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (m->cfg.residency != ZO_RESIDENT) return fail(ZO_ESTATE, "a streamed model always defers its updates");
    if (!on) ZO_TRY(apply_pending_resident(m));
    m->deferred = on != 0;
    return ZO_OK;
}

extern "C" int zo_set_writeback_interval(zo_model *m, int steps)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (m->cfg.residency != ZO_STREAMED) return fail(ZO_ESTATE, "not a streamed model");
    if (steps < 1 || steps > kMaxPending) return fail(ZO_EINVAL, "write-back interval %d outside 1 .. %d", steps, kMaxPending);
    if (m->step_open || m->pend_n != 0) return fail(ZO_ESTATE, "updates are pending: call zo_flush_pending first");
    m->wb_interval = steps;
    return ZO_OK;
}

extern "C" int zo_set_stream_lookahead(zo_model *m, int steps)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (m->cfg.residency != ZO_STREAMED) return fail(ZO_ESTATE, "not a streamed model");
    if (steps < 0 || steps > 1) return fail(ZO_EINVAL, "look-ahead of %d steps: 0 or 1", steps);
    m->lookahead = steps;
    return ZO_OK;
}

extern "C" int zo_flush_pending(zo_model *m)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (m->cfg.residency == ZO_RESIDENT) return apply_pending_resident(m);
    if (m->pend_n == 0) return ZO_OK;
    if (m->step_open) return fail(ZO_ESTATE, "a streamed step is open");
    const int lnf = 2 + kPerBlock * m->cfg.n_layers;
    if (m->resident_pending) {
        ZO_TRY(axpy_range(m, 0, 2, m->pend_seed[m->pend_n - 1], 0.0f, m->s_pend + (m->pend_n - 1), true));
        ZO_TRY(axpy_range(m, lnf, 2, m->pend_seed[m->pend_n - 1], 0.0f, m->s_pend + (m->pend_n - 1), true));
        m->resident_pending = false;
    }
    m->up_next = 0;
    ZO_TRY(stream_fill(m));
    for (int l = 0; l < m->cfg.n_layers; ++l) {
        ZO_TRY(stream_compute(m, l, false, true));
        ZO_TRY(stream_writeback(m, l));
        ZO_TRY(stream_fill(m));
    }
    ZO_HIP(hipStreamSynchronize(m->download));
    ZO_HIP(hipStreamSynchronize(m->compute));
    m->pend_n = 0;
    return ZO_OK;
}

extern "C" int zo_device_flags(zo_model *m, uint32_t *host_flags)
{
    if (!m || !host_flags) return fail(ZO_EINVAL, "NULL argument");
    ZO_HIP(hipMemcpyAsync(host_flags, m->flags, sizeof(uint32_t), hipMemcpyDeviceToHost, m->compute));
    ZO_HIP(hipStreamSynchronize(m->compute));
    return ZO_OK;
}

extern "C" int zo_profile_begin(zo_model *m, int max_launches)
{
    if (!m) return fail(ZO_EINVAL, "model is NULL");
    if (max_launches < 1 || max_launches > (1 << 20)) return fail(ZO_EINVAL, "max_launches %d out of range", max_launches);
    while ((int)m->prof_ev.size() < 2 * max_launches) {
        hipEvent_t ev;
        ZO_HIP(hipEventCreate(&ev));
        m->prof_ev.push_back(ev);
    }
    m->prof_cls.assign(max_launches, 0);
    m->prof_work.assign(max_launches, 0.0);
    m->prof_n = 0;
    for (auto &sp : m->spans) { (void)hipEventDestroy(sp.t0); (void)hipEventDestroy(sp.t1); }
    m->spans.clear();
    m->prof_on = true;
    return ZO_OK;
}

extern "C" int zo_profile_end(zo_model *m, double *ms, uint64_t *launches, double *work)
{
    if (!m || !ms || !launches || !work) return fail(ZO_EINVAL, "NULL argument");
    if (!m->prof_on) return fail(ZO_ESTATE, "profiling was not started");
    m->prof_on = false;
    ZO_HIP(hipStreamSynchronize(m->compute));
    for (int c = 0; c < ZO_K_CLASSES; ++c) { ms[c] = 0.0; launches[c] = 0; work[c] = 0.0; }
    for (int i = 0; i < m->prof_n; ++i) {
        float t = 0.0f;
        ZO_HIP(hipEventElapsedTime(&t, m->prof_ev[2 * i], m->prof_ev[2 * i + 1]));
        const int c = m->prof_cls[i];
        ms[c] += t; launches[c] += 1; work[c] += m->prof_work[i];
    }
    return ZO_OK;
}

extern "C" int zo_profile_spans(zo_model *m, int max_spans, int32_t *kind, int32_t *block, double *start_ms, double *end_ms, int *n_spans)
{
    if (!m || !kind || !block || !start_ms || !end_ms || !n_spans || max_spans < 0) return fail(ZO_EINVAL, "bad argument");
    if (m->prof_on) return fail(ZO_ESTATE, "profiling is still on: call zo_profile_end first");
    if (m->upload) ZO_HIP(hipStreamSynchronize(m->upload));
    if (m->download) ZO_HIP(hipStreamSynchronize(m->download));
    ZO_HIP(hipStreamSynchronize(m->compute));
    const int n = (int)m->spans.size() < max_spans ? (int)m->spans.size() : max_spans;
    // time zero: the earliest start among the records
    int first = 0;
    for (int i = 1; i < (int)m->spans.size(); ++i) {
        float t = 0.0f;
        ZO_HIP(hipEventElapsedTime(&t, m->spans[first].t0, m->spans[i].t0));
        if (t < 0.0f) first = i;
    }
    for (int i = 0; i < n; ++i) {
        float a = 0.0f, b = 0.0f;
        ZO_HIP(hipEventElapsedTime(&a, m->spans[first].t0, m->spans[i].t0));
        ZO_HIP(hipEventElapsedTime(&b, m->spans[first].t0, m->spans[i].t1));
        kind[i] = m->spans[i].kind; block[i] = m->spans[i].block; start_ms[i] = a; end_ms[i] = b;
    }
    *n_spans = n;
    return ZO_OK;
}

// ------------------------------------------------------------------ kernel-level entry points
static int check_dtype(int dtype) { return dtype >= 0 && dtype <= 2 ? ZO_OK : fail(ZO_EINVAL, "dtype %d unknown", dtype); }

extern "C" int zo_kernel_z(float *out, uint64_t n, uint64_t seed, uint32_t tensor_id, uint64_t first, void *stream)
{
    if (!out && n) return fail(ZO_EINVAL, "out is NULL");
    ZO_HIP(launch_z(out, n, seed, tensor_id, first, (hipStream_t)stream));
    return ZO_OK;
}

extern "C" int zo_kernel_normal_pairs(const uint32_t *words, float *z, uint64_t n_pairs, void *stream)
{
    if ((!words || !z) && n_pairs) return fail(ZO_EINVAL, "NULL argument");
    ZO_HIP(launch_normal_pairs(words, z, n_pairs, (hipStream_t)stream));
    return ZO_OK;
}

extern "C" int zo_kernel_axpy_z(const void *src, void *dst, int dtype, uint64_t n, uint64_t seed, uint32_t tensor_id, float scale,
                                const float *dev_scale, void *stream)
{
    ZO_TRY(check_dtype(dtype));
    if (n == 0) return ZO_OK;
    if (!src || !dst) return fail(ZO_EINVAL, "NULL argument");
    if ((uintptr_t)src % 16 || (uintptr_t)dst % 16) return fail(ZO_EINVAL, "buffers must be 16-byte aligned");
    TensorDesc d{src, dst, n, 0, tensor_id, 0};
    ZO_HIP(launch_axpy_single(d, dtype, seed, scale, dev_scale, false, (hipStream_t)stream));
    return ZO_OK;
}

extern "C" int zo_kernel_axpy_z_sr(const void *src, void *dst, int dtype, uint64_t n, uint64_t seed, uint32_t tensor_id, float scale,
                                   const float *dev_scale, void *stream)
{
    if (dtype != ZO_BF16 && dtype != ZO_FP16) return fail(ZO_EINVAL, "stochastic rounding is for ZO_BF16 / ZO_FP16 storage (dtype %d)", dtype);
    if (n == 0) return ZO_OK;
    if (!src || !dst) return fail(ZO_EINVAL, "NULL argument");
    if ((uintptr_t)src % 16 || (uintptr_t)dst % 16) return fail(ZO_EINVAL, "buffers must be 16-byte aligned");
    TensorDesc d{src, dst, n, 0, tensor_id, 0};
    ZO_HIP(launch_axpy_single(d, dtype, seed, scale, dev_scale, true, (hipStream_t)stream));
    return ZO_OK;
}

extern "C" int zo_kernel_stage_pm(const void *theta, void *w_plus, void *w_minus, int dtype, int rows, int cols, int transpose,
                                  uint64_t seed, uint32_t tensor_id, float eps, void *stream)
{
    ZO_TRY(check_dtype(dtype));
    if (!theta || !w_plus || !w_minus) return fail(ZO_EINVAL, "NULL argument");
    if (rows < 1 || cols < 1) return fail(ZO_EINVAL, "bad shape %d x %d", rows, cols);
    if (transpose && cols % 4) return fail(ZO_EINVAL, "transposed staging needs cols %% 4 == 0");
    if ((uintptr_t)theta % 16 || (uintptr_t)w_plus % 16 || (uintptr_t)w_minus % 16) return fail(ZO_EINVAL, "buffers must be 16-byte aligned");
    StageBatch b{};
    stage_batch_add(b, theta, w_plus, w_minus, rows, cols, tensor_id, transpose != 0);
    ZO_HIP(launch_stage(b, dtype, seed, eps, false, (hipStream_t)stream));
    return ZO_OK;
}

extern "C" int zo_kernel_stage_update_pm(void *theta, void *w_plus, void *w_minus, int dtype, int rows, int cols, int transpose,
                                         uint64_t seed, uint32_t tensor_id, float eps, uint64_t upd_seed, const float *dev_scale,
                                         int stochastic, void *stream)
{
    ZO_TRY(check_dtype(dtype));
    if (!theta || !w_plus || !w_minus || !dev_scale) return fail(ZO_EINVAL, "NULL argument");
    if (rows < 1 || cols < 1) return fail(ZO_EINVAL, "bad shape %d x %d", rows, cols);
    if (transpose && cols % 4) return fail(ZO_EINVAL, "transposed staging needs cols %% 4 == 0");
    if (stochastic && dtype == ZO_FP32) return fail(ZO_EINVAL, "stochastic rounding is for ZO_BF16 / ZO_FP16 storage");
    if ((uintptr_t)theta % 16 || (uintptr_t)w_plus % 16 || (uintptr_t)w_minus % 16) return fail(ZO_EINVAL, "buffers must be 16-byte aligned");
    StageBatch b{};
    stage_batch_add(b, theta, w_plus, w_minus, rows, cols, tensor_id, transpose != 0);
    ZO_HIP(launch_stage(b, dtype, seed, eps, false, (hipStream_t)stream, stochastic ? 2 : 1, upd_seed, dev_scale));
    return ZO_OK;
}

extern "C" int zo_kernel_linear_pm(const void *x, const void *wt_plus, const void *wt_minus, const void *b_plus, const void *b_minus,
                                   void *y, int dtype, int m_half, int n, int k, int epilogue, void *stream)
{
    ZO_TRY(check_dtype(dtype));
    if (!x || !wt_plus || !wt_minus || !y) return fail(ZO_EINVAL, "NULL argument");
    if (epilogue < 0 || epilogue > 3) return fail(ZO_EINVAL, "epilogue %d unknown", epilogue);
    if (epilogue != 3 && (!b_plus || !b_minus)) return fail(ZO_EINVAL, "bias is NULL");
    if (m_half < 1 || n < 1 || k < 1) return fail(ZO_EINVAL, "bad shape");
    if (dtype != ZO_FP32 && (n % 8 || k % 8)) return fail(ZO_EINVAL, "n and k must be multiples of 8 for 2-byte types");
    if (dtype != ZO_FP32 && ((uintptr_t)x % 16 || (uintptr_t)wt_plus % 16 || (uintptr_t)wt_minus % 16 || (uintptr_t)y % 16 ||
                             (uintptr_t)b_plus % 16 || (uintptr_t)b_minus % 16))
        return fail(ZO_EINVAL, "buffers must be 16-byte aligned");
    ZO_HIP(launch_linear(x, wt_plus, wt_minus, b_plus, b_minus, y, dtype, 2, m_half, n, k, epilogue, true, (hipStream_t)stream));
    return ZO_OK;
}

extern "C" int zo_kernel_layernorm_pm(const void *resid, const void *g_plus, const void *g_minus, const void *b_plus, const void *b_minus,
                                      void *y, int dtype, int m_half, int d, float ln_eps, void *stream)
{
    ZO_TRY(check_dtype(dtype));
    if (!resid || !g_plus || !g_minus || !b_plus || !b_minus || !y) return fail(ZO_EINVAL, "NULL argument");
    if (m_half < 1 || d < 1) return fail(ZO_EINVAL, "bad shape");
    ZO_HIP(launch_layernorm(resid, g_plus, g_minus, b_plus, b_minus, y, dtype, 2, m_half, d, ln_eps, (hipStream_t)stream));
    return ZO_OK;
}

extern "C" int zo_kernel_attention(const void *qkv, void *out, int dtype, int n_seq, int seq, int n_heads, int d_head, void *stream)
{
    ZO_TRY(check_dtype(dtype));
    if (!qkv || !out) return fail(ZO_EINVAL, "NULL argument");
    if (n_seq < 1 || seq < 1 || n_heads < 1 || d_head < 1 || d_head > 128) return fail(ZO_EINVAL, "bad shape");
    if (dtype != ZO_FP32 && d_head % 8) return fail(ZO_EINVAL, "d_head must be a multiple of 8 for 2-byte types");
    ZO_HIP(launch_attention(qkv, out, dtype, n_seq, seq, n_heads, d_head, true, (hipStream_t)stream));
    return ZO_OK;
}

static int lmhead_rows(int m_half) { return m_half < 2048 ? m_half : 2048; }

static int check_lmhead_args(const void *x, const void *e_plus, const void *e_minus, const int32_t *target, double *row_loss, int dtype,
                             int m_half, int d, int vocab)
{
    ZO_TRY(check_dtype(dtype));
    if (!x || !e_plus || !e_minus || !target || !row_loss) return fail(ZO_EINVAL, "NULL argument");
    if (m_half < 1 || d < 1 || vocab < 2) return fail(ZO_EINVAL, "bad shape");
    if (dtype != ZO_FP32 && (d % 8 || vocab % 8)) return fail(ZO_EINVAL, "d and vocab must be multiples of 8 for 2-byte types");
    return ZO_OK;
}

extern "C" size_t zo_kernel_lmhead_scratch_bytes(int dtype, int m_half, int vocab)
{
    if (dtype < 0 || dtype > 2 || m_half < 1 || vocab < 1) return 0;
    return lmhead_region_bytes(dtype, 2 * (size_t)m_half, vocab);
}

extern "C" int zo_kernel_lmhead_ce(const void *x, const void *e_plus, const void *e_minus, const int32_t *target, double *row_loss,
                                   void *scratch_mem, int dtype, int m_half, int d, int vocab, void *stream)
{
    ZO_TRY(check_lmhead_args(x, e_plus, e_minus, target, row_loss, dtype, m_half, d, vocab));
    if (!scratch_mem) return fail(ZO_EINVAL, "NULL argument");
    return lmhead_ce(nullptr, (hipStream_t)stream, x, e_plus, e_minus, target, row_loss, scratch_mem, lmhead_rows(m_half), dtype, 2, m_half, d, vocab, true);
}

// ------------------------------------------------------------------ the entry point that allocates nothing
// The LM head's partial results (per-row, per-strip (max, sum-exp) pairs and target logits, or a chunk of logits)
// in a buffer that belongs to the library instead of the caller: one array per GPU, created when the code object
// is loaded on it and held until the process ends.  `scratch` is only the host-side name of that array; what
// kernels and copies take is the device address hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[ZO_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, looked up once per device
std::mutex g_scratch_mutex;

int static_scratch(void **out)
{
    int dev = -1;
    ZO_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(ZO_EINVAL, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        ZO_HIP(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(ZO_EHIP, "hipGetSymbolAddress gave no address for the scratch array on device %d", dev);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ZO_OK;
}
}  // namespace

extern "C" int zo_kernel_lmhead_ce_noalloc(const void *x, const void *e_plus, const void *e_minus, const int32_t *target,
                                           double *row_loss, int dtype, int m_half, int d, int vocab, void *stream)
{
    ZO_TRY(check_lmhead_args(x, e_plus, e_minus, target, row_loss, dtype, m_half, d, vocab));
    // what this call's path really needs: the fused 16-bit head keeps (max, sum-exp) pairs and a target logit per row;
    // the other path a chunk of logits, whose row count is cut down to what the buffer holds
    const size_t cap = (size_t)ZO_NOALLOC_SCRATCH_BYTES, rows = 2 * (size_t)m_half;
    int chunk_rows = lmhead_rows(m_half);
    if (dtype != ZO_FP32 && mfma_linear_supported(m_half, vocab, d)) {
        const size_t need = align_up(rows * (size_t)mfma_ce_partials(2, m_half, vocab, d) * 8) + rows * 4;
        if (need > cap)
            return fail(ZO_ENOMEM, "m_half %d x vocab %d needs %zu bytes of partial results, the built-in buffer holds %zu: use "
                        "zo_kernel_lmhead_ce", m_half, vocab, need, cap);
    } else {
        const size_t per_row = (size_t)vocab * acc_bytes(dtype);
        if (per_row > cap)
            return fail(ZO_ENOMEM, "one row of %d logits needs %zu bytes, the built-in buffer holds %zu: use zo_kernel_lmhead_ce",
                        vocab, per_row, cap);
        if ((size_t)chunk_rows * per_row > cap) chunk_rows = (int)(cap / per_row);
    }
    void *buf = nullptr;
    ZO_TRY(static_scratch(&buf));
    // every byte of the buffer that a launch reads was written by an earlier kernel of the same call (the partials
    // and target logits by the GEMM epilogue, the logits chunk by the GEMM): nothing has to start at zero
    return lmhead_ce(nullptr, (hipStream_t)stream, x, e_plus, e_minus, target, row_loss, buf, chunk_rows, dtype, 2, m_half, d, vocab, true);
}
