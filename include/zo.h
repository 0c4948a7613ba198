/*
 * libzo -- the single-GPU hot path of zeroth-order (ZO-SGD) fine-tuning of an
 * OPT-style decoder on AMD MI355X (gfx950), after DistZO2 (arXiv 2507.03211).
 *
 * One ZO-SGD step (Preliminaries, Eq. 1-2; App. A, Alg. 1):
 *     z ~ N(0, I) from the step's seed,
 *     l+ = L(theta + eps z),  l- = L(theta - eps z),
 *     g  = (l+ - l-) / (2 eps),
 *     theta <- theta - lr g z          (the same z, regenerated, never stored).
 *
 * Conventions of every entry point
 *   - Plain C ABI: raw pointers and sizes.  "device" pointers are HIP device
 *     addresses (e.g. torch.Tensor.data_ptr() of a tensor on the GPU), "host"
 *     pointers are ordinary host addresses; "pinned host" means page-locked
 *     memory obtained from hipHostMalloc (or torch's pin_memory).
 *   - Every call returns a zo_status.  Nothing throws or aborts across the
 *     boundary; zo_last_error() gives a thread-local description of the last
 *     failure.  Arguments are checked on the host before anything is enqueued.
 *   - Work is enqueued on the streams given to zo_init_model and is
 *     asynchronous with respect to the host unless a non-NULL host
 *     out-pointer is passed, in which case the call synchronises the compute
 *     stream before writing through it.
 *   - Ownership: the caller owns all parameter, token and workspace memory and
 *     must keep it alive until zo_free.  The library owns only the opaque
 *     handle and a few HIP events.
 *
 * Parameter tensors, canonical order (tensor id = position in this list):
 *     0  embed_tokens [vocab, d_model]     (also the LM head: tied)
 *     1  embed_pos    [max_pos, d_model]   (row t serves position t)
 *     2 + 16*l + k, k = 0..15, for block l:
 *        ln1_g[d] ln1_b[d] wq[d,d] bq[d] wk[d,d] bk[d] wv[d,d] bv[d] wo[d,d] bo[d]
 *        ln2_g[d] ln2_b[d] w1[ffn,d] b1[ffn] w2[d,ffn] b2[d]
 *     2 + 16*L, 3 + 16*L: final LayerNorm gain and bias.
 *   Linear weights are row-major [out, in]:  y = x W^T + b, the order in which
 *   the OPT checkpoints of the paper's experiments (Sec. 7) keep them.  All
 *   tensors are contiguous and stored in cfg.dtype.
 *
 * The random direction (what "the same seed gives the same z" means here):
 *   z of element i of tensor t under seed s is word-pair (i%4)/2 of
 *   Philox4x32-10(counter = (j lo, j hi, t, 0), key = (s lo, s hi)), j = i/4,
 *   turned into two normals by a Box-Muller transform with fully specified
 *   fp32 arithmetic.  It is a pure function of (s, t, i): regenerating it in
 *   another pass, kernel, chunking or step costs no state.
 */
#ifndef ZO_H
#define ZO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZO_OK = 0,
    ZO_EINVAL = 1,   /* bad argument (NULL, shape, range); nothing was enqueued */
    ZO_ENOMEM = 2,   /* workspace too small */
    ZO_EHIP = 3,     /* a HIP runtime call failed; zo_last_error() names it */
    ZO_ESTATE = 4    /* call not valid in the model's current state (e.g. streaming order) */
} zo_status;

enum { ZO_FP32 = 0, ZO_BF16 = 1, ZO_FP16 = 2 };
enum { ZO_RESIDENT = 0, ZO_STREAMED = 1 };
enum { ZO_MODE_LITERAL = 0, ZO_MODE_FUSED = 1 };
enum { ZO_PHASE_PREFETCH = 1, ZO_PHASE_COMPUTE = 2, ZO_PHASE_WRITEBACK = 4 };

typedef struct zo_model zo_model;

typedef struct {
    int32_t n_layers, d_model, n_heads, d_ffn, vocab, max_pos;
    int32_t dtype;       /* ZO_FP32 / ZO_BF16 / ZO_FP16: storage type of every parameter */
    int32_t residency;   /* ZO_RESIDENT: all parameters in HBM.
                            ZO_STREAMED: the 16 tensors of a block live in pinned host
                            memory, one contiguous region per block in canonical order, and are
                            uploaded for every visit (Alg. 3 uploads only the blocks W_i);
                            embeddings and the final LayerNorm stay in HBM.  Any block may be
                            given in device memory instead (all 16 tensors; they need not be
                            adjacent): it then stays in HBM and costs no transfer, so a model that
                            does not fit streams only the blocks that HBM has no room for. */
    float   ln_eps;      /* LayerNorm epsilon (OPT: 1e-5) */
} zo_config;

/* Bytes of device workspace zo_init_model needs for batches of up to `batch` x `seq` tokens: the
 * activations of the dual forward (Eq. 1 evaluates L twice; both signs are resident at once), the
 * staged W+- of one block (PertP workflow, Step 2) and, for ZO_STREAMED, the two upload slots of
 * App. A, Alg. 3.  Returns 0 if cfg is invalid. */
size_t zo_workspace_bytes(const zo_config *cfg, int batch, int seq);

/* Create a model handle over caller-owned memory: the inputs of App. A, Alg. 1 / Alg. 2 (theta, and where each
 * module's parameters live: Alg. 3 keeps the blocks W_i in host memory and uploads them per visit).
 *   tensor_ptrs[n_tensors]  canonical order.  ZO_RESIDENT: all device pointers.
 *                           ZO_STREAMED: ids 0, 1 and the last two are device pointers;
 *                           the 16 tensors of a block are either pinned-host pointers, adjacent
 *                           in memory in canonical order, or all device pointers (the block
 *                           stays in HBM).  Where a block lives is read off its pointers.
 *   workspace               device memory, >= zo_workspace_bytes(cfg, batch, seq), 256-byte aligned.
 *   compute_stream          hipStream_t on which all kernels run (NULL = the null stream).
 *   copy_stream             hipStream_t for host<->device block copies; required (and
 *                           different from compute_stream) when ZO_STREAMED, else ignored.
 * Errors: ZO_EINVAL (NULL, n_tensors != 4+16*n_layers, d_model % n_heads, dims not
 * multiples of 8, head size > 128, batch*seq == 0, seq > max_pos), ZO_ENOMEM, ZO_EHIP. */
int zo_init_model(const zo_config *cfg, void *const *tensor_ptrs, int n_tensors,
                  void *workspace, size_t workspace_bytes, int batch, int seq,
                  void *compute_stream, void *copy_stream, zo_model **out);

/* Alg. 1, PerturbParameters / UpdateParameters:  theta_t <- rn(fma(scale, z_t, theta_t)) in
 * place for tensors first_tensor .. first_tensor + n_tensors - 1, z from `seed`; one fp32
 * fma per element, rounded to nearest-even into the storage type.  scale = +eps, -2 eps,
 * +eps gives the three perturbations, scale = -(lr g) the update of Eq. 2.
 * ZO_STREAMED models: only device-resident tensors may be named (ZO_ESTATE otherwise). */
int zo_perturb(zo_model *m, uint64_t seed, float scale, int first_tensor, int n_tensors);

/* Eq. 1's two evaluations: l+ = L(theta + eps z; tokens), l- = L(theta - eps z; tokens),
 * L = mean next-token cross entropy over batch x (seq-1) positions.
 *   tokens        device, int32 [batch, seq], values in [0, vocab)
 *   mode          ZO_MODE_FUSED: both signs in one batched pass over W+- = rn(theta +- eps z),
 *                 theta untouched (PertP workflow Step 2, on one device).
 *                 ZO_MODE_LITERAL: Alg. 1 as printed: +eps in place, forward, -2 eps, forward,
 *                 +eps (theta returns to within rounding).  ZO_RESIDENT only.
 *   dev_loss_pm   device, double[2], receives (l+, l-); may be NULL
 *   host_loss_pm  host, double[2]; if non-NULL the call waits for the result
 * A token id outside [0, vocab) makes both losses NaN. */
int zo_dual_forward(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed,
                    float eps, int mode, double *dev_loss_pm, double *host_loss_pm);

/* One whole step: zo_dual_forward, g = (l+ - l-)/(2 eps) and s = -(lr g) on the device,
 * then theta <- rn(fma(s, z, theta)) for every tensor.  A non-finite g skips the update
 * (s = 0).  ZO_RESIDENT: the update is applied at once (unless zo_set_deferred_update).  ZO_STREAMED (Alg. 2 / Alg. 3):
 * blocks are uploaded one ahead of the computation, each block's update from the previous
 * step is applied right after its upload and written back, and this step's update stays
 * pending until the next zo_step or zo_flush_pending.
 *   host_g, host_loss_pm   host, double[1] / double[2], nullable; non-NULL synchronises.
 * A ZO_STREAMED step returns with its kernels finished unless zo_set_stream_lookahead allows it to run ahead.  If a HIP call fails inside a streamed step, the step is closed and the upload slots are
 * emptied before the error is returned; theta is then partly updated and has to be restored by the caller. */
int zo_step(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed,
            float eps, float lr, int mode, double *host_g, double *host_loss_pm);

/* Alg. 3's three operations on one block of a ZO_STREAMED model, for callers that drive
 * the schedule themselves (zo_step does this internally):
 *   PREFETCH   U(W_block): enqueue the host->device copy into slot block % 2 on the copy stream.
 *   COMPUTE    C(W_block): on the compute stream, wait for the upload, apply the updates the host
 *              copy lacks (if any), then the dual forward of this block on the activations left by
 *              the previous COMPUTE.  Blocks must be computed in order 0,1,..,L-1 after
 *              zo_stream_begin.
 *   WRITEBACK  O(W_block): wait for COMPUTE, copy the updated block back to its pinned-host home
 *              (nothing to do in a step that does not close a write-back interval).
 * Flags may be OR-ed; they are issued in the order PREFETCH, COMPUTE, WRITEBACK.
 * ZO_ESTATE: not a streamed model, no step open, COMPUTE of a block that was not prefetched or
 * out of order, PREFETCH into a slot whose occupant still awaits COMPUTE. */
int zo_stream_block(zo_model *m, int block, int phase_flags);

/* Open / close a manually scheduled streamed step around zo_stream_block calls:
 * begin = embedding DualForward (Alg. 2, first module), end = LM head, losses, g and the
 * new pending update.  Same argument meaning as zo_step. */
int zo_stream_begin(zo_model *m, const int32_t *tokens, int batch, int seq, uint64_t seed, float eps);
int zo_stream_end(zo_model *m, float lr, double *host_g, double *host_loss_pm);

/* Apply the updates that the host copies of a streamed model still lack (as printed, Alg. 2 never
 * applies the last one) and write every block back; for a resident model with deferred updates, apply the
 * pending one.  No-op when nothing is pending. */
int zo_flush_pending(zo_model *m);

/* Resident model: defer the update of Eq. 2 the way Alg. 2 does.  With `on` non-zero a ZO_MODE_FUSED zo_step computes
 * L+-, g and the step scalar, and leaves theta as it was: the update theta <- rn(theta + s z) is applied by the next
 * zo_step / zo_dual_forward in ZO_MODE_FUSED, inside the staging pass that reads every parameter anyway (one read
 * and one write of theta less per step, the same bits in theta afterwards), or by zo_flush_pending.  Until then
 * the caller's tensors are one update behind.  zo_perturb and the ZO_MODE_LITERAL paths apply a pending update
 * first; a ZO_MODE_LITERAL zo_step updates at once, as without this setting.  The rounding mode of a pending update
 * is the one that was set when its step ran.  `on` == 0 applies what is pending and returns to immediate updates.
 * ZO_ESTATE for a streamed model (it always defers). */
int zo_set_deferred_update(zo_model *m, int on);

/* Streamed models: how often the updated blocks go back to pinned host memory.  1 (the default) is Alg. 3 as
 * printed: every block is written back in every step, so the host link carries each block both ways.  With
 * `steps` = K > 1 the host copies are left up to K steps behind: a block takes all the updates it lacks, in
 * order, right after each upload (theta and the losses are bit for bit those of K = 1), and is written back
 * only in every K-th step, which takes the download traffic off the link in the others.  zo_flush_pending
 * brings the host copies up to date at any time.  1 <= steps <= 16.  ZO_ESTATE on a resident model or while
 * updates are pending (flush first). */
int zo_set_writeback_interval(zo_model *m, int steps);

/* Streamed models: how many steps the host may run ahead of the device in zo_step when no host out-pointer makes the
 * call wait anyway.  0 (the default): every zo_step returns with its kernels finished (its last write-backs may still
 * be running), which is what keeps the device on the schedule of App. A, Alg. 3.  1: the call that enqueues step j
 * returns once step j - 2 has finished, so the first uploads and launches of the next step are already queued when
 * a step ends; on the PCIe-bound configuration this measured slower (the queued copies of two steps share the
 * link less evenly), so it is an option, not the default.  Results are bit-identical either way.  ZO_EINVAL outside
 * 0..1, ZO_ESTATE on a resident model. */
int zo_set_stream_lookahead(zo_model *m, int steps);

/* How the update of Eq. 2 is rounded into a 16-bit storage type.  ZO_ROUND_NEAREST (the default, and the
 * only rounding of every perturbation) is round-to-nearest-even.  ZO_ROUND_STOCHASTIC is an opt-in
 * variant that is not in the paper: at its learning rates a nearest-rounded update of a 16-bit weight
 * is almost always lost, the stochastic one is unbiased.  With |v| = (n + f) u, u the type's spacing at
 * |v| = |fma(s, z, theta)|, the magnitude becomes (n + 1) u when the top 24 bits of the element's random
 * word are below floor(f 2^24) and n u otherwise; the word of element i is word i % 4 of the Philox block
 * with counter (i / 4, tensor id, tag 3) under the step's seed.  Applies to every later update of this
 * model, deferred ones included.  ZO_EINVAL for a ZO_FP32 model or an unknown mode. */
#define ZO_ROUND_NEAREST 0
#define ZO_ROUND_STOCHASTIC 1
int zo_set_update_rounding(zo_model *m, int mode);

/* Device-side status word accumulated by the kernels: bit 0 = non-finite loss / skipped
 * update, bit 1 = token id out of range.  Synchronises the compute stream. */
int zo_device_flags(zo_model *m, uint32_t *host_flags);

/* Per-launch timing of the model's kernels with HIP events on the compute stream, by class.
 * Between begin and end every kernel the model launches is bracketed by two events (up to
 * max_launches launches; later ones are not recorded).  zo_profile_end synchronises the compute
 * stream and fills three host arrays of ZO_K_CLASSES entries: summed kernel milliseconds, number
 * of launches, and summed algorithmic work (FLOP for LINEAR and ATTENTION -- 2 m n k, causal half
 * for attention -- bytes that must cross HBM for the others). */
enum { ZO_K_LINEAR = 0, ZO_K_ATTENTION = 1, ZO_K_STAGE = 2, ZO_K_UPDATE = 3, ZO_K_NORM = 4, ZO_K_CE = 5, ZO_K_OTHER = 6,
       ZO_K_CLASSES = 7 };
int zo_profile_begin(zo_model *m, int max_launches);
int zo_profile_end(zo_model *m, double *ms, uint64_t *launches, double *work);

/* ZO_STREAMED models: the timeline of App. A, Alg. 3's three operations over the steps that ran between
 * zo_profile_begin and zo_profile_end, from HIP events on the stream each one ran on.  One record per upload U(W_i)
 * (ZO_SPAN_UPLOAD), per block's kernels C(W_i) (ZO_SPAN_COMPUTE: pending updates, staging, dual forward) and per
 * write-back O(W_i) (ZO_SPAN_WRITEBACK), in the order they were enqueued; blocks that live in HBM have compute records
 * only.  Times are milliseconds since the earliest recorded start.  Host arrays of max_spans entries; *n_spans
 * receives the number filled (at most 4096 are kept).  Synchronises all three streams.  ZO_ESTATE while profiling
 * is still on. */
enum { ZO_SPAN_UPLOAD = 0, ZO_SPAN_COMPUTE = 1, ZO_SPAN_WRITEBACK = 2 };
int zo_profile_spans(zo_model *m, int max_spans, int32_t *kind, int32_t *block, double *start_ms, double *end_ms, int *n_spans);

int zo_free(zo_model *m);
const char *zo_last_error(void);

/* ------------------------------------------------------------------------
 * Kernel-level entry points.  They run exactly the kernels the calls above
 * use, on caller-provided buffers, so that each can be checked against the
 * oracle and timed against its roofline at real shapes.  All pointers are
 * device pointers; `stream` is a hipStream_t (NULL = null stream); dtype is
 * ZO_FP32 / ZO_BF16 / ZO_FP16.
 * ---------------------------------------------------------------------- */

/* z itself (fp32) for elements [first, first+n) of tensor `tensor_id` (Eq. 1: z ~ N(0, I)). */
int zo_kernel_z(float *out, uint64_t n, uint64_t seed, uint32_t tensor_id, uint64_t first, void *stream);

/* The normal transform alone: z[2i], z[2i+1] from the word pair (words[2i], words[2i+1]). */
int zo_kernel_normal_pairs(const uint32_t *words, float *z, uint64_t n_pairs, void *stream);

/* dst <- rn(fma(scale, z, src)) over one tensor of n elements (dst may equal src): the
 * perturb/update stream of Alg. 1 on a bare buffer.  If dev_scale is non-NULL the scalar is
 * read from device memory instead (as the update inside zo_step does). */
int zo_kernel_axpy_z(const void *src, void *dst, int dtype, uint64_t n, uint64_t seed,
                     uint32_t tensor_id, float scale, const float *dev_scale, void *stream);

/* The same with the stochastic rounding of zo_set_update_rounding (ZO_BF16 / ZO_FP16 only). */
int zo_kernel_axpy_z_sr(const void *src, void *dst, int dtype, uint64_t n, uint64_t seed,
                        uint32_t tensor_id, float scale, const float *dev_scale, void *stream);

/* W+ = rn(theta + eps z), W- = rn(theta - eps z) (PertP workflow, Step 2; Alg. 1 PerturbParameters out of place)
 * for a [rows, cols] row-major tensor, z of element i as everywhere: drawn at the element's index in theta.  Written
 * in the same layout, or transposed ([cols, rows]) when `transpose` is non-zero (needs cols % 4 == 0): for a caller
 * that keeps a matrix [in, out] and wants the [out, in] the GEMMs read.  The model's own tensors are [out, in]
 * already and are staged with transpose = 0.  All three buffers: device, 16-byte aligned, not overlapping. */
int zo_kernel_stage_pm(const void *theta, void *w_plus, void *w_minus, int dtype, int rows, int cols,
                       int transpose, uint64_t seed, uint32_t tensor_id, float eps, void *stream);

/* The staging pass with a pending update of Eq. 2 folded in: first theta <- rn(fma(*dev_scale, z', theta)) in place,
 * z' drawn from `upd_seed` (round to nearest, or stochastic rounding with the words of stream 3 when `stochastic` is
 * non-zero: 16-bit types only), then W+- = rn(theta +- eps z) from the updated theta, z drawn from `seed`, as
 * zo_kernel_stage_pm writes them.  theta, w_plus, w_minus: device, 16-byte aligned; dev_scale: one float on the
 * device.  The same bits as zo_kernel_axpy_z(_sr) followed by zo_kernel_stage_pm. */
int zo_kernel_stage_update_pm(void *theta, void *w_plus, void *w_minus, int dtype, int rows, int cols, int transpose,
                              uint64_t seed, uint32_t tensor_id, float eps, uint64_t upd_seed,
                              const float *dev_scale, int stochastic, void *stream);

/* Sign-batched linear layer (the QKV / out / FFN projections of a module's DualForward, App. A, Alg. 2:
 * both evaluations of Eq. 1 in one launch):  rows [0, m_half) of x use (wt_plus, b_plus), rows
 * [m_half, 2 m_half) use (wt_minus, b_minus):  y = x W + b with W given transposed as
 * wt[n, k].  x is [2 m_half, k].  2-byte dtypes run on MFMA with fp32 accumulation;
 * ZO_FP32 takes fp64 activations (x, y are double) and accumulates in fp64.
 *   epilogue 0: y[.., n] = acc + b           (y in the activation type)
 *            1: y = relu(acc + b)
 *            2: resid += acc + b             (y = resid: fp32, or fp64 for ZO_FP32)
 *            3: y = acc                      (fp32 out, or fp64 for ZO_FP32; bias ignored)
 * 2-byte dtypes: n and k multiples of 8 and every buffer 16-byte aligned (ZO_EINVAL otherwise). */
int zo_kernel_linear_pm(const void *x, const void *wt_plus, const void *wt_minus,
                        const void *b_plus, const void *b_minus, void *y,
                        int dtype, int m_half, int n, int k, int epilogue, void *stream);

/* LayerNorm of the OPT decoder block (Sec. 7, experimental set-up: OPT family) inside DualForward (App. A, Alg. 2),
 * over the last dimension of resid [2 m_half, d] (fp32; fp64 for ZO_FP32) with
 * per-sign gain and bias, output in the activation type. */
int zo_kernel_layernorm_pm(const void *resid, const void *g_plus, const void *g_minus,
                           const void *b_plus, const void *b_minus, void *y,
                           int dtype, int m_half, int d, float ln_eps, void *stream);

/* Causal multi-head attention of the decoder block inside DualForward (App. A, Alg. 2; both signs are
 * simply more sequences): qkv [n_seq * seq, 3 d] (q | k | v, heads contiguous inside each)
 * -> out [n_seq * seq, d], softmax(q k^T / sqrt(d_head)) v per (sequence, head). */
int zo_kernel_attention(const void *qkv, void *out, int dtype, int n_seq, int seq, int n_heads,
                        int d_head, void *stream);

/* Tied LM head + cross entropy, the last module of App. A, Alg. 2 ("LM head") and the loss L of Eq. 1:
 * for each row r of x [2 m_half, d] (already final-LayerNormed),
 * logits = x[r] . E+-^T over the vocabulary, row_loss[r] = logsumexp(logits) - logits[target[r]];
 * target[r] < 0 marks a row that does not count (row_loss = 0).  row_loss is double[2 m_half].
 * `scratch` is device memory of zo_kernel_lmhead_scratch_bytes(...) bytes. */
size_t zo_kernel_lmhead_scratch_bytes(int dtype, int m_half, int vocab);
int zo_kernel_lmhead_ce(const void *x, const void *e_plus, const void *e_minus, const int32_t *target,
                        double *row_loss, void *scratch, int dtype, int m_half, int d, int vocab,
                        void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): zo_kernel_lmhead_ce without the scratch argument.  The partial results
 * live in a buffer that is part of the library, ZO_NOALLOC_SCRATCH_BYTES of device memory per GPU, held from
 * the moment the library is loaded on that GPU until the process ends.  The call allocates and frees nothing,
 * on the device or through any library; the first call on a device looks the buffer's address up once.
 * Same arguments, results and errors as zo_kernel_lmhead_ce, and additionally
 *   ZO_ENOMEM  the call's partial results do not fit ZO_NOALLOC_SCRATCH_BYTES (nothing is enqueued).  ZO_BF16 /
 *              ZO_FP16 with d a multiple of 64: 2 m_half rows of P (max, sum-exp) pairs of 8 bytes plus 4 bytes,
 *              P = 2 ceil(vocab / 256) when the 256-wide tiling runs (at least 128 tiles and d >= 192), else
 *              2 ceil(vocab / 128): at vocab 50272 up to m_half = 5315, or 2666 with the 128-wide tiling.  Other
 *              shapes and ZO_FP32 go through logits in row chunks that are cut to fit, and fail only when a
 *              single row of vocab logits (4 bytes each, 8 for ZO_FP32) does not fit.
 *   ZO_EHIP    the buffer's address cannot be obtained.
 * All calls on one GPU share that GPU's buffer: calls whose kernels may overlap (different streams, or several
 * host threads) race on it; serialise them.  The buffer keeps the previous call's contents; every word a call
 * reads it has written first, so nothing needs clearing between calls. */
#define ZO_NOALLOC_SCRATCH_BYTES (32u << 20)
int zo_kernel_lmhead_ce_noalloc(const void *x, const void *e_plus, const void *e_minus, const int32_t *target,
                                double *row_loss, int dtype, int m_half, int d, int vocab, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ZO_H */
