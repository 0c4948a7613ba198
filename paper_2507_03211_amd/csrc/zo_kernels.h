// Host-side launchers of the library's kernels (internal).  Each returns the HIP status of
// the launch; all work goes to `stream`.  Shapes are validated by the callers in zo_api.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zo {

// ---- perturb / update streams (zo_stream_kernels.hip) ----
struct TensorDesc {          // one tensor of an in-place pass
    const void *src;
    void *dst;
    uint64_t numel;
    uint64_t first_chunk;    // index of this tensor's first chunk in the launch
    uint32_t tid;
    uint32_t pad;
};
#ifndef ZO_AXPY_CHUNK
#define ZO_AXPY_CHUNK 8192
#endif
constexpr uint32_t kAxpyChunk = ZO_AXPY_CHUNK;   // elements per chunk (one workgroup iteration)

struct StageDesc {           // one tensor of an out-of-place W+- staging pass
    const void *src;
    void *dst_plus;
    void *dst_minus;         // unused when staging a single copy
    uint32_t rows, cols;     // source is [rows, cols] row-major
    uint32_t tid;
    uint32_t transpose;      // write [cols, rows]
    uint32_t first_tile;
    uint32_t tiles_c;        // tiles along cols (transpose) ; unused otherwise
};
constexpr int kStageMaxDesc = 16;
struct StageBatch { StageDesc d[kStageMaxDesc]; int n; uint32_t total_tiles; };
constexpr uint32_t kStageTile = 64;          // transposing tile edge
constexpr uint32_t kStageFlatTile = 8192;    // consecutive elements per tile when not transposing

hipError_t launch_z(float *out, uint64_t n, uint64_t seed, uint32_t tid, uint64_t first, hipStream_t s);
hipError_t launch_normal_pairs(const uint32_t *words, float *z, uint64_t n_pairs, hipStream_t s);
// descs in device memory: n_desc consecutive entries whose chunks are chunk_offset .. chunk_offset + total_chunks - 1
hipError_t launch_axpy_multi(const TensorDesc *dev_descs, int n_desc, uint64_t chunk_offset, uint64_t total_chunks,
                             int dtype, uint64_t seed, float scale, const float *dev_scale, bool stochastic, hipStream_t s);
// the same over several updates in one pass: theta <- rn(fma(dev_scales[j], z(seeds[j]), theta)), j = 0 .. n-1 in order
constexpr int kMaxUpdates = 16;
struct UpdateSeeds { int n; uint64_t seed[kMaxUpdates]; };
hipError_t launch_axpy_updates(const TensorDesc *dev_descs, int n_desc, uint64_t chunk_offset, uint64_t total_chunks, int dtype,
                               const UpdateSeeds &upd, const float *dev_scales, bool stochastic, hipStream_t s);
hipError_t launch_axpy_single(const TensorDesc &d, int dtype, uint64_t seed, float scale,
                              const float *dev_scale, bool stochastic, hipStream_t s);
// both signs (eps) or a plain (transposing) copy when single_copy
// upd_mode 0: stage only.  1 / 2: first theta <- rn(fma(*dev_scale, z(upd_seed), theta)) in place (round to nearest /
// stochastic rounding), then W+- from the updated theta, in the same pass (`src` of every descriptor is written).
hipError_t launch_stage(const StageBatch &b, int dtype, uint64_t seed, float eps, bool single_copy, hipStream_t s, int upd_mode = 0,
                        uint64_t upd_seed = 0, const float *dev_scale = nullptr);
void stage_batch_add(StageBatch &b, const void *src, void *dp, void *dm, uint32_t rows, uint32_t cols,
                     uint32_t tid, bool transpose);

// ---- forward (zo_forward_kernels.hip, zo_gemm_mfma.hip, zo_attn_mfma.hip) ----
// rows are laid out sign-major: row = sign * m_half + b * seq + t.
hipError_t launch_embed(const int32_t *tokens, const void *e_p, const void *e_m, const void *pos_p,
                        const void *pos_m, void *resid, int32_t *target, uint32_t *flags, int dtype,
                        int n_sign, int batch, int seq, int d, int vocab, hipStream_t s);
hipError_t launch_layernorm(const void *resid, const void *g_p, const void *g_m, const void *b_p,
                            const void *b_m, void *y, int dtype, int n_sign, int m_half, int d, float eps,
                            hipStream_t s);
hipError_t launch_linear(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m,
                         void *y, int dtype, int n_sign, int m_half, int n, int k, int epilogue,
                         bool allow_mfma, hipStream_t s);
hipError_t launch_attention(const void *qkv, void *out, int dtype, int n_seq, int seq, int n_heads, int d_head,
                            bool allow_mfma, hipStream_t s);
hipError_t launch_ce_rows(const void *logits, const int32_t *target, double *row_loss, int dtype, int rows,
                          int vocab, hipStream_t s);
hipError_t launch_loss_reduce(const double *row_loss, int n_sign, int m_half, int count_per_sign, double *loss_pm,
                              hipStream_t s);
hipError_t launch_g_scalar(const double *loss_pm, float eps, float lr, double *g_out, float *s_out,
                           uint32_t *flags, hipStream_t s);

// MFMA paths (2-byte dtypes).  *_supported report whether the shape fits the kernel's tiling.
bool mfma_linear_supported(int m_half, int n, int k);
hipError_t launch_linear_mfma(const void *x, const void *wt_p, const void *wt_m, const void *b_p, const void *b_m,
                              void *y, int dtype, int n_sign, int m_half, int n, int k, int epilogue,
                              hipStream_t s);
// Epilogue 4 of launch_linear_mfma (LM head fused with the cross-entropy reduction): instead of logits it
// leaves mfma_ce_partials(...) (max, sum-exp) pairs per row in `y` (float2[rows][pairs]) and the target
// logit of each row in `b_m` (float[rows]); `b_p` carries the int32 targets.  launch_ce_finish merges them.
int mfma_ce_partials(int n_sign, int m_half, int n, int k);
hipError_t launch_ce_finish(const void *partials, int n_partial, const float *target_logit, const int32_t *target,
                            double *row_loss, int rows, hipStream_t s);
bool mfma_attention_supported(int seq, int d_head);
hipError_t launch_attention_mfma(const void *qkv, void *out, int dtype, int n_seq, int seq, int n_heads,
                                 int d_head, hipStream_t s);

}  // namespace zo
