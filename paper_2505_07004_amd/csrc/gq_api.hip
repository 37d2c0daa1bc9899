// C ABI of libgq: argument validation and dispatch to the gfx950 kernels.
// Every entry point checks its arguments on the host, enqueues work on the caller's
// stream and returns without synchronising.
#include "gq_internal.hpp"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }
inline size_t elem_size(gq_dtype dt) { return dt == GQ_BF16 ? 2 : 4; }
inline bool valid_dtype(int dt) { return dt == GQ_F32 || dt == GQ_BF16; }
inline int from_hip(hipError_t e) { return e == hipSuccess ? GQ_OK : GQ_ERR_HIP; }

}  // namespace

extern "C" {

int gq_version(void) { return 100; }  // 0.1.0

const char* gq_status_string(int status) {
  switch (status) {
    case GQ_OK: return "ok";
    case GQ_ERR_NULLPTR: return "a required pointer is NULL";
    case GQ_ERR_SHAPE: return "invalid shape (sizes must be positive, G must divide d_out, ld >= width)";
    case GQ_ERR_DTYPE: return "unknown dtype";
    case GQ_ERR_ALIGN: return "pointer or row pitch not 16-byte aligned";
    case GQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GQ_ERR_HIP: return "HIP runtime error";
    case GQ_ERR_UNSUPPORTED: return "unsupported request";
    default: return "unknown status";
  }
}

int gq_group_weights(const void* dZ, gq_dtype dz_dtype, int64_t n, int64_t d_out, int64_t ld_dz, int32_t G,
                     float grad_scale, float* s, void* hip_stream) {
  if (!valid_dtype((int)dz_dtype)) return GQ_ERR_DTYPE;
  if (n < 0 || d_out <= 0 || G <= 0 || d_out % G != 0 || ld_dz < d_out) return GQ_ERR_SHAPE;
  if (n == 0) return GQ_OK;
  if (!dZ || !s) return GQ_ERR_NULLPTR;
  if (!aligned16(dZ) || ((size_t)ld_dz * elem_size(dz_dtype)) % 16 != 0) return GQ_ERR_ALIGN;
  return from_hip(gq::launch_group_weights(dZ, dz_dtype, n, d_out, ld_dz, G, grad_scale, s, G, (hipStream_t)hip_stream));
}

int gq_group_weights_strided(const void* dZ, gq_dtype dz_dtype, int64_t n, int64_t d_out, int64_t ld_dz, int32_t G,
                             float grad_scale, float* s, int64_t ld_s, void* hip_stream) {
  if (!valid_dtype((int)dz_dtype)) return GQ_ERR_DTYPE;
  if (n < 0 || d_out <= 0 || G <= 0 || d_out % G != 0 || ld_dz < d_out || ld_s < G) return GQ_ERR_SHAPE;
  if (n == 0) return GQ_OK;
  if (!dZ || !s) return GQ_ERR_NULLPTR;
  if (!aligned16(dZ) || ((size_t)ld_dz * elem_size(dz_dtype)) % 16 != 0) return GQ_ERR_ALIGN;
  return from_hip(gq::launch_group_weights(dZ, dz_dtype, n, d_out, ld_dz, G, grad_scale, s, ld_s, (hipStream_t)hip_stream));
}

size_t gq_fisher_gram_workspace_bytes(gq_dtype x_dtype, int64_t n, int64_t d_in, int32_t G) {
  if (!valid_dtype((int)x_dtype) || n < 0 || d_in <= 0 || G <= 0) return 0;
  return x_dtype == GQ_BF16 ? gq::fisher_gram_heavy_workspace(n, d_in, G) : 0;
}

int gq_fisher_gram(const void* X, gq_dtype x_dtype, int64_t n, int64_t d_in, int64_t ld_x, const float* s, int32_t G,
                   float* H, uint32_t flags, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!valid_dtype((int)x_dtype)) return GQ_ERR_DTYPE;
  if (n < 0 || d_in <= 0 || G <= 0 || ld_x < d_in) return GQ_ERR_SHAPE;
  if (flags & ~(uint32_t)(GQ_ACCUMULATE | GQ_MIRROR | GQ_TWO_TERMS | GQ_HEAVY_TWO_TERMS)) return GQ_ERR_UNSUPPORTED;
  if (!H) return GQ_ERR_NULLPTR;
  if (n > 0 && (!X || !s)) return GQ_ERR_NULLPTR;
  if (!aligned16(H)) return GQ_ERR_ALIGN;
  if (n > 0 && (!aligned16(X) || ((size_t)ld_x * elem_size(x_dtype)) % 16 != 0)) return GQ_ERR_ALIGN;
  // the bf16 kernel addresses a stage of 32 token rows with 32-bit byte offsets and counts stages in 32 bits
  if (x_dtype == GQ_BF16 && (ld_x >= ((int64_t)1 << 26) || n >= ((int64_t)1 << 28))) return GQ_ERR_UNSUPPORTED;
  const size_t need = gq_fisher_gram_workspace_bytes(x_dtype, n, d_in, G);
  if (need > 0 && (!workspace || workspace_bytes < need || !aligned256(workspace))) return GQ_ERR_WORKSPACE;

  hipStream_t st = (hipStream_t)hip_stream;
  const bool accumulate = (flags & GQ_ACCUMULATE) != 0;
  hipError_t e = hipSuccess;
  if (n == 0) {
    if (!accumulate) e = gq::launch_zero_upper(H, d_in, G, st);
  } else if (x_dtype == GQ_F32) {
    e = gq::launch_fisher_gram_f32((const float*)X, n, d_in, ld_x, s, G, H, accumulate, st);
  } else if ((flags & GQ_HEAVY_TWO_TERMS) && !(flags & GQ_TWO_TERMS)) {
    e = gq::launch_fisher_gram_bf16_heavy(X, n, d_in, ld_x, s, G, H, accumulate, workspace, st);
  } else {
    e = gq::launch_fisher_gram_bf16(X, n, d_in, ld_x, s, G, H, accumulate, (flags & GQ_TWO_TERMS) != 0, workspace,
                                    false, st);
  }
  if (e != hipSuccess) return GQ_ERR_HIP;
  if (flags & GQ_MIRROR) e = gq::launch_mirror(H, d_in, G, st);
  return from_hip(e);
}

size_t gq_fisher_gram_heavy_pool_bytes(int64_t d_in, int32_t G, int64_t pool_rows) {
  if (d_in <= 0 || G <= 0 || pool_rows < 32 || pool_rows % 32 != 0 || pool_rows >= ((int64_t)1 << 28)) return 0;
  return gq::fisher_gram_heavy_pool_bytes(d_in, G, pool_rows);
}

int gq_fisher_gram_heavy_deferred(const void* X, gq_dtype x_dtype, int64_t n, int64_t d_in, int64_t ld_x, const float* s,
                                  int32_t G, float* H, uint32_t flags, void* workspace, size_t workspace_bytes, void* pool,
                                  int64_t pool_rows, void* hip_stream) {
  if (!valid_dtype((int)x_dtype)) return GQ_ERR_DTYPE;
  if (x_dtype != GQ_BF16) return GQ_ERR_UNSUPPORTED;
  if (n < 0 || d_in <= 0 || G <= 0 || ld_x < d_in) return GQ_ERR_SHAPE;
  if (pool_rows < 32 || pool_rows % 32 != 0 || pool_rows >= ((int64_t)1 << 28)) return GQ_ERR_SHAPE;
  if (flags & ~(uint32_t)(GQ_ACCUMULATE | GQ_HEAVY_TWO_TERMS)) return GQ_ERR_UNSUPPORTED;
  if (!H || !pool) return GQ_ERR_NULLPTR;
  if (n > 0 && (!X || !s)) return GQ_ERR_NULLPTR;
  if (!aligned16(H) || !aligned256(pool)) return GQ_ERR_ALIGN;
  if (n > 0 && (!aligned16(X) || ((size_t)ld_x * 2) % 16 != 0)) return GQ_ERR_ALIGN;
  if (ld_x >= ((int64_t)1 << 26) || n >= ((int64_t)1 << 28)) return GQ_ERR_UNSUPPORTED;
  const size_t need = gq_fisher_gram_workspace_bytes(x_dtype, n, d_in, G);
  if (need > 0 && (!workspace || workspace_bytes < need || !aligned256(workspace))) return GQ_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool accumulate = (flags & GQ_ACCUMULATE) != 0;
  if (n == 0) return accumulate ? GQ_OK : from_hip(gq::launch_zero_upper(H, d_in, G, st));
  return from_hip(gq::launch_fisher_gram_bf16_heavy_deferred(X, n, d_in, ld_x, s, G, H, accumulate, workspace, pool, pool_rows, st));
}

int gq_fisher_gram_heavy_flush(void* pool, int64_t pool_rows, int64_t d_in, int32_t G, float* H, uint32_t flags,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (d_in <= 0 || G <= 0 || pool_rows < 32 || pool_rows % 32 != 0 || pool_rows >= ((int64_t)1 << 28)) return GQ_ERR_SHAPE;
  if (flags & ~(uint32_t)GQ_MIRROR) return GQ_ERR_UNSUPPORTED;
  if (!H || !pool) return GQ_ERR_NULLPTR;
  if (!aligned16(H) || !aligned256(pool)) return GQ_ERR_ALIGN;
  const size_t need = gq_fisher_gram_workspace_bytes(GQ_BF16, pool_rows, d_in, G);
  if (!workspace || workspace_bytes < need || !aligned256(workspace)) return GQ_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  hipError_t e = gq::launch_fisher_gram_bf16_heavy_flush(pool, pool_rows, d_in, G, H, workspace, st);
  if (e != hipSuccess) return GQ_ERR_HIP;
  if (flags & GQ_MIRROR) e = gq::launch_mirror(H, d_in, G, st);
  return from_hip(e);
}

int gq_fisher_gram_set_xcd_speeds(const float* speeds) {
  if (speeds)
    for (int i = 0; i < 8; ++i)
      if (!(speeds[i] >= 0.5f && speeds[i] <= 2.0f)) return GQ_ERR_SHAPE;
  return from_hip(gq::fisher_gram_set_xcd_speeds(speeds));
}

int gq_fisher_gram_measured_xcd_speeds(int64_t n, int64_t d_in, int32_t G, const void* workspace, float* speeds) {
  if (n <= 0 || d_in <= 0 || G <= 0) return GQ_ERR_SHAPE;
  if (!workspace || !speeds) return GQ_ERR_NULLPTR;
  const hipError_t e = gq::fisher_gram_measured_xcd_speeds(n, d_in, G, workspace, speeds);
  if (e == hipErrorInvalidValue) return GQ_ERR_UNSUPPORTED;
  return from_hip(e);
}

int gq_fisher_mirror(float* H, int64_t d_in, int32_t G, void* hip_stream) {
  if (d_in <= 0 || G <= 0) return GQ_ERR_SHAPE;
  if (!H) return GQ_ERR_NULLPTR;
  if (!aligned16(H)) return GQ_ERR_ALIGN;
  return from_hip(gq::launch_mirror(H, d_in, G, (hipStream_t)hip_stream));
}

int gq_damp_diagonal(float* H, int64_t d_in, int32_t G, double damp_rel, double damp_abs, void* hip_stream) {
  if (d_in <= 0 || G <= 0 || !(damp_rel >= 0.0) || !(damp_abs >= 0.0)) return GQ_ERR_SHAPE;
  if (!H) return GQ_ERR_NULLPTR;
  return from_hip(gq::launch_damp_diagonal(H, d_in, G, damp_rel, damp_abs, (hipStream_t)hip_stream));
}

size_t gq_objective_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0) return 0;
  return gq::objective_workspace(d_out, d_in, G);
}

int gq_objective(const float* W, const float* What, int64_t d_out, int64_t d_in, int64_t ld_w, const float* H,
                 int32_t G, double* obj, float* obj_row, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0 || ld_w < d_in) return GQ_ERR_SHAPE;
  if (!W || !What || !H || !obj) return GQ_ERR_NULLPTR;
  if (!aligned16(W) || !aligned16(What) || !aligned16(H) || ((size_t)ld_w * 4) % 16 != 0) return GQ_ERR_ALIGN;
  const size_t need = gq_objective_workspace_bytes(d_out, d_in, G);
  if (!workspace || workspace_bytes < need || !aligned256(workspace)) return GQ_ERR_WORKSPACE;
  return from_hip(gq::launch_objective(W, What, d_out, d_in, ld_w, H, G, obj, obj_row, workspace,
                                       (hipStream_t)hip_stream));
}

size_t gq_cd_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0) return 0;
  return gq::cd_workspace(d_out, d_in, G);
}

int gq_cd_assign(const float* W, float* What, const float* codebook, int32_t n_levels, int64_t d_out, int64_t d_in,
                 int64_t ld_w, const float* H, int32_t G, int32_t n_cycles, uint8_t* Q, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0 || ld_w < d_in || n_cycles < 0 || n_levels <= 0)
    return GQ_ERR_SHAPE;
  if (n_levels > 16 || d_out > 65535) return GQ_ERR_UNSUPPORTED;
  if (!W || !What || !codebook || !H) return GQ_ERR_NULLPTR;
  if (!aligned16(W) || !aligned16(What) || !aligned16(H) || ((size_t)ld_w * 4) % 16 != 0) return GQ_ERR_ALIGN;
  const size_t need = gq_cd_workspace_bytes(d_out, d_in, G);
  if (!workspace || workspace_bytes < need || !aligned256(workspace)) return GQ_ERR_WORKSPACE;
  if (n_cycles == 0) return GQ_OK;
  return from_hip(gq::launch_cd_assign(W, What, codebook, n_levels, d_out, d_in, ld_w, H, G, n_cycles, Q, workspace, false,
                                       (hipStream_t)hip_stream));
}

size_t gq_cholesky_workspace_bytes(int64_t d_in, int32_t G) {
  if (d_in <= 0 || G <= 0) return 0;
  return gq::cholesky_workspace(d_in, G);
}

int gq_damped_cholesky(const float* H, int64_t d_in, int32_t G, double damp_rel, double damp_abs, uint32_t flags,
                       float* F, int32_t* info, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (d_in <= 0 || G <= 0 || !(damp_rel >= 0.0) || !(damp_abs >= 0.0)) return GQ_ERR_SHAPE;
  if (flags & ~(uint32_t)GQ_CHOL_REVERSE) return GQ_ERR_UNSUPPORTED;
  if (!H || !F) return GQ_ERR_NULLPTR;
  if (H == F) return GQ_ERR_SHAPE;
  if (!aligned16(H) || !aligned16(F)) return GQ_ERR_ALIGN;
  const size_t need = gq_cholesky_workspace_bytes(d_in, G);
  if (!workspace || workspace_bytes < need || !aligned256(workspace)) return GQ_ERR_WORKSPACE;
  return from_hip(gq::launch_damped_cholesky(H, d_in, G, damp_rel, damp_abs, (flags & GQ_CHOL_REVERSE) != 0, F, info,
                                             workspace, (hipStream_t)hip_stream));
}

int gq_ldlq_assign(const float* W, float* What, const float* codebook, int32_t n_levels, int64_t d_out, int64_t d_in,
                   int64_t ld_w, const float* R, int32_t G, uint8_t* Q, void* workspace, size_t workspace_bytes,
                   void* hip_stream) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0 || ld_w < d_in || n_levels <= 0) return GQ_ERR_SHAPE;
  if (n_levels > 16 || d_out > 65535) return GQ_ERR_UNSUPPORTED;
  if (!W || !What || !codebook || !R) return GQ_ERR_NULLPTR;
  if (W == What) return GQ_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(What) || !aligned16(R) || ((size_t)ld_w * 4) % 16 != 0) return GQ_ERR_ALIGN;
  const size_t need = gq_cd_workspace_bytes(d_out, d_in, G);
  if (!workspace || workspace_bytes < need || !aligned256(workspace)) return GQ_ERR_WORKSPACE;
  return from_hip(gq::launch_ldlq_assign(W, What, codebook, n_levels, d_out, d_in, ld_w, R, G, Q, workspace,
                                         (hipStream_t)hip_stream));
}

size_t gq_lnq_codebook_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G, int32_t n_levels) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0 || n_levels <= 0 || n_levels > 16) return 0;
  return gq::lnq_codebook_workspace(d_out, d_in, G, n_levels);
}

int gq_lnq_codebook(const float* W, int64_t d_out, int64_t d_in, int64_t ld_w, const uint8_t* Q, const float* H,
                    int32_t G, int32_t n_levels, double lam, float* codebook, float* What, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0 || ld_w < d_in || n_levels <= 0 || !(lam >= 0.0))
    return GQ_ERR_SHAPE;
  if (n_levels > 16 || d_out > 65535) return GQ_ERR_UNSUPPORTED;
  if (!W || !Q || !H || !codebook) return GQ_ERR_NULLPTR;
  if (!aligned16(W) || (What && !aligned16(What)) || !aligned16(H) || ((size_t)ld_w * 4) % 16 != 0)
    return GQ_ERR_ALIGN;
  const size_t need = gq_lnq_codebook_workspace_bytes(d_out, d_in, G, n_levels);
  if (!workspace || workspace_bytes < need || !aligned256(workspace)) return GQ_ERR_WORKSPACE;
  return from_hip(gq::launch_lnq_codebook(W, d_out, d_in, ld_w, Q, H, G, n_levels, lam, codebook, What, workspace, false,
                                          (hipStream_t)hip_stream));
}

// gq_lnq keeps the two steps' preparations of H (split coefficients of the CD step, the three bf16 terms of
// the codebook step) side by side, so that only the first round of the alternation builds them.
static size_t lnq_cd_part(int64_t d_out, int64_t d_in, int32_t G) {
  return (gq_cd_workspace_bytes(d_out, d_in, G) + 255) / 256 * 256;
}

size_t gq_lnq_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G, int32_t n_levels) {
  const size_t a = gq_cd_workspace_bytes(d_out, d_in, G), b = gq_lnq_codebook_workspace_bytes(d_out, d_in, G, n_levels);
  if (a == 0 || b == 0) return 0;
  return lnq_cd_part(d_out, d_in, G) + b;
}

int gq_lnq(const float* W, float* What, uint8_t* Q, float* codebook, int32_t n_levels, int64_t d_out, int64_t d_in,
           int64_t ld_w, const float* H, int32_t G, int32_t n_iters, int32_t n_cycles, double lam, void* workspace,
           size_t workspace_bytes, void* hip_stream) {
  if (d_out <= 0 || d_in <= 0 || G <= 0 || d_out % G != 0 || ld_w < d_in || n_levels <= 0 || n_iters < 0 ||
      n_cycles < 0 || !(lam >= 0.0))
    return GQ_ERR_SHAPE;
  if (n_levels > 16 || d_out > 65535) return GQ_ERR_UNSUPPORTED;
  if (!W || !What || !Q || !codebook || !H) return GQ_ERR_NULLPTR;
  if (W == What) return GQ_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(What) || !aligned16(H) || ((size_t)ld_w * 4) % 16 != 0) return GQ_ERR_ALIGN;
  const size_t need = gq_lnq_workspace_bytes(d_out, d_in, G, n_levels);
  if (!workspace || workspace_bytes < need || !aligned256(workspace)) return GQ_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  void* ws_cd = workspace;
  void* ws_cb = (char*)workspace + lnq_cd_part(d_out, d_in, G);
  hipError_t e = hipSuccess;
  for (int t = 0; t < n_iters && e == hipSuccess; ++t) {
    e = gq::launch_lnq_codebook(W, d_out, d_in, ld_w, Q, H, G, n_levels, lam, codebook, What, ws_cb, t > 0, st);
    if (e == hipSuccess && n_cycles > 0)
      e = gq::launch_cd_assign(W, What, codebook, n_levels, d_out, d_in, ld_w, H, G, n_cycles, Q, ws_cd, t > 0, st);
  }
  if (e == hipSuccess)
    e = gq::launch_lnq_codebook(W, d_out, d_in, ld_w, Q, H, G, n_levels, lam, codebook, What, ws_cb, n_iters > 0, st);
  return from_hip(e);
}

}  // extern "C"
