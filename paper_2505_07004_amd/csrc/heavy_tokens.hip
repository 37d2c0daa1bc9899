// GQ_HEAVY_TWO_TERMS: positive definiteness of the bf16 Gram for little extra work.
//
// The bf16 path of H[k] = X^T Diag(s[:,k]) X (Algorithm 1, line 4) rounds one operand of every
// product, bf16(s*x).  When the token weights are heavy-tailed (a few tokens carry most of a
// group's weight, as squared output gradients do) the rounding errors of those few tokens do not
// average out, and the result is indefinite by far more than the "small constant on the
// diagonal" of Section 4.2 covers.  Carrying the scaled operand as two bf16 terms repairs that
// at twice the matrix-core work.  The errors that matter belong to the heavy tokens, though:
// here those tokens are taken out of the main call (weight 0) and their rows are gathered into
// a small second call that runs with two terms.  The sum is the same H; only the arithmetic
// of the heavy tokens' products differs.
//
//   heavy(i)  <=>  s[i,k] > kHeavyFactor * mean_i s[i,k]  for some group k   (mean over this call's n tokens)
//
// The first heavy_capacity(n) heavy tokens in token order are gathered; further ones, if any,
// stay in the main call.  Everything is decided on the device in a fixed order (no atomics),
// so identical arguments give identical bits.
//
// Chunked calls.  The second call adds to every entry of H, so a caller that feeds the tokens in chunks pays a
// read-modify-write of the whole H per chunk for a few dozen rows.  The deferred form gathers the heavy rows of
// every chunk into a pool the caller keeps (header: the number of rows in use; then the rows' weights, then the
// rows) and the second call runs once, over the pool, when the caller flushes it.  A full pool leaves further
// heavy tokens in the main calls, as a full capacity does.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr float kHeavyFactor = 16.f;
constexpr int kTokensPerBlock = 1024;                 // of the marking kernels: 256 threads x 4 tokens

inline size_t up256(size_t b) { return (b + 255) & ~(size_t)255; }

struct HeavyLayout {
  int64_t n_blocks, n_cap, ld_h;
  size_t off_sums, off_counts, off_idx, off_smain, off_sh, off_xh, bytes;
};

HeavyLayout heavy_layout(int64_t n, int64_t d_in, int G) {
  HeavyLayout L;
  L.n_blocks = (n + kTokensPerBlock - 1) / kTokensPerBlock;
  L.n_cap = heavy_capacity(n);
  L.ld_h = (d_in + 7) / 8 * 8;
  size_t o = 0;
  L.off_sums = o;   o += up256((size_t)L.n_blocks * G * sizeof(double));
  L.off_counts = o; o += up256(((size_t)L.n_blocks + 1) * sizeof(int));          // [n_blocks] + the total taken
  L.off_idx = o;    o += up256((size_t)L.n_cap * sizeof(int));
  L.off_smain = o;  o += up256((size_t)n * G * sizeof(float));
  L.off_sh = o;     o += up256((size_t)L.n_cap * G * sizeof(float));
  L.off_xh = o;     o += up256((size_t)L.n_cap * L.ld_h * 2);
  L.bytes = o;
  return L;
}

// Per block of 1024 tokens and group: the sum of the weights in fp64, threads in a fixed tree.
__global__ __launch_bounds__(256) void heavy_sums_kernel(const float* __restrict__ s, int64_t n, int G,
                                                         double* __restrict__ sums) {
  __shared__ double red[256];
  const int64_t t0 = (int64_t)blockIdx.x * kTokensPerBlock;
  for (int k = 0; k < G; ++k) {
    double a = 0.0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t t = t0 + threadIdx.x + 256 * u;
      if (t < n) a += (double)s[t * G + k];
    }
    red[threadIdx.x] = a;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0) sums[(int64_t)blockIdx.x * G + k] = red[0];
    __syncthreads();
  }
}

// The threshold of group k: kHeavyFactor times the mean.  Thread t adds the block sums t, t + 256, ... in
// that order, then the 256 partial sums are added in a fixed tree (fp64).
__device__ inline void heavy_thresholds(const double* __restrict__ sums, int64_t n_blocks, int64_t n, int G,
                                        float* thr /* LDS, G entries */) {
  __shared__ double tred[256];
  for (int k = 0; k < G; ++k) {
    double a = 0.0;
    for (int64_t b = threadIdx.x; b < n_blocks; b += 256) a += sums[b * G + k];
    tred[threadIdx.x] = a;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w) tred[threadIdx.x] += tred[threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0) thr[k] = (float)(tred[0] / (double)n) * kHeavyFactor;
    __syncthreads();
  }
}

__device__ inline bool heavy_token(const float* __restrict__ s, int64_t t, int G, const float* thr) {
  bool h = false;
  for (int k = 0; k < G; ++k) h = h || (s[t * G + k] > thr[k]);
  return h;
}

// counts[b] = heavy tokens among the 1024 of block b.
__global__ __launch_bounds__(256) void heavy_count_kernel(const float* __restrict__ s, int64_t n, int G,
                                                          const double* __restrict__ sums, int64_t n_blocks,
                                                          int* __restrict__ counts) {
  extern __shared__ float thr[];
  __shared__ int red[256];
  heavy_thresholds(sums, n_blocks, n, G, thr);
  const int64_t t0 = (int64_t)blockIdx.x * kTokensPerBlock + 4 * (int64_t)threadIdx.x;
  int c = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (t0 + u < n && heavy_token(s, t0 + u, G, thr)) ++c;
  red[threadIdx.x] = c;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) counts[blockIdx.x] = red[0];
}

// Positions in token order: heavy token number q < n_cap goes to idx[q] and gets weight 0 in
// s_main; all other tokens keep their weights.  counts[n_blocks] receives min(total, n_cap).
__global__ __launch_bounds__(256) void heavy_assign_kernel(const float* __restrict__ s, int64_t n, int G,
                                                           const double* __restrict__ sums, int64_t n_blocks,
                                                           int* __restrict__ counts, int n_cap, int* __restrict__ idx,
                                                           float* __restrict__ s_main, const int* __restrict__ pool_cursor,
                                                           int pool_rows) {
  if (pool_cursor) {                                 // deferred form: no more than the pool still takes
    const int room = pool_rows - *pool_cursor;
    n_cap = room < n_cap ? (room > 0 ? room : 0) : n_cap;
  }
  extern __shared__ float thr[];
  __shared__ long long red[256];
  __shared__ int scan[256];
  heavy_thresholds(sums, n_blocks, n, G, thr);
  // heavy tokens before this block (thread-strided partial sums, fixed tree; integers, so exact)
  long long before = 0;
  for (int64_t b = threadIdx.x; b < (int64_t)blockIdx.x; b += 256) before += counts[b];
  red[threadIdx.x] = before;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  const long long base = red[0];
  const int64_t t0 = (int64_t)blockIdx.x * kTokensPerBlock + 4 * (int64_t)threadIdx.x;
  bool h[4];
  int c = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    h[u] = t0 + u < n && heavy_token(s, t0 + u, G, thr);
    c += h[u] ? 1 : 0;
  }
  scan[threadIdx.x] = c;
  __syncthreads();
  for (int w = 1; w < 256; w <<= 1) {                       // inclusive scan over the threads
    const int v = (int)threadIdx.x >= w ? scan[threadIdx.x - w] : 0;
    __syncthreads();
    scan[threadIdx.x] += v;
    __syncthreads();
  }
  long long q = base + scan[threadIdx.x] - c;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t t = t0 + u;
    if (t >= n) break;
    const bool take = h[u] && q < n_cap;
    if (take) idx[q] = (int)t;
    if (h[u]) ++q;
    for (int k = 0; k < G; ++k) s_main[t * G + k] = take ? 0.f : s[t * G + k];
  }
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 255) {
    const long long total = base + scan[255];
    counts[n_blocks] = (int)(total < n_cap ? total : n_cap);
  }
}

// Row r of the gathered operands: token idx[r] for r < taken, else a row of zeros with weight 0.
// 16 bytes per thread and step; ld of X and ld_h are multiples of 8 elements.
__global__ __launch_bounds__(256) void heavy_gather_kernel(const __bf16* __restrict__ X, int64_t d_in, int64_t ld,
                                                           const float* __restrict__ s, int G,
                                                           const int* __restrict__ idx, const int* __restrict__ taken,
                                                           int64_t ld_h, __bf16* __restrict__ Xh, float* __restrict__ sh) {
  const int r = blockIdx.x;
  const bool live = r < *taken;
  const int64_t t = live ? idx[r] : 0;
  const uint4* src = reinterpret_cast<const uint4*>(X + t * ld);
  uint4* dst = reinterpret_cast<uint4*>(Xh + (int64_t)r * ld_h);
  const int64_t chunks = ld_h / 8, src_chunks = (d_in + 7) / 8;     // the last source chunk lies within the row pitch
  for (int64_t c = threadIdx.x; c < chunks; c += 256) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (live && c < src_chunks) v = src[c];
    dst[c] = v;
  }
  for (int k = threadIdx.x; k < G; k += 256) sh[(int64_t)r * G + k] = live ? s[t * G + k] : 0.f;
}

// ---- the pool of the deferred form ---------------------------------------------------------------
struct PoolLayout {
  int64_t ld_h;
  size_t off_s, off_x, bytes;
};
PoolLayout pool_layout(int64_t d_in, int G, int64_t rows) {
  PoolLayout P;
  P.ld_h = (d_in + 7) / 8 * 8;
  size_t o = 256;                                             // header: [0] = rows in use
  P.off_s = o; o += up256((size_t)rows * G * sizeof(float));
  P.off_x = o; o += up256((size_t)rows * P.ld_h * 2);
  P.bytes = o;
  return P;
}

// Row r of this call's heavy tokens goes to pool row cursor + r; the rows from there up to the next multiple
// of 32 are cleared (weights 0), so that the pass over the pool can always run whole token steps.
__global__ __launch_bounds__(256) void heavy_gather_pool_kernel(const __bf16* __restrict__ X, int64_t d_in, int64_t ld,
                                                                const float* __restrict__ s, int G,
                                                                const int* __restrict__ idx, const int* __restrict__ taken,
                                                                const int* __restrict__ cursor, int64_t ld_h,
                                                                __bf16* __restrict__ Xp, float* __restrict__ sp) {
  const int r = blockIdx.x, n_taken = *taken, base = *cursor;
  const int end32 = (base + n_taken + 31) / 32 * 32;
  const bool live = r < n_taken;
  if (!live && base + r >= end32) return;                      // uniform for the block
  const int64_t t = live ? idx[r] : 0;
  const uint4* src = reinterpret_cast<const uint4*>(X + t * ld);
  uint4* dst = reinterpret_cast<uint4*>(Xp + (int64_t)(base + r) * ld_h);
  const int64_t chunks = ld_h / 8, src_chunks = (d_in + 7) / 8;
  for (int64_t c = threadIdx.x; c < chunks; c += 256) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (live && c < src_chunks) v = src[c];
    dst[c] = v;
  }
  for (int k = threadIdx.x; k < G; k += 256) sp[(int64_t)(base + r) * G + k] = live ? s[t * G + k] : 0.f;
}
__global__ void heavy_pool_advance_kernel(int* __restrict__ cursor, const int* __restrict__ taken) {
  if (threadIdx.x == 0 && blockIdx.x == 0) *cursor += *taken;
}
// An empty pool: no rows in use, and a first token step of weight 0 (the pass over the pool runs at least one).
__global__ __launch_bounds__(256) void heavy_pool_reset_kernel(int* __restrict__ cursor, float* __restrict__ sp, int G) {
  for (int i = threadIdx.x; i < 32 * G; i += 256) sp[i] = 0.f;
  if (threadIdx.x == 0) *cursor = 0;
}

}  // namespace

size_t fisher_gram_heavy_pool_bytes(int64_t d_in, int G, int64_t rows) { return pool_layout(d_in, G, rows).bytes; }

hipError_t launch_fisher_gram_bf16_heavy_deferred(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                                  float* H, bool accumulate, void* ws, void* pool, int64_t pool_rows,
                                                  hipStream_t st) {
  const HeavyLayout L = heavy_layout(n, d_in, G);
  const PoolLayout P = pool_layout(d_in, G, pool_rows);
  const size_t a = fisher_gram_bf16_workspace(n, d_in, G), b = fisher_gram_bf16_workspace(L.n_cap, d_in, G);
  char* hw = (char*)ws + up256(a > b ? a : b);
  double* sums = (double*)(hw + L.off_sums);
  int* counts = (int*)(hw + L.off_counts);
  int* idx = (int*)(hw + L.off_idx);
  float* s_main = (float*)(hw + L.off_smain);
  int* cursor = (int*)pool;
  float* s_p = (float*)((char*)pool + P.off_s);
  __bf16* X_p = (__bf16*)((char*)pool + P.off_x);
  const dim3 grid((unsigned)L.n_blocks), block(256);
  const size_t thr_bytes = (size_t)G * sizeof(float);
  heavy_sums_kernel<<<grid, block, 0, st>>>(s, n, G, sums);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  heavy_count_kernel<<<grid, block, thr_bytes, st>>>(s, n, G, sums, L.n_blocks, counts);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  heavy_assign_kernel<<<grid, block, thr_bytes, st>>>(s, n, G, sums, L.n_blocks, counts, (int)L.n_cap, idx, s_main, cursor,
                                                      (int)pool_rows);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  heavy_gather_pool_kernel<<<dim3((unsigned)(L.n_cap + 32)), block, 0, st>>>((const __bf16*)X, d_in, ld, s, G, idx,
                                                                           counts + L.n_blocks, cursor, P.ld_h, X_p, s_p);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  heavy_pool_advance_kernel<<<dim3(1), dim3(64), 0, st>>>(cursor, counts + L.n_blocks);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return launch_fisher_gram_bf16(X, n, d_in, ld, s_main, G, H, accumulate, false, ws, false, st);
}

hipError_t launch_fisher_gram_bf16_heavy_flush(void* pool, int64_t pool_rows, int64_t d_in, int G, float* H, void* ws,
                                               hipStream_t st) {
  const PoolLayout P = pool_layout(d_in, G, pool_rows);
  int* cursor = (int*)pool;
  float* s_p = (float*)((char*)pool + P.off_s);
  const __bf16* X_p = (const __bf16*)((char*)pool + P.off_x);
  hipError_t e = launch_fisher_gram_bf16(X_p, pool_rows, d_in, P.ld_h, s_p, G, H, true, true, ws, false, st, cursor);
  if (e != hipSuccess) return e;
  heavy_pool_reset_kernel<<<dim3(1), dim3(256), 0, st>>>(cursor, s_p, G);
  return hipGetLastError();
}

int64_t heavy_capacity(int64_t n) { return 32 * ((n + 2047) / 2048 > 0 ? (n + 2047) / 2048 : 1); }

size_t fisher_gram_heavy_workspace(int64_t n, int64_t d_in, int G) {
  const HeavyLayout L = heavy_layout(n, d_in, G);
  const size_t a = fisher_gram_bf16_workspace(n, d_in, G), b = fisher_gram_bf16_workspace(L.n_cap, d_in, G);
  return up256(a > b ? a : b) + L.bytes;
}

hipError_t launch_fisher_gram_bf16_heavy(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                         float* H, bool accumulate, void* ws, hipStream_t st) {
  const HeavyLayout L = heavy_layout(n, d_in, G);
  const size_t a = fisher_gram_bf16_workspace(n, d_in, G), b = fisher_gram_bf16_workspace(L.n_cap, d_in, G);
  char* hw = (char*)ws + up256(a > b ? a : b);
  double* sums = (double*)(hw + L.off_sums);
  int* counts = (int*)(hw + L.off_counts);
  int* idx = (int*)(hw + L.off_idx);
  float* s_main = (float*)(hw + L.off_smain);
  float* s_h = (float*)(hw + L.off_sh);
  __bf16* X_h = (__bf16*)(hw + L.off_xh);
  const dim3 grid((unsigned)L.n_blocks), block(256);
  const size_t thr_bytes = (size_t)G * sizeof(float);
  heavy_sums_kernel<<<grid, block, 0, st>>>(s, n, G, sums);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  heavy_count_kernel<<<grid, block, thr_bytes, st>>>(s, n, G, sums, L.n_blocks, counts);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  heavy_assign_kernel<<<grid, block, thr_bytes, st>>>(s, n, G, sums, L.n_blocks, counts, (int)L.n_cap, idx, s_main,
                                                      nullptr, 0);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  heavy_gather_kernel<<<dim3((unsigned)L.n_cap), block, 0, st>>>((const __bf16*)X, d_in, ld, s, G, idx,
                                                                counts + L.n_blocks, L.ld_h, X_h, s_h);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  e = launch_fisher_gram_bf16(X, n, d_in, ld, s_main, G, H, accumulate, false, ws, false, st);
  if (e != hipSuccess) return e;
  // the gathered rows past the number taken are zero: the second pass runs over the token steps in use only
  return launch_fisher_gram_bf16(X_h, L.n_cap, d_in, L.ld_h, s_h, G, H, true, true, ws, false, st, counts + L.n_blocks);
}

}  // namespace gq
