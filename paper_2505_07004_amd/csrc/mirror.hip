// Triangle utilities for the cached Hessians H[G, d_in, d_in]:
//  - mirror: H[k][b,a] = H[k][a,b] for a < b (the paper stores full squares; the Gram
//    kernels only produce the upper triangle),
//  - zero_upper: clear the upper triangle (an overwrite call with no tokens).
// Both are HBM-bound copies through a padded LDS tile.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kT = 64;  // tile edge

__global__ __launch_bounds__(256) void mirror_kernel(float* __restrict__ H, int64_t d, int64_t n_tri) {
  __shared__ float tile[kT][kT + 1];
  const int k = blockIdx.y;
  float* Hk = H + (int64_t)k * d * d;
  int ti, tj;
  tri_decode(blockIdx.x, ti, tj);  // ti <= tj
  const int64_t r0 = (int64_t)ti * kT, c0 = (int64_t)tj * kT;
  const int tx = threadIdx.x % kT, ty = threadIdx.x / kT;  // 64 x 4
  // branch-free (clamped addresses): the 16 loads of a thread are in flight together
#pragma unroll
  for (int u = 0; u < kT / 4; ++u) {
    const int r = ty + 4 * u;
    const int64_t a = r0 + r, b = c0 + tx;
    const int64_t ac = a < d ? a : d - 1, bc = b < d ? b : d - 1;
    tile[r][tx] = Hk[ac * d + bc];
  }
  __syncthreads();
  // write the transposed tile: rows b in tile tj, columns a in tile ti
  for (int r = ty; r < kT; r += 4) {
    const int64_t b = c0 + r, a = r0 + tx;
    if (a < d && b < d && a < b) Hk[b * d + a] = tile[tx][r];
  }
}

__global__ __launch_bounds__(256) void zero_upper_kernel(float* __restrict__ H, int64_t d) {
  const int k = blockIdx.y;
  float* Hk = H + (int64_t)k * d * d;
  int ti, tj;
  tri_decode(blockIdx.x, ti, tj);
  const int64_t r0 = (int64_t)ti * kT, c0 = (int64_t)tj * kT;
  const int tx = threadIdx.x % kT, ty = threadIdx.x / kT;
  for (int r = ty; r < kT; r += 4) {
    const int64_t a = r0 + r, b = c0 + tx;
    if (a < d && b < d && a <= b) Hk[a * d + b] = 0.f;
  }
}

// H[k][i][i] += damp_abs + damp_rel * mean_i H[k][i][i].  One workgroup per group: the mean in fp64
// in a fixed order, then the diagonal.
__global__ __launch_bounds__(256) void damp_diagonal_kernel(float* __restrict__ H, int64_t d, double damp_rel,
                                                            double damp_abs) {
  __shared__ double part[256];
  float* Hk = H + (int64_t)blockIdx.x * d * d;
  double acc = 0.0;
  for (int64_t i = threadIdx.x; i < d; i += 256) acc += (double)Hk[i * d + i];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  const double eps = damp_abs + damp_rel * (part[0] / (double)d);
  for (int64_t i = threadIdx.x; i < d; i += 256) Hk[i * d + i] = (float)((double)Hk[i * d + i] + eps);
}

}  // namespace

hipError_t launch_damp_diagonal(float* H, int64_t d_in, int G, double damp_rel, double damp_abs, hipStream_t st) {
  damp_diagonal_kernel<<<dim3((unsigned)G), dim3(256), 0, st>>>(H, d_in, damp_rel, damp_abs);
  return hipGetLastError();
}

hipError_t launch_mirror(float* H, int64_t d_in, int G, hipStream_t st) {
  const int64_t T = (d_in + kT - 1) / kT;
  mirror_kernel<<<dim3((unsigned)tri_count(T), (unsigned)G), dim3(256), 0, st>>>(H, d_in, tri_count(T));
  return hipGetLastError();
}

hipError_t launch_zero_upper(float* H, int64_t d_in, int G, hipStream_t st) {
  const int64_t T = (d_in + kT - 1) / kT;
  zero_upper_kernel<<<dim3((unsigned)tri_count(T), (unsigned)G), dim3(256), 0, st>>>(H, d_in);
  return hipGetLastError();
}

}  // namespace gq
