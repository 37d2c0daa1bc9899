// fp32 path of the grouped Fisher Gram, H[k] (+)= X^T Diag(s[:,k]) X on upper-triangle
// tiles (GuidedQuant, Algorithm 1, line 4).
//
// One workgroup (4 waves, 2x2) owns one 128x128 output tile of one group and walks over
// the tokens in steps of 16.  Rows of X are staged through LDS exactly as they lie in
// memory ([token][column]); the "row" operand is multiplied by s[token, k] in fp32 while
// it is staged.  The contraction runs on the fp32 matrix cores (v_mfma_f32_32x32x2_f32),
// whose operand layout (lane -> column l%32, token l/32) reads that LDS tile row-wise, so no
// transpose is needed.  Accumulators are flushed into a second-level sum every 2048
// tokens to keep fp32 accumulation error well below the 1e-5 parity bar at large n.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kTile = 128;          // output tile edge
constexpr int kStep = 16;           // tokens per LDS stage
constexpr int kPitch = kTile + 32;  // floats; +32 keeps the two token rows of one MFMA read on disjoint banks
constexpr int kFlush = 2048 / kStep;

__device__ inline f32x4 load_row4(const float* __restrict__ X, int64_t ld, int64_t n, int64_t d, int64_t i,
                                  int64_t c) {
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (i < n) {
    const float* p = X + i * ld + c;
    if (c + 4 <= d) {
      v = *reinterpret_cast<const f32x4*>(p);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (c + e < d) v[e] = p[e];
    }
  }
  return v;
}

__global__ __launch_bounds__(256) void fisher_gram_f32_kernel(const float* __restrict__ X, int64_t n, int64_t d,
                                                              int64_t ld, const float* __restrict__ s, int G,
                                                              float* __restrict__ H, int accumulate) {
  __shared__ __attribute__((aligned(16))) float As[2][kStep][kPitch];
  __shared__ __attribute__((aligned(16))) float Bs[2][kStep][kPitch];

  const int k = blockIdx.y;
  int ti, tj;
  tri_decode(blockIdx.x, ti, tj);  // ti <= tj
  const int64_t a0 = (int64_t)ti * kTile, b0 = (int64_t)tj * kTile;

  const int tid = threadIdx.x;
  const int lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / 2, wn = wave % 2;  // wave's 64x64 quadrant

  // staging assignment: 16 rows x 32 float4 per operand = 512 float4, two per thread
  const int lrow = tid / 32;        // 0..7 (and +8)
  const int lcol = (tid % 32) * 4;  // column inside the tile

  f32x16 acc[2][2], tot[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[x][y][r] = 0.f; tot[x][y][r] = 0.f; }

  const int64_t steps = (n + kStep - 1) / kStep;
  f32x4 ra[2], rb[2];
  float rs[2];
  auto fetch = [&](int64_t step) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int64_t i = step * kStep + lrow + 8 * h;
      ra[h] = load_row4(X, ld, n, d, i, a0 + lcol);
      rb[h] = load_row4(X, ld, n, d, i, b0 + lcol);
      rs[h] = (i < n) ? s[i * G + k] : 0.f;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      f32x4 sa = {ra[h][0] * rs[h], ra[h][1] * rs[h], ra[h][2] * rs[h], ra[h][3] * rs[h]};
      *reinterpret_cast<f32x4*>(&As[buf][lrow + 8 * h][lcol]) = sa;
      *reinterpret_cast<f32x4*>(&Bs[buf][lrow + 8 * h][lcol]) = rb[h];
    }
  };

  if (steps > 0) {
    fetch(0);
    stash(0);
  }
  __syncthreads();
  for (int64_t step = 0; step < steps; ++step) {
    const int buf = (int)(step & 1);
    if (step + 1 < steps) fetch(step + 1);
#pragma unroll
    for (int kk = 0; kk < kStep; kk += 2) {
      float av[2], bv[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) av[x] = As[buf][kk + lane / 32][wm * 64 + x * 32 + lane % 32];
#pragma unroll
      for (int y = 0; y < 2; ++y) bv[y] = Bs[buf][kk + lane / 32][wn * 64 + y * 32 + lane % 32];
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[x], bv[y], acc[x][y], 0, 0, 0);
    }
    if ((step + 1) % kFlush == 0) {
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
          tot[x][y] += acc[x][y];
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;
        }
    }
    if (step + 1 < steps) stash(buf ^ 1);
    __syncthreads();
  }

  // epilogue: accumulator register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32
  float* Hk = H + (int64_t)k * d * d;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int64_t col = b0 + wn * 64 + y * 32 + lane % 32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = a0 + wm * 64 + x * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        if (row < d && col < d && row <= col) {
          float v = tot[x][y][r] + acc[x][y][r];
          float* p = Hk + row * d + col;
          if (accumulate) v += *p;
          *p = v;
        }
      }
    }
}

}  // namespace

hipError_t launch_fisher_gram_f32(const float* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                  float* H, bool accumulate, hipStream_t st) {
  const int64_t T = (d_in + kTile - 1) / kTile;
  fisher_gram_f32_kernel<<<dim3((unsigned)tri_count(T), (unsigned)G), dim3(256), 0, st>>>(X, n, d_in, ld, s, G, H,
                                                                                         accumulate ? 1 : 0);
  return hipGetLastError();
}

}  // namespace gq
