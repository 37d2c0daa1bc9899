// GuidedQuant layer objective (Eq. "ours2", Section 3.2):
//   obj_row[j] = delta_j^T H[k(j)] delta_j,  delta_j = W[j,:] - What[j,:],  obj[k] = sum_{j in J_k} obj_row[j].
//
// Only the upper triangle of H is read:  delta^T H delta = sum_{a<=b in tile terms} ... =
//   2 * sum_{tiles ta < tb} delta_a^T H[ta,tb] delta_b + sum_{tb} delta_b^T H[tb,tb] delta_b,
// where the diagonal tile is completed to a full symmetric tile while it is staged.
// A workgroup owns 128 channels (rows j) x one 128-wide column tile tb of one group and
// contracts over all tiles ta <= tb on the fp32 matrix cores (v_mfma_f32_32x32x2_f32):
//   Y[j,b] = 2 * sum_{a in tiles < tb} delta[j,a] H[a,b] + sum_{a in tile tb} delta[j,a] Hsym[a,b]
// then partial[tb][j] = sum_b Y[j,b] * delta[j,b].  A second kernel adds the partials of a
// row in fixed order (fp32 obj_row) and the rows of a group in fp64 (obj): deterministic.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kTile = 128;
constexpr int kStep = 16;
constexpr int kDPitch = kStep + 1;    // delta tile [128 rows j][16 a], odd pitch: column reads hit distinct banks
constexpr int kHPitch = kTile + 32;   // H tile [16 a][128 b]

__global__ __launch_bounds__(256) void objective_partial_kernel(const float* __restrict__ W,
                                                                const float* __restrict__ What, int64_t d_out,
                                                                int64_t d, int64_t ld, const float* __restrict__ H,
                                                                int G, int n_tb, int n_rb, float* __restrict__ partial) {
  __shared__ float Ds[2][kTile][kDPitch];
  __shared__ __attribute__((aligned(16))) float Hs[2][kStep][kHPitch];
  __shared__ float red[2][kTile];

  const int tb = n_tb - 1 - (int)(blockIdx.x % n_tb);  // heavy column tiles first
  const int rb = (int)(blockIdx.x / n_tb);
  const int k = blockIdx.y;
  const int64_t m = d_out / G;
  const int64_t j0 = (int64_t)k * m + (int64_t)rb * kTile;  // first channel of this block
  const int64_t j_end = (int64_t)(k + 1) * m;               // rows >= j_end belong to another group
  const int64_t b0 = (int64_t)tb * kTile;
  const float* Hk = H + (int64_t)k * d * d;

  const int tid = threadIdx.x;
  const int lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / 2, wn = wave % 2;

  f32x16 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // staging assignment.  delta: 128 rows x 16 a = 512 float4 -> 2 per thread (row = q/4, a4 = q%4).
  // H: 16 a x 128 b = 512 float4 -> 2 per thread (row = q/32, b4 = q%32).
  f32x4 rd[2], rh[2];
  auto fetch = [&](int ta, int kk) {  // kk: a-offset inside tile ta
    const int64_t abase = (int64_t)ta * kTile + kk;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int q = tid + 256 * h;
      {  // delta
        const int64_t j = j0 + q / 4;
        const int64_t a = abase + 4 * (q % 4);
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (j < j_end) {
          const float* pw = W + j * ld + a;
          const float* ph = What + j * ld + a;
          if (a + 4 <= d) {
            f32x4 w4 = *reinterpret_cast<const f32x4*>(pw);
            f32x4 h4 = *reinterpret_cast<const f32x4*>(ph);
            v = w4 - h4;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (a + e < d) v[e] = pw[e] - ph[e];
          }
        }
        rd[h] = v;
      }
      {  // H rows a, columns b0.. ; on the diagonal tile entries below the diagonal come from the transpose
        const int64_t a = abase + q / 32;
        const int64_t b = b0 + 4 * (q % 32);
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (a < d) {
          if (ta != tb && b + 4 <= d && (d & 3) == 0) {
            v = *reinterpret_cast<const f32x4*>(Hk + a * d + b);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int64_t bb = b + e;
              if (bb < d) v[e] = (a <= bb) ? Hk[a * d + bb] : Hk[bb * d + a];
            }
          }
        }
        rh[h] = v;
      }
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int q = tid + 256 * h;
#pragma unroll
      for (int e = 0; e < 4; ++e) Ds[buf][q / 4][4 * (q % 4) + e] = rd[h][e];
      *reinterpret_cast<f32x4*>(&Hs[buf][q / 32][4 * (q % 32)]) = rh[h];
    }
  };

  constexpr int kSub = kTile / kStep;  // 8 stages per a-tile
  const int total = (tb + 1) * kSub;
  fetch(0, 0);
  stash(0);
  __syncthreads();
  for (int it = 0; it < total; ++it) {
    const int buf = it & 1;
    const int ta = it / kSub;
    if (it + 1 < total) fetch((it + 1) / kSub, ((it + 1) % kSub) * kStep);
#pragma unroll
    for (int kk = 0; kk < kStep; kk += 2) {
      float av[2], bv[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) av[x] = Ds[buf][wm * 64 + x * 32 + lane % 32][kk + lane / 32];
#pragma unroll
      for (int y = 0; y < 2; ++y) bv[y] = Hs[buf][kk + lane / 32][wn * 64 + y * 32 + lane % 32];
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[x], bv[y], acc[x][y], 0, 0, 0);
    }
    // all strictly-upper tiles are done: they count twice (their mirror images are never visited)
    if (ta < tb && (it + 1) / kSub == tb) {
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] *= 2.f;
    }
    if (it + 1 < total) stash(buf ^ 1);
    __syncthreads();
  }

  // row dot with delta[j, b]: register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32
  float rowsum[2][16];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t j = j0 + wm * 64 + x * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
      float v = 0.f;
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        const int64_t b = b0 + wn * 64 + y * 32 + lane % 32;
        if (j < j_end && b < d) v += acc[x][y][r] * (W[j * ld + b] - What[j * ld + b]);
      }
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
      rowsum[x][r] = v;
    }
  if (lane % 32 == 0) {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        red[wn][wm * 64 + x * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4)] = rowsum[x][r];
  }
  __syncthreads();
  if (tid < kTile) {
    const int64_t j = j0 + tid;
    if (j < j_end) partial[(int64_t)tb * d_out + j] = red[0][tid] + red[1][tid];
  }
}

// obj_row[j] = sum_tb partial[tb][j] (fixed order); obj[k] = fp64 sum over the group's rows.
__global__ __launch_bounds__(256) void objective_reduce_kernel(const float* __restrict__ partial, int64_t d_out,
                                                               int G, int n_tb, float* __restrict__ obj_row,
                                                               double* __restrict__ obj) {
  __shared__ double red[256];
  const int k = blockIdx.x;
  const int64_t m = d_out / G;
  double acc = 0.0;
  for (int64_t jj = threadIdx.x; jj < m; jj += 256) {
    const int64_t j = (int64_t)k * m + jj;
    float v = 0.f;
    for (int tb = 0; tb < n_tb; ++tb) v += partial[(int64_t)tb * d_out + j];
    if (obj_row) obj_row[j] = v;
    acc += (double)v;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) obj[k] = red[0];
}

}  // namespace

size_t objective_workspace(int64_t d_out, int64_t d_in, int G) {
  (void)G;
  const int64_t n_tb = (d_in + kTile - 1) / kTile;
  return (size_t)(n_tb * d_out) * sizeof(float);
}

hipError_t launch_objective(const float* W, const float* What, int64_t d_out, int64_t d_in, int64_t ld,
                            const float* H, int G, double* obj, float* obj_row, void* ws, hipStream_t st) {
  const int64_t m = d_out / G;
  const int n_tb = (int)((d_in + kTile - 1) / kTile);
  const int n_rb = (int)((m + kTile - 1) / kTile);
  float* partial = (float*)ws;
  objective_partial_kernel<<<dim3((unsigned)(n_tb * n_rb), (unsigned)G), dim3(256), 0, st>>>(
      W, What, d_out, d_in, ld, H, G, n_tb, n_rb, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  objective_reduce_kernel<<<dim3((unsigned)G), dim3(256), 0, st>>>(partial, d_out, G, n_tb, obj_row, obj);
  return hipGetLastError();
}

}  // namespace gq
