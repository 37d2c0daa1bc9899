// GuidedQuant layer objective (Eq. "ours2", Section 3.2):
//   obj_row[j] = delta_j^T H[k(j)] delta_j,  delta_j = W[j,:] - What[j,:],  obj[k] = sum_{j in J_k} obj_row[j].
//
// The contraction Y = Delta_k H_k (2 d_out d_in^2 flop) runs on the bf16 matrix cores at
// fp32-grade accuracy by splitting both operands into two bf16 terms, x = hi + lo with
// hi = bf16(x), lo = bf16(x - hi) (together 16 mantissa bits), and summing the three products
// hi*hi + hi*lo + lo*hi in fp32 accumulators (the dropped lo*lo term is below 2^-16 relative).
// Only the upper triangle of H is read.  In tile terms
//   delta^T H delta = 2 * sum_{ta < tb} delta_a^T H[ta,tb] delta_b + sum_tb delta_b^T H[tb,tb] delta_b,
// so a workgroup that owns 128 channels (rows j) and one 128-wide column tile tb contracts only
// over a < (tb+1)*128, doubles its accumulators before the diagonal tile, and finishes with
// partial[tb][j] = sum_b Y[j,b] * delta[j,b] in fp32.
//
// Kernels: (1) split delta into hi/lo bf16 [d_out, d_in]; (2) split H into hi/lo bf16 written
// TRANSPOSED (Hs[k][b][a] = H[k][a][b] for a <= b, the diagonal 128-tiles completed to full
// squares), which makes both MFMA operands contiguous along the contraction index a;
// (3) the MFMA kernel; (4) a two-step reduction that adds the partials of a row in fixed order
// (fp32 obj_row) and the rows of a group in fp64 (obj).  Everything is deterministic.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kTile = 128;            // rows j and columns b per workgroup
constexpr int kKS = 32;               // contraction elements per LDS stage (2 stages x 4 tiles = 80 KiB: two workgroups per CU)
constexpr int kPitch = kKS * 2 + 16;  // LDS bytes per tile row: an odd number (5) of 16-byte granules => conflict-free b128 reads
constexpr int kChunks = kKS / 8;      // 16-byte chunks per tile row
constexpr int kTileLoads = kTile * kChunks / 256;   // chunks per thread and tile
constexpr int kTileBytes = kTile * kPitch;

__device__ inline void split_bf16(float x, unsigned short& hi, unsigned short& lo) {
  const __bf16 h = (__bf16)x;
  const __bf16 l = (__bf16)(x - (float)h);
  hi = __builtin_bit_cast(unsigned short, h);
  lo = __builtin_bit_cast(unsigned short, l);
}

// Dh/Dl[j, a] = hi/lo of W[j,a] - What[j,a]; row pitch ldp (multiple of kKS, zero padded).
__global__ __launch_bounds__(256) void split_delta_kernel(const float* __restrict__ W, const float* __restrict__ What,
                                                          int64_t d_out, int64_t d, int64_t ld, int64_t ldp,
                                                          unsigned short* __restrict__ Dh,
                                                          unsigned short* __restrict__ Dl) {
  const int64_t j = blockIdx.y;
  for (int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x; a < ldp; a += (int64_t)gridDim.x * 256) {
    const float v = a < d ? W[j * ld + a] - What[j * ld + a] : 0.f;
    unsigned short h, l;
    split_bf16(v, h, l);
    Dh[j * ldp + a] = h;
    Dl[j * ldp + a] = l;
  }
}

// Hh/Hl[k][b][a] = hi/lo of H[k][a][b] for a <= b; inside a diagonal 128-tile also [a][b].
// One workgroup per 64x64 tile (ti <= tj) of the upper triangle, transposed through LDS.
__global__ __launch_bounds__(256) void split_h_kernel(const float* __restrict__ H, int64_t d, int64_t ldp,
                                                      unsigned short* __restrict__ Hh,
                                                      unsigned short* __restrict__ Hl) {
  __shared__ float tile[64][65];
  const int k = blockIdx.y;
  const float* Hk = H + (int64_t)k * d * d;
  unsigned short* Hhk = Hh + (int64_t)k * ldp * ldp;
  unsigned short* Hlk = Hl + (int64_t)k * ldp * ldp;
  int ti, tj;
  tri_decode(blockIdx.x, ti, tj);
  const int64_t r0 = (int64_t)ti * 64, c0 = (int64_t)tj * 64;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  for (int r = ty; r < 64; r += 4) {
    const int64_t a = r0 + r, b = c0 + tx;
    tile[r][tx] = (a < d && b < d && a <= b) ? Hk[a * d + b] : 0.f;
  }
  __syncthreads();
  const bool same128 = (ti / 2 == tj / 2);
  for (int r = ty; r < 64; r += 4) {
    // transposed position: row b = c0 + r, column a = r0 + tx
    const int64_t b = c0 + r, a = r0 + tx;
    if (a < ldp && b < ldp) {
      float v = 0.f;
      if (a <= b) v = tile[tx][r];
      else if (ti == tj) v = tile[r][tx];          // below the diagonal inside a diagonal 64-tile: the mirror image
      if (a <= b || ti == tj) {
        unsigned short h, l;
        split_bf16(v, h, l);
        Hhk[b * ldp + a] = h;
        Hlk[b * ldp + a] = l;
      }
    }
    // the upper off-diagonal 64-tile of a diagonal 128-tile is needed as well (untransposed)
    if (same128 && ti != tj) {
      const int64_t a2 = r0 + r, b2 = c0 + tx;
      if (a2 < ldp && b2 < ldp) {
        unsigned short h, l;
        split_bf16(tile[r][tx], h, l);
        Hhk[a2 * ldp + b2] = h;
        Hlk[a2 * ldp + b2] = l;
      }
    }
  }
}

// Y tile [128 j][128 b] over a < (tb+1)*128 on bf16 MFMA with split operands, then the row dot.
__global__ __launch_bounds__(256, 2) void objective_mfma_kernel(const unsigned short* __restrict__ Dh,
                                                             const unsigned short* __restrict__ Dl,
                                                             const unsigned short* __restrict__ Hh,
                                                             const unsigned short* __restrict__ Hl,
                                                             const float* __restrict__ W, const float* __restrict__ What,
                                                             int64_t d_out, int64_t d, int64_t ld, int64_t ldp, int G,
                                                             int n_tb, int n_rb, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) char smem[2][4][kTileBytes];   // stage x {Dh, Dl, Hh, Hl}
  // the row-sum exchange at the end reuses the staging memory (all waves are past the last
  // barrier of the main loop by then), which keeps the workgroup at exactly 80 KiB
  float (*red)[kTile] = reinterpret_cast<float (*)[kTile]>(&smem[0][0][0]);

  // Work order: group, then column tile (heavy ones first), then row block, so that the row
  // blocks that read the same H tiles run side by side; workgroup ids are dealt round-robin to
  // the 8 XCDs (each with its own L2), so the id is first remapped to give every XCD one
  // contiguous stretch of that order.
  int k, tb, rb;
  {
    constexpr int kXcd = 8;
    const int64_t total = gridDim.x, id = blockIdx.x;
    const int64_t x = id % kXcd, idx = id / kXcd, q = total / kXcd, r = total % kXcd;
    const int64_t logical = x * q + (x < r ? x : r) + idx;
    const int64_t per_group = (int64_t)n_tb * n_rb;
    k = (int)(logical / per_group);
    const int64_t rem = logical - (int64_t)k * per_group;
    tb = n_tb - 1 - (int)(rem / n_rb);
    rb = (int)(rem % n_rb);
  }
  const int64_t m = d_out / G;
  const int64_t j0 = (int64_t)k * m + (int64_t)rb * kTile;  // first channel of this block
  const int64_t j_end = (int64_t)(k + 1) * m;               // rows >= j_end belong to another group
  const int64_t b0 = (int64_t)tb * kTile;
  const unsigned short* Hhk = Hh + (int64_t)k * ldp * ldp;
  const unsigned short* Hlk = Hl + (int64_t)k * ldp * ldp;

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

  // staging: every tile is 128 rows x kChunks chunks of 16 B; thread -> (row q/kChunks, chunk q%kChunks), q = tid + 256 h
  u32x4 rg[4][kTileLoads];
  auto fetch = [&](int64_t a0) {
#pragma unroll
    for (int h = 0; h < kTileLoads; ++h) {
      const int q = tid + 256 * h;
      const int r = q / kChunks, c = q % kChunks;
      const int64_t a = a0 + 8 * c;                       // a0 + kKS <= ldp always (ldp is padded to 128)
      int64_t j = j0 + r;
      j = j < d_out ? j : d_out - 1;                      // rows past the group are masked at the end
      int64_t b = b0 + r;
      b = b < ldp ? b : ldp - 1;
      rg[0][h] = *reinterpret_cast<const u32x4*>(Dh + j * ldp + a);
      rg[1][h] = *reinterpret_cast<const u32x4*>(Dl + j * ldp + a);
      rg[2][h] = *reinterpret_cast<const u32x4*>(Hhk + b * ldp + a);
      rg[3][h] = *reinterpret_cast<const u32x4*>(Hlk + b * ldp + a);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int h = 0; h < kTileLoads; ++h) {
        const int q = tid + 256 * h;
        *reinterpret_cast<u32x4*>(&smem[buf][t][(q / kChunks) * kPitch + (q % kChunks) * 16]) = rg[t][h];
      }
  };
  auto frag = [&](int buf, int t, int row0, int ks) -> bf16x8 {   // rows row0 + lane%32, k = 16 ks + 8 (lane/32) ..
    const u32x4 v = *reinterpret_cast<const u32x4*>(&smem[buf][t][(row0 + lane % 32) * kPitch + (2 * ks + lane / 32) * 16]);
    return __builtin_bit_cast(bf16x8, v);
  };

  const int64_t stages = (int64_t)(tb + 1) * (kTile / kKS);
  const int64_t first_diag = (int64_t)tb * (kTile / kKS);
  fetch(0);
  stash(0);
  __syncthreads();
  for (int64_t it = 0; it < stages; ++it) {
    const int buf = (int)(it & 1);
    if (it + 1 < stages) fetch((it + 1) * kKS);
    if (it == first_diag && tb > 0) {
      // all strictly-upper tiles are done: they count twice (their mirror images are never visited)
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) acc[x][y] *= 2.f;
    }
#pragma unroll
    for (int ks = 0; ks < kKS / 16; ++ks) {
      bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        ah[x] = frag(buf, 0, wm * 64 + x * 32, ks);
        al[x] = frag(buf, 1, wm * 64 + x * 32, ks);
      }
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        bh[y] = frag(buf, 2, wn * 64 + y * 32, ks);
        bl[y] = frag(buf, 3, wn * 64 + y * 32, ks);
      }
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y) {
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[x], bh[y], acc[x][y], 0, 0, 0);
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[x], bl[y], acc[x][y], 0, 0, 0);
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[x], bh[y], acc[x][y], 0, 0, 0);
        }
    }
    if (it + 1 < stages) stash(buf ^ 1);
    __syncthreads();
  }

  // row dot with delta[j, b] (fp32): register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32
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

// obj_row[j] = sum_tb partial[tb][j] (fixed order) for 256 rows per workgroup, and the fp64 sum
// of those rows (fixed tree) into block_sum[k][block].
__global__ __launch_bounds__(256) void objective_rows_kernel(const float* __restrict__ partial, int64_t d_out, int G,
                                                             int n_tb, float* __restrict__ obj_row,
                                                             double* __restrict__ block_sum) {
  __shared__ double red[256];
  const int k = blockIdx.y;
  const int64_t m = d_out / G;
  const int64_t jj = (int64_t)blockIdx.x * 256 + threadIdx.x;
  double acc = 0.0;
  if (jj < m) {
    const int64_t j = (int64_t)k * m + jj;
    float v = 0.f;
    for (int tb = 0; tb < n_tb; ++tb) v += partial[(int64_t)tb * d_out + j];
    if (obj_row) obj_row[j] = v;
    acc = (double)v;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) block_sum[(int64_t)k * gridDim.x + blockIdx.x] = red[0];
}

// obj[k] = sum of the group's block sums, in block order.
__global__ void objective_groups_kernel(const double* __restrict__ block_sum, int n_blocks, double* __restrict__ obj) {
  const int k = blockIdx.x;
  if (threadIdx.x != 0) return;
  double acc = 0.0;
  for (int b = 0; b < n_blocks; ++b) acc += block_sum[(int64_t)k * n_blocks + b];
  obj[k] = acc;
}

struct Layout {
  int64_t ldp, n_tb;
  int64_t n_blocks;                             // 256-row blocks per group in the final reduction
  size_t partial_bytes, sums_bytes, delta_bytes, h_bytes;   // delta_bytes / h_bytes: one of the hi/lo arrays
};
Layout make_layout(int64_t d_out, int64_t d_in, int G) {
  Layout L;
  L.n_tb = (d_in + kTile - 1) / kTile;
  L.ldp = L.n_tb * kTile;                       // padded so that every 128 x 64 operand tile is in range
  L.partial_bytes = ((size_t)(L.n_tb * d_out) * sizeof(float) + 255) / 256 * 256;
  L.n_blocks = (d_out / G + 255) / 256;
  L.sums_bytes = ((size_t)(L.n_blocks * G) * sizeof(double) + 255) / 256 * 256;
  L.delta_bytes = ((size_t)(d_out * L.ldp) * 2 + 255) / 256 * 256;
  L.h_bytes = ((size_t)((int64_t)G * L.ldp * L.ldp) * 2 + 255) / 256 * 256;
  return L;
}

}  // namespace

size_t objective_workspace(int64_t d_out, int64_t d_in, int G) {
  const Layout L = make_layout(d_out, d_in, G);
  return L.partial_bytes + L.sums_bytes + 2 * L.delta_bytes + 2 * L.h_bytes;
}

hipError_t launch_objective(const float* W, const float* What, int64_t d_out, int64_t d_in, int64_t ld,
                            const float* H, int G, double* obj, float* obj_row, void* ws, hipStream_t st) {
  const Layout L = make_layout(d_out, d_in, G);
  char* p = (char*)ws;
  float* partial = (float*)p;
  p += L.partial_bytes;
  double* block_sum = (double*)p;
  p += L.sums_bytes;
  unsigned short* Dh = (unsigned short*)p;
  p += L.delta_bytes;
  unsigned short* Dl = (unsigned short*)p;
  p += L.delta_bytes;
  unsigned short* Hh = (unsigned short*)p;
  p += L.h_bytes;
  unsigned short* Hl = (unsigned short*)p;

  const int64_t m = d_out / G;
  const int n_tb = (int)L.n_tb;
  const int n_rb = (int)((m + kTile - 1) / kTile);
  hipError_t e;
  {
    int64_t bx = (L.ldp + 255) / 256;
    if (bx > 64) bx = 64;
    split_delta_kernel<<<dim3((unsigned)bx, (unsigned)d_out), dim3(256), 0, st>>>(W, What, d_out, d_in, ld, L.ldp, Dh, Dl);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    const int64_t T = L.ldp / 64;
    split_h_kernel<<<dim3((unsigned)tri_count(T), (unsigned)G), dim3(256), 0, st>>>(H, d_in, L.ldp, Hh, Hl);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  objective_mfma_kernel<<<dim3((unsigned)((int64_t)n_tb * n_rb * G)), dim3(256), 0, st>>>(
      Dh, Dl, Hh, Hl, W, What, d_out, d_in, ld, L.ldp, G, n_tb, n_rb, partial);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  objective_rows_kernel<<<dim3((unsigned)L.n_blocks, (unsigned)G), dim3(256), 0, st>>>(partial, d_out, G, n_tb, obj_row,
                                                                                       block_sum);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  objective_groups_kernel<<<dim3((unsigned)G), dim3(64), 0, st>>>(block_sum, (int)L.n_blocks, obj);
  return hipGetLastError();
}

}  // namespace gq
