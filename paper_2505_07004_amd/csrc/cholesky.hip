// Damped Cholesky factorization of the group Hessians (Algorithm 2, line 1; Section 4.2: a small
// constant on the diagonal makes the matrix positive definite):
//     A_k = H[k] + eps_k I,   eps_k = damp_abs + damp_rel * mean_i H[k][i][i],
//     A_k = L L^T  (L lower triangular)    or    A_k = R R^T  (R UPPER triangular: the factorization
//     taken from the last coordinate backwards, whose columns are the feedback coefficients of
//     sequential rounding in the order 0, 1, ..., d_in-1).
//
// Both are one algorithm on a working matrix A' = U^T U, U upper triangular, processed by block rows
// of 128 in fp32:  A' = A gives L = U^T;  A'[a][b] = A[d-1-a][d-1-b] gives R[i][j] = U[d-1-j][d-1-i].
// Per block row:  (1) the 128 x 128 diagonal block is factored and (2) the panel to its right is solved
// against it, U12 = U11^-T A12, in one launch (both with the block in registers, 8 x 8 per thread, eight
// rows at a time published through LDS);
// (3) the trailing upper triangle is updated, A22 -= U12^T U12, on the bf16 matrix cores at fp32
// accuracy (U12 as three bf16 terms, six products).
// Only the upper triangle of H is read.  A non-positive pivot is recorded in info[k] (its
// coordinate + 1, the first one) and replaced by 1 so that everything stays finite.
#include <mutex>

#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kNb = 128;             // block size
constexpr int kPair = 2 * kNb;       // rows of U that one trailing update applies (a pair of block rows)

// eps[k] and info[k] = 0.  One workgroup per group; fixed-order fp64 sum of the diagonal.
__global__ __launch_bounds__(256) void chol_eps_kernel(const float* __restrict__ H, int64_t d, double damp_rel,
                                                       double damp_abs, double* __restrict__ eps,
                                                       int* __restrict__ info) {
  __shared__ double part[256];
  const int k = blockIdx.x;
  const float* Hk = H + (int64_t)k * d * d;
  double acc = 0.0;
  for (int64_t i = threadIdx.x; i < d; i += 256) acc += (double)Hk[i * d + i];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    eps[k] = damp_abs + damp_rel * (part[0] / (double)d);
    if (info) info[k] = 0;
  }
}

// Working matrix, upper triangle: Uw[r][c] = A'[r][c] for r <= c.  One workgroup per 64 x 64 tile; the grid's
// y range selects the tile rows by0, by0 + 1, ...
__global__ __launch_bounds__(256) void chol_load_kernel(const float* __restrict__ H, int64_t d, int reverse,
                                                        const double* __restrict__ eps, float* __restrict__ Uw, int by0) {
  __shared__ float tile[64][65];
  const int k = blockIdx.z;
  const int by = by0 + blockIdx.y, bx = blockIdx.x;        // tile of rows r (from tile row by0 on), of columns c
  if (by > bx) return;
  const float* Hk = H + (int64_t)k * d * d;
  float* Uk = Uw + (int64_t)k * d * d;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  const int64_t r0 = (int64_t)by * 64, c0 = (int64_t)bx * 64;
  const double e = eps[k];
  if (!reverse) {
    for (int lr = ty; lr < 64; lr += 4) {
      const int64_t r = r0 + lr, c = c0 + tx;
      if (r < d && c < d && r <= c) {
        const float h = Hk[r * d + c];
        Uk[r * d + c] = r == c ? (float)((double)h + e) : h;
      }
    }
    return;
  }
  // A'[r][c] = A[d-1-r][d-1-c] = (upper triangle of H)[d-1-c][d-1-r]
  for (int lc = ty; lc < 64; lc += 4) {
    const int64_t sr = d - 1 - (c0 + lc), sc = d - 1 - (r0 + tx);
    tile[lc][tx] = (sr >= 0 && sc >= 0 && sr <= sc) ? Hk[sr * d + sc] : 0.f;
  }
  __syncthreads();
  for (int lr = ty; lr < 64; lr += 4) {
    const int64_t r = r0 + lr, c = c0 + tx;
    if (r < d && c < d && r <= c) {
      const float h = tile[tx][lr];
      Uk[r * d + c] = r == c ? (float)((double)h + e) : h;
    }
  }
}

// The rows of U12 as three bf16 terms, for the trailing update: per group and term, for every step of 16
// contraction elements (rows of U12), all columns one after the other with their 16 elements (32 bytes).
// A workgroup's operand tile for a step (128 columns) is one contiguous 4 KiB run, so every 1 KiB direct
// load moves whole cache lines.
constexpr int kP3Step = 16;
__device__ __forceinline__ int64_t p3_index(int64_t k, int term, int64_t row, int64_t col, int64_t ldc) {
  return ((((k * 3 + term) * (kPair / kP3Step) + row / kP3Step) * ldc + col) * kP3Step) + row % kP3Step;
}

// the value a register holds in lane `l` of the wave (l uniform)
__device__ __forceinline__ float lane_value(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
// between an LDS write by one lane and the read of it by another lane of the same wave
__device__ __forceinline__ void wave_lds_fence() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
}

// (1) + (2) One block row: the diagonal block A11 = U11^T U11 at (r0, r0) and the panel to its right,
// U12 = U11^-T A12, in one launch.  A workgroup owns 128 columns of the panel; its threads 256..511 hold
// that 128 x 128 tile of A12 in registers (thread (tr, tc) of 16 x 16 the 8 x 8 tile at rows 8 tr, columns
// 8 tc), its threads 0..255 hold the diagonal block the same way: every workgroup factors the diagonal
// block again beside its panel (the two halves run on different waves, so this costs no time and saves
// the launch and the round trip of U11 through memory that a separate kernel needs).  Eight rows at a time:
//   a. the thread of the diagonal 8 x 8 tile factors it on its own (eight pivots, no barrier) and
//      publishes the 8 x 8 factor;
//   b. the other owners of these eight rows, of the diagonal block and of the panel alike, solve their
//      tiles against it (forward substitution, eight steps, no barrier) and publish the finished rows;
//   c. every tile further down subtracts the product of its eight row entries (from the diagonal
//      block's rows) and its eight column entries: a rank-8 update.
// Two barriers per eight rows (the published data alternate between two buffers).  Launched with 256
// threads there is no panel (the last block row).  Workgroup 0 stores U11 and reports bad pivots; U11
// goes to a buffer of its own (Ud[k][block][128][128]), not over A11, which workgroups that start
// later still have to read.
// Rows and columns past the end of the matrix are those of the identity.
__global__ __launch_bounds__(512) void chol_block_row_kernel(float* __restrict__ Uw, int64_t d, int64_t r0,
                                                             float* __restrict__ Ud, unsigned short* __restrict__ P3,
                                                             int64_t ldc, int koff, int* __restrict__ info) {
  __shared__ __attribute__((aligned(16))) float dtile[2][8][8];
  __shared__ __attribute__((aligned(16))) float draw[8][8];            // the diagonal tile of a pass before it is factored
  __shared__ __attribute__((aligned(16))) float rows[2][8][2 * kNb];   // columns 0..127: diagonal block, 128..255: panel
  __shared__ int bad;
  const int k = blockIdx.y;
  float* Uk = Uw + (int64_t)k * d * d;
  const int tid = threadIdx.x, role = tid / 256, tr = (tid % 256) / 16, tc = tid % 16;
  const int cb = role * kNb + 8 * tc;                                    // this thread's columns in `rows`
  const int64_t c0 = role == 0 ? r0 : r0 + kNb + (int64_t)blockIdx.x * kNb;   // first global column of this half's tile
  if (tid == 0) bad = -1;
  // The thread's 8 x 8 tile: 32 bytes per row, as two 16-byte loads where the rows are 16-byte aligned
  // (d a multiple of 4) and the eight columns lie inside the matrix; all loads in flight at once.
  const bool vec_rows = d % 4 == 0;                          // uniform
  float a[8][8];
  {
    const int64_t gc0 = c0 + 8 * tc;
    const bool whole = vec_rows && gc0 + 7 < d;
    f32x4 in4[8][2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t gr = r0 + 8 * tr + i;
      if (whole && gr < d) {
        in4[i][0] = *reinterpret_cast<const f32x4*>(Uk + gr * d + gc0);
        in4[i][1] = *reinterpret_cast<const f32x4*>(Uk + gr * d + gc0 + 4);
      } else {
#pragma unroll
        for (int l = 0; l < 8; ++l) in4[i][l / 4][l % 4] = (gr < d && gc0 + l < d) ? Uk[gr * d + gc0 + l] : 0.f;
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int l = 0; l < 8; ++l) {
        const int r = 8 * tr + i, c = 8 * tc + l;
        const bool in = r0 + r < d && gc0 + l < d && (role == 1 || r <= c);
        a[i][l] = in ? in4[i][l / 4][l % 4] : ((role == 0 && r == c) ? 1.f : 0.f);
      }
  }
  __syncthreads();
  for (int jb = 0; jb < 16; ++jb) {
    const int buf = jb & 1;
    if (role == 0 && tr / 4 == jb / 4) {                      // a. the diagonal tile (uniform: the wave that holds it)
      // Its owner hands the tile to eight lanes of its wave (those of tile row jb, columns 0..7 of it), one
      // column each; the eight pivots then cost one cross-lane read each instead of a chain through all
      // 36 elements in one lane.  Same operations on the same values as the factorization of an 8 x 8 tile
      // by one thread.  LDS accesses of one wave execute in order; the fence only stops the compiler.
      if (tr == jb && tc == jb) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          *reinterpret_cast<f32x4*>(&draw[i][0]) = f32x4{a[i][0], a[i][1], a[i][2], a[i][3]};
          *reinterpret_cast<f32x4*>(&draw[i][4]) = f32x4{a[i][4], a[i][5], a[i][6], a[i][7]};
        }
      }
      wave_lds_fence();
      const int hl = tc & 7;
      float col[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) col[i] = draw[i][hl];
      const int lane_base = 16 * (jb % 4);                    // lane of (tile row jb, tile column 0) in this wave
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        float p = lane_value(col[jj], lane_base + jj);
        const bool ok = p > 0.f;                              // false for NaN as well (uniform)
        if (!ok && tr == jb && tc == 0 && bad < 0) bad = 8 * jb + jj;
        p = ok ? p : 1.f;
        const float sp = __builtin_amdgcn_sqrtf(p), isp = __builtin_amdgcn_rcpf(sp);
        const float u = hl == jj ? sp : col[jj] * isp;        // row jj of the factor, this lane's column
        col[jj] = u;
#pragma unroll
        for (int i = jj + 1; i < 8; ++i) col[i] -= lane_value(u, lane_base + i) * u;
      }
      if (tr == jb && tc < 8) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float v = hl >= i ? col[i] : 0.f;
          dtile[buf][i][hl] = v;
          rows[buf][i][8 * jb + hl] = v;
        }
      }
      wave_lds_fence();
      if (tr == jb && tc == jb) {                             // the owner takes the factored tile back
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const f32x4 lo = *reinterpret_cast<const f32x4*>(&dtile[buf][i][0]);
          const f32x4 hi = *reinterpret_cast<const f32x4*>(&dtile[buf][i][4]);
#pragma unroll
          for (int l = 0; l < 4; ++l) {
            a[i][l] = lo[l];
            a[i][4 + l] = hi[l];
          }
        }
      }
    }
    __syncthreads();
    if (tr == jb && (role == 1 || tc > jb)) {                 // b. the rest of the eight rows: U_dd^T X = A
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const float rp = __builtin_amdgcn_rcpf(dtile[buf][jj][jj]);
#pragma unroll
        for (int l = 0; l < 8; ++l) {
          float v = a[jj][l];
#pragma unroll
          for (int i = 0; i < jj; ++i) v -= dtile[buf][i][jj] * a[i][l];
          a[jj][l] = v * rp;
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        *reinterpret_cast<f32x4*>(&rows[buf][i][cb]) = f32x4{a[i][0], a[i][1], a[i][2], a[i][3]};
        *reinterpret_cast<f32x4*>(&rows[buf][i][cb + 4]) = f32x4{a[i][4], a[i][5], a[i][6], a[i][7]};
      }
    }
    __syncthreads();
    if (tr > jb && (role == 1 || tc >= tr)) {                 // c. rank-8 update of everything further down
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        float f[8], cl[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = rows[buf][jj][8 * tr + i];
#pragma unroll
        for (int l = 0; l < 8; ++l) cl[l] = rows[buf][jj][cb + l];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
          for (int l = 0; l < 8; ++l) a[i][l] -= f[i] * cl[l];
      }
    }
  }
  if (role == 1) {
    const int64_t gc0 = c0 + 8 * tc;
    const bool whole = vec_rows && gc0 + 7 < d;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t gr = r0 + 8 * tr + i;
      if (whole && gr < d) {
        *reinterpret_cast<f32x4*>(Uk + gr * d + gc0) = f32x4{a[i][0], a[i][1], a[i][2], a[i][3]};
        *reinterpret_cast<f32x4*>(Uk + gr * d + gc0 + 4) = f32x4{a[i][4], a[i][5], a[i][6], a[i][7]};
      } else {
#pragma unroll
        for (int l = 0; l < 8; ++l)
          if (gr < d && gc0 + l < d) Uk[gr * d + gc0 + l] = a[i][l];
      }
    }
    // ... and once more for the trailing update: three bf16 terms in the order the update consumes them
    // (p3_index): a thread's eight rows of one column are 16 bytes per term
#pragma unroll
    for (int l = 0; l < 8; ++l) {
      unsigned short t[3][8];
#pragma unroll
      for (int i = 0; i < 8; ++i) split3_bf16(a[i][l], t[0][i], t[1][i], t[2][i]);
      const int64_t gc = c0 + 8 * tc + l;                         // < ldc: the buffer covers whole panels
#pragma unroll
      for (int term = 0; term < 3; ++term) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (unsigned)t[term][2 * e] | ((unsigned)t[term][2 * e + 1] << 16);
        *reinterpret_cast<u32x4*>(P3 + p3_index(k, term, koff + 8 * tr, gc, ldc)) = w;
      }
    }
  } else if (blockIdx.x == 0) {
    float* Ub = Ud + ((int64_t)k * ((d + kNb - 1) / kNb) + r0 / kNb) * (kNb * kNb);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      f32x4 o[2];
#pragma unroll
      for (int l = 0; l < 8; ++l) o[l / 4][l % 4] = (8 * tr + i <= 8 * tc + l) ? a[i][l] : 0.f;
      *reinterpret_cast<f32x4*>(Ub + (8 * tr + i) * kNb + 8 * tc) = o[0];
      *reinterpret_cast<f32x4*>(Ub + (8 * tr + i) * kNb + 8 * tc + 4) = o[1];
    }
  }
  __syncthreads();
  if (tid == 0 && blockIdx.x == 0 && bad >= 0 && info && info[k] == 0) info[k] = (int)(r0 + bad) + 1;
}

// (3) Trailing update: for 128 x 128 tiles (ti <= tj) of the upper triangle with origin t0,
//   A[a][b] -= sum_{k < n_k} U[r0 + k][a] * U[r0 + k][b],     n_k = 128 or 256.
// Block rows are processed in pairs: after the first of a pair only the strip of the second one is
// updated (strip = 1: the tiles of the first tile row, 128 rows of U), after the second everything
// behind the pair with the 256 rows of both at once, which halves the read-modify-write traffic of the
// trailing matrix.  The rows of U arrive as three bf16 terms each, contraction-major (P3, written by
// the block-row kernel), and the product runs on the bf16 matrix cores at fp32 accuracy: of the nine
// term products the six that matter (hi*hi, hi*mid, mid*hi, hi*lo, lo*hi, mid*mid; the others are
// below 2^-24 of the result) -- 2.7 times fewer matrix-core cycles than the fp32 instruction.
// 4 waves of 64 x 64; a stage is 32 contraction elements of the 2 x 3 x 128 operand rows (48 KiB,
// global_load_lds_dwordx4), ring of three stages.
// The tile itself is read and written through a buffer resource, 32 loads in flight, no branch.
constexpr int kSK = 32;                               // contraction elements per stage
constexpr int kSTile = kNb * kSK * 2;                 // one staged term of one side (8 KiB)
constexpr int kSStage = 6 * kSTile;                   // {row side, column side} x {hi, mid, lo}: 48 KiB
constexpr int kSRing = 3;
constexpr int kSLoads = 12;                           // 1 KiB loads per wave and stage
constexpr int kBufferWord3 = 0x00020000;              // raw buffer, 32-bit elements
constexpr unsigned kBufferOutside = 0x7ffffff0u;

__global__ __launch_bounds__(256) void chol_syrk_kernel(float* __restrict__ Uw, int64_t d, const unsigned short* __restrict__ P3,
                                                        int64_t ldc, int n_k, int64_t t0, int strip) {
  __shared__ __attribute__((aligned(1024))) char smem[kSRing * kSStage];
  const int k = blockIdx.y;
  float* Uk = Uw + (int64_t)k * d * d;
  int ti = 0, tj = (int)blockIdx.x;                          // strip: the first tile row only
  if (!strip) tri_decode(blockIdx.x, ti, tj);                // ti <= tj
  const int64_t a0 = t0 + (int64_t)ti * kNb, b0 = t0 + (int64_t)tj * kNb;
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / 2, wn = wave % 2;
  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;

  // staging: a staged tile (one term of one side, 8 KiB) is two halves of 16 contraction elements, each
  // [128 rows][32 bytes] as it lies in P3; load g = 12 wave + i of a stage moves rows 32 (g % 4) .. + 31 of
  // half (g / 4) % 2 of tile g / 8 (tiles 0..2: the three terms of the tile's rows a0.., 3..5: of its
  // columns b0..); chunk c (of two) of row r sits at position c ^ ((r >> 2) & 1)
  const unsigned short* lsrc[kSLoads];
  unsigned ldst[kSLoads];
#pragma unroll
  for (int i = 0; i < kSLoads; ++i) {
    const int g = wave * kSLoads + i, tile = g / 8, half = (g / 4) % 2, i4 = g % 4;
    const int r = 32 * i4 + lane / 2;
    const int c = (lane % 2) ^ ((r >> 2) & 1);
    const int64_t col = (tile < 3 ? a0 : b0) + r;               // < ldc
    lsrc[i] = P3 + p3_index(k, tile % 3, kP3Step * half + 8 * c, col, ldc);
    ldst[i] = tile * kSTile + half * (kSTile / 2) + i4 * 1024;
  }
  const int64_t stage_pitch = (kSK / kP3Step) * ldc * kP3Step;  // elements from one stage to the next
  auto issue = [&](int stage, int slot) {
#pragma unroll
    for (int i = 0; i < kSLoads; ++i) dma16(lsrc[i] + stage * stage_pitch, smem_base + slot * kSStage + ldst[i]);
  };
  const int lrow = lane % 32;
  auto frag = [&](int slot, int tile, int row0, int t) -> bf16x8 {
    const int pos = (lane / 32) ^ ((lrow >> 2) & 1);
    const u32x4 v = *reinterpret_cast<const u32x4*>(
        &smem[slot * kSStage + tile * kSTile + t * (kSTile / 2) + (row0 + lrow) * 32 + pos * 16]);
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  const int n_stages = n_k / kSK;                               // 4 or 8
  issue(0, 0);
  issue(1, 1);
  for (int s = 0; s < n_stages; ++s) {
    const int slot = s % kSRing;
    if (s + 1 < n_stages) wait_vmcnt<kSLoads>();                // the next stage may still be in flight
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();                               // everyone's part of stage s is there; stage s - 1 is done with
    if (s + 2 < n_stages) issue(s + 2, (s + 2) % kSRing);
#pragma unroll
    for (int t = 0; t < kSK / 16; ++t) {
      bf16x8 a[2][3], b[2][3];
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int term = 0; term < 3; ++term) {
          a[x][term] = frag(slot, term, wm * 64 + x * 32, t);
          b[x][term] = frag(slot, 3 + term, wn * 64 + x * 32, t);
        }
      // smallest products first; (row term, column term): (0,2) (2,0) (1,1) (0,1) (1,0) (0,0)
      constexpr int kTa[6] = {0, 2, 1, 0, 1, 0}, kTb[6] = {2, 0, 1, 1, 0, 0};
#pragma unroll
      for (int pr = 0; pr < 6; ++pr)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
          for (int x = 0; x < 2; ++x)
            acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x][kTa[pr]], b[y][kTb[pr]], acc[x][y], 0, 0, 0);
    }
  }

  // accumulator register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32.
  // Straight-line code with every lane active: the trailing matrix is addressed through a buffer
  // resource that spans the valid rows of this wave's 64-row block; an entry below the diagonal or
  // right of column d gets an offset outside it (such a load returns 0, such a store is dropped).
  const int64_t row_w = a0 + wm * 64;
  const int64_t rows_valid = (d - row_w) < 64 ? (d - row_w) : 64;
  const int records = rows_valid > 0 ? (int)(rows_valid * d * (int64_t)sizeof(float)) : 0;
  const __amdgpu_buffer_rsrc_t res =
      __builtin_amdgcn_make_buffer_rsrc(Uk + (rows_valid > 0 ? row_w : 0) * d, 0, records, kBufferWord3);
  const unsigned dbytes = (unsigned)(d * (int64_t)sizeof(float));
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    float old[2][16];
    unsigned off[2][16];
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int64_t col = b0 + wn * 64 + y * 32 + lane % 32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int lr = x * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        const bool keep = (row_w + lr < d) & (col < d) & (row_w + lr <= col);
        off[y][r] = keep ? (unsigned)lr * dbytes + (unsigned)(col * (int64_t)sizeof(float)) : kBufferOutside;
        old[y][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(res, off[y][r], 0, 0));
      }
    }
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float val = acc[x][y][r];
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, old[y][r] - val), res, off[y][r], 0, 0);
      }
  }
}

// The same update for tiles of 256 rows by 128 columns (used for the update with both block rows of a
// pair, where it is nearly all of the work): a workgroup then pulls 3 x (256 + 128) operand rows for
// twice the products, a quarter less per product, and the update is bound by exactly that traffic.
// Tile row p covers the block rows 2p and 2p + 1 of the trailing matrix and the block columns tj >= 2p
// (for tj = 2p the lower half lies below the diagonal and is masked like every entry there).
// 4 waves of 128 x 64; a stage is 16 contraction elements (9 terms-of-128-rows of 4 KiB: 36 KiB), ring of
// four, the loads of a stage issued two stages ahead and before the wait for the current one; chunk c
// (of two) of row r sits at position c ^ ((r >> 2) & 1).
constexpr int kS2K = 16;
constexpr int kS2Tile = kNb * kS2K * 2;               // 4 KiB
constexpr int kS2Stage = 9 * kS2Tile;                 // 36 KiB
constexpr int kS2Ring = 4;
constexpr int kS2Loads = 9;                           // 1 KiB loads per wave and stage
__global__ __launch_bounds__(256) void chol_syrk2_kernel(float* __restrict__ Uw, int64_t d,
                                                         const unsigned short* __restrict__ P3, int64_t ldc, int n_k,
                                                         int64_t t0, int nb) {
  __shared__ __attribute__((aligned(1024))) char smem[kS2Ring * kS2Stage];
  const int k = blockIdx.y;
  float* Uk = Uw + (int64_t)k * d * d;
  int p = 0, tj = (int)blockIdx.x;                            // tile row p holds nb - 2p tiles (uniform loop)
  while (2 * p < nb && tj >= nb - 2 * p) {
    tj -= nb - 2 * p;
    ++p;
  }
  if (2 * p >= nb) return;                                    // (the grid holds exactly the tiles there are)
  tj += 2 * p;
  const int64_t a0 = t0 + (int64_t)(2 * p) * kNb, b0 = t0 + (int64_t)tj * kNb;
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / 2, wn = wave % 2;
  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;

  // staging: load g = 9 wave + i of a stage moves rows 32 (g % 4) .. + 31 of staged tile g / 4
  // (tiles 0..2: the three terms of rows a0 .. a0 + 127, 3..5: of rows a0 + 128 .., 6..8: of columns b0 ..)
  const unsigned short* lsrc[kS2Loads];
  unsigned ldst[kS2Loads];
#pragma unroll
  for (int i = 0; i < kS2Loads; ++i) {
    const int g = wave * kS2Loads + i, tile = g / 4, i4 = g % 4;
    const int r = 32 * i4 + lane / 2;
    const int c = (lane % 2) ^ ((r >> 2) & 1);
    int64_t col = (tile < 6 ? a0 + (int64_t)(tile / 3) * kNb : b0) + r;
    col = col < ldc ? col : ldc - 1;                          // a second block row past the matrix: masked below
    lsrc[i] = P3 + p3_index(k, tile % 3, 8 * c, col, ldc);
    ldst[i] = tile * kS2Tile + i4 * 1024;
  }
  static_assert(kS2K == kP3Step, "one step of P3 per stage");
  const int64_t stage_pitch = ldc * kP3Step;                    // elements from one stage to the next
  auto issue = [&](int stage) {
    const int slot = stage % kS2Ring;
#pragma unroll
    for (int i = 0; i < kS2Loads; ++i) dma16(lsrc[i] + stage * stage_pitch, smem_base + slot * kS2Stage + ldst[i]);
  };
  const int lrow = lane % 32;
  auto frag = [&](int slot, int tile, int row0) -> bf16x8 {
    const int pos = (lane / 32) ^ ((lrow >> 2) & 1);
    const u32x4 v = *reinterpret_cast<const u32x4*>(&smem[slot * kS2Stage + tile * kS2Tile + (row0 + lrow) * 32 + pos * 16]);
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[4][2];
#pragma unroll
  for (int x = 0; x < 4; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  const int n_stages = n_k / kS2K;
  issue(0);
  if (n_stages > 1) issue(1);
  for (int s = 0; s < n_stages; ++s) {
    const int slot = s % kS2Ring;
    if (s + 2 < n_stages) {                                     // uniform
      issue(s + 2);                                             // its slot's last readers were two barriers ago
      wait_vmcnt<2 * kS2Loads>();
    } else if (s + 1 < n_stages) {
      wait_vmcnt<kS2Loads>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();                               // everyone's part of stage s is there
    bf16x8 a[4][3], b[2][3];
#pragma unroll
    for (int term = 0; term < 3; ++term) {
#pragma unroll
      for (int x = 0; x < 4; ++x) a[x][term] = frag(slot, 3 * wm + term, 32 * x);
#pragma unroll
      for (int y = 0; y < 2; ++y) b[y][term] = frag(slot, 6 + term, wn * 64 + 32 * y);
    }
    // smallest products first; (row term, column term): (0,2) (2,0) (1,1) (0,1) (1,0) (0,0)
    constexpr int kTa[6] = {0, 2, 1, 0, 1, 0}, kTb[6] = {2, 0, 1, 1, 0, 0};
#pragma unroll
    for (int pr = 0; pr < 6; ++pr)
#pragma unroll
      for (int y = 0; y < 2; ++y)
#pragma unroll
        for (int x = 0; x < 4; ++x)
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x][kTa[pr]], b[y][kTb[pr]], acc[x][y], 0, 0, 0);
  }

  // accumulator register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32; the epilogue of the
  // 128 x 128 kernel, over the wave's 128 rows
  const int64_t row_w = a0 + wm * kNb;
  const int64_t rows_valid = (d - row_w) < kNb ? (d - row_w) : kNb;
  const int records = rows_valid > 0 ? (int)(rows_valid * d * (int64_t)sizeof(float)) : 0;
  const __amdgpu_buffer_rsrc_t res =
      __builtin_amdgcn_make_buffer_rsrc(Uk + (rows_valid > 0 ? row_w : 0) * d, 0, records, kBufferWord3);
  const unsigned dbytes = (unsigned)(d * (int64_t)sizeof(float));
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    float old[2][16];
    unsigned off[2][16];
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      const int64_t col = b0 + wn * 64 + y * 32 + lane % 32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int lr = x * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        const bool keep = (row_w + lr < d) & (col < d) & (row_w + lr <= col);
        off[y][r] = keep ? (unsigned)lr * dbytes + (unsigned)(col * (int64_t)sizeof(float)) : kBufferOutside;
        old[y][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(res, off[y][r], 0, 0));
      }
    }
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float val = acc[x][y][r];
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, old[y][r] - val), res, off[y][r], 0, 0);
      }
  }
}

// The factor in the requested form, every entry of F written: L[i][j] = U[j][i] (i >= j), zeros above
// the diagonal; or R[i][j] = U[d-1-j][d-1-i] (i <= j), zeros below.  One workgroup per 64 x 64 tile of F.
// A launch writes the columns [j_lo, j_hi) of F (a column of F is a row of U, so finished block rows can
// leave while later ones are still being factored); blockIdx.x counts tile columns from j_lo / 64.
__global__ __launch_bounds__(256) void chol_emit_kernel(const float* __restrict__ Uw, const float* __restrict__ Ud,
                                                        int64_t d, int reverse, float* __restrict__ F, int64_t j_lo,
                                                        int64_t j_hi) {
  __shared__ float tile[64][65];
  const int k = blockIdx.z;
  const float* Uk = Uw + (int64_t)k * d * d;
  float* Fk = F + (int64_t)k * d * d;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  const int64_t i0 = (int64_t)blockIdx.y * 64, j0 = (j_lo / 64 + (int64_t)blockIdx.x) * 64;   // tile of F: rows i, columns j
  // source entry of F[i0+li][j0+lj]:  U[sr][sc], sr = j (or d-1-j), sc = i (or d-1-i); tile[lj][li]
  for (int lj = ty; lj < 64; lj += 4) {
    const int64_t j = j0 + lj, i = i0 + tx;
    const int64_t sr = reverse ? d - 1 - j : j, sc = reverse ? d - 1 - i : i;
    const bool in = i < d && j < d && sr >= 0 && sc >= 0 && sr <= sc;
    const int64_t srr = in ? sr : 0, scc = in ? sc : 0;
    const float* src = (srr / kNb == scc / kNb)                // entries of a diagonal block live in Ud
                           ? Ud + (((int64_t)k * ((d + kNb - 1) / kNb) + srr / kNb) * kNb + srr % kNb) * kNb + scc % kNb
                           : Uk + srr * d + scc;
    const float v = *src;
    tile[lj][tx] = in ? v : 0.f;
  }
  __syncthreads();
  for (int li = ty; li < 64; li += 4) {
    const int64_t i = i0 + li, j = j0 + tx;
    if (i < d && j >= j_lo && j < j_hi) Fk[i * d + j] = tile[tx][li];
  }
}

struct Layout {
  int64_t ldc;
  size_t u_bytes, ud_bytes, p3_bytes, eps_bytes;
};
Layout make_layout(int64_t d, int G) {
  auto up = [](size_t b) { return (b + 255) / 256 * 256; };
  Layout L;
  L.u_bytes = up((size_t)G * d * d * sizeof(float));
  L.ud_bytes = up((size_t)G * ((d + kNb - 1) / kNb) * kNb * kNb * sizeof(float));
  L.ldc = (d + kNb - 1) / kNb * kNb;
  L.p3_bytes = up((size_t)G * 3 * L.ldc * kPair * sizeof(unsigned short));
  L.eps_bytes = up((size_t)G * sizeof(double));
  return L;
}

// A second stream and a few events per device, created on first use and kept for the life of the process
// (see the order of work below).  Calls are enqueued under the mutex, so the record / wait pairs of one
// call never interleave with another's.
constexpr int kMaxDevices = 64;
struct Aux {
  hipStream_t side = nullptr;
  hipEvent_t fork = nullptr, strip_done = nullptr, rest_done = nullptr;
};
std::mutex g_aux_mutex;
Aux g_aux[kMaxDevices];

hipError_t aux_of_current_device(Aux** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  Aux& a = g_aux[dev];
  if (!a.side) {
    if ((e = hipStreamCreateWithFlags(&a.side, hipStreamNonBlocking)) != hipSuccess) return e;
    if ((e = hipEventCreateWithFlags(&a.fork, hipEventDisableTiming)) != hipSuccess) return e;
    if ((e = hipEventCreateWithFlags(&a.strip_done, hipEventDisableTiming)) != hipSuccess) return e;
    if ((e = hipEventCreateWithFlags(&a.rest_done, hipEventDisableTiming)) != hipSuccess) return e;
  }
  *out = &a;
  return hipSuccess;
}

}  // namespace

size_t cholesky_workspace(int64_t d, int G) {
  const Layout L = make_layout(d, G);
  return L.u_bytes + L.ud_bytes + 2 * L.p3_bytes + L.eps_bytes;
}

// Order of work.  Block rows go in pairs (r0, t0 = r0 + 128); t1 = r0 + 256 is the next pair's first.  The
// chain that nothing can shorten runs on the caller's stream:
//   factor r0 -> strip of t0 (128 rows of U) -> factor t0 -> strip of t1 (the pair's 256 rows) -> factor t1 -> ...
// (a block row can be factored once every earlier block row has been subtracted from it).  Everything else runs
// beside it on a second stream, forked after "factor t0":
//   the pair's update of block row t1 + 128        needed before the next pair's "strip of t0"     (strip_done)
//   the pair's update of all rows from t1 + 256 on  needed before the next pair's "strip of t1"     (rest_done)
//   the pair's finished rows of U leave for F       needed at the end
// and, before the first pair, the load of everything but the first block row (the first pair treats it like a
// previous pair's update).  The two pairs in flight write their panels (three bf16 terms) to alternating buffers.
hipError_t launch_damped_cholesky(const float* H, int64_t d, int G, double damp_rel, double damp_abs, bool reverse,
                                  float* F, int* info, void* ws, hipStream_t st) {
  const Layout L = make_layout(d, G);
  float* Uw = (float*)ws;
  float* Ud = (float*)((char*)ws + L.u_bytes);
  unsigned short* P3buf[2] = {(unsigned short*)((char*)ws + L.u_bytes + L.ud_bytes),
                              (unsigned short*)((char*)ws + L.u_bytes + L.ud_bytes + L.p3_bytes)};
  double* eps = (double*)((char*)ws + L.u_bytes + L.ud_bytes + 2 * L.p3_bytes);
  std::lock_guard<std::mutex> lock(g_aux_mutex);
  Aux* aux = nullptr;
  hipError_t e = aux_of_current_device(&aux);
  if (e != hipSuccess) return e;
  hipStream_t side = aux->side;
  const unsigned t64 = (unsigned)((d + 63) / 64);
  const int rev = reverse ? 1 : 0;
  bool wait_strip = false, wait_rest = false;                 // work on the second stream that this stream has not waited for yet
  auto fork = [&]() -> hipError_t {
    hipError_t f = hipEventRecord(aux->fork, st);
    return f != hipSuccess ? f : hipStreamWaitEvent(side, aux->fork, 0);
  };
  auto join_strip = [&]() -> hipError_t {
    if (!wait_strip) return hipSuccess;
    wait_strip = false;
    return hipStreamWaitEvent(st, aux->strip_done, 0);
  };
  auto join_rest = [&]() -> hipError_t {
    if (!wait_rest) return hipSuccess;
    wait_rest = false;
    return hipStreamWaitEvent(st, aux->rest_done, 0);
  };
  // the columns of F that hold the rows [u_lo, u_hi) of U
  auto emit = [&](int64_t u_lo, int64_t u_hi, hipStream_t s) -> hipError_t {
    if (u_hi > d) u_hi = d;
    if (u_hi <= u_lo) return hipSuccess;
    const int64_t j_lo = reverse ? d - u_hi : u_lo, j_hi = reverse ? d - u_lo : u_hi;
    const unsigned cols = (unsigned)((j_hi - 1) / 64 - j_lo / 64 + 1);
    chol_emit_kernel<<<dim3(cols, t64, (unsigned)G), dim3(256), 0, s>>>(Uw, Ud, d, rev, F, j_lo, j_hi);
    return hipGetLastError();
  };

  chol_eps_kernel<<<dim3((unsigned)G), dim3(256), 0, st>>>(H, d, damp_rel, damp_abs, eps, info);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const unsigned first_tiles = t64 < 2 ? t64 : 2;             // the first block row: two tile rows of 64
  chol_load_kernel<<<dim3(t64, first_tiles, (unsigned)G), dim3(256), 0, st>>>(H, d, rev, eps, Uw, 0);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (t64 > first_tiles) {
    if ((e = fork()) != hipSuccess) return e;
    chol_load_kernel<<<dim3(t64, t64 - first_tiles, (unsigned)G), dim3(256), 0, side>>>(H, d, rev, eps, Uw, (int)first_tiles);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = hipEventRecord(aux->strip_done, side)) != hipSuccess) return e;
    if ((e = hipEventRecord(aux->rest_done, side)) != hipSuccess) return e;
    wait_strip = wait_rest = true;
  }
  // one block row: its diagonal block and, if there is anything to its right, the panel
  auto block_row = [&](int64_t r0, int koff, unsigned short* P3) -> hipError_t {
    const int64_t trail = d - (r0 + kNb);
    const int64_t tt = trail > 0 ? (trail + kNb - 1) / kNb : 0;
    chol_block_row_kernel<<<dim3((unsigned)(tt > 0 ? tt : 1), (unsigned)G), dim3(tt > 0 ? 512 : 256), 0, st>>>(
        Uw, d, r0, Ud, P3, L.ldc, koff, info);
    return hipGetLastError();
  };
  int64_t emitted = 0;                                        // rows of U already on their way to F
  int pair = 0;
  for (int64_t r0 = 0; r0 < d; r0 += 2 * kNb, ++pair) {
    unsigned short* P3 = P3buf[pair % 2];
    if ((e = block_row(r0, 0, P3)) != hipSuccess) return e;
    const int64_t t0 = r0 + kNb, trail = d - t0;
    if (trail <= 0) break;
    if ((e = join_strip()) != hipSuccess) return e;           // block row t0 has everything from before this pair
    const int64_t tt = (trail + kNb - 1) / kNb;
    chol_syrk_kernel<<<dim3((unsigned)tt, (unsigned)G), dim3(256), 0, st>>>(Uw, d, P3, L.ldc, kNb, t0, 1);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = block_row(t0, kNb, P3)) != hipSuccess) return e;
    const int64_t t1 = t0 + kNb, trail1 = d - t1;
    if (trail1 <= 0) break;
    const int64_t tt1 = (trail1 + kNb - 1) / kNb;
    // (waited for here, before this pair's events are recorded: a wait refers to the latest record)
    if ((e = join_rest()) != hipSuccess) return e;            // the previous pair's update of block row t1 (and beyond) is in
    // ---- second stream: the pair's updates from block row t1 + 128 on, then its finished rows to F
    if ((e = fork()) != hipSuccess) return e;
    if (tt1 > 1) {
      const int64_t t2 = t1 + kNb;
      chol_syrk_kernel<<<dim3((unsigned)(tt1 - 1), (unsigned)G), dim3(256), 0, side>>>(Uw, d, P3, L.ldc, kPair, t2, 1);
      if ((e = hipGetLastError()) != hipSuccess) return e;
      if ((e = hipEventRecord(aux->strip_done, side)) != hipSuccess) return e;
      wait_strip = true;
    }
    if (tt1 > 2) {
      const int64_t t3 = t1 + 2 * kNb, tt3 = tt1 - 2;
      // Large trailing matrices take the 256 x 128 tiles (less operand traffic per product); small ones, where
      // a launch is only a few rounds of workgroups, the 128 x 128 tiles (twice as many, shorter workgroups).
      // Measured cross-over on MI355X: about 3000 workgroups of the smaller kind.
      if (tri_count(tt3) * G >= 3000) {
        int64_t n_tiles2 = 0;                                 // tile row p has tt3 - 2p tiles
        for (int64_t p = 0; 2 * p < tt3; ++p) n_tiles2 += tt3 - 2 * p;
        chol_syrk2_kernel<<<dim3((unsigned)n_tiles2, (unsigned)G), dim3(256), 0, side>>>(Uw, d, P3, L.ldc, kPair, t3, (int)tt3);
      } else {
        chol_syrk_kernel<<<dim3((unsigned)tri_count(tt3), (unsigned)G), dim3(256), 0, side>>>(Uw, d, P3, L.ldc, kPair, t3, 0);
      }
      if ((e = hipGetLastError()) != hipSuccess) return e;
      if ((e = hipEventRecord(aux->rest_done, side)) != hipSuccess) return e;
      wait_rest = true;
    }
    if ((e = emit(emitted, t1, side)) != hipSuccess) return e;
    emitted = t1;
    // ---- this stream: the strip of the next pair's first block row, with the 256 rows of this pair at once
    chol_syrk_kernel<<<dim3((unsigned)tt1, (unsigned)G), dim3(256), 0, st>>>(Uw, d, P3, L.ldc, kPair, t1, 1);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // the rows of U not yet sent to F, and nothing of this call may outlive the caller's stream
  if ((e = emit(emitted, d, st)) != hipSuccess) return e;
  if ((e = hipEventRecord(aux->rest_done, side)) != hipSuccess) return e;
  return hipStreamWaitEvent(st, aux->rest_done, 0);
}

}  // namespace gq
