// Closed-form codebook update of LNQ for fixed assignments (Section 4.2, Eq. "conti-sol";
// Algorithm 2, lines 4 and 14), against the group Hessians:
//     c^(j) = (P^T H P + lam I)^-1 P^T H w_j,      P[i][q] = 1 if Q[j][i] == q else 0.
//
// With E_j = P^T (one-hot rows, one per grid point) the two small quantities of a channel are
//     T_j = E_j H            [m, d_in]      (row q: the sum of the rows of H assigned to q)
//     A_j[q][q'] = sum_{i : Q[j][i] == q'} T_j[q][i],      b_j[q] = sum_i T_j[q][i] * w_j[i].
// T for all channels of a group is ONE contraction (d_out/G * m rows) x d_in x d_in on the bf16
// matrix cores: the one-hot operand is exact in bf16, H is split into three bf16 terms
// (24 mantissa bits), so every product is exact and only the fp32 accumulation rounds.  A
// second kernel bins T into A and b (one workgroup per channel, fixed-order reductions) and
// solves the m x m system in fp64 by Gaussian elimination with partial pivoting.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kTile = 128;                           // rows (channel, grid point) and columns per workgroup
constexpr int kK = 64;                               // contraction elements per stage
constexpr int kTileBytes = kTile * kK * 2;           // one staged operand tile (16 KiB)
constexpr int kStageBytes = 4 * kTileBytes;          // {E, H hi, H mid, H lo}: 64 KiB
constexpr unsigned short kOneBf16 = 0x3F80;

// x = hi + mid + lo, three bf16 terms (exact for every fp32 x whose exponent leaves room).
__device__ inline void split3_bf16(float x, unsigned short& hi, unsigned short& mid, unsigned short& lo) {
  const __bf16 h = (__bf16)x;
  const float r1 = x - (float)h;
  const __bf16 m = (__bf16)r1;
  const __bf16 l = (__bf16)(r1 - (float)m);
  hi = __builtin_bit_cast(unsigned short, h);
  mid = __builtin_bit_cast(unsigned short, m);
  lo = __builtin_bit_cast(unsigned short, l);
}

// The full symmetric H[k] from its upper triangle, split into three bf16 terms,
// [G][ldp][ldp] each, zero padded.  One workgroup per 64 x 64 tile.
__global__ __launch_bounds__(256) void lnq_split_h_kernel(const float* __restrict__ H, int64_t d, int64_t ldp,
                                                          unsigned short* __restrict__ Hh,
                                                          unsigned short* __restrict__ Hm,
                                                          unsigned short* __restrict__ Hl) {
  __shared__ float tile[64][65];
  const int k = blockIdx.z;
  const int ti = blockIdx.y, tj = blockIdx.x;
  const float* Hk = H + (int64_t)k * d * d;
  const int tmin = ti < tj ? ti : tj, tmax = ti < tj ? tj : ti;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
#pragma unroll
  for (int u = 0; u < 16; ++u) {                            // the tile on or above the diagonal; clamped, branch-free
    const int r = ty + 4 * u;
    const int64_t a = (int64_t)tmin * 64 + r, b = (int64_t)tmax * 64 + tx;
    const int64_t ac = a < d ? a : d - 1, bc = b < d ? b : d - 1;
    const float v = Hk[ac * d + bc];
    tile[r][tx] = (a < d && b < d) ? v : 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int li = ty + 4 * u, lj = tx;
    const int64_t i = (int64_t)ti * 64 + li, ip = (int64_t)tj * 64 + lj;
    float h;
    if (ti < tj) h = tile[li][lj];
    else if (ti > tj) h = tile[lj][li];
    else h = li <= lj ? tile[li][lj] : tile[lj][li];
    unsigned short a, b, c;
    split3_bf16(h, a, b, c);
    const int64_t off = (int64_t)k * ldp * ldp + i * ldp + ip;
    Hh[off] = a;
    Hm[off] = b;
    Hl[off] = c;
  }
}

// E[(j*m + q)][i] = 1 if Q[j][i] == q else 0 (bf16), row pitch ldp, zero padded.
__global__ __launch_bounds__(256) void lnq_onehot_kernel(const unsigned char* __restrict__ Q, int64_t d, int64_t ldp,
                                                         int n_levels, unsigned short* __restrict__ E) {
  const int64_t j = blockIdx.y;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < ldp; i += (int64_t)gridDim.x * 256) {
    const int code = i < d ? (int)Q[j * d + i] : -1;
    for (int q = 0; q < n_levels; ++q) E[(j * n_levels + q) * ldp + i] = (q == code) ? kOneBf16 : (unsigned short)0;
  }
}

// T[r][i] = sum_{i'} E[r][i'] * H[k(r)][i][i']  for a 128 x 128 tile of (rows r, columns i).
// Both operands are contraction-major; a stage is 64 contraction elements = one whole
// 128-byte line of each of the 4 x 128 operand rows (E; H hi, mid, lo), copied straight into
// LDS (global_load_lds_dwordx4, 8 lanes per row, wave w copies operand w) into a ring of two
// stages with one barrier per stage; chunk c of row r sits at position c ^ ((r >> 1) & 7).
// 4 waves of 64 x 64; three MFMAs per fragment pair (E * hi, E * mid, E * lo).
__global__ __launch_bounds__(256) void lnq_gemm_kernel(const unsigned short* __restrict__ E,
                                                       const unsigned short* __restrict__ Hh,
                                                       const unsigned short* __restrict__ Hm,
                                                       const unsigned short* __restrict__ Hl, int64_t rows_per_group,
                                                       int64_t ldp, int n_rt, float* __restrict__ T) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * kStageBytes];
  const int k = blockIdx.x / n_rt, rt = blockIdx.x % n_rt;
  const int64_t r0 = (int64_t)k * rows_per_group + (int64_t)rt * kTile, r_last = (int64_t)(k + 1) * rows_per_group - 1;
  const int64_t c0 = (int64_t)blockIdx.y * kTile;
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / 2, wn = wave % 2;
  const int64_t n_stages = ldp / kK;

  const unsigned short* src = wave == 0 ? E : (wave == 1 ? Hh : wave == 2 ? Hm : Hl) + (int64_t)k * ldp * ldp;
  const int64_t row_first = wave == 0 ? r0 : c0, row_last = wave == 0 ? r_last : ldp - 1;
  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;
  auto issue = [&](int64_t stage, int slot) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = 8 * i + lane / 8;
      const int c = (lane % 8) ^ ((r >> 1) & 7);
      int64_t row = row_first + r;
      row = row < row_last ? row : row_last;             // rows past the group: repeat its last row (never stored)
      dma16(src + row * ldp + stage * kK + 8 * c, smem_base + slot * kStageBytes + wave * kTileBytes + i * 1024);
    }
  };
  const int lrow = lane % 32;
  auto frag = [&](int slot, int tile, int row0, int t) -> bf16x8 {
    const int pos = (2 * t + lane / 32) ^ ((lrow >> 1) & 7);
    const u32x4 v = *reinterpret_cast<const u32x4*>(&smem[slot * kStageBytes + tile * kTileBytes + (row0 + lrow) * 128 + pos * 16]);
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  issue(0, 0);
  for (int64_t s = 0; s < n_stages; ++s) {
    const int slot = (int)(s & 1);
    wait_vmcnt<0>();                                      // this wave's loads of stage s have landed
    __builtin_amdgcn_s_barrier();                         // everyone's have; and everyone is done with the other slot
    if (s + 1 < n_stages) issue(s + 1, slot ^ 1);
#pragma unroll
    for (int t = 0; t < kK / 16; ++t) {
      bf16x8 a[2], bh[2], bm[2], bl[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) a[x] = frag(slot, 0, wm * 64 + x * 32, t);
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        bh[y] = frag(slot, 1, wn * 64 + y * 32, t);
        bm[y] = frag(slot, 2, wn * 64 + y * 32, t);
        bl[y] = frag(slot, 3, wn * 64 + y * 32, t);
      }
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], bl[y], acc[0][y], 0, 0, 0);
        acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], bl[y], acc[1][y], 0, 0, 0);
        acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], bm[y], acc[0][y], 0, 0, 0);
        acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], bm[y], acc[1][y], 0, 0, 0);
        acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], bh[y], acc[0][y], 0, 0, 0);
        acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], bh[y], acc[1][y], 0, 0, 0);
      }
    }
  }

  // register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32 of a 32 x 32 block
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int64_t row = r0 + wm * 64 + 32 * x + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
      if (row <= r_last) {
#pragma unroll
        for (int y = 0; y < 2; ++y) T[row * ldp + c0 + wn * 64 + 32 * y + lane % 32] = acc[x][y][r];
      }
    }
}

// One workgroup per channel: bins its m rows of T into A (m x m) and b (m), solves
// (A + lam I) c = b in fp64 (Gauss-Jordan elimination with partial pivoting, the workgroup's
// threads sharing the entries of the system), and writes the grid values and, if wanted,
// What[j][i] = c[Q[j][i]].  Wave w bins the rows q = w, w + 4, ... on its own: a fixed order
// of additions (per lane, then an xor tree over the lanes), no barrier until the solve.
// LV = 4, 8 or 16 bounds the number of grid points.
template <int LV>
__global__ __launch_bounds__(256) void lnq_solve_kernel(const float* __restrict__ T, const unsigned char* __restrict__ Q,
                                                        const float* __restrict__ W, int64_t d, int64_t ld, int64_t ldp,
                                                        int n_levels, double lam, float* __restrict__ codebook,
                                                        float* __restrict__ What) {
  __shared__ double sys[LV][LV + 1];                       // the system; column LV holds b
  __shared__ float cval[LV];
  const int64_t j = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const unsigned char* Qj = Q + j * d;
  const float* Wj = W + j * ld;
  const int64_t d4 = d / 4 * 4;

  for (int q = wave; q < n_levels; q += 4) {                // row q of T_j
    const float* Tq = T + (j * n_levels + q) * ldp;
    float bins[LV], dot = 0.f;
#pragma unroll
    for (int u = 0; u < LV; ++u) bins[u] = 0.f;
    for (int64_t i = 4 * lane; i < d4; i += 4 * kWave) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(Tq + i);
      const f32x4 w = *reinterpret_cast<const f32x4*>(Wj + i);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float ve = v[e];
        const int code = Qj[i + e];
        dot += ve * w[e];
#pragma unroll
        for (int u = 0; u < LV; ++u) bins[u] += (code == u) ? ve : 0.f;
      }
    }
    if (lane < d - d4) {                                    // the last d % 4 coordinates
      const int64_t i = d4 + lane;
      const float ve = Tq[i];
      const int code = Qj[i];
      dot += ve * Wj[i];
#pragma unroll
      for (int u = 0; u < LV; ++u) bins[u] += (code == u) ? ve : 0.f;
    }
#pragma unroll
    for (int u = 0; u <= LV; ++u) {
      float v = u < LV ? bins[u] : dot;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
      if (lane == 0) sys[q][u] = (double)v + ((u == q) ? lam : 0.0);
    }
  }
  __syncthreads();

  // Gauss-Jordan: at step p the pivot is the largest entry of column p among the rows not yet
  // used; every other row is cleared in that column.  Rows are never moved: `mine` remembers,
  // in thread p, which row became the pivot of column p.  A step reads column p and the pivot
  // row and writes neither, so one barrier per step is enough.
  const int n = n_levels;
  unsigned used = 0;
  int mine = 0;
  for (int p = 0; p < n; ++p) {
    int best = 0;
    double bv = -1.0;
    for (int r = 0; r < n; ++r) {
      const double v = fabs(sys[r][p]);
      const bool take = (((used >> r) & 1u) == 0) & (v > bv);
      bv = take ? v : bv;
      best = take ? r : best;
    }
    used |= 1u << best;
    if (tid == p) mine = best;
    const double piv = sys[best][p];
    const double inv = piv != 0.0 ? 1.0 / piv : 0.0;
    for (int e = tid; e < n * (LV + 1); e += 256) {
      const int r = e / (LV + 1), c = e % (LV + 1);
      if (r != best && c > p && (c < n || c == LV)) sys[r][c] -= sys[r][p] * inv * sys[best][c];
    }
    __syncthreads();
  }
  if (tid < n) {
    const double piv = sys[mine][tid];
    const float c = piv != 0.0 ? (float)(sys[mine][LV] / piv) : 0.f;
    cval[tid] = c;
    codebook[j * n_levels + tid] = c;
  }
  __syncthreads();
  if (What) {
    for (int64_t i = tid; i < d; i += 256) {
      const int code = Qj[i];
      What[j * ld + i] = code < n_levels ? cval[code < LV ? code : 0] : 0.f;
    }
  }
}

struct Layout {
  int64_t ldp;
  int n_rt;
  size_t h_bytes, e_bytes, t_bytes;
};
Layout make_layout(int64_t d_out, int64_t d_in, int G, int n_levels) {
  Layout L;
  L.ldp = (d_in + kTile - 1) / kTile * kTile;
  const int64_t rows_per_group = d_out / G * n_levels;
  L.n_rt = (int)((rows_per_group + kTile - 1) / kTile);
  auto up = [](size_t b) { return (b + 255) / 256 * 256; };
  L.h_bytes = up((size_t)G * L.ldp * L.ldp * 2);
  L.e_bytes = up((size_t)d_out * n_levels * L.ldp * 2);
  L.t_bytes = up((size_t)d_out * n_levels * L.ldp * sizeof(float));
  return L;
}

}  // namespace

size_t lnq_codebook_workspace(int64_t d_out, int64_t d_in, int G, int n_levels) {
  const Layout L = make_layout(d_out, d_in, G, n_levels);
  return 3 * L.h_bytes + L.e_bytes + L.t_bytes;
}

hipError_t launch_lnq_codebook(const float* W, int64_t d_out, int64_t d_in, int64_t ld, const unsigned char* Q,
                               const float* H, int G, int n_levels, double lam, float* codebook, float* What,
                               void* ws, hipStream_t st) {
  const Layout L = make_layout(d_out, d_in, G, n_levels);
  char* p = (char*)ws;
  unsigned short* Hh = (unsigned short*)p;
  p += L.h_bytes;
  unsigned short* Hm = (unsigned short*)p;
  p += L.h_bytes;
  unsigned short* Hl = (unsigned short*)p;
  p += L.h_bytes;
  unsigned short* E = (unsigned short*)p;
  p += L.e_bytes;
  float* T = (float*)p;

  hipError_t e;
  const unsigned t64 = (unsigned)(L.ldp / 64);
  lnq_split_h_kernel<<<dim3(t64, t64, (unsigned)G), dim3(256), 0, st>>>(H, d_in, L.ldp, Hh, Hm, Hl);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  {
    int64_t bx = (L.ldp + 255) / 256;
    if (bx > 64) bx = 64;
    lnq_onehot_kernel<<<dim3((unsigned)bx, (unsigned)d_out), dim3(256), 0, st>>>(Q, d_in, L.ldp, n_levels, E);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  lnq_gemm_kernel<<<dim3((unsigned)(L.n_rt * G), (unsigned)(L.ldp / kTile)), dim3(256), 0, st>>>(
      E, Hh, Hm, Hl, d_out / G * n_levels, L.ldp, L.n_rt, T);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (n_levels <= 4)
    lnq_solve_kernel<4><<<dim3((unsigned)d_out), dim3(256), 0, st>>>(T, Q, W, d_in, ld, L.ldp, n_levels, lam, codebook, What);
  else if (n_levels <= 8)
    lnq_solve_kernel<8><<<dim3((unsigned)d_out), dim3(256), 0, st>>>(T, Q, W, d_in, ld, L.ldp, n_levels, lam, codebook, What);
  else
    lnq_solve_kernel<16><<<dim3((unsigned)d_out), dim3(256), 0, st>>>(T, Q, W, d_in, ld, L.ldp, n_levels, lam, codebook, What);
  return hipGetLastError();
}

}  // namespace gq
