// Closed-form codebook update of LNQ for fixed assignments (Section 4.2, Eq. "conti-sol";
// Algorithm 2, lines 4 and 14), against the group Hessians:
//     c^(j) = (P^T H P + lam I)^-1 P^T H w_j,      P[i][q] = 1 if Q[j][i] == q else 0.
//
// With E_j = P^T (one-hot rows, one per grid point) the two small quantities of a channel are
//     T_j = E_j H            [m, d_in]      (row q: the sum of the rows of H assigned to q)
//     A_j[q][q'] = sum_{i : Q[j][i] == q'} T_j[q][i],      b_j[q] = sum_i T_j[q][i] * w_j[i].
// T for all channels of a group is ONE contraction (d_out/G * m rows) x d_in x d_in on the bf16
// matrix cores: the one-hot operand is exact in bf16, H is split into three bf16 terms
// (24 mantissa bits), so every product is exact and only the fp32 accumulation rounds.  The
// one-hot operand never exists in memory: every lane builds its fragment from eight code bytes
// with a few integer operations, so only H travels from L2 to LDS.  T never exists in memory
// either: a workgroup bins every 256 x 128 tile of it into its share of A and b while the
// tile is still on chip (through LDS; A by one more one-hot product on the matrix cores, b by
// a plain dot, both in a fixed order) and carries the sums over the column tiles it works
// through; what leaves the kernel is one partial [m][m + 1] system per channel and chunk of
// column tiles.  A second kernel adds the partial
// systems in chunk order and solves the m x m system in fp64 by Gauss-Jordan elimination
// with partial pivoting.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kRows = 256;                           // rows (channel, grid point) of T per workgroup
constexpr int kCols = 128;                           // columns of T (= rows of H) per workgroup
constexpr int kK = 64;                               // contraction elements per stage
constexpr int kHTile = kCols * kK * 2;               // one staged term of H (16 KiB)
constexpr int kHStage = 3 * kHTile;                  // hi, mid, lo: 48 KiB
constexpr int kMaxCh = 64;                           // channels per workgroup at most
constexpr int kQStage = kMaxCh * kK;                 // their codes for one stage (4 KiB)
constexpr int kRing = 3;                             // stages in flight
constexpr int kLoadsPerStage = 7;                    // per wave: 6 pieces of H, 1 of the codes
constexpr unsigned kPadCode = 0x7F;                  // a code no grid point has
constexpr unsigned kNoLevel = 0x7E7E7E7Eu;           // a grid point no code has (rows past the tile's channels)

// Rows [row0, row0 + 64 * gridDim.y) of the full symmetric H[k0 + z] (from its upper triangle), split into
// three bf16 terms, [gridDim.z][pass_rows][ldp] each, zero padded.  One workgroup per 64 x 64 tile.
__global__ __launch_bounds__(256) void lnq_split_h_kernel(const float* __restrict__ H, int64_t d, int64_t ldp, int k0,
                                                          int64_t row0, int64_t pass_rows,
                                                          unsigned short* __restrict__ Hh,
                                                          unsigned short* __restrict__ Hm,
                                                          unsigned short* __restrict__ Hl) {
  __shared__ float tile[64][65];
  const int kk = blockIdx.z;
  const int ti = (int)(row0 / 64) + blockIdx.y, tj = blockIdx.x;
  const float* Hk = H + (int64_t)(k0 + kk) * d * d;
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
    const int64_t il = (int64_t)blockIdx.y * 64 + li, ip = (int64_t)tj * 64 + lj;
    float h;
    if (ti < tj) h = tile[li][lj];
    else if (ti > tj) h = tile[lj][li];
    else h = li <= lj ? tile[li][lj] : tile[lj][li];
    unsigned short a, b, c;
    split3_bf16(h, a, b, c);
    const int64_t off = ((int64_t)kk * pass_rows + il) * ldp + ip;
    Hh[off] = a;
    Hm[off] = b;
    Hl[off] = c;
  }
}

// Qp[j][i] = Q[j][i] for i < d and Q[j][i] < n_levels, else the pad code; row pitch ldp.
__global__ __launch_bounds__(256) void lnq_pad_codes_kernel(const unsigned char* __restrict__ Q, int64_t d, int64_t ldp,
                                                            int n_levels, unsigned char* __restrict__ Qp) {
  const int64_t j = blockIdx.y;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < ldp; i += (int64_t)gridDim.x * 256) {
    const int64_t ic = i < d ? i : d - 1;
    const unsigned code = Q[j * d + ic];
    Qp[j * ldp + i] = (unsigned char)((i < d && code < (unsigned)n_levels) ? code : kPadCode);
  }
}

// Eight bf16 values, 1.0 where the code byte equals the lane's grid point (qrep = that point in
// every byte), else 0.  All bytes involved are below 0x80, so adding 0x7F to a byte sets its
// top bit exactly when the byte is non-zero and never carries into the next byte.
__device__ inline bf16x8 onehot_frag(unsigned c0, unsigned c1, unsigned qrep) {
  const unsigned m0 = ~((c0 ^ qrep) + 0x7F7F7F7Fu) & 0x80808080u;        // 0x80 in every matching byte
  const unsigned m1 = ~((c1 ^ qrep) + 0x7F7F7F7Fu) & 0x80808080u;
  auto one = [](unsigned s) { return (s << 7) - s; };                    // 0x0080 -> 0x3F80 in both halves
  u32x4 v;
  v[0] = one(__builtin_amdgcn_perm(0u, m0, 0x0C010C00u));                 // bytes 0, 1 -> the low bytes of the halves
  v[1] = one(__builtin_amdgcn_perm(0u, m0, 0x0C030C02u));
  v[2] = one(__builtin_amdgcn_perm(0u, m1, 0x0C010C00u));
  v[3] = one(__builtin_amdgcn_perm(0u, m1, 0x0C030C02u));
  return __builtin_bit_cast(bf16x8, v);
}

// T[r][i] = sum_{i'} E[r][i'] * H[k][i][i']  for the rows r = (channel, grid point) of up to 64
// whole channels (256 rows at most) and 128 columns i at a time.  8 waves of 64 x 64 (4 along
// the rows, 2 along the columns).  A stage is 64 contraction elements: one whole 128-byte line
// of each of the 3 x 128 rows of the terms of H, copied straight into LDS
// (global_load_lds_dwordx4; chunk c of row r at position c ^ ((r >> 1) & 7)), and 64 code bytes
// of every channel; a ring of three stages, one barrier per stage.  A lane's contraction
// elements within a stage are the 32 consecutive ones of its half-wave (the matrix cores do not
// care about the order as long as both operands agree), so its codes are two 16-byte reads.
// Three MFMAs per fragment pair (E * lo, E * mid, E * hi).
//
// A workgroup works through `cts_per` consecutive column tiles.  After each, the tile of T goes
// to LDS (the ring is idle then) and is binned where it lies:
//   A[r][u] += sum_i T[r][i] * [Q[j(r)][i] == u]  is one more product with one-hot rows: the rows of
//   the tile are cut into blocks of whole channels (at most 32 rows); for a block, T (split into
//   three bf16 terms, so that the one-hot products are exact again) times the transposed one-hot rows
//   of the same block gives a 32 x 32 result whose entry (r, n) with r and n in the same channel is
//   A[r][level of n].  Wave w owns blocks w and w + 8 and keeps their results in matrix-core
//   accumulators over all column tiles: the order of additions is fixed by the instruction stream.
//   b[r] += sum_i T[r][i] * w[j(r)][i]  in fp32 by two threads per row, 64 columns each, in column order.
// At the end both are written (or, in a later pass over the same channels, added) to row r of
// part[chunk][channel * n_levels + q][LV + 1] (b in column LV).  One launch covers the groups
// [k0, k0 + Gp) and the column tiles [ct0, ct0 + n_ct) whose rows of H the split buffers hold
// ([Gp][pass_rows][ldp]).  Workgroups are renumbered so that each XCD works through chunks of its
// own: a block of H is fetched into one L2 only.
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
constexpr int kTilePitch = kCols + 4;                 // floats per row of the tile of T in LDS (16-byte aligned rows)
template <int LV>
__global__ __launch_bounds__(512) void lnq_gemm_kernel(const unsigned char* __restrict__ Qp,
                                                       const unsigned short* __restrict__ Hh,
                                                       const unsigned short* __restrict__ Hm,
                                                       const unsigned short* __restrict__ Hl,
                                                       const float* __restrict__ W, int64_t ld, int64_t d,
                                                       int64_t per_group, int n_levels, int n_ch, int n_rt, int k0,
                                                       int Gp, int ct0, int n_ct, int cts_per, int n_chunks,
                                                       int64_t ldp, int64_t pass_rows, int64_t part_rows,
                                                       int accumulate, float* __restrict__ part) {
  __shared__ __attribute__((aligned(1024))) char smem[kRing * (kHStage + kQStage)];
  static_assert(kRows * kTilePitch * 4 <= kRing * (kHStage + kQStage), "the tile of T must fit the idle ring");
  const int n_blocks = n_rt * Gp * n_chunks;
  const int per_xcd = (n_blocks + 7) / 8;
  const int v = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
  if (v >= n_blocks) return;                                   // the whole workgroup, before any barrier
  const int chunk = v / (n_rt * Gp), rtg = v % (n_rt * Gp);
  const int kk = rtg / n_rt, rt = rtg % n_rt;
  const int k = k0 + kk;
  const int64_t j0 = (int64_t)k * per_group + (int64_t)rt * n_ch, j_last = (int64_t)(k + 1) * per_group - 1;
  const int64_t ch_left = per_group - (int64_t)rt * n_ch;
  const int rows_here = (int)(ch_left < n_ch ? ch_left : n_ch) * n_levels;   // rows of this tile that exist
  const int ct_first = chunk * cts_per;
  const int ct_end = ct_first + cts_per < n_ct ? ct_first + cts_per : n_ct;
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / 2, wn = wave % 2;
  const int n_stages = (int)(ldp / kK);
  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;
  const unsigned q_base = smem_base + kRing * kHStage;

  // this lane's six 16-byte pieces of a stage of H (for column tile 0) and one of the codes
  const unsigned short* hsrc[6];
  unsigned hdst[6];
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    const int g = wave * 6 + i, term = g / 16, i16 = g % 16;
    const int r = 8 * i16 + lane / 8;
    const int c = (lane % 8) ^ ((r >> 1) & 7);
    const unsigned short* base = term == 0 ? Hh : (term == 1 ? Hm : Hl);
    hsrc[i] = base + ((int64_t)kk * pass_rows + r) * ldp + 8 * c;
    hdst[i] = term * kHTile + i16 * 1024;
  }
  const unsigned char* qsrc;
  {
    const int piece = tid % 256;
    int64_t ch = j0 + piece / 4;
    ch = ch < j_last ? ch : j_last;                            // channels past the group: repeat its last one (never stored)
    qsrc = Qp + ch * ldp + 16 * (piece % 4);
  }
  const unsigned qdst = (wave % 4) * 1024;

  // the two rows of E this lane supplies: channel and grid point
  unsigned qrep[2];
  int qoff[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const int lr = wm * 64 + 32 * x + lane % 32;
    const bool valid = lr < rows_here;
    const int ch = valid ? lr / n_levels : 0;
    qrep[x] = valid ? (unsigned)(lr % n_levels) * 0x01010101u : kNoLevel;
    qoff[x] = ch * kK + 32 * (lane / 32);
  }
  const int lrow = lane % 32;
  auto hfrag = [&](int slot, int term, int row0, int t) -> bf16x8 {
    const int pos = (4 * (lane / 32) + t) ^ ((lrow >> 1) & 7);
    const u32x4 w = *reinterpret_cast<const u32x4*>(&smem[slot * kHStage + term * kHTile + (row0 + lrow) * 128 + pos * 16]);
    return __builtin_bit_cast(bf16x8, w);
  };

  // binning blocks: whole channels, at most 32 rows; this wave owns blocks wave and wave + 8
  const int rpb = (32 / n_levels) * n_levels;
  const int n_bb = (rows_here + rpb - 1) / rpb;                // at most 12 for n_levels <= 16
  float* tile = reinterpret_cast<float*>(smem);
  f32x16 bacc[2];
  int b_arow[2], b_ch[2], b_lvl[2];
  bool b_valid[2];
  unsigned b_qrep[2];
  const unsigned char* b_q[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
#pragma unroll
    for (int r = 0; r < 16; ++r) bacc[x][r] = 0.f;
    const int bb = wave + 8 * x;
    const int nrow = bb * rpb + lane % 32;                     // the row this lane stands for, as A row and as column n
    b_valid[x] = bb < n_bb && lane % 32 < rpb && nrow < rows_here;
    b_arow[x] = nrow < kRows ? nrow : kRows - 1;
    b_ch[x] = b_valid[x] ? nrow / n_levels : 0;
    b_lvl[x] = b_valid[x] ? nrow % n_levels : 0;
    b_qrep[x] = b_valid[x] ? (unsigned)b_lvl[x] * 0x01010101u : kNoLevel;
    b_q[x] = Qp + (j0 + b_ch[x]) * ldp + 8 * (lane / 32);
  }
  // b: two threads per row, 64 columns each
  const int brow = tid / 2, bhalf = tid % 2;
  const bool brow_valid = brow < rows_here;
  const int64_t bj = j0 + (brow_valid ? brow / n_levels : 0);
  float dot = 0.f;

  for (int ct = ct_first; ct < ct_end; ++ct) {
    const int64_t c0 = (int64_t)(ct0 + ct) * kCols;           // first column of T (= row of H) of this tile
    auto issue = [&](int stage, int slot) {
#pragma unroll
      for (int i = 0; i < 6; ++i)
        dma16(hsrc[i] + (int64_t)ct * kCols * ldp + (int64_t)stage * kK, smem_base + slot * kHStage + hdst[i]);
      dma16(qsrc + (int64_t)stage * kK, q_base + slot * kQStage + qdst);
    };
    f32x16 acc[2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

    issue(0, 0);
    issue(n_stages > 1 ? 1 : 0, 1);
    for (int s = 0; s < n_stages; ++s) {
      const int slot = s % kRing;
      wait_vmcnt<kLoadsPerStage>();                         // all but the youngest stage's loads of this wave have landed
      __builtin_amdgcn_s_barrier();                         // everyone's have; and everyone is done with stage s - 1
      issue(s + 2 < n_stages ? s + 2 : n_stages - 1, (s + 2) % kRing);   // past the end: a harmless repeat keeps the count uniform
      u32x4 codes[2][2];
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int h = 0; h < 2; ++h)
          codes[x][h] = *reinterpret_cast<const u32x4*>(&smem[kRing * kHStage + slot * kQStage + qoff[x] + 16 * h]);
#pragma unroll
      for (int t = 0; t < kK / 16; ++t) {
        bf16x8 a[2], bh[2], bm[2], bl[2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const unsigned cl = codes[x][t / 2][2 * (t % 2)], chi = codes[x][t / 2][2 * (t % 2) + 1];
          a[x] = onehot_frag(cl, chi, qrep[x]);
        }
#pragma unroll
        for (int y = 0; y < 2; ++y) {
          bh[y] = hfrag(slot, 0, wn * 64 + y * 32, t);
          bm[y] = hfrag(slot, 1, wn * 64 + y * 32, t);
          bl[y] = hfrag(slot, 2, wn * 64 + y * 32, t);
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
    wait_vmcnt<0>();                                        // the repeats issued past the end
    __syncthreads();                                        // every wave is done with the ring: it becomes the tile of T

    // register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32 of a 32 x 32 block
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int lr = wm * 64 + 32 * x + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
#pragma unroll
        for (int y = 0; y < 2; ++y) tile[lr * kTilePitch + wn * 64 + 32 * y + lane % 32] = acc[x][y][r];
      }
    __builtin_amdgcn_sched_barrier(0);                      // the accumulators are dead from here on: no load moves above
    // the codes of the binning blocks are fetched before the barrier and used after it
    unsigned bcodes[2][8][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
      if (wave + 8 * x < n_bb) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const uint2 cc = *reinterpret_cast<const uint2*>(b_q[x] + c0 + 16 * ks);
          bcodes[x][ks][0] = cc.x;
          bcodes[x][ks][1] = cc.y;
        }
      }
    __syncthreads();
    // the weights of this thread's 64 columns, 32 at a time
    f32x4 wv[8];
    auto fetch_w = [&](int piece) {
      const float* wrow = W + bj * ld;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const int64_t i = c0 + 64 * bhalf + 32 * piece + 4 * c;
        if (i + 3 < d) {
          wv[c] = *reinterpret_cast<const f32x4*>(wrow + i);
        } else {                                            // the ragged end: any finite value will do past d (T is 0 there)
#pragma unroll
          for (int e = 0; e < 4; ++e) wv[c][e] = wrow[i + e < d ? i + e : d - 1];
        }
      }
    };
    if (brow_valid) fetch_w(0);
#pragma unroll
    for (int x = 0; x < 2; ++x)
      if (wave + 8 * x < n_bb) {                              // wave-uniform
        const float* ta = tile + b_arow[x] * kTilePitch + 8 * (lane / 32);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const f32x4 t0 = *reinterpret_cast<const f32x4*>(ta + 16 * ks);
          const f32x4 t1 = *reinterpret_cast<const f32x4*>(ta + 16 * ks + 4);
          u16x8 ah, am, al;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            unsigned short h, m, l;
            split3_bf16(e < 4 ? t0[e] : t1[e - 4], h, m, l);
            ah[e] = h;
            am[e] = m;
            al[e] = l;
          }
          const bf16x8 onehot = onehot_frag(bcodes[x][ks][0], bcodes[x][ks][1], b_qrep[x]);
          bacc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, al), onehot, bacc[x], 0, 0, 0);
          bacc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, am), onehot, bacc[x], 0, 0, 0);
          bacc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ah), onehot, bacc[x], 0, 0, 0);
        }
      }
    __builtin_amdgcn_sched_barrier(0);
    if (brow_valid) {
      const float* trow = tile + brow * kTilePitch + 64 * bhalf;
#pragma unroll
      for (int c = 0; c < 32; ++c) dot += trow[c] * wv[c / 4][c % 4];   // T is exactly 0 in the padded columns
      fetch_w(1);
#pragma unroll
      for (int c = 0; c < 32; ++c) dot += trow[32 + c] * wv[c / 4][c % 4];
    }
    __syncthreads();                                        // the ring is free again
  }

  float* prow = part + ((int64_t)chunk * part_rows + j0 * n_levels) * (LV + 1);
  dot += __shfl_xor(dot, 1, kWave);
  if (brow_valid && bhalf == 0) {
    float* dst = prow + (int64_t)brow * (LV + 1) + LV;
    *dst = accumulate ? *dst + dot : dot;
  }
  // register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32 of a block's 32 x 32 result
#pragma unroll
  for (int x = 0; x < 2; ++x)
    if (b_valid[x]) {
      const int r0 = (wave + 8 * x) * rpb;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        const int row = r0 + rl;
        if (rl < rpb && row < rows_here && row / n_levels == b_ch[x]) {
          float* dst = prow + (int64_t)row * (LV + 1) + b_lvl[x];
          *dst = accumulate ? *dst + bacc[x][r] : bacc[x][r];
        }
      }
    }
}

// One workgroup per channel: adds the partial systems of its m rows in chunk order (A: m x m, b: m),
// solves (A + lam I) c = b in fp64 (Gauss-Jordan elimination with partial pivoting, the
// workgroup's threads sharing the entries of the system), and writes the grid values and, if
// wanted, What[j][i] = c[Q[j][i]].  LV = 4, 8 or 16 bounds the number of grid points.
template <int LV>
__global__ __launch_bounds__(256) void lnq_solve_kernel(const float* __restrict__ part, int n_chunks, int64_t part_rows,
                                                        const unsigned char* __restrict__ Q, int64_t d, int64_t ld,
                                                        int n_levels, double lam, float* __restrict__ codebook,
                                                        float* __restrict__ What) {
  __shared__ double sys[LV][LV + 1];                       // the system; column LV holds b
  __shared__ float cval[LV];
  const int64_t j = blockIdx.x;
  const int tid = threadIdx.x;
  const unsigned char* Qj = Q + j * d;

  for (int e = tid; e < n_levels * (LV + 1); e += 256) {
    const int q = e / (LV + 1), u = e % (LV + 1);
    double a = 0.0;
    if (u < n_levels || u == LV)                             // columns n_levels .. LV - 1 do not exist
      for (int c = 0; c < n_chunks; ++c) a += (double)part[((int64_t)c * part_rows + j * n_levels + q) * (LV + 1) + u];
    sys[q][u] = a + ((u == q) ? lam : 0.0);
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

// The three bf16 terms of H are staged in passes: all groups at once if that fits kSplitBudget,
// else one group and a range of column tiles (= rows of H) at a time.
constexpr size_t kSplitBudget = (size_t)512 << 20;

struct Layout {
  int64_t ldp, part_rows, pass_rows;
  int n_ch, n_rt, n_ct, groups_per_pass, pass_cts, cts_per, chunks_per_pass, lv;
  size_t h_bytes, q_bytes, part_bytes;
};
Layout make_layout(int64_t d_out, int64_t d_in, int G, int n_levels) {
  Layout L;
  L.ldp = (d_in + kCols - 1) / kCols * kCols;
  const int64_t per_group = d_out / G;
  L.n_ch = kRows / n_levels < kMaxCh ? kRows / n_levels : kMaxCh;          // whole channels per workgroup
  L.n_rt = (int)((per_group + L.n_ch - 1) / L.n_ch);
  L.n_ct = (int)(L.ldp / kCols);
  const size_t per_tile_row = (size_t)3 * 2 * L.ldp * kCols;               // bytes of the three terms of one column tile
  if (per_tile_row * L.n_ct * G <= kSplitBudget) {
    L.groups_per_pass = G;
    L.pass_cts = L.n_ct;
  } else {                                                                  // passes of equal size
    L.groups_per_pass = 1;
    int64_t fit = (int64_t)(kSplitBudget / per_tile_row);
    fit = fit < 1 ? 1 : fit;
    const int64_t n_passes = (L.n_ct + fit - 1) / fit;
    L.pass_cts = (int)((L.n_ct + n_passes - 1) / n_passes);
  }
  // Column tiles per chunk: one workgroup per (row block, chunk), one workgroup per compute unit at a time.
  // Chunks stay short (at most 4 tiles): the workgroups of an XCD share a tile's rows of H in their L2 only
  // while they work on the same tile, and they drift apart over a long chunk (16 tiles per chunk ran at half
  // the speed of 1).  Of 4, 3, 2, 1 the first that fills whole rounds of 256 workgroups to 93 %, because
  // every chunk costs a partial system per channel; if none does, the best filled one.
  const int64_t row_blocks = (int64_t)L.n_rt * L.groups_per_pass;
  int best = 1;
  double best_eff = -1.0;
  for (int per = L.pass_cts < 4 ? L.pass_cts : 4; per >= 1; --per) {
    const int64_t chunks = (L.pass_cts + per - 1) / per;
    const int64_t wgs = row_blocks * chunks, rounds = (wgs + 255) / 256;
    const double eff = (double)wgs / (double)(rounds * 256);
    if (wgs >= 256 && eff >= 0.93) {
      best = per;
      break;
    }
    if (eff > best_eff + 1e-9) {
      best_eff = eff;
      best = per;
    }
  }
  L.cts_per = best;
  L.chunks_per_pass = (L.pass_cts + L.cts_per - 1) / L.cts_per;
  L.pass_rows = (int64_t)L.pass_cts * kCols;
  L.lv = n_levels <= 4 ? 4 : (n_levels <= 8 ? 8 : 16);
  L.part_rows = d_out * n_levels;
  auto up = [](size_t b) { return (b + 255) / 256 * 256; };
  L.h_bytes = up((size_t)L.groups_per_pass * L.pass_rows * L.ldp * 2);
  L.q_bytes = up((size_t)d_out * L.ldp);
  L.part_bytes = up((size_t)L.chunks_per_pass * L.part_rows * (L.lv + 1) * sizeof(float));
  return L;
}

}  // namespace

size_t lnq_codebook_workspace(int64_t d_out, int64_t d_in, int G, int n_levels) {
  const Layout L = make_layout(d_out, d_in, G, n_levels);
  return 3 * L.h_bytes + L.q_bytes + L.part_bytes;
}

hipError_t launch_lnq_codebook(const float* W, int64_t d_out, int64_t d_in, int64_t ld, const unsigned char* Q,
                               const float* H, int G, int n_levels, double lam, float* codebook, float* What,
                               void* ws, bool splits_done, hipStream_t st) {
  const Layout L = make_layout(d_out, d_in, G, n_levels);
  // splits_done: an earlier call with the same H and this workspace has left the three terms of H in place
  // (they survive a call only when one pass holds all of them)
  const bool keep_splits = splits_done && L.groups_per_pass == G && L.pass_cts == L.n_ct;
  char* p = (char*)ws;
  unsigned short* Hh = (unsigned short*)p;
  p += L.h_bytes;
  unsigned short* Hm = (unsigned short*)p;
  p += L.h_bytes;
  unsigned short* Hl = (unsigned short*)p;
  p += L.h_bytes;
  unsigned char* Qp = (unsigned char*)p;
  p += L.q_bytes;
  float* part = (float*)p;

  hipError_t e;
  {
    int64_t bx = (L.ldp + 255) / 256;
    if (bx > 64) bx = 64;
    lnq_pad_codes_kernel<<<dim3((unsigned)bx, (unsigned)d_out), dim3(256), 0, st>>>(Q, d_in, L.ldp, n_levels, Qp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  for (int k0 = 0; k0 < G; k0 += L.groups_per_pass) {
    for (int ct0 = 0; ct0 < L.n_ct; ct0 += L.pass_cts) {
      const int n_ct = ct0 + L.pass_cts <= L.n_ct ? L.pass_cts : L.n_ct - ct0;
      const int n_chunks = (n_ct + L.cts_per - 1) / L.cts_per;
      if (!keep_splits) {
        lnq_split_h_kernel<<<dim3((unsigned)(L.ldp / 64), (unsigned)(n_ct * (kCols / 64)), (unsigned)L.groups_per_pass),
                             dim3(256), 0, st>>>(H, d_in, L.ldp, k0, (int64_t)ct0 * kCols, L.pass_rows, Hh, Hm, Hl);
        if ((e = hipGetLastError()) != hipSuccess) return e;
      }
      const int64_t n_blocks = (int64_t)L.n_rt * L.groups_per_pass * n_chunks;
      const int64_t grid = (n_blocks + 7) / 8 * 8;
      if (grid > 0x7fffffff) return hipErrorInvalidValue;
      const int accumulate = ct0 > 0 ? 1 : 0;
#define GQ_LNQ_GEMM(LV)                                                                                                \
  lnq_gemm_kernel<LV><<<dim3((unsigned)grid), dim3(512), 0, st>>>(Qp, Hh, Hm, Hl, W, ld, d_in, d_out / G, n_levels,     \
                                                                  L.n_ch, L.n_rt, k0, L.groups_per_pass, ct0, n_ct,     \
                                                                  L.cts_per, n_chunks, L.ldp, L.pass_rows, L.part_rows, \
                                                                  accumulate, part);
      if (L.lv == 4) {
        GQ_LNQ_GEMM(4)
      } else if (L.lv == 8) {
        GQ_LNQ_GEMM(8)
      } else {
        GQ_LNQ_GEMM(16)
      }
#undef GQ_LNQ_GEMM
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  if (L.lv == 4)
    lnq_solve_kernel<4><<<dim3((unsigned)d_out), dim3(256), 0, st>>>(part, L.chunks_per_pass, L.part_rows, Q, d_in, ld,
                                                                   n_levels, lam, codebook, What);
  else if (L.lv == 8)
    lnq_solve_kernel<8><<<dim3((unsigned)d_out), dim3(256), 0, st>>>(part, L.chunks_per_pass, L.part_rows, Q, d_in, ld,
                                                                   n_levels, lam, codebook, What);
  else
    lnq_solve_kernel<16><<<dim3((unsigned)d_out), dim3(256), 0, st>>>(part, L.chunks_per_pass, L.part_rows, Q, d_in, ld,
                                                                    n_levels, lam, codebook, What);
  return hipGetLastError();
}

}  // namespace gq
