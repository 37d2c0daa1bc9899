// bf16 matrix-core path of the grouped Fisher Gram (GuidedQuant, Algorithm 1, line 4):
//   H[k][a,b] (+)= sum_i bf16_rne(s[i,k] * X[i,a]) * X[i,b]     for a <= b,  fp32 accumulation.
//
// Work decomposition.  The upper triangle of every H[k] is cut into tiles of TM rows by
// 256 columns.  A workgroup of 4 waves owns one tile for GPC groups at once
// (GPC * TM = 256): every wave computes a 64 x 256 block for ONE group, so the 256-column
// "raw" operand staged in LDS is shared by all groups and each wave scales only its own
// 64-row operand.  The contraction index is the token, which is the strided dimension of
// the row-major X; tiles are therefore staged in LDS exactly as they lie in memory
// ([token][column], 16-byte chunks XOR-swizzled against bank conflicts) and the
// token-major MFMA operands are produced by the CDNA4 transposing LDS read
// (ds_read_b64_tr_b16).  s[i,k] is applied in registers between that read and the MFMA:
// bf16 -> fp32, one fp32 multiply, round-to-nearest-even back to bf16.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kTN = 256;            // tile columns (raw operand)
constexpr int kStep = 32;           // tokens per LDS stage
constexpr int kRowBytes = kTN * 2;  // LDS bytes per token row (both operand tiles use this pitch)
constexpr int kTileBytes = kStep * kRowBytes;
constexpr int kNB = kTN / 32;       // raw-operand MFMA fragments per wave
constexpr int kMA = 2;              // scaled-operand MFMA fragments per wave (64 rows)

// Byte offset of 16-byte chunk c of token row r inside a staged tile.  XOR-ing bits 2..3 of
// the chunk index with r%4 spreads the four token rows of one transposing read over all banks.
__device__ inline int lds_chunk_off(int r, int c) { return r * kRowBytes + 16 * (c ^ (4 * (r & 3))); }

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;

__device__ inline u32x2 lds_read_tr(const char* base, int byte_off) {
  bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(base + byte_off));
  return __builtin_bit_cast(u32x2, v);
}

// 8 bf16 (as 4 dwords) of tokens t..t+7 times their 8 fp32 weights, rounded to bf16 (RNE).
__device__ inline bf16x8 scale_frag(u32x2 lo, u32x2 hi, f32x4 s0, f32x4 s1) {
  unsigned int w[4] = {lo[0], lo[1], hi[0], hi[1]};
  float sc[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
  u32x4 out;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    f32x2 f;
    f[0] = __builtin_bit_cast(float, w[q] << 16) * sc[2 * q];
    f[1] = __builtin_bit_cast(float, w[q] & 0xffff0000u) * sc[2 * q + 1];
    bf16x2 p = __builtin_convertvector(f, bf16x2);
    out[q] = __builtin_bit_cast(unsigned int, p);
  }
  return __builtin_bit_cast(bf16x8, out);
}

__device__ inline u32x4 load_chunk(const __bf16* __restrict__ X, int64_t ld, int64_t n, int64_t d, int64_t i,
                                   int64_t c) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (i < n && c < d) {
    const __bf16* p = X + i * ld + c;
    if (c + 8 <= d) {
      v = *reinterpret_cast<const u32x4*>(p);
    } else {
      unsigned short h[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int e = 0; e < 8; ++e)
        if (c + e < d) h[e] = __builtin_bit_cast(unsigned short, p[e]);
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = (unsigned int)h[2 * q] | ((unsigned int)h[2 * q + 1] << 16);
    }
  }
  return v;
}

template <int GPC>
__global__ __launch_bounds__(256) void fisher_gram_bf16_kernel(const __bf16* __restrict__ X, int64_t n, int64_t d,
                                                               int64_t ld, const float* __restrict__ s, int G,
                                                               float* __restrict__ H, int accumulate) {
  constexpr int RB = 4 / GPC;          // 64-row blocks per workgroup tile
  constexpr int TM = 64 * RB;          // tile rows
  constexpr int kAChunks = TM / 8;     // 16-byte chunks per token row of the scaled operand
  constexpr int kALoads = (kStep * kAChunks) / 256;  // per thread: 1, 2 or 4
  constexpr int kBLoads = (kStep * (kTN / 8)) / 256; // 4

  __shared__ __attribute__((aligned(16))) char As[2][kTileBytes];
  __shared__ __attribute__((aligned(16))) char Bs[2][kTileBytes];
  __shared__ __attribute__((aligned(16))) float Ss[2][GPC][kStep];

  // ---- which tile --------------------------------------------------------------------
  int I, J;
  {
    const int64_t t = blockIdx.x;
    int dummy;
    tri_decode(t / GPC, dummy, J);
    I = (int)(t - (int64_t)GPC * tri_count(J));
  }
  const int64_t row_t = (int64_t)I * TM;   // first row of the tile
  const int64_t col_t = (int64_t)J * kTN;  // first column of the tile
  const int gbase = blockIdx.y * GPC;

  const int tid = threadIdx.x;
  const int lane = tid % kWave, wave = tid / kWave;
  const int g_local = wave % GPC;
  const int sub = wave / GPC;
  const int64_t row_w = row_t + 64 * sub;  // first row of this wave's block
  // fragments of 32 columns that lie entirely below the diagonal are never needed
  int y_first = 0;
  if (row_w > col_t) y_first = (int)((row_w - col_t) / 32);
  const bool wave_active = row_w < d;

  // ---- per-lane LDS read offsets (loop invariant) ---------------------------------------
  const int t16 = lane % 16;
  const int krl = 8 * (lane / 32) + t16 / 4;                  // token row inside a 16-token sub-step
  const int clane = 2 * ((lane / 16) % 2) + (t16 % 4) / 2;    // chunk bits 0..1
  const int boff = ((4 * (t16 % 4)) % 8) * 2;                 // byte inside the chunk
  int offA[kMA], offB[kNB];
#pragma unroll
  for (int x = 0; x < kMA; ++x) offA[x] = lds_chunk_off(krl, 8 * sub + 4 * x + clane) + boff;
#pragma unroll
  for (int y = 0; y < kNB; ++y) offB[y] = lds_chunk_off(krl, 4 * y + clane) + boff;
  const int offS = (8 * (lane / 32)) * 4;

  f32x16 acc[kMA][kNB];
#pragma unroll
  for (int x = 0; x < kMA; ++x)
#pragma unroll
    for (int y = 0; y < kNB; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // ---- staging ------------------------------------------------------------------------------
  u32x4 ra[kALoads], rb[kBLoads];
  float rs = 0.f;
  auto fetch = [&](int64_t step) {
    const int64_t i0 = step * kStep;
#pragma unroll
    for (int h = 0; h < kALoads; ++h) {
      const int q = tid + 256 * h;
      ra[h] = load_chunk(X, ld, n, d, i0 + q / kAChunks, row_t + 8 * (q % kAChunks));
    }
#pragma unroll
    for (int h = 0; h < kBLoads; ++h) {
      const int q = tid + 256 * h;
      rb[h] = load_chunk(X, ld, n, d, i0 + q / (kTN / 8), col_t + 8 * (q % (kTN / 8)));
    }
    if (tid < GPC * kStep) {
      const int64_t i = i0 + tid % kStep;
      rs = (i < n) ? s[i * G + gbase + tid / kStep] : 0.f;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int h = 0; h < kALoads; ++h) {
      const int q = tid + 256 * h;
      *reinterpret_cast<u32x4*>(&As[buf][lds_chunk_off(q / kAChunks, q % kAChunks)]) = ra[h];
    }
#pragma unroll
    for (int h = 0; h < kBLoads; ++h) {
      const int q = tid + 256 * h;
      *reinterpret_cast<u32x4*>(&Bs[buf][lds_chunk_off(q / (kTN / 8), q % (kTN / 8))]) = rb[h];
    }
    if (tid < GPC * kStep) Ss[buf][tid / kStep][tid % kStep] = rs;
  };

  const int64_t steps = (n + kStep - 1) / kStep;
  if (steps > 0) {
    fetch(0);
    stash(0);
  }
  __syncthreads();
  for (int64_t step = 0; step < steps; ++step) {
    const int buf = (int)(step & 1);
    if (step + 1 < steps) fetch(step + 1);
    if (wave_active) {
      const char* Ab = As[buf];
      const char* Bb = Bs[buf];
      const char* Sb = reinterpret_cast<const char*>(&Ss[buf][g_local][0]);
#pragma unroll
      for (int ks = 0; ks < kStep / 16; ++ks) {
        const int roff = ks * 16 * kRowBytes;
        const f32x4 s0 = *reinterpret_cast<const f32x4*>(Sb + offS + ks * 64);
        const f32x4 s1 = *reinterpret_cast<const f32x4*>(Sb + offS + ks * 64 + 16);
        bf16x8 a[kMA];
#pragma unroll
        for (int x = 0; x < kMA; ++x) {
          u32x2 lo = lds_read_tr(Ab, offA[x] + roff);
          u32x2 hi = lds_read_tr(Ab, offA[x] + roff + 4 * kRowBytes);
          a[x] = scale_frag(lo, hi, s0, s1);
        }
#pragma unroll
        for (int y = 0; y < kNB; ++y) {
          if (y >= y_first) {
            u32x2 lo = lds_read_tr(Bb, offB[y] + roff);
            u32x2 hi = lds_read_tr(Bb, offB[y] + roff + 4 * kRowBytes);
            u32x4 bw = {lo[0], lo[1], hi[0], hi[1]};
            bf16x8 b = __builtin_bit_cast(bf16x8, bw);
#pragma unroll
            for (int x = 0; x < kMA; ++x)
              acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[x], b, acc[x][y], 0, 0, 0);
          }
        }
      }
    }
    if (step + 1 < steps) stash(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32 ------
  if (!wave_active) return;
  float* Hk = H + (int64_t)(gbase + g_local) * d * d;
#pragma unroll
  for (int y = 0; y < kNB; ++y) {
    if (y < y_first) continue;
    const int64_t col = col_t + 32 * y + lane % 32;
#pragma unroll
    for (int x = 0; x < kMA; ++x) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = row_w + 32 * x + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        if (row < d && col < d && row <= col) {
          float v = acc[x][y][r];
          float* p = Hk + row * d + col;
          if (accumulate) v += *p;
          *p = v;
        }
      }
    }
  }
}

int groups_per_workgroup(int G) { return (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1; }

int64_t tile_count(int64_t d, int gpc) {
  const int64_t TM = 64 * (4 / gpc);
  const int64_t last = (d + kTN - 1) / kTN - 1;
  int64_t rows_last = (d + TM - 1) / TM;
  if (rows_last > (last + 1) * gpc) rows_last = (last + 1) * gpc;
  return (int64_t)gpc * tri_count(last) + rows_last;
}

}  // namespace

size_t fisher_gram_bf16_workspace(int64_t, int64_t, int) { return 0; }

hipError_t launch_fisher_gram_bf16(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                   float* H, bool accumulate, void*, size_t, hipStream_t st) {
  const int gpc = groups_per_workgroup(G);
  const dim3 grid((unsigned)tile_count(d_in, gpc), (unsigned)(G / gpc));
  const __bf16* Xb = (const __bf16*)X;
  const int acc = accumulate ? 1 : 0;
  if (gpc == 4)
    fisher_gram_bf16_kernel<4><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, s, G, H, acc);
  else if (gpc == 2)
    fisher_gram_bf16_kernel<2><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, s, G, H, acc);
  else
    fisher_gram_bf16_kernel<1><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, s, G, H, acc);
  return hipGetLastError();
}

}  // namespace gq
