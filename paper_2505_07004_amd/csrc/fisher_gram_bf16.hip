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
//
// Pipeline.  Tokens are consumed 32 at a time through a ring of LDS stages (7 deep when four
// groups share a workgroup).  Stages are filled by direct global->LDS loads
// (global_load_lds_dwordx4: 16 bytes per lane, no VGPR staging), issued 5-6 stages ahead of
// their use so that HBM/L2 latency is covered by a single wave per SIMD; the swizzle is
// applied by choosing which global chunk each lane fetches.  Completion is tracked with an
// explicit s_waitcnt vmcnt(N) per stage followed by the one workgroup barrier of the stage.
// The loop is free of bounds branches: rows past the last token are clamped to the last row
// and get weight 0 (the weights are first repacked group-major and zero-padded into the
// workspace), columns past d_in are clamped into the row pitch and only ever feed outputs
// that are not stored.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kTN = 256;            // tile columns (raw operand)
constexpr int kStep = 32;           // tokens per LDS stage
constexpr int kNB = kTN / 32;       // raw-operand MFMA fragments per wave
constexpr int kMA = 2;              // scaled-operand MFMA fragments per wave (64 rows)
constexpr int kMaxStages = 8;       // upper bound of the ring depth (sizes the weight padding)
constexpr int kLdsBudget = 150 * 1024;

// Byte offset of 16-byte chunk c of token row r in a staged tile whose rows hold CHUNKS
// chunks.  The XOR spreads the four token rows touched by one transposing read (64 bytes
// each per half-wave) over all 64 banks.  It is an involution in c, so the same function maps
// a physical slot back to the logical chunk it holds.
template <int CHUNKS>
__device__ inline int swizzle(int r, int c) {
  if (CHUNKS >= 16) return c ^ (4 * (r & 3));
  return c ^ (4 * ((r >> 1) & 1));
}
template <int CHUNKS>
__device__ inline int lds_chunk_off(int r, int c) {
  return r * (CHUNKS * 16) + 16 * swizzle<CHUNKS>(r, c);
}

typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
typedef char __attribute__((address_space(3))) * lds_char_ptr;

__device__ inline u32x2 lds_read_tr(const char* p) {
  bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)p);
  return __builtin_bit_cast(u32x2, v);
}

// Direct global->LDS load: every active lane moves 16 bytes from its own global address to
// LDS address lds_base + 16*lane (lds_base is wave-uniform and travels in M0).  Tracked by vmcnt.
__device__ inline void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
// Same with 4 bytes per lane (LDS address lds_base + 4*lane).
__device__ inline void dma4(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
template <int N>
__device__ inline void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
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

// Operands of one 16-token sub-step of a wave: the two 64-row fragments already scaled, the
// eight raw 32-column fragments as read.
struct Operands {
  bf16x8 a[kMA];
  u32x2 b[kNB][2];
};
struct RawA {
  u32x2 a[kMA][2];
  f32x4 s[2];
};

template <int GPC>
struct Cfg {
  static constexpr int RB = 4 / GPC;                 // 64-row blocks per workgroup tile
  static constexpr int TM = 64 * RB;                 // tile rows
  static constexpr int kAChunks = TM / 8;            // 16-byte chunks per token row, scaled operand
  static constexpr int kBChunks = kTN / 8;           // 32
  static constexpr int kALoads = (kStep * kAChunks) / 256;  // wave-level 1 KiB loads per wave and stage
  static constexpr int kBLoads = (kStep * kBChunks) / 256;  // 4
  static constexpr int kLoads = kALoads + kBLoads + 1;      // + one 4-byte-per-lane load of the wave's weights
  static constexpr int kABytes = kStep * kAChunks * 16;
  static constexpr int kBBytes = kStep * kBChunks * 16;
  static constexpr int kSBytes = 4 * 64 * 4;         // per wave 64 floats: its 32 weights + 32 of the next stage (unused)
  static constexpr int kStageBytes = kABytes + kBBytes + kSBytes;
  static constexpr int kStages = (kLdsBudget / kStageBytes) < kMaxStages ? (kLdsBudget / kStageBytes) : kMaxStages;
  static_assert(kStages >= 4, "ring too shallow");
  static_assert((kStages - 3) * kLoads <= 63, "vmcnt is a 6-bit counter");
};

// Weights repacked group-major with zero padding: sp[g][i] = s[i][g] for i < n, 0 for n <= i < n_pad.
__global__ __launch_bounds__(256) void pack_weights_kernel(const float* __restrict__ s, int64_t n, int G,
                                                           int64_t n_pad, float* __restrict__ sp) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_pad) return;
  for (int g = 0; g < G; ++g) sp[(int64_t)g * n_pad + i] = (i < n) ? s[i * G + g] : 0.f;
}

template <int GPC>
__global__ __launch_bounds__(256) void fisher_gram_bf16_kernel(const __bf16* __restrict__ X, int64_t n, int64_t d,
                                                               int64_t ld, const float* __restrict__ sp,
                                                               int64_t n_pad, float* __restrict__ H, int accumulate, int n_gsets) {
  using C = Cfg<GPC>;
  constexpr int TM = C::TM, kAChunks = C::kAChunks, kBChunks = C::kBChunks;
  constexpr int kABytes = C::kABytes, kBBytes = C::kBBytes, kStageBytes = C::kStageBytes, NS = C::kStages;

  __shared__ __attribute__((aligned(1024))) char smem[NS * kStageBytes];

  // ---- which tile --------------------------------------------------------------------
  // Workgroups are handed to the 8 XCDs round-robin by their linear id, and every XCD has its
  // own L2.  The id is therefore remapped so that each XCD walks one contiguous range of the
  // work list (ordered by tile column J, then tile row I, then group set): workgroups that are
  // resident on an XCD at the same time share the 256-column raw panel, and both group sets of
  // a tile read identical data.
  int I, J, gset;
  {
    constexpr int kXcd = 8;
    const int64_t total = gridDim.x;
    const int64_t id = blockIdx.x;
    const int64_t x = id % kXcd, idx = id / kXcd;
    const int64_t q = total / kXcd, r = total % kXcd;
    const int64_t logical = x * q + (x < r ? x : r) + idx;
    gset = (int)(logical % n_gsets);
    const int64_t t = logical / n_gsets;
    int dummy;
    tri_decode(t / GPC, dummy, J);
    I = (int)(t - (int64_t)GPC * tri_count(J));
  }
  const int64_t row_t = (int64_t)I * TM;   // first row of the tile
  const int64_t col_t = (int64_t)J * kTN;  // first column of the tile
  const int gbase = gset * GPC;

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int g_local = wave % GPC;
  const int sub = wave / GPC;
  const int64_t row_w = row_t + 64 * sub;  // first row of this wave's block

  // ---- per-lane LDS read offsets (loop invariant) ---------------------------------------
  const int t16 = lane % 16;
  const int krl = 8 * (lane / 32) + t16 / 4;                  // token row inside a 16-token sub-step
  const int clane = 2 * ((lane / 16) % 2) + (t16 % 4) / 2;    // chunk bits 0..1
  const int boff = ((4 * (t16 % 4)) % 8) * 2;                 // byte inside the chunk
  // Fragment y of the raw operand sits at chunk 4*(y ^ q) + clane of its token row, q = krl & 3
  // (the swizzle); only the two low bits of y interact with q, so four per-lane bases plus
  // immediate offsets (256 B per unit of y/4, whole rows per sub-step) address all of them.
  int offA[kMA], offB[4];
#pragma unroll
  for (int x = 0; x < kMA; ++x) offA[x] = lds_chunk_off<kAChunks>(krl, 8 * sub + 4 * x + clane) + boff;
#pragma unroll
  for (int y = 0; y < 4; ++y) offB[y] = kABytes + lds_chunk_off<kBChunks>(krl, 4 * y + clane) + boff;
  const int offS = kABytes + kBBytes + wave * 256 + (8 * (lane / 32)) * 4;

  f32x16 acc[kMA][kNB];
#pragma unroll
  for (int x = 0; x < kMA; ++x)
#pragma unroll
    for (int y = 0; y < kNB; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // ---- direct global->LDS staging -------------------------------------------------------------
  // Wave w issues, per stage, kALoads + kBLoads loads of 1 KiB (64 lanes x 16 B) plus one
  // 8-lane load of its own 32 weights.  LDS slot q (16 B units) of a tile holds token row
  // q / CHUNKS and physical chunk q % CHUNKS; the lane fetches the logical chunk that the
  // swizzle stores there.
  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;
  const int64_t last_row = n - 1;
  const int64_t full_steps = n / kStep;          // stages below this index need no row clamp
  const char* pa[C::kALoads];                    // running global address, stage 0 .. (valid while unclamped)
  const char* pb[C::kBLoads];
  int ra_[C::kALoads], rb_[C::kBLoads];          // token row inside the stage
  int64_t ca_[C::kALoads], cb_[C::kBLoads];      // clamped first column of the lane's chunk
#pragma unroll
  for (int h = 0; h < C::kALoads; ++h) {
    const int q = (wave * C::kALoads + h) * 64 + lane;
    const int r = q / kAChunks;
    int64_t c = row_t + 8 * swizzle<kAChunks>(r, q % kAChunks);
    if (c + 8 > ld) c = ld - 8;                  // stays inside the row pitch; feeds only unstored outputs
    ra_[h] = r;
    ca_[h] = c;
    pa[h] = reinterpret_cast<const char*>(X + (int64_t)r * ld + c);
  }
#pragma unroll
  for (int h = 0; h < C::kBLoads; ++h) {
    const int q = (wave * C::kBLoads + h) * 64 + lane;
    const int r = q / kBChunks;
    int64_t c = col_t + 8 * swizzle<kBChunks>(r, q % kBChunks);
    if (c + 8 > ld) c = ld - 8;
    rb_[h] = r;
    cb_[h] = c;
    pb[h] = reinterpret_cast<const char*>(X + (int64_t)r * ld + c);
  }
  const int64_t step_bytes = (int64_t)kStep * ld * 2;
  // weights: lane l of every wave fetches float l of the wave's group from the current stage on
  // (64 floats: the second half belongs to the next stage and is never read from this slot)
  const char* ps = reinterpret_cast<const char*>(sp + (int64_t)(gbase + g_local) * n_pad + lane);

  // Addresses of the loads of one stage, fixed at the top of the step that issues them.
  const char* cur_ptr[C::kLoads];
  auto prepare = [&](int64_t step) {
    const bool full = step < full_steps;
    const int64_t i0 = step * kStep;
#pragma unroll
    for (int h = 0; h < C::kALoads; ++h) {
      int64_t i = i0 + ra_[h];
      i = i < last_row ? i : last_row;       // only the ragged last stage and stages past the end clamp
      cur_ptr[h] = full ? pa[h] : reinterpret_cast<const char*>(X + i * ld + ca_[h]);
      pa[h] += step_bytes;
    }
#pragma unroll
    for (int h = 0; h < C::kBLoads; ++h) {
      int64_t i = i0 + rb_[h];
      i = i < last_row ? i : last_row;
      cur_ptr[C::kALoads + h] = full ? pb[h] : reinterpret_cast<const char*>(X + i * ld + cb_[h]);
      pb[h] += step_bytes;
    }
    cur_ptr[C::kLoads - 1] = ps;
    ps += kStep * 4;
  };
  auto issue_one = [&](int k, int slot) {     // k-th load of the prepared stage into ring slot `slot`
    const unsigned stage = smem_base + (unsigned)slot * kStageBytes;
    if (k < C::kALoads)
      dma16(cur_ptr[k], stage + (wave * C::kALoads + k) * 1024);
    else if (k < C::kALoads + C::kBLoads)
      dma16(cur_ptr[k], stage + kABytes + (wave * C::kBLoads + (k - C::kALoads)) * 1024);
    else
      dma4(cur_ptr[k], stage + kABytes + kBBytes + wave * 256);
  };
  auto issue = [&](int64_t step, int slot) {
    prepare(step);
#pragma unroll
    for (int k = 0; k < C::kLoads; ++k) issue_one(k, slot);
  };
  auto read_raw_a = [&](RawA& f, const char* stage, int ks) {
    f.s[0] = *reinterpret_cast<const f32x4*>(stage + offS + ks * 64);
    f.s[1] = *reinterpret_cast<const f32x4*>(stage + offS + ks * 64 + 16);
#pragma unroll
    for (int x = 0; x < kMA; ++x) {
      f.a[x][0] = lds_read_tr(stage + offA[x] + ks * 16 * (kAChunks * 16));
      f.a[x][1] = lds_read_tr(stage + offA[x] + (ks * 16 + 4) * (kAChunks * 16));
    }
  };
  auto read_b1 = [&](Operands& o, const char* stage, int ks, int y) {
    const char* p = stage + offB[y % 4] + (y / 4) * 256;
    o.b[y][0] = lds_read_tr(p + ks * 16 * (kBChunks * 16));
    o.b[y][1] = lds_read_tr(p + (ks * 16 + 4) * (kBChunks * 16));
  };
  // One dword (two tokens) of a scaled fragment: bf16 -> fp32, times the token weights, RNE -> bf16.
  auto scale1 = [&](const RawA& f, int x, int q) -> unsigned int {
    const unsigned int w = f.a[x][q / 2][q % 2];
    const f32x4 sv = f.s[q / 2];
    f32x2 v;
    v[0] = __builtin_bit_cast(float, w << 16) * sv[2 * (q % 2)];
    v[1] = __builtin_bit_cast(float, w & 0xffff0000u) * sv[2 * (q % 2) + 1];
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2));
  };
  auto mfma1 = [&](const Operands& o, int i) {   // MFMA number i of a sub-step: fragment pair (x, y) = (i%2, i/2)
    const int x = i % 2, y = i / 2;
    u32x4 bw = {o.b[y][0][0], o.b[y][0][1], o.b[y][1][0], o.b[y][1][1]};
    acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[x], __builtin_bit_cast(bf16x8, bw), acc[x][y], 0, 0, 0);
  };
  // One 16-token sub-step in its exact issue order (scheduling fences keep the compiler from
  // regrouping it): the 16 MFMAs on the current operands, each occupying the matrix core for
  // 32 cycles, with the next sub-step's work slotted in between them: after MFMA 0 the six LDS
  // reads of the next scaled operand and its weights, after MFMAs 1..8 the reads of one raw
  // fragment each, after MFMAs 8..15 one eighth of the scaling (5 VALU operations) each.
  // The direct loads of the stage NS-1 ahead are spread over the two sub-steps (one after every
  // third MFMA or so): issued back to back they would fill the address queue of the memory
  // pipeline and hold the wave, and with it its MFMAs, at the issue stage.
  auto sub_step = [&](const Operands& cur, Operands& nxt, RawA& raw, const char* stage, int ks, int dma_first,
                      int dma_count, int slot) {
    u32x4 an[kMA];
    mfma1(cur, 0);
    read_raw_a(raw, stage, ks);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 1; i <= 8; ++i) {
      mfma1(cur, i);
      read_b1(nxt, stage, ks, i - 1);
      if (i == 8) {
        an[0][0] = scale1(raw, 0, 0);
        asm volatile("" : "+v"(an[0][0]));           // keeps the scaling where it is written (see below)
      }
      if (i % 3 == 2 && i / 3 < dma_count) issue_one(dma_first + i / 3, slot);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 9; i <= 15; ++i) {
      mfma1(cur, i);
      const int piece = i - 8;                       // 1..7
      an[piece / 4][piece % 4] = scale1(raw, piece / 4, piece % 4);
      // an empty asm that "uses" the value: without it the optimiser sinks all the scaling
      // below the last MFMA of the sub-step, where nothing hides it
      asm volatile("" : "+v"(an[piece / 4][piece % 4]));
      if (i % 3 == 2 && i / 3 < dma_count) issue_one(dma_first + i / 3, slot);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int x = 0; x < kMA; ++x) nxt.a[x] = __builtin_bit_cast(bf16x8, an[x]);
  };

  // Stage t lives in ring slot t % NS.  Loads of stages 0 .. NS-2 are issued up front; in
  // iteration t the wave first waits until its own loads of stage t+1 have landed (at most
  // NS-3 younger stages may still be in flight), the barrier then makes every wave's part of
  // stage t+1 visible and proves that stage t-1 is no longer being read, so its slot is
  // refilled with stage t+NS-1.
  const int64_t steps = (n + kStep - 1) / kStep;
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) issue(t, t);
  wait_vmcnt<(NS - 3) * C::kLoads>();
  __builtin_amdgcn_s_barrier();
  int slot_cur = 0, slot_nxt = 1, slot_fill = NS - 1;
  Operands o0, o1;
  RawA raw;
  read_raw_a(raw, smem, 0);
#pragma unroll
  for (int y = 0; y < kNB; ++y) read_b1(o0, smem, 0, y);
#pragma unroll
  for (int x = 0; x < kMA; ++x) o0.a[x] = scale_frag(raw.a[x][0], raw.a[x][1], raw.s[0], raw.s[1]);
  for (int64_t step = 0; step < steps; ++step) {
    wait_vmcnt<(NS - 3) * C::kLoads>();
    __builtin_amdgcn_s_barrier();
    prepare(step + NS - 1);            // past the end this re-reads the last row with weight 0: harmless
    const char* st_cur = smem + slot_cur * kStageBytes;
    const char* st_nxt = smem + slot_nxt * kStageBytes;
    constexpr int kFirstHalf = (C::kLoads + 1) / 2;
    __builtin_amdgcn_sched_barrier(0);
    // tokens 0..15 of the stage; fetches tokens 16..31
    sub_step(o0, o1, raw, st_cur, 1, 0, kFirstHalf, slot_fill);
    // tokens 16..31; fetches tokens 0..15 of the next stage (complete since the barrier)
    sub_step(o1, o0, raw, st_nxt, 0, kFirstHalf, C::kLoads - kFirstHalf, slot_fill);
    slot_fill = slot_cur;
    slot_cur = slot_nxt;
    slot_nxt = (slot_nxt + 1 == NS) ? 0 : slot_nxt + 1;
  }
  wait_vmcnt<0>();   // no load may still be writing this workgroup's LDS when it is released

  // ---- epilogue: register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32 ------
  float* Hk = H + (int64_t)(gbase + g_local) * d * d;
#pragma unroll
  for (int y = 0; y < kNB; ++y) {
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

int64_t padded_tokens(int64_t n) { return (n + kStep - 1) / kStep * kStep + (int64_t)kStep * kMaxStages; }

}  // namespace

size_t fisher_gram_bf16_workspace(int64_t n, int64_t, int G) {
  return (size_t)(padded_tokens(n) * G) * sizeof(float);
}

hipError_t launch_fisher_gram_bf16(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                   float* H, bool accumulate, void* ws, size_t, hipStream_t st) {
  const int64_t n_pad = padded_tokens(n);
  float* sp = (float*)ws;
  pack_weights_kernel<<<dim3((unsigned)((n_pad + 255) / 256)), dim3(256), 0, st>>>(s, n, G, n_pad, sp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int gpc = groups_per_workgroup(G);
  const int n_gsets = G / gpc;
  const dim3 grid((unsigned)(tile_count(d_in, gpc) * n_gsets));
  const __bf16* Xb = (const __bf16*)X;
  const int acc = accumulate ? 1 : 0;
  if (gpc == 4)
    fisher_gram_bf16_kernel<4><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, sp, n_pad, H, acc, n_gsets);
  else if (gpc == 2)
    fisher_gram_bf16_kernel<2><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, sp, n_pad, H, acc, n_gsets);
  else
    fisher_gram_bf16_kernel<1><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, sp, n_pad, H, acc, n_gsets);
  return hipGetLastError();
}

}  // namespace gq
