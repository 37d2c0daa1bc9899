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
typedef const f32x4 __attribute__((address_space(3))) * lds_f32x4_ptr;
// Transposing LDS read at a 32-bit LDS byte address.
__device__ inline u32x2 lds_read_tr(unsigned addr) {
  bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(reinterpret_cast<lds_bf16x4_ptr>(addr));
  return __builtin_bit_cast(u32x2, v);
}
// Per-lane LDS byte addresses of one ring stage: the two scaled-operand fragments, the four
// swizzle classes of the raw fragments, the wave's weights.
struct LBase {
  unsigned a[2];
  unsigned b[4];
  unsigned s;
};

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
  bf16x8 a2[kMA];        // second bf16 term of the scaled operand (two-term mode only)
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

// Weights repacked group-major with zero padding: sp[g][i] = s[i][g] for i < n, 0 for n <= i < n_pad
// (ld_s: the row pitch of s in floats).
__global__ __launch_bounds__(256) void pack_weights_kernel(const float* __restrict__ s, int64_t ld_s, int64_t n, int G,
                                                           int64_t n_pad, float* __restrict__ sp) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_pad) return;
  for (int g = 0; g < G; ++g) sp[(int64_t)g * n_pad + i] = (i < n) ? s[i * ld_s + g] : 0.f;
}

// A work item is one tile (TM rows x 256 columns of the upper triangle) for one set of GPC
// groups.  The group set is the fastest index (both sets of a tile read identical data), the
// tiles follow the banded order of band_decode.
struct Item {
  int64_t row_t, col_t;
  int gbase;
};
template <int GPC>
__device__ inline Item decode_item(int64_t item, int n_gsets, int64_t d) {
  const int gset = (int)(item % n_gsets);
  const int64_t t = item / n_gsets;
  int I, J;
  band_decode(t, GPC, (d + kTN - 1) / kTN, I, J);
  Item it;
  it.row_t = (int64_t)I * (64 * (4 / GPC));
  it.col_t = (int64_t)J * kTN;
  it.gbase = gset * GPC;
  return it;
}

// First unit of persistent workgroup p when `units` units are dealt evenly to P workgroups.
__host__ __device__ inline int64_t first_unit(int64_t p, int64_t units, int64_t P) { return p * units / P; }

// Word 3 of a gfx950 raw buffer resource (32-bit untyped data), and a byte offset that lies
// outside every resource built here (each spans at most 64 rows of H).
constexpr int kBufferWord3 = 0x00020000;
constexpr unsigned kBufferOutside = 0x7ffffff0u;

constexpr int kTileFloats = 4 * kMA * kNB * 16 * 64;   // accumulators of one workgroup tile (256 KiB)

// Persistent kernel with a hybrid work split.  P workgroups are resident (one per compute unit).
// With T items of `steps` token steps each, every workgroup first computes floor(T/P) whole
// items, all starting at token 0 at the same time: workgroups that share column panels then
// sweep the tokens in lockstep and find each other's rows in L2.  The T mod P left-over items
// are cut stream-K fashion: their items x steps "units" are dealt out as one contiguous run
// per workgroup, so every compute unit stays busy to the end.  A run that covers all steps of
// an item goes straight into H; a partial run is parked in the workspace and a second small
// kernel adds the parts of every split item in a fixed order.  No workgroup ever waits for
// another one.
// Fewer items than workgroups: there is no whole round then, every item would be cut at token positions that
// differ from workgroup to workgroup and nobody would find a neighbour's rows in L2.  Such a call cuts the
// token steps of every item into `segs` segments of seg_steps steps; the units (segment, item), numbered
// segment-major, take the place of the items (one lock-step round of P units, the rest in runs).  No unit is a
// whole item, so every part is parked -- a unit that one workgroup computes whole in slot 2 P + unit (there are
// fewer than 2 P units) -- and the second kernel writes every item.  The last segment may be shorter than the
// others; the left-over units all belong to it (the plan sees to that), so they are all equally long.
// segs == 1, seg_steps == steps otherwise.
// SPLIT: the scaled operand s * x is carried as TWO bf16 terms (hi + lo, 16 mantissa bits) and every
// fragment pair takes two MFMAs: twice the matrix-core work for products that are exact to 2^-17, so
// that the result is positive semidefinite up to ~1e-5 of its largest eigenvalue instead of ~5e-4.
// The number of token rows a call really holds when only the device knows it (n_dev != nullptr: the rows of the
// heaviest tokens gathered by the call before; the rows past *n_dev are zero with zero weights, so leaving their
// token steps out changes nothing): *n_dev rounded up to whole steps, at least one step, at most n.
__device__ __forceinline__ int64_t tokens_in_use(int64_t n, const int* __restrict__ n_dev) {
  if (!n_dev) return n;
  const int64_t t = *n_dev < 1 ? 1 : *n_dev;
  const int64_t whole = (t + kStep - 1) / kStep * kStep;
  return whole < n ? whole : n;
}

template <int GPC, bool SPLIT>
__global__ __launch_bounds__(256) void fisher_gram_bf16_kernel(const __bf16* __restrict__ X, int64_t n, int64_t d,
                                                               int64_t ld, const float* __restrict__ sp,
                                                               int64_t n_pad, float* __restrict__ H, int accumulate,
                                                               int n_gsets, int64_t n_items, float* __restrict__ partial,
                                                               int segs, int seg_steps, const int* __restrict__ n_dev) {
  using C = Cfg<GPC>;
  n = tokens_in_use(n, n_dev);
  constexpr int kAChunks = C::kAChunks, kBChunks = C::kBChunks;
  constexpr int kABytes = C::kABytes, kBBytes = C::kBBytes, kStageBytes = C::kStageBytes, NS = C::kStages;

  __shared__ __attribute__((aligned(1024))) char smem[NS * kStageBytes];

  // Workgroups are handed to the 8 XCDs round-robin by their id, and every XCD has its own L2.
  // The id is remapped so that each XCD owns one contiguous eighth of the unit range:
  // workgroups resident on an XCD then share raw panels (and both group sets of a tile read
  // identical data).
  const int64_t P = gridDim.x;
  int64_t p;
  {
    constexpr int kXcd = 8;
    const int64_t id = blockIdx.x;
    const int64_t x = id % kXcd, idx = id / kXcd;
    const int64_t q = P / kXcd, r = P % kXcd;
    p = x * q + (x < r ? x : r) + idx;
  }
  const int64_t steps = (n + kStep - 1) / kStep;
  // Without a place to park partial tiles (partial == nullptr: the entry point that allocates nothing)
  // every item is computed whole: ceil(n_items / P) rounds, the last one not full, no left-over runs.
  const int64_t n_units = n_items * segs;
  const int64_t rounds = partial ? n_units / P : (n_units + P - 1) / P;     // whole units per workgroup
  const int tail_steps = (int)(steps - (int64_t)(segs - 1) * seg_steps);    // steps of a unit of the last segment
  const int64_t units = partial ? (n_units - rounds * P) * tail_steps : 0;  // left-over work, dealt out in runs
  const int64_t u_begin = first_unit(p, units, P), u_end = first_unit(p + 1, units, P);

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int g_local = wave % GPC;
  const int sub = wave / GPC;

  // ---- per-lane LDS read offsets (invariant) ----------------------------------------------
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

  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;
  const int64_t last_row = n - 1;
  const int64_t step_bytes = (int64_t)kStep * ld * 2;

  f32x16 acc[kMA][kNB];

  int64_t round = 0;
  for (int64_t u = u_begin; round < rounds || u < u_end;) {
    // the unit and the steps [r0, r1) of it that this pass computes: all uniform, 32-bit, in scalar registers
    auto uniform = [](int64_t v) { return (int)__builtin_amdgcn_readfirstlane((int)v); };
    int unit, r0, r1;
    const bool in_round = round < rounds;
    if (in_round) {                  // a whole unit, in step with every other workgroup
      if (round * P + p >= n_units) break;    // the last round of the schedule without left-over runs
      unit = uniform(round * P + p);
      r0 = 0;
      r1 = -1;                       // all of it
    } else {                         // (part of) a left-over unit
      const int64_t j = u / tail_steps;
      unit = uniform(rounds * P + j);
      r0 = uniform(u - j * tail_steps);
      const int64_t len = (tail_steps - r0) < (u_end - u) ? (tail_steps - r0) : (u_end - u);
      r1 = r0 + uniform(len);
      u += len;                      // the next part starts here
    }
    const int n_items_i = uniform(n_items);
    const int seg = unit / n_items_i, item = unit - seg * n_items_i;
    const int unit_steps = seg == segs - 1 ? tail_steps : seg_steps;
    if (in_round) r1 = unit_steps;
    // Where the result is parked if it is not a whole item: the first part of a workgroup's run in slot 2p, a
    // later one that is not a whole unit (necessarily the last) in 2p+1, a unit computed whole here (in the
    // round, or inside a run) that is a segment of an item in its own slot.  Fixed now: one scalar register
    // across the token loop instead of what it is made of.
    const bool first_part = !in_round && u - (r1 - r0) == u_begin;
    const bool covers_unit = r0 == 0 && r1 == unit_steps;
    const int slot_i = uniform((segs > 1 && covers_unit) ? 2 * P + unit : 2 * p + (first_part ? 0 : 1));
    const int64_t k0 = seg * seg_steps + r0, k1 = seg * seg_steps + r1;
    if (in_round) ++round;
    const Item it = decode_item<GPC>(item, n_gsets, d);
    const int64_t row_t = it.row_t, col_t = it.col_t;
    const int gbase = it.gbase;
    const int64_t row_w = row_t + 64 * sub;      // first row of this wave's block

#pragma unroll
    for (int x = 0; x < kMA; ++x)
#pragma unroll
      for (int y = 0; y < kNB; ++y)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

    // ---- direct global->LDS staging -----------------------------------------------------------
    // Wave w issues, per stage, kALoads + kBLoads loads of 1 KiB (64 lanes x 16 B) plus one
    // 4-byte-per-lane load of its group's weights.  LDS slot q (16 B units) of a tile holds
    // token row q / CHUNKS and physical chunk q % CHUNKS; the lane fetches the logical chunk
    // that the swizzle stores there.
    // Every load is "wave-uniform base + 32-bit byte offset of the lane": the base is the first
    // token row of the stage and lives in scalar registers (advancing a stage is scalar
    // arithmetic), the offset (token row inside the stage x pitch + column) is fixed for the
    // whole item.  Stages past the last one re-read the last one (their data is never used);
    // in the last stage, rows past the last token are read from that token's row instead (their
    // weight is 0): a second set of offsets, swapped in once when the fill reaches that stage.
    unsigned vo[C::kLoads - 1], vo_last[C::kLoads - 1];
    const int r_last = (int)(last_row - (steps - 1) * kStep);      // last valid row of the last stage
#pragma unroll
    for (int h = 0; h < C::kALoads; ++h) {
      const int q = (wave * C::kALoads + h) * 64 + lane;
      const int r = q / kAChunks;
      int64_t c = row_t + 8 * swizzle<kAChunks>(r, q % kAChunks);
      if (c + 8 > ld) c = ld - 8;                  // stays inside the row pitch; feeds only unstored outputs
      vo[h] = (unsigned)((r * ld + c) * 2);
      vo_last[h] = (unsigned)(((r < r_last ? r : r_last) * ld + c) * 2);
    }
#pragma unroll
    for (int h = 0; h < C::kBLoads; ++h) {
      const int q = (wave * C::kBLoads + h) * 64 + lane;
      const int r = q / kBChunks;
      int64_t c = col_t + 8 * swizzle<kBChunks>(r, q % kBChunks);
      if (c + 8 > ld) c = ld - 8;
      vo[C::kALoads + h] = (unsigned)((r * ld + c) * 2);
      vo_last[C::kALoads + h] = (unsigned)(((r < r_last ? r : r_last) * ld + c) * 2);
    }
    // weights: lane l of every wave fetches float l of the wave's group from the stage's first token
    // on (64 floats: the second half belongs to the next stage and is never read from this slot);
    // the padding of the repacked weights makes every such read valid, also past the last stage
    const char* const spg = reinterpret_cast<const char*>(sp + (int64_t)(gbase + g_local) * n_pad);
    unsigned vo_w = (unsigned)lane * 4u;
    asm volatile("" : "+v"(vo_w));       // a fresh live range per item (see the LDS offsets below)
    const char* fbase = nullptr;     // first token row of the stage being filled (scalar)
    const char* wbase = nullptr;     // its weights
    // Point the loads at stage `si` (wave-uniform).
    const int steps32 = (int)steps, k0_32 = (int)k0, k1_32 = (int)k1;   // token steps fit 32 bits (checked on the host)
    auto set_fill = [&](int si) {
      const int se = si < steps32 - 1 ? si : steps32 - 1;
      fbase = reinterpret_cast<const char*>(X) + (int64_t)se * step_bytes;
      wbase = spg + (int64_t)si * (kStep * 4);
      if (se == steps32 - 1) {
#pragma unroll
        for (int k = 0; k < C::kLoads - 1; ++k) vo[k] = vo_last[k];
      }
    };

    // k-th load of the stage set_fill points at, into ring slot `slot`: one scalar move and one
    // memory instruction, small enough to sit between two MFMAs
    auto issue_one = [&](int k, int slot) {
      const unsigned stage = smem_base + (unsigned)slot * kStageBytes;
      if (k < C::kLoads - 1) {
        if (k < C::kALoads)
          dma16s(fbase, vo[k], stage + (wave * C::kALoads + k) * 1024);
        else
          dma16s(fbase, vo[k], stage + kABytes + (wave * C::kBLoads + (k - C::kALoads)) * 1024);
      } else {
        dma4s(wbase, vo_w, stage + kABytes + kBBytes + wave * 256);
      }
    };
    auto issue = [&](int slot) {
#pragma unroll
      for (int k = 0; k < C::kLoads; ++k) issue_one(k, slot);
    };
    // LDS reads of a stage go through per-lane byte addresses (`LBase`: the lane's invariant
    // offsets plus the stage's position in the ring, formed once per stage); everything else is
    // an immediate offset.
    // The lane's invariant offsets, re-defined here for the allocator: their live ranges then start
    // at the token loop that uses them, not at the top of the kernel (where they were being spilled
    // and re-loaded inside the loop, and a scratch re-load waits for every direct load in flight).
    unsigned la[kMA], lb[4], ls = (unsigned)offS;
#pragma unroll
    for (int x = 0; x < kMA; ++x) {
      la[x] = (unsigned)offA[x];
      asm volatile("" : "+v"(la[x]));
    }
#pragma unroll
    for (int y = 0; y < 4; ++y) {
      lb[y] = (unsigned)offB[y];
      asm volatile("" : "+v"(lb[y]));
    }
    asm volatile("" : "+v"(ls));
    auto stage_base = [&](int slot) {
      LBase b;
      const unsigned st = smem_base + (unsigned)slot * kStageBytes;
#pragma unroll
      for (int x = 0; x < kMA; ++x) b.a[x] = st + la[x];
#pragma unroll
      for (int y = 0; y < 4; ++y) b.b[y] = st + lb[y];
      b.s = st + ls;
      return b;
    };
    auto read_raw_a = [&](RawA& f, const LBase& b, int ks) {
      f.s[0] = *reinterpret_cast<lds_f32x4_ptr>(b.s + ks * 64);
      f.s[1] = *reinterpret_cast<lds_f32x4_ptr>(b.s + ks * 64 + 16);
#pragma unroll
      for (int x = 0; x < kMA; ++x) {
        f.a[x][0] = lds_read_tr(b.a[x] + ks * 16 * (kAChunks * 16));
        f.a[x][1] = lds_read_tr(b.a[x] + (ks * 16 + 4) * (kAChunks * 16));
      }
    };
    auto read_b1 = [&](Operands& o, const LBase& b, int ks, int y) {
      const unsigned pp = b.b[y % 4] + (y / 4) * 256;
      o.b[y][0] = lds_read_tr(pp + ks * 16 * (kBChunks * 16));
      o.b[y][1] = lds_read_tr(pp + (ks * 16 + 4) * (kBChunks * 16));
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
    // The two terms of one dword of a scaled fragment: hi = bf16(s * x), lo = bf16(s * x - hi).
    auto scale2 = [&](const RawA& f, int x, int q) -> u32x2 {
      const unsigned int w = f.a[x][q / 2][q % 2];
      const f32x4 sv = f.s[q / 2];
      f32x2 v, r;
      v[0] = __builtin_bit_cast(float, w << 16) * sv[2 * (q % 2)];
      v[1] = __builtin_bit_cast(float, w & 0xffff0000u) * sv[2 * (q % 2) + 1];
      const unsigned int hi = __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2));
      r[0] = v[0] - __builtin_bit_cast(float, hi << 16);
      r[1] = v[1] - __builtin_bit_cast(float, hi & 0xffff0000u);
      const unsigned int lo = __builtin_bit_cast(unsigned int, __builtin_convertvector(r, bf16x2));
      return u32x2{hi, lo};
    };
    // Slot i of a sub-step.  One term: MFMA number i, fragment pair (x, y) = (i%2, i/2).  Two terms: slot
    // i works on y = i/2 for both x, first with the hi term (i even), then with the lo term (i odd), so
    // that the two MFMAs into one accumulator are two MFMAs apart.
    auto mfma1 = [&](const Operands& o, int i) {
      const int y = i / 2;
      u32x4 bw = {o.b[y][0][0], o.b[y][0][1], o.b[y][1][0], o.b[y][1][1]};
      const bf16x8 b8 = __builtin_bit_cast(bf16x8, bw);
      if constexpr (SPLIT) {
        if (i % 2 == 0) {
          acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[0], b8, acc[0][y], 0, 0, 0);
          acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[1], b8, acc[1][y], 0, 0, 0);
        } else {
          acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a2[0], b8, acc[0][y], 0, 0, 0);
          acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a2[1], b8, acc[1][y], 0, 0, 0);
        }
      } else {
        const int x = i % 2;
        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[x], b8, acc[x][y], 0, 0, 0);
      }
    };
    // One 16-token sub-step in its exact issue order (scheduling fences keep the compiler from
    // regrouping it): the 16 MFMAs on the current operands, each occupying the matrix core for
    // 32 cycles, with the next sub-step's work slotted in between them: after MFMA 0 the six LDS
    // reads of the next scaled operand and its weights; after every odd MFMA the reads of the
    // raw fragment that MFMA was the last to use, for the next sub-step, INTO THE SAME registers
    // (one set of raw fragments, refreshed in place: 32 registers less than two alternating sets);
    // after MFMAs 8..15 one eighth of the scaling (5 VALU operations) each.
    // The direct loads of the stage NS-1 ahead are spread over the two sub-steps (one after
    // every third MFMA): issued back to back they would queue up in the memory pipeline.
    auto sub_step = [&](Operands& o, RawA& raw, const LBase& stage, int ks, int dma_first, int dma_count, int slot) {
      u32x4 an[kMA], an2[kMA];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        mfma1(o, i);
        if (i == 0) read_raw_a(raw, stage, ks);
        if (i % 2 == 1) read_b1(o, stage, ks, i / 2);
        if (i >= 8) {
          const int piece = i - 8;                       // 0..7
          if constexpr (SPLIT) {
            const u32x2 hl = scale2(raw, piece / 4, piece % 4);
            an[piece / 4][piece % 4] = hl[0];
            an2[piece / 4][piece % 4] = hl[1];
            asm volatile("" : "+v"(an2[piece / 4][piece % 4]));
          } else {
            an[piece / 4][piece % 4] = scale1(raw, piece / 4, piece % 4);
          }
          // an empty asm that "uses" the value: without it the optimiser sinks all the scaling
          // below the last MFMA of the sub-step, where nothing hides it
          asm volatile("" : "+v"(an[piece / 4][piece % 4]));
        }
        if (i % 3 == 2 && i / 3 < dma_count) issue_one(dma_first + i / 3, slot);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int x = 0; x < kMA; ++x) {
        o.a[x] = __builtin_bit_cast(bf16x8, an[x]);
        if constexpr (SPLIT) o.a2[x] = __builtin_bit_cast(bf16x8, an2[x]);
      }
    };

    // Token step k0 + t of the run lives in ring slot t % NS.  Loads of the first NS-1 stages are
    // issued up front; in iteration t the wave first waits until its own loads of stage t+1
    // have landed (at most NS-3 younger stages may still be in flight), the barrier then makes
    // every wave's part of stage t+1 visible and proves that stage t-1 is no longer being
    // read, so its slot is refilled with stage t+NS-1.
#pragma unroll
    for (int t = 0; t < NS - 1; ++t) {
      set_fill(k0_32 + t);
      issue(t);
    }
    wait_vmcnt<(NS - 3) * C::kLoads>();
    __builtin_amdgcn_s_barrier();
    int slot_cur = 0, slot_nxt = 1, slot_fill = NS - 1;
    Operands o0;
    RawA raw;
    const LBase lb0 = stage_base(0);
    read_raw_a(raw, lb0, 0);
#pragma unroll
    for (int y = 0; y < kNB; ++y) read_b1(o0, lb0, 0, y);
#pragma unroll
    for (int x = 0; x < kMA; ++x) {
      if constexpr (SPLIT) {
        u32x4 h4, l4;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const u32x2 hl = scale2(raw, x, q);
          h4[q] = hl[0];
          l4[q] = hl[1];
        }
        o0.a[x] = __builtin_bit_cast(bf16x8, h4);
        o0.a2[x] = __builtin_bit_cast(bf16x8, l4);
      } else {
        o0.a[x] = scale_frag(raw.a[x][0], raw.a[x][1], raw.s[0], raw.s[1]);
      }
    }
    for (int step = k0_32; step < k1_32; ++step) {
      wait_vmcnt<(NS - 3) * C::kLoads>();
      __builtin_amdgcn_s_barrier();
      set_fill(step + (NS - 1));
      const LBase cur = stage_base(slot_cur), nxt = stage_base(slot_nxt);
      constexpr int kFirstHalf = (C::kLoads + 1) / 2;
      __builtin_amdgcn_sched_barrier(0);
      // tokens 0..15 of the stage; fetches tokens 16..31
      sub_step(o0, raw, cur, 1, 0, kFirstHalf, slot_fill);
      // tokens 16..31; fetches tokens 0..15 of the next stage (complete since the barrier)
      sub_step(o0, raw, nxt, 0, kFirstHalf, C::kLoads - kFirstHalf, slot_fill);
      slot_fill = slot_cur;
      slot_cur = slot_nxt;
      slot_nxt = (slot_nxt + 1 == NS) ? 0 : slot_nxt + 1;
    }
    wait_vmcnt<0>();   // no load may still be writing the ring when it is reused or released

    // ---- epilogue: register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4), column l%32 ------
    if (k0 == 0 && k1 == steps) {
      // Straight-line code with every lane active: H is addressed through a buffer resource
      // that spans exactly the valid rows of this wave's 64-row block, and a lane whose entry
      // lies below the diagonal or right of column d gets an offset outside it (the hardware
      // returns 0 for such a load and drops such a store).  No branch depends on the lane.
      const int64_t rows_valid = (d - row_w) < 64 ? (d - row_w) : 64;
      float* base = H + (int64_t)(gbase + g_local) * d * d + row_w * d;
      const int records = rows_valid > 0 ? (int)(rows_valid * d * (int64_t)sizeof(float)) : 0;
      const __amdgpu_buffer_rsrc_t hres = __builtin_amdgcn_make_buffer_rsrc(base, 0, records, kBufferWord3);
      const int lrow = 4 * (lane / 32), lcol = lane % 32;
      const int delta = lrow - lcol + (int)(row_w - col_t);        // row <= col  <=>  delta + c <= 32 y
      const int cols_left = (int)(d - col_t) - lcol;               // col < d     <=>  32 y < cols_left
      const unsigned off0 = (unsigned)(((int64_t)lrow * d + col_t + lcol) * (int64_t)sizeof(float));
      const unsigned dbytes = (unsigned)(d * (int64_t)sizeof(float));
#pragma unroll
      for (int y = 0; y < kNB; ++y) {
#pragma unroll
        for (int x = 0; x < kMA; ++x) {
          unsigned off[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int c = 32 * x + 8 * (r / 4) + (r % 4);          // row inside the block, less lrow
            const bool keep = (delta + c <= 32 * y) && (32 * y < cols_left);
            off[r] = keep ? off0 + (unsigned)c * dbytes + (unsigned)(32 * y * (int)sizeof(float)) : kBufferOutside;
          }
          if (accumulate) {
            float old[16];
#pragma unroll
            for (int r = 0; r < 16; ++r)
              old[r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(hres, off[r], 0, 0));
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[x][y][r] += old[r];
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float v = acc[x][y][r];   // a scalar copy: a bit cast applied to the vector element itself reads element 0
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), hres, off[r], 0, 0);
          }
        }
      }
    } else {
      float* slot = partial + (size_t)slot_i * kTileFloats + (size_t)wave * (kTileFloats / 4);
#pragma unroll
      for (int x = 0; x < kMA; ++x)
#pragma unroll
        for (int y = 0; y < kNB; ++y)
#pragma unroll
          for (int r = 0; r < 16; ++r) slot[((x * kNB + y) * 16 + r) * 64 + lane] = acc[x][y][r];
    }
    __syncthreads();   // every wave is done with the ring before the next run refills it
  }
}

// Adds the parked parts of every item that was split between workgroups, in a fixed order, and stores the
// sum into H.  blockIdx.x: the left-over item (segs == 1) or the item (segs > 1: every item is split then);
// blockIdx.y: one 32 x 32 accumulator fragment of every wave.  Order: the item's segments by token position,
// the parts of a left-over unit in workgroup order.
template <int GPC>
__global__ __launch_bounds__(256) void fisher_gram_fixup_kernel(int64_t n, int64_t d, float* __restrict__ H,
                                                                int accumulate, int n_gsets, int64_t n_items, int64_t P,
                                                                const float* __restrict__ partial, int segs,
                                                                int seg_steps, const int* __restrict__ n_dev) {
  n = tokens_in_use(n, n_dev);
  const int64_t steps = (n + kStep - 1) / kStep;
  const bool split = segs > 1;
  const int64_t rounds = n_items * segs / P;
  const int64_t tail_steps = steps - (int64_t)(segs - 1) * seg_steps;   // every left-over unit is one of the last segment
  const int64_t units = (n_items * segs - rounds * P) * tail_steps;
  const int64_t item = split ? (int64_t)blockIdx.x : rounds * P + blockIdx.x;
  const Item it = decode_item<GPC>(item, n_gsets, d);
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int g_local = wave % GPC, sub = wave / GPC;
  const int64_t row_w = it.row_t + 64 * sub;
  float* Hk = H + (int64_t)(it.gbase + g_local) * d * d;
  // blockIdx.y picks one 32x32 accumulator fragment (x, y) of every wave
  const int x = blockIdx.y / kNB, y = blockIdx.y % kNB;
  const size_t in_tile = (size_t)wave * (kTileFloats / 4) + lane + (size_t)((x * kNB + y) * 16) * 64;
  const int64_t col = it.col_t + 32 * y + lane % 32;
  float v[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = 0.f;
  for (int seg = 0; seg < segs; ++seg) {
    const int64_t unit = (int64_t)seg * n_items + item;
    if (unit < rounds * P) {                                       // (split only) a whole unit of the lock-step round
      const float* part = partial + (size_t)(2 * P + unit) * kTileFloats + in_tile;
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] += part[r * 64];
      continue;
    }
    const int64_t j = unit - rounds * P;                           // index among the left-over units
    const int64_t lo = j * tail_steps, hi = lo + tail_steps;       // its place in the runs
    // first workgroup whose run reaches into the unit
    int64_t q0 = lo * P / units;
    if (q0 >= P) q0 = P - 1;
    while (q0 > 0 && first_unit(q0, units, P) > lo) --q0;
    while (q0 + 1 < P && first_unit(q0 + 1, units, P) <= lo) ++q0;
    if (!split && first_unit(q0, units, P) <= lo && first_unit(q0 + 1, units, P) >= hi) return;   // one run covers the item: already in H
    for (int64_t q = q0; q < P; ++q) {
      const int64_t b0 = first_unit(q, units, P), b1 = first_unit(q + 1, units, P);
      if (b0 >= hi) break;
      if (b1 == b0) continue;                                      // this workgroup had no left-over run
      const int64_t r0 = (b0 > lo ? b0 : lo) - lo, r1 = (b1 < hi ? b1 : hi) - lo;   // its part of the unit
      // a run parks its first part in slot 2q and a later (necessarily last) part in 2q+1; with segments, a
      // part that is the whole unit in the unit's own slot
      const int64_t slot_i = (split && r0 == 0 && r1 == tail_steps) ? 2 * P + unit : 2 * q + (b0 >= lo ? 0 : 1);
      const float* part = partial + (size_t)slot_i * kTileFloats + in_tile;
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] += part[r * 64];
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int64_t row = row_w + 32 * x + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
    if (row < d && col < d && row <= col) {
      float* ph = Hk + row * d + col;
      *ph = accumulate ? *ph + v[r] : v[r];
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

constexpr int kMaxWorkgroups = 256;   // one persistent workgroup per compute unit of an MI355X
constexpr int kMinUnitsPerWorkgroup = 32;

constexpr int64_t kMinSegmentSteps = 32;   // a segment of an item's token steps is at least 1024 tokens
constexpr int64_t kMaxSegments = 3;        // more of them cost more in parked tiles than the shared panels save
struct Plan {
  int gpc, n_gsets, segs;
  int64_t n_pad, n_items, P, seg_steps;
  size_t sp_bytes, partial_bytes;
  int64_t n_units() const { return n_items * segs; }
};
// with_workspace: the call can park partial tiles (runs of left-over units, segments of items)
Plan make_plan(int64_t n, int64_t d_in, int G, bool with_workspace = true) {
  Plan pl;
  pl.gpc = groups_per_workgroup(G);
  pl.n_gsets = G / pl.gpc;
  pl.n_pad = padded_tokens(n);
  const int64_t steps = (n + kStep - 1) / kStep;
  pl.n_items = tile_count(d_in, pl.gpc) * pl.n_gsets;
  int64_t P = pl.n_items * steps / kMinUnitsPerWorkgroup;
  if (P < 1) P = 1;
  if (P > kMaxWorkgroups) P = kMaxWorkgroups;
  pl.segs = 1;
  pl.seg_steps = steps;
  if (with_workspace && pl.n_items < P) {                   // no whole round of items: segments of their token steps
    const int64_t want = (P + pl.n_items - 1) / pl.n_items;
    const int64_t len = (steps + want - 1) / want;
    const int64_t count = (steps + len - 1) / len;           // no empty last segment
    // fewer than 2 P units: one slot per unit behind the 2 P slots of the runs; the lock-step round takes all
    // units of the segments before the last one, so that the left-over units are equally long
    if (len >= kMinSegmentSteps && count <= kMaxSegments && count * pl.n_items < 2 * P &&
        (count * pl.n_items / P) * P >= (count - 1) * pl.n_items) {
      pl.seg_steps = len;
      pl.segs = (int)count;
    }
  }
  if (!with_workspace) P = pl.n_items < kMaxWorkgroups ? pl.n_items : kMaxWorkgroups;   // whole items only
  pl.P = P;
  pl.sp_bytes = ((size_t)(pl.n_pad * G) * sizeof(float) + 255) / 256 * 256;
  pl.partial_bytes = (size_t)((pl.segs > 1 ? 4 : 2) * P) * kTileFloats * sizeof(float);
  return pl;
}

}  // namespace

// An odd group count from 3 on whose even part the wide kernel takes: that part runs there and the last group
// on the narrow kernel (one-term calls).  Three groups on X[65536,5120]: 4.5 ms instead of 5.0.
static bool runs_in_two_parts(int64_t n, int64_t d_in, int G, bool two_terms) {
  return !two_terms && G >= 3 && G % 2 == 1 && fisher_gram_bf16_wide_chosen(n, d_in, G - 1, false);
}

// Bytes of the repacked weights alone (what a call without partial tiles needs), for either kernel.
size_t fisher_gram_bf16_weights_bytes(int64_t n, int G) {
  if (n <= 0) return 0;
  const size_t narrow = make_plan(n, 8, G).sp_bytes;
  size_t wide = fisher_gram_bf16_wide_applies(n, G, false) ? fisher_gram_bf16_wide_weights_bytes(n, G) : 0;
  // an odd group count may run as its even part on the wide kernel (d_in is not known here)
  if (G >= 3 && G % 2 == 1 && fisher_gram_bf16_wide_applies(n, G - 1, false)) wide = fisher_gram_bf16_wide_weights_bytes(n, G - 1);
  return narrow > wide ? narrow : wide;
}

size_t fisher_gram_bf16_workspace(int64_t n, int64_t d_in, int G) {
  if (n <= 0) return 0;
  const Plan pl = make_plan(n, d_in, G);
  size_t need = pl.sp_bytes + pl.partial_bytes;
  if (fisher_gram_bf16_wide_chosen(n, d_in, G, false)) {      // the flags are not known here: enough for either kernel
    const size_t wide = fisher_gram_bf16_wide_workspace(n, d_in, G);
    if (wide > need) need = wide;
  }
  if (runs_in_two_parts(n, d_in, G, false)) {                 // one part after the other in the same workspace
    const size_t even = fisher_gram_bf16_workspace(n, d_in, G - 1), last = fisher_gram_bf16_workspace(n, d_in, 1);
    if (even > need) need = even;
    if (last > need) need = last;
  }
  return need;
}

namespace {
// G groups whose weights are the columns s[:, 0 .. G-1] of an array with row pitch ld_s, into H[0 .. G-1]
hipError_t launch_groups(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int64_t ld_s, int G, float* H,
                         bool accumulate, bool two_terms, void* ws, bool no_partials, hipStream_t st, const int* n_dev) {
  if (fisher_gram_bf16_wide_chosen(n, d_in, G, two_terms))
    return launch_fisher_gram_bf16_wide(X, n, d_in, ld, s, ld_s, G, H, accumulate, ws, no_partials, st);
  const Plan pl = make_plan(n, d_in, G, !no_partials);
  float* sp = (float*)ws;
  float* partial = no_partials ? nullptr : (float*)((char*)ws + pl.sp_bytes);
  pack_weights_kernel<<<dim3((unsigned)((pl.n_pad + 255) / 256)), dim3(256), 0, st>>>(s, ld_s, n, G, pl.n_pad, sp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t left_over = no_partials ? 0 : pl.n_units() % pl.P;
  const int64_t fix_items = pl.segs > 1 ? pl.n_items : left_over;   // segments: every item is summed from its parts
  const dim3 grid((unsigned)pl.P), fix((unsigned)(fix_items > 0 ? fix_items : 1), (unsigned)(kMA * kNB));
  const int segs = pl.segs, seg_steps = (int)pl.seg_steps;
  const __bf16* Xb = (const __bf16*)X;
  const int acc = accumulate ? 1 : 0;
#define GQ_LAUNCH_GRAM(GPC)                                                                                     \
  if (two_terms)                                                                                                \
    fisher_gram_bf16_kernel<GPC, true><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, sp, pl.n_pad, H, acc,        \
                                                                   pl.n_gsets, pl.n_items, partial, segs,        \
                                                                   seg_steps, n_dev);                            \
  else                                                                                                          \
    fisher_gram_bf16_kernel<GPC, false><<<grid, dim3(256), 0, st>>>(Xb, n, d_in, ld, sp, pl.n_pad, H, acc,       \
                                                                    pl.n_gsets, pl.n_items, partial, segs,       \
                                                                    seg_steps, nullptr);                         \
  e = hipGetLastError();                                                                                        \
  if (e == hipSuccess && fix_items > 0) {                                                                       \
    fisher_gram_fixup_kernel<GPC><<<fix, dim3(256), 0, st>>>(n, d_in, H, acc, pl.n_gsets, pl.n_items, pl.P,      \
                                                             partial, segs, seg_steps, n_dev);                  \
    e = hipGetLastError();                                                                                      \
  }
  if (pl.gpc == 4) {
    GQ_LAUNCH_GRAM(4)
  } else if (pl.gpc == 2) {
    GQ_LAUNCH_GRAM(2)
  } else {
    GQ_LAUNCH_GRAM(1)
  }
#undef GQ_LAUNCH_GRAM
  return e;
}
}  // namespace

hipError_t launch_fisher_gram_bf16(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                   float* H, bool accumulate, bool two_terms, void* ws, bool no_partials, hipStream_t st,
                                   const int* n_dev) {
  if (n_dev && !two_terms) return hipErrorInvalidValue;        // only the two-term pass over gathered rows uses it
  if (!runs_in_two_parts(n, d_in, G, two_terms))
    return launch_groups(X, n, d_in, ld, s, G, G, H, accumulate, two_terms, ws, no_partials, st, n_dev);
  // the even part, then the last group; the second launch reuses the workspace once the first is through with it
  // (same stream)
  hipError_t e = launch_groups(X, n, d_in, ld, s, G, G - 1, H, accumulate, false, ws, no_partials, st, nullptr);
  if (e != hipSuccess) return e;
  return launch_groups(X, n, d_in, ld, s + (G - 1), G, 1, H + (int64_t)(G - 1) * d_in * d_in, accumulate, false, ws,
                       no_partials, st, nullptr);
}

}  // namespace gq
