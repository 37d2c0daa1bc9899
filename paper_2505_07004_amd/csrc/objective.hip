// GuidedQuant layer objective (Eq. "ours2", Section 3.2):
//   obj_row[j] = delta_j^T H[k(j)] delta_j,  delta_j = W[j,:] - What[j,:],  obj[k] = sum_{j in J_k} obj_row[j].
//
// The contraction Y = Delta_k H_k (2 d_out d_in^2 flop) runs on the bf16 matrix cores at
// fp32-grade accuracy by splitting both operands into two bf16 terms, x = hi + lo with
// hi = bf16(x), lo = bf16(x - hi) (together 16 mantissa bits), and summing the three products
// hi*hi + hi*lo + lo*hi in fp32 accumulators (the dropped lo*lo term is below 2^-16 relative).
// Only the upper triangle of H is read.  In tile terms
//   delta^T H delta = 2 * sum_{ta < tb} delta_a^T H[ta,tb] delta_b + sum_tb delta_b^T H[tb,tb] delta_b,
// so a workgroup that owns 256 channels (rows j) and a pair of 128-wide column tiles
// (tb = 2P, 2P+1) contracts over a < (2P+2)*128; the accumulators of a column tile are doubled
// once the contraction reaches that tile's diagonal block (everything before it lies strictly
// above the diagonal), the first tile of the pair reads zeros past its diagonal block, and the
// workgroup finishes with partial[P][j] = sum_b Y[j,b] * delta[j,b] in fp32.
//
// Kernels: (1) split delta into hi/lo bf16; (2) split H into hi/lo bf16, TRANSPOSED
// (Hs[k][b][a] = H[k][a][b] for a <= b, the diagonal 128-tiles completed to full squares), so
// that both MFMA operands run along the contraction index a; both are written in the order the
// MFMA kernel consumes them: one contiguous 4 KiB block per (128-row tile, 16 contraction
// elements), already in the swizzled LDS layout, so staging is a linear copy of whole cache
// lines; (3) the MFMA kernel; (4) a two-step reduction that adds the partials of a row in fixed
// order (fp32 obj_row) and the rows of a group in fp64 (obj).  Everything is deterministic.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kTile = 128;            // rows of a staged tile (channels j, or columns b of H)
constexpr int kKS = 16;               // contraction elements per LDS stage (one MFMA deep)
constexpr int kRowBytes = kKS * 2;    // a staged tile row: two 16-byte chunks
constexpr int kTileBytes = kTile * kRowBytes;       // 4 KiB
constexpr int kStageTiles = 8;                      // {Dh, Dl} x 2 row blocks, {Hh, Hl} x 2 column tiles
constexpr int kStageBytes = kStageTiles * kTileBytes;   // 32 KiB
constexpr int kStages = 5;                          // ring depth: 160 KiB, all of a CU
constexpr int kLoadsPerStage = kTileBytes / 1024;   // 1 KiB direct loads per wave and stage (wave w fills tile w)
constexpr int kPairStages = 2 * kTile / kKS;        // stages per pair of 128-tiles along the contraction (16)
constexpr int kOrderP = 4, kOrderR = 8;             // workgroups are ordered in blocks of 4 tile pairs x 8 row blocks
constexpr int kTileElems = kTile * kKS;             // bf16 elements of one staged tile

// Element offset, inside a staged tile, of contraction element e (0..15) of row r (0..127): a row
// is two 16-byte chunks, and rows 8..15 of every 16 keep them swapped, so that the 16-byte
// fragment reads of 16 consecutive rows fall into 16 different bank groups.
__host__ __device__ inline int tile_pos(int r, int e) { return r * kKS + ((((e >> 3) ^ (r >> 3)) & 1) << 3) + (e & 7); }

// Staged tiles of delta: block (k, rb) holds channels k*m + rb*128 + r, r < 128 (zero past the
// end of the group), stage st the contraction elements 16 st .. 16 st + 15 (zero past d):
//   Dh/Dl[((k*n_rb + rb) * n_st + st) * kTileElems + tile_pos(r, e)].
// One workgroup turns 128 rows x 64 contraction elements (four stages) through LDS: a wave
// reads 256 contiguous bytes of a row of W and of What, and writes 1 KiB contiguous.
__global__ __launch_bounds__(256) void split_delta_kernel(const float* __restrict__ W, const float* __restrict__ What,
                                                          int64_t d_out, int64_t d, int64_t ld, int G, int n_rb,
                                                          int64_t n_st, unsigned short* __restrict__ Dh,
                                                          unsigned short* __restrict__ Dl) {
  __shared__ float tile[kTile][64 + 1];
  const int64_t blk = blockIdx.y;
  const int k = (int)(blk / n_rb), rb = (int)(blk % n_rb);
  const int64_t m = d_out / G;
  const int64_t j0 = (int64_t)k * m + (int64_t)rb * kTile, j_end = (int64_t)(k + 1) * m;
  const int64_t a0 = (int64_t)blockIdx.x * 64;
  const int t = threadIdx.x;
  // branch-free (clamped addresses, values selected afterwards) so that all 32 x 2 loads of a thread are in flight together
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const int idx = t + 256 * i;
    const int r = idx / 64, ac = idx % 64;
    const int64_t j = j0 + r, a = a0 + ac;
    const int64_t jc = j < j_end ? j : j_end - 1, acl = a < d ? a : d - 1;
    const float v = W[jc * ld + acl] - What[jc * ld + acl];
    tile[r][ac] = (j < j_end && a < d) ? v : 0.f;
  }
  __syncthreads();
  const int r = t / 2, c = t % 2;
#pragma unroll
  for (int i = 0; i < 4; ++i) {                             // stage i of the block
    u32x4 h4, l4;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      unsigned short h0, l0, h1, l1;
      split_bf16(tile[r][16 * i + 8 * c + e], h0, l0);
      split_bf16(tile[r][16 * i + 8 * c + e + 1], h1, l1);
      h4[e / 2] = (unsigned)h0 | ((unsigned)h1 << 16);
      l4[e / 2] = (unsigned)l0 | ((unsigned)l1 << 16);
    }
    const int64_t st = a0 / kKS + i;
    const int64_t off = (blk * n_st + st) * kTileElems + tile_pos(r, 8 * c);
    *reinterpret_cast<u32x4*>(Dh + off) = h4;
    *reinterpret_cast<u32x4*>(Dl + off) = l4;
  }
}

// Staged tiles of the transposed H: column tile tb holds columns b = 128 tb + r as its rows,
// stage st the contraction elements a = 16 st .. 16 st + 15, for st < 16 (tb / 2 + 1):
//   Hh/Hl[k][(tb * n_st + st) * kTileElems + tile_pos(r, e)] = hi/lo of H[k][a][b]  (a <= b),
// of H[k][b][a] below the diagonal of the diagonal 128-tile, 0 past d; an even tile tb also
// gets eight stages of zeros after its diagonal block.  One workgroup turns a
// block of 64 a x 128 b (four stages) through LDS: coalesced reads along b, 1 KiB contiguous
// writes per wave.
__global__ __launch_bounds__(256) void split_h_kernel(const float* __restrict__ H, int64_t d, int64_t ldp, int64_t n_st,
                                                      unsigned short* __restrict__ Hh,
                                                      unsigned short* __restrict__ Hl) {
  __shared__ float tile[64][kTile + 1];
  const int k = blockIdx.y;
  const float* Hk = H + (int64_t)k * d * d;
  unsigned short* Hhk = Hh + (int64_t)k * ldp * ldp;
  unsigned short* Hlk = Hl + (int64_t)k * ldp * ldp;
  // 128-tiles (ta, tb) with ta/2 <= tb/2: the tile below the diagonal of a pair (ta = tb + 1) is
  // written as zeros, the MFMA kernel runs both column tiles of a pair over the same range
  int ta, tb;
  {
    int pa, pb;
    tri_decode(blockIdx.x / 8, pa, pb);
    const int sub = (blockIdx.x / 2) % 4;
    ta = 2 * pa + (sub & 1);
    tb = 2 * pb + (sub >> 1);
  }
  const int64_t a0 = (int64_t)ta * kTile + 64 * (blockIdx.x % 2), b0 = (int64_t)tb * kTile;
  const int t = threadIdx.x;
  // branch-free inside (clamped addresses, values selected afterwards): all 32 loads of a thread in flight together
  if (ta <= tb) {                                           // uniform; the tile below a pair's diagonal is all zeros
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const int idx = t + 256 * i;
      const int ar = idx / kTile, bc = idx % kTile;
      const int64_t a = a0 + ar, b = b0 + bc;
      const int64_t lo = a < b ? a : b, hi = a < b ? b : a;   // below the diagonal of a diagonal tile: the mirror image
      const int64_t lc = lo < d ? lo : d - 1, hc = hi < d ? hi : d - 1;
      const float v = Hk[lc * d + hc];
      tile[ar][bc] = (hi < d) ? v : 0.f;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 32; ++i) tile[(t + 256 * i) / kTile][(t + 256 * i) % kTile] = 0.f;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {                             // stage i of the block; thread: row t/2, chunk t%2
    const int r = t / 2, c = t % 2;
    u32x4 h4, l4;
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      unsigned short h0, l0, h1, l1;
      split_bf16(tile[16 * i + 8 * c + e][r], h0, l0);
      split_bf16(tile[16 * i + 8 * c + e + 1][r], h1, l1);
      h4[e / 2] = (unsigned)h0 | ((unsigned)h1 << 16);
      l4[e / 2] = (unsigned)l0 | ((unsigned)l1 << 16);
    }
    const int64_t st = a0 / kKS + i;
    const int64_t off = ((int64_t)tb * n_st + st) * kTileElems + tile_pos(r, 8 * c);
    *reinterpret_cast<u32x4*>(Hhk + off) = h4;
    *reinterpret_cast<u32x4*>(Hlk + off) = l4;
  }
}

// Y tile [256 j][256 b] for one pair P of column tiles, on bf16 MFMA with split operands, then
// the row dot.  8 waves: wave (wm, wn) owns rows 64 wm .. 64 wm + 63 and column tile 2P + wn.
//
// Staging.  The eight operand tiles of a stage (128 rows x 16 contraction elements each, 4 KiB
// contiguous in the split arrays and already in LDS order) go from global memory straight into
// LDS (global_load_lds_dwordx4: wave w copies tile w with four 1 KiB loads), kStages - 1 stages
// ahead of their use, tracked by an explicit vmcnt wait and one workgroup barrier per stage.
__global__ __launch_bounds__(512) void objective_mfma_kernel(const unsigned short* __restrict__ Dh,
                                                             const unsigned short* __restrict__ Dl,
                                                             const unsigned short* __restrict__ Hh,
                                                             const unsigned short* __restrict__ Hl,
                                                             const float* __restrict__ W, const float* __restrict__ What,
                                                             int64_t d_out, int64_t d, int64_t ld, int64_t ldp, int G,
                                                             int n_pairs, int n_rb2, int chunk, int n_slots,
                                                             int deal, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(1024))) char smem[kStages * kStageBytes];
  // (the row-sum exchange at the end reuses the staging memory, after a barrier)

  // Work order.  Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2), so
  // the id is first remapped to give every XCD one contiguous stretch of the logical order.
  // That order walks, per group, blocks of kOrderP tile pairs x kOrderR row blocks (heavy pairs
  // first): the workgroups resident on an XCD then share both their H tiles and their delta
  // tiles through its L2.
  // The contraction of pair P (P + 1 pair blocks of 16 stages) is cut into slots of at most
  // `chunk` pair blocks: workgroups of similar length keep pace with their neighbours (and keep
  // sharing tiles), and small problems still give every CU several workgroups; slot 0 is the
  // last (diagonal) part of the heaviest pair.
  int k, sl, rb2;
  {
    constexpr int kXcd = 8, kDeal = kOrderP * kOrderR;      // 32: what the 32 CUs of an XCD run at a time
    const int64_t total = gridDim.x, id = blockIdx.x;
    const int64_t x = id % kXcd, idx = id / kXcd, q = total / kXcd, r = total % kXcd;
    // Large grids (`deal`): stretches of 32 consecutive workgroups of the logical order go to the XCDs in
    // turn; the order is heavy first, so every XCD gets the same share of the work and runs one stretch
    // (one block of pairs x row blocks) at a time.  Small grids: one contiguous stretch per XCD.
    const int64_t dealt = total / (kXcd * kDeal) * (kXcd * kDeal);
    const int64_t logical = !deal ? x * q + (x < r ? x : r) + idx
                                  : (id < dealt ? ((idx / kDeal) * kXcd + x) * kDeal + idx % kDeal : id);
    const int64_t per_group = (int64_t)n_slots * n_rb2;
    k = (int)(logical / per_group);
    int64_t rem = logical - (int64_t)k * per_group;
    // bands of kOrderP slots; the first band holds the remainder
    const int n_bands = (n_slots + kOrderP - 1) / kOrderP;
    const int first_w = n_slots - (n_bands - 1) * kOrderP;
    int band, pw;
    if (rem < (int64_t)first_w * n_rb2) {
      band = 0;
      pw = first_w;
    } else {
      rem -= (int64_t)first_w * n_rb2;
      band = 1 + (int)(rem / ((int64_t)kOrderP * n_rb2));
      rem = rem % ((int64_t)kOrderP * n_rb2);
      pw = kOrderP;
    }
    const int s_lo = band == 0 ? 0 : first_w + (band - 1) * kOrderP;   // first slot of the band
    const int rblk = (int)(rem / ((int64_t)pw * kOrderR));
    const int off = (int)(rem % ((int64_t)pw * kOrderR));
    const int rw = (n_rb2 - rblk * kOrderR) < kOrderR ? (n_rb2 - rblk * kOrderR) : kOrderR;
    sl = s_lo + off / rw;
    rb2 = rblk * kOrderR + off % rw;
  }
  // slot -> (pair, part): pairs from the heaviest down, the parts of a pair from its diagonal end down
  int P = n_pairs - 1, part;
  {
    int rem = sl;
    while (rem >= (P + chunk) / chunk) {                   // number of parts of pair P = ceil((P + 1) / chunk)
      rem -= (P + chunk) / chunk;
      --P;
    }
    part = (P + chunk) / chunk - 1 - rem;
  }
  const int pb_begin = part * chunk;                                        // first pair block of this part
  const bool last_part = (part + 1) * chunk >= P + 1;                       // it ends with the diagonal pair block
  const int64_t m = d_out / G;
  const int64_t j0 = (int64_t)k * m + (int64_t)rb2 * 2 * kTile;   // first channel of this block
  const int64_t j_end = (int64_t)(k + 1) * m;                     // rows >= j_end belong to another group
  const int64_t b0 = (int64_t)P * 2 * kTile;

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / 2, wn = wave % 2;

  // ---- this wave's share of the staging: tile `wave` of every stage, 16 bytes per lane -------
  const int64_t n_st = ldp / kKS;
  const unsigned short* gp[kLoadsPerStage];
  {
    const int which = (wave % 4) / 2;                       // row block / column tile of the pair
    const unsigned short* src =
        wave < 4 ? (wave % 2 == 0 ? Dh : Dl) + (((int64_t)k * n_rb2 + rb2) * 2 + which) * n_st * kTileElems
                 : (wave % 2 == 0 ? Hh : Hl) + (int64_t)k * ldp * ldp + ((int64_t)P * 2 + which) * n_st * kTileElems;
#pragma unroll
    for (int i = 0; i < kLoadsPerStage; ++i) gp[i] = src + (int64_t)pb_begin * kPairStages * kTileElems + i * 512 + lane * 8;
  }
  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;
  // Requests the next stage of the contraction into ring slot `slot`; `advance` is false once
  // the last stage has been requested (later calls fetch it again into a free slot, which
  // keeps the number of loads in flight, and with it the vmcnt arithmetic, constant).
  auto issue = [&](int slot, bool advance) {
    const int step_elems = advance ? kTileElems : 0;
#pragma unroll
    for (int i = 0; i < kLoadsPerStage; ++i) {
      dma16(gp[i], smem_base + slot * kStageBytes + wave * kTileBytes + i * 1024);
      gp[i] += step_elems;
    }
  };

  // ---- fragment addresses: row l % 32 of a 32-row block, chunk l / 32 -----------------------
  const int lrow = lane % 32;
  const int frag_off = lrow * kRowBytes + (((lane / 32) ^ ((lrow >> 3) & 1)) * 16);
  const int a_off = (wm / 2) * 2 * kTileBytes + (wm % 2) * 64 * kRowBytes + frag_off;   // Dh tile; Dl follows it
  const int b_off = (4 + 2 * wn) * kTileBytes + frag_off;                               // Hh tile; Hl follows it
  auto frag = [&](int slot, int off) -> bf16x8 {
    const u32x4 v = *reinterpret_cast<const u32x4*>(&smem[slot * kStageBytes + off]);
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[2][4];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 4; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // Fragments of one stage: rows of delta (hi, lo) and of the transposed H tile (hi, lo).
  struct Frags {
    bf16x8 ah[2], al[2], bh[4], bl[4];
  };
  // The three products of the two 32 x 32 blocks of column block y, interleaved so that
  // consecutive MFMAs never update the same accumulator.
  auto mma = [&](const Frags& f, int y) {
    acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.al[0], f.bh[y], acc[0][y], 0, 0, 0);
    acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.al[1], f.bh[y], acc[1][y], 0, 0, 0);
    acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[0], f.bl[y], acc[0][y], 0, 0, 0);
    acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[1], f.bl[y], acc[1][y], 0, 0, 0);
    acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[0], f.bh[y], acc[0][y], 0, 0, 0);
    acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[1], f.bh[y], acc[1][y], 0, 0, 0);
  };
  auto read_a = [&](Frags& f, int slot, int x) {
    f.ah[x] = frag(slot, a_off + x * 32 * kRowBytes);
    f.al[x] = frag(slot, a_off + kTileBytes + x * 32 * kRowBytes);
  };
  auto read_b = [&](Frags& f, int slot, int y) {
    f.bh[y] = frag(slot, b_off + y * 32 * kRowBytes);
    f.bl[y] = frag(slot, b_off + kTileBytes + y * 32 * kRowBytes);
  };
  auto read_all = [&](Frags& f, int slot) {
#pragma unroll
    for (int x = 0; x < 2; ++x) read_a(f, slot, x);
#pragma unroll
    for (int y = 0; y < 4; ++y) read_b(f, slot, y);
  };
  auto twice = [&]() {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 4; ++y) acc[x][y] *= 2.f;
  };

  // Every kernel argument the epilogue needs is pulled into registers here: a scalar load left
  // pending across the loops would turn the partial LDS-counter waits inside them into full ones.
  asm volatile("" ::"s"(partial), "s"(W), "s"(What), "s"(ld), "s"(d), "s"(d_out), "s"(j_end));

  const int stages = (last_part ? P + 1 : (part + 1) * chunk) * kPairStages;   // end of this part; it has >= 16 stages
#pragma unroll
  for (int t = 0; t < kStages - 1; ++t) issue(t, true);
  int slot_next = 1, slot_fill = kStages - 1;               // ring slots of stage it + 1 and of stage it - 1

  // One step: the MFMAs of stage `it` run on fragments read during the previous step, while
  // the fragments of stage it + 1 are read and stage it + kStages - 1 is requested.  The step
  // is branch-free (past the end it reads a stale slot and requests the last stage again).
  // All eight waves leave the barrier together, so every wave first queues MFMAs and then
  // slips its loads and LDS reads in between groups of six MFMAs, in the order in which the
  // next step consumes them: the matrix pipe has work while the LDS serves the reads, and at
  // most 12 LDS reads are in flight (the counter that tracks them has 4 bits).
  auto fence = [&]() { __builtin_amdgcn_sched_barrier(0); };
  auto step = [&](const Frags& cur, Frags& nxt, int it) {
    wait_vmcnt<(kStages - 3) * kLoadsPerStage>();   // this wave's loads of stage it + 1 have landed
    // everyone's have; and everyone has issued the MFMAs of stage it - 1, so its slot is free
    __builtin_amdgcn_s_barrier();
    fence();
    mma(cur, 0);
    fence();
    issue(slot_fill, it + kStages < stages);
    read_a(nxt, slot_next, 0);
    read_a(nxt, slot_next, 1);
    fence();
    mma(cur, 1);
    fence();
    read_b(nxt, slot_next, 0);
    read_b(nxt, slot_next, 1);
    fence();
    mma(cur, 2);
    fence();
    read_b(nxt, slot_next, 2);
    read_b(nxt, slot_next, 3);
    fence();
    mma(cur, 3);
    fence();
    slot_fill = slot_fill + 1 == kStages ? 0 : slot_fill + 1;
    slot_next = slot_next + 1 == kStages ? 0 : slot_next + 1;
  };

  Frags f0, f1;
  wait_vmcnt<(kStages - 2) * kLoadsPerStage>();
  __builtin_amdgcn_s_barrier();
  read_all(f0, 0);
  int it = pb_begin * kPairStages;
  const int diag0 = P * kPairStages, diag1 = diag0 + kPairStages / 2;
  const int upper_end = last_part ? diag0 : stages;
  for (; it < upper_end; it += 2) {      // strictly above the diagonal for both column tiles
    step(f0, f1, it);
    step(f1, f0, it + 1);
  }
  // what came before counts twice (its mirror image is never visited)
  if (!last_part || (wn == 0 && P > 0)) twice();
  if (last_part) {
    for (; it < diag1; it += 2) {        // diagonal block of the first tile, still above the second's
      step(f0, f1, it);
      step(f1, f0, it + 1);
    }
    if (wn == 1) twice();
    for (; it < stages; it += 2) {       // diagonal block of the second tile (zeros for the first)
      step(f0, f1, it);
      step(f1, f0, it + 1);
    }
  }
  wait_vmcnt<0>();   // the repeated requests of the last stage
  __syncthreads();   // the ring is idle: `red` may reuse it

  // Row dot with delta[j, b] (fp32).  Register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4),
  // column l%32 of a 32 x 32 block.  Branch-free: addresses are clamped into the matrix, which
  // is harmless because Y is exactly 0 in columns b >= d (the padded rows of the transposed H
  // are zeros) and rows j >= j_end are dropped at the final store.
  float v[2][16];
  {
    const int64_t bl = b0 + wn * kTile + lane % 32;
    int64_t bcol[4];
#pragma unroll
    for (int y = 0; y < 4; ++y) bcol[y] = (bl + 32 * y) < d ? (bl + 32 * y) : d - 1;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int64_t j = j0 + wm * 64 + x * 32 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        j = j < j_end ? j : j_end - 1;
        float t = 0.f;
#pragma unroll
        for (int y = 0; y < 4; ++y) t += acc[x][y][r] * (W[j * ld + bcol[y]] - What[j * ld + bcol[y]]);
        v[x][r] = t;
      }
  }
  // Sum over the 32 lanes of each half-wave, for all 32 rows at once: every lane parks its 32
  // values as a column of a 32 x 32 array (pitch 33 floats), then adds up one row of it.
  constexpr int kPitch = 33;
  float* park = reinterpret_cast<float*>(&smem[0]) + (wave * 2 + lane / 32) * 32 * kPitch;
  float (*red)[2 * kTile] = reinterpret_cast<float (*)[2 * kTile]>(&smem[8 * 2 * 32 * kPitch * sizeof(float)]);
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 16; ++r) park[(x * 16 + r) * kPitch + lane % 32] = v[x][r];
  float sum = 0.f;   // no barrier: a wave reads back only what it wrote itself, and its LDS accesses stay in order
#pragma unroll
  for (int c = 0; c < 32; ++c) sum += park[(lane % 32) * kPitch + c];
  {
    const int xr = lane % 32;   // this lane now owns block x = xr / 16, register r = xr % 16 of its half-wave
    red[wn][wm * 64 + (xr / 16) * 32 + 8 * ((xr % 16) / 4) + 4 * (lane / 32) + (xr % 4)] = sum;
  }
  __syncthreads();
  if (tid < 2 * kTile) {
    const int64_t j = j0 + tid;
    if (j < j_end) partial[(int64_t)sl * d_out + j] = red[0][tid] + red[1][tid];
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
    // the partials are added in the order tb = 0, 1, ...; eight loads at a time are in flight (a loop of one load
    // and one add per turn waits for every load in turn)
    float v = 0.f;
    int tb = 0;
    for (; tb + 8 <= n_tb; tb += 8) {
      float p[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) p[u] = partial[(int64_t)(tb + u) * d_out + j];
#pragma unroll
      for (int u = 0; u < 8; ++u) v += p[u];
    }
    for (; tb < n_tb; ++tb) v += partial[(int64_t)tb * d_out + j];
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
  int64_t ldp, n_pairs, n_rb2;
  int chunk, n_slots, deal;                     // pair blocks per workgroup, workgroups per (group, row block), XCD mapping
  int64_t n_blocks;                             // 256-row blocks per group in the final reduction
  size_t partial_bytes, sums_bytes, delta_bytes, h_bytes;   // delta_bytes / h_bytes: one of the hi/lo arrays
};
Layout make_layout(int64_t d_out, int64_t d_in, int G) {
  Layout L;
  L.n_pairs = (d_in + 2 * kTile - 1) / (2 * kTile);
  L.ldp = L.n_pairs * 2 * kTile;                // contraction length padded to whole tile pairs
  L.n_rb2 = (d_out / G + 2 * kTile - 1) / (2 * kTile);
  // Slots of at most `chunk` pair blocks (measured on MI355X over the 7B ... 70B shapes, chunk 1 ... 32, both
  // mappings): grids of a thousand workgroups and more run fastest with 12 and stretches dealt to the XCDs in
  // turn (the order is heavy first; a contiguous eighth per XCD leaves the XCD with the heavy pairs up to 30 %
  // behind); small grids (a few workgroups per CU) with three tenths of the pairs per slot and one contiguous
  // stretch per XCD.
  auto slots_with = [&](int64_t c) {
    int64_t n = 0;
    for (int64_t P = 0; P < L.n_pairs; ++P) n += (P + c) / c;
    return n;
  };
  L.chunk = (int)(L.n_pairs < 12 ? L.n_pairs : 12);
  L.deal = slots_with(L.chunk) * L.n_rb2 * G >= 1024 ? 1 : 0;
  if (!L.deal) {
    L.chunk = (int)((3 * L.n_pairs + 9) / 10);
    if (L.chunk < 2) L.chunk = (int)(L.n_pairs < 2 ? L.n_pairs : 2);
  }
  L.n_slots = 0;
  for (int64_t P = 0; P < L.n_pairs; ++P) L.n_slots += (int)((P + L.chunk) / L.chunk);
  L.partial_bytes = ((size_t)((int64_t)L.n_slots * d_out) * sizeof(float) + 255) / 256 * 256;
  L.n_blocks = (d_out / G + 255) / 256;
  L.sums_bytes = ((size_t)(L.n_blocks * G) * sizeof(double) + 255) / 256 * 256;
  L.delta_bytes = ((size_t)((int64_t)G * L.n_rb2 * 2 * kTile * L.ldp) * 2 + 255) / 256 * 256;
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

  const int n_pairs = (int)L.n_pairs, n_rb2 = (int)L.n_rb2;
  hipError_t e;
  const int64_t n_st = L.ldp / kKS;
  split_delta_kernel<<<dim3((unsigned)(n_st / 4), (unsigned)(G * n_rb2 * 2)), dim3(256), 0, st>>>(W, What, d_out, d_in, ld, G,
                                                                                                 n_rb2 * 2, n_st, Dh, Dl);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  split_h_kernel<<<dim3((unsigned)(8 * tri_count(n_pairs)), (unsigned)G), dim3(256), 0, st>>>(H, d_in, L.ldp, n_st, Hh, Hl);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  objective_mfma_kernel<<<dim3((unsigned)((int64_t)L.n_slots * n_rb2 * G)), dim3(512), 0, st>>>(
      Dh, Dl, Hh, Hl, W, What, d_out, d_in, ld, L.ldp, G, n_pairs, n_rb2, L.chunk, L.n_slots, L.deal, partial);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  objective_rows_kernel<<<dim3((unsigned)L.n_blocks, (unsigned)G), dim3(256), 0, st>>>(partial, d_out, G, L.n_slots, obj_row,
                                                                                       block_sum);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  objective_groups_kernel<<<dim3((unsigned)G), dim3(64), 0, st>>>(block_sum, (int)L.n_blocks, obj);
  return hipGetLastError();
}

}  // namespace gq
