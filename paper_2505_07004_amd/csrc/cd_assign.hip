// Cyclic coordinate descent on the assignments against the group Hessians (Section 4.2:
// Algorithm 2 lines 6-12, coordinate update of Eq. "cd_closed_par"; evaluated block-wise in
// the spirit of Algorithms 3 and 4).
//
// For output channel j of group k, with delta = what_j - w_j and Ht[i][i'] = H[k][i][i'] / H[k][i][i]
// (zero diagonal), coordinate i is replaced by the grid point nearest to
//     t = w[i] - sum_{i' != i} Ht[i][i'] * delta[i'],
// coordinates in increasing order, every channel independently.
//
// The coordinates are processed in blocks of 128.  For a block, one GEMM gives
//     B0[j][i] = sum_{i'} delta[j][i'] * Ht[i][i']            (all i', current delta)
// for its 128 coordinates at once (bf16 matrix cores at fp32-grade accuracy: both operands
// split into hi + lo bf16 terms, three products), and a walk goes through the block
// sequentially, four lanes per channel: after coordinate i changes by eps, the targets of the
// later coordinates i'' of the block move by -eps * Ht[i''][i].  The block's new delta is
// written back (split) for the later GEMMs.  The GEMM of block b + 1 runs in the same launch as
// the walk of block b (other workgroups) and leaves out block b's 128 contraction elements; the
// walk of b ends by computing their share from its own fresh values, as one more partial sum of
// block b + 1.
// Compared with Algorithm 4 the bookkeeping differs (the part of the sum that lies outside
// the block is recomputed per block from the current weights instead of being carried along
// and corrected after each block; the flop count is the same), the update rule does not.
#include "gq_internal.hpp"

namespace gq {
namespace {

constexpr int kBlk = 128;             // coordinates per block
constexpr int kRows = 64;             // channels per workgroup of the walk
constexpr int kMaxLevels = 16;        // most grid points per channel (4 bits)

// Ht is stored in the order the GEMM consumes it: per group and block of 128 rows i, for every stage
// of 32 contraction elements i', the 128 rows one after the other, each with its 32 hi halves followed
// by its 32 lo halves (128 bytes): a workgroup's operand tile for a stage is one contiguous 16 KiB run.
// Htl = Hth + 32.
__device__ __forceinline__ int64_t ht_index(int64_t k, int64_t i, int64_t ip, int64_t ldp) {
  return (((k * (ldp / 128) + i / 128) * (ldp / 32) + ip / 32) * 128 + i % 128) * 64 + ip % 32;
}

// Eight consecutive elements i' = ip .. ip + 7 (ip a multiple of 8) of row i: two 16-byte stores, and the
// fp32 copy for the diagonal block's coefficient tile.
__device__ __forceinline__ void store_ht8(int64_t k, int64_t i, int64_t ip, int64_t ldp, const float (&v)[8],
                                          unsigned short* __restrict__ Hth, unsigned short* __restrict__ Htl,
                                          float* __restrict__ Cd) {
  unsigned short hi[8], lo[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) split_bf16(v[e], hi[e], lo[e]);
  u32x4 h, l;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    h[e] = hi[2 * e] | ((unsigned)hi[2 * e + 1] << 16);
    l[e] = lo[2 * e] | ((unsigned)lo[2 * e + 1] << 16);
  }
  const int64_t off = ht_index(k, i, ip, ldp);
  *reinterpret_cast<u32x4*>(Hth + off) = h;
  *reinterpret_cast<u32x4*>(Htl + off) = l;
  if (i / kBlk == ip / kBlk) {
    const int64_t base = (k * (ldp / kBlk) + i / kBlk) * kBlk * kBlk;
#pragma unroll
    for (int e = 0; e < 8; ++e) Cd[base + ((ip + e) % kBlk) * kBlk + (i % kBlk)] = v[e];
  }
}

// Ht (hi/lo bf16, zero diagonal and zero padding, in the order of ht_index) and
// the fp32 coefficients of every diagonal block,
//   Cd[k][blk][a][b] = Ht[blk*128 + b][blk*128 + a]
// (what the target of coordinate b moves by, per unit change of coordinate a; row a contiguous over b).
// Only the upper triangle of H is read, every 64 x 64 tile of it once: its workgroup writes the two
// tiles of Ht it determines.
__global__ __launch_bounds__(256) void cd_prep_kernel(const float* __restrict__ H, int64_t d, int64_t ldp,
                                                      unsigned short* __restrict__ Hth,
                                                      unsigned short* __restrict__ Htl, float* __restrict__ Cd) {
  __shared__ float tile[64][65];
  __shared__ float diag[2][64];
  const int k = blockIdx.z;
  // The tile (ta, tb) of H on or above the diagonal is read once and gives both Ht(ta, tb) and Ht(tb, ta).
  // Consecutive workgroups take consecutive tiles of one tile row, so that together they stream whole rows of H.
  const int n_t = (int)(ldp / 64);
  int ta, tb;
  tri_decode(blockIdx.x, tb, ta);
  ta = n_t - 1 - ta;
  tb = n_t - 1 - tb;
  const float* Hk = H + (int64_t)k * d * d;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  float in[16];                                            // all 16 loads of the thread in flight at once
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int64_t a = (int64_t)ta * 64 + ty + 4 * u, b = (int64_t)tb * 64 + tx;
    in[u] = (a < d && b < d) ? Hk[a * d + b] : 0.f;
  }
#pragma unroll
  for (int u = 0; u < 16; ++u) tile[ty + 4 * u][tx] = in[u];
  if (threadIdx.x < 128) {
    const int64_t i = (int64_t)(threadIdx.x < 64 ? ta : tb) * 64 + threadIdx.x % 64;
    diag[threadIdx.x / 64][threadIdx.x % 64] = i < d ? Hk[i * d + i] : 1.f;
  }
  __syncthreads();
  for (int side = 0; side < (ta == tb ? 1 : 2); ++side) {   // side 0: rows i in tile ta; side 1: rows i in tile tb (transposed)
    const int ti = side == 0 ? ta : tb, tj = side == 0 ? tb : ta;
    for (int idx = threadIdx.x; idx < 64 * 8; idx += 256) {   // local row i, eight local columns i'
      const int li = idx / 8, lj0 = 8 * (idx % 8);
      const int64_t i = (int64_t)ti * 64 + li;
      const float rd = 1.f / diag[side][li];                // one division per row; the products differ from
      float v[8];                                           // the quotients by at most one unit in the last place
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int lj = lj0 + e;
        const int64_t ip = (int64_t)tj * 64 + lj;
        float h;
        if (ta == tb) h = li <= lj ? tile[li][lj] : tile[lj][li];
        else h = side == 0 ? tile[li][lj] : tile[lj][li];
        v[e] = (i < d && ip < d && i != ip) ? h * rd : 0.f;
      }
      store_ht8(k, i, (int64_t)tj * 64 + lj0, ldp, v, Hth, Htl, Cd);
    }
  }
}

// The same two outputs for sequential rounding with error feedback (GPTQ / LDLQ) from the upper
// triangular factor R of the damped matrix, A = R R^T: the feedback a coordinate i receives from an
// EARLIER coordinate i' is R[i'][i] / R[i][i] per unit of error, later coordinates give none:
//   Ht[i][i'] = R[i'][i] / R[i][i]  for i' < i,  0 otherwise.
__global__ __launch_bounds__(256) void ldlq_prep_kernel(const float* __restrict__ R, int64_t d, int64_t ldp,
                                                        unsigned short* __restrict__ Hth,
                                                        unsigned short* __restrict__ Htl, float* __restrict__ Cd) {
  __shared__ float tile[64][65];
  __shared__ float diag[64];
  const int k = blockIdx.z;
  const int ti = blockIdx.y, tj = blockIdx.x;              // tile of rows i, of columns i'
  const float* Rk = R + (int64_t)k * d * d;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  float in[16];                                            // R[i'][i]: rows from the tile of i', columns from the tile of i;
#pragma unroll                                             // all 16 loads of the thread in flight at once
  for (int u = 0; u < 16; ++u) {
    const int64_t a = (int64_t)tj * 64 + ty + 4 * u, b = (int64_t)ti * 64 + tx;
    in[u] = (tj <= ti && a < d && b < d) ? Rk[a * d + b] : 0.f;
  }
#pragma unroll
  for (int u = 0; u < 16; ++u) tile[ty + 4 * u][tx] = in[u];
  if (threadIdx.x < 64) {
    const int64_t i = (int64_t)ti * 64 + threadIdx.x;
    diag[threadIdx.x] = i < d ? Rk[i * d + i] : 1.f;
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < 64 * 8; idx += 256) {   // local row i, eight local columns i'
    const int li = idx / 8, lj0 = 8 * (idx % 8);
    const int64_t i = (int64_t)ti * 64 + li;
    const float rd = 1.f / diag[li];
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int64_t ip = (int64_t)tj * 64 + lj0 + e;
      v[e] = (i < d && ip < i) ? tile[lj0 + e][li] * rd : 0.f;
    }
    store_ht8(k, i, (int64_t)tj * 64 + lj0, ldp, v, Hth, Htl, Cd);
  }
}

// The split delta is stored in the order the GEMM consumes it: for every stage of 32 contraction
// elements, all channels one after the other, each with its 32 hi halves followed by its 32 lo
// halves (128 bytes).  A workgroup's operand tile for a stage (128 channels) is then one contiguous
// 16 KiB run of memory instead of 256 pieces of 64 bytes a whole matrix row apart.  Dl = Dh + 32.
__device__ __forceinline__ int64_t delta_index(int64_t j, int64_t a, int64_t d_out) {
  return ((a >> 5) * d_out + j) * 64 + (a & 31);
}

// Sequential rounding starts from the weights themselves: What = W, no error yet.
__global__ __launch_bounds__(256) void ldlq_init_kernel(const float* __restrict__ W, float* __restrict__ What,
                                                        int64_t d, int64_t ld, int64_t ldp,
                                                        unsigned short* __restrict__ Dh,
                                                        unsigned short* __restrict__ Dl) {
  const int64_t j = blockIdx.y;
  for (int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x; a < ldp; a += (int64_t)gridDim.x * 256) {
    if (a < d) What[j * ld + a] = W[j * ld + a];
    Dh[delta_index(j, a, gridDim.y)] = 0;
    Dl[delta_index(j, a, gridDim.y)] = 0;
  }
}

// Dh/Dl = hi/lo of What[j][a] - W[j][a], a < ldp, zero padded, in the staged order of delta_index.
__global__ __launch_bounds__(256) void cd_delta_kernel(const float* __restrict__ W, const float* __restrict__ What,
                                                       int64_t d, int64_t ld, int64_t ldp,
                                                       unsigned short* __restrict__ Dh,
                                                       unsigned short* __restrict__ Dl) {
  const int64_t j = blockIdx.y;
  for (int64_t a = (int64_t)blockIdx.x * 256 + threadIdx.x; a < ldp; a += (int64_t)gridDim.x * 256) {
    const float v = a < d ? What[j * ld + a] - W[j * ld + a] : 0.f;
    unsigned short h, l;
    split_bf16(v, h, l);
    Dh[delta_index(j, a, gridDim.y)] = h;
    Dl[delta_index(j, a, gridDim.y)] = l;
  }
}

// Partial sums of B0 for block `blk`:  C[part][walk tile][j][i] = sum over this part's contraction
// range of delta[j][i'] * Ht[blk*128 + i][i'],  i < 128, j a channel slot of a 64-channel walk tile
// (the layout of W: coordinates contiguous), WITHOUT the 128 contraction elements of block `excl`:
// those belong to the block that is being walked while this runs, and that walk supplies their
// share itself, as one more part, once they are final.
// A workgroup owns 128 channels of one group and all 128 coordinates of the block; its 4
// waves compute 64 x 64 each.  Both operands are contraction-major in memory; a stage is 32
// contraction elements = one 128-byte line (hi halves, lo halves) of each of the 2 x 128 operand
// rows (delta, Ht), copied straight into LDS (global_load_lds_dwordx4: 8 lanes per row)
// into a ring of four stages.  The loads of a stage are issued two stages ahead, BEFORE the wait
// for the current one, so the memory pipe never runs dry, and a slot is not written again before
// the barrier after its last reader: one barrier per stage.  The parts split the contraction; the
// walk adds them in a fixed order.
constexpr int kGemmRows = 128;                       // channels per workgroup
constexpr int kGemmK = 32;                           // contraction elements per stage
constexpr int kGemmTile = 128 * kGemmK * 2;          // bytes of one staged operand tile (8 KiB)
constexpr int kGemmStage = 4 * kGemmTile;            // 32 KiB
constexpr int kGemmRing = 4;
constexpr int kGemmLoads = kGemmTile / 1024;         // direct loads per lane and stage
constexpr int kBlkStages = kBlk / kGemmK;            // stages per block of coordinates
__device__ __forceinline__ void gemm_far_body(char* smem, int gidx, int part, int n_parts,
                                              const unsigned short* __restrict__ Dh,
                                              const unsigned short* __restrict__ Dl,
                                              const unsigned short* __restrict__ Hth,
                                              const unsigned short* __restrict__ Htl, int64_t d_out, int64_t ldp,
                                              int G, int n_gt, int n_rt, int blk, int excl, int k_stages,
                                              float* __restrict__ C) {
  const int k = gidx / n_gt, gt = gidx % n_gt;
  const int64_t m = d_out / G;
  const int64_t j0 = (int64_t)k * m + (int64_t)gt * kGemmRows, j_last = (int64_t)(k + 1) * m - 1;
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / 2, wn = wave % 2;

  // contraction range of this part, in stages: the first k_stages of the matrix (all of it, or for the
  // strictly lower triangular Ht of sequential rounding the part that is not zero); the excluded block's
  // stages are stepped over
  const int64_t n_stages = k_stages - (excl >= 0 ? kBlkStages : 0);
  const int64_t s0 = (int64_t)part * n_stages / n_parts, s1 = ((int64_t)part + 1) * n_stages / n_parts;
  const int64_t skip_from = excl >= 0 ? kBlkStages * (int64_t)excl : n_stages;   // excl < 0: nothing is stepped over

  // ---- staging: a row of an operand in a stage is one 128-byte line (32 hi halves, then 32 lo halves) and
  // is staged as it lies in memory, so every direct load moves 8 whole lines: waves 0 and 1 copy rows 0..63
  // and 64..127 of delta, waves 2 and 3 of Ht; load number i moves rows 8 i .. 8 i + 7 of the wave's 64,
  // lane -> (row 8 i + lane / 8, position lane % 8).  Logical 16-byte chunk c of row r sits at position
  // c ^ (r & 7): the fragment reads of 8 consecutive rows are conflict-free (the loading lane applies the
  // same XOR when it picks its global chunk; 8 i is a multiple of 8, so its chunk is the same for every load).
  const int op = wave / 2;                                  // 0: delta (over all channels), 1: Ht (the block's 128 rows)
  const unsigned short* src = op == 0 ? Dh : Hth + ht_index(k, (int64_t)blk * kBlk, 0, ldp);
  const int64_t row_first = op == 0 ? j0 : 0, row_last = op == 0 ? j_last : kBlk - 1;
  const int64_t row_pitch = 2 * kGemmK, stage_pitch = (op == 0 ? d_out : (int64_t)kBlk) * 2 * kGemmK;
  const unsigned smem_base = (unsigned)(uintptr_t)(lds_char_ptr)smem;
  const unsigned short* lane_src[kGemmLoads];               // this lane's chunk in stage 0, per load
#pragma unroll
  for (int i = 0; i < kGemmLoads; ++i) {
    const int r = 64 * (wave % 2) + 8 * i + lane / 8;
    const int c = (lane % 8) ^ (r & 7);
    int64_t row = row_first + r;
    row = row < row_last ? row : row_last;                  // rows past the group: repeat its last row
    lane_src[i] = src + row * row_pitch + 8 * c;
  }
  auto issue = [&](int64_t stage) {
    const int slot = (int)((stage - s0) % kGemmRing);
    const int64_t off = (stage < skip_from ? stage : stage + kBlkStages) * stage_pitch;
#pragma unroll
    for (int i = 0; i < kGemmLoads; ++i)
      dma16(lane_src[i] + off, smem_base + slot * kGemmStage + op * (2 * kGemmTile) + (64 * (wave % 2) + 8 * i) * 128);
  };

  // ---- fragments: row l % 32 of a 32-row block, chunk 2 t + l / 32 of the 32 contraction elements of
  // term `term` (0: hi, 1: lo) of operand `o`
  const int lrow = lane % 32;
  auto frag = [&](int slot, int tile, int row0, int t) -> bf16x8 {
    const int o = tile / 2, term = tile % 2;
    const int pos = (4 * term + 2 * t + lane / 32) ^ (lrow & 7);
    const u32x4 v = *reinterpret_cast<const u32x4*>(&smem[slot * kGemmStage + o * (2 * kGemmTile) + (row0 + lrow) * 128 + pos * 16]);
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  if (s0 < s1) issue(s0);
  if (s0 + 1 < s1) issue(s0 + 1);
  for (int64_t s = s0; s < s1; ++s) {
    const int slot = (int)((s - s0) % kGemmRing);
    if (s + 2 < s1) {                                     // uniform
      issue(s + 2);                                       // its slot's last readers were two barriers ago
      wait_vmcnt<2 * kGemmLoads>();                       // this wave's loads of stage s have landed
    } else if (s + 1 < s1) {
      wait_vmcnt<kGemmLoads>();
    } else {
      wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();                         // everyone's have
#pragma unroll
    for (int t = 0; t < kGemmK / 16; ++t) {
      bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        ah[x] = frag(slot, 0, wm * 64 + x * 32, t);
        al[x] = frag(slot, 1, wm * 64 + x * 32, t);
      }
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        bh[y] = frag(slot, 2, wn * 64 + y * 32, t);
        bl[y] = frag(slot, 3, wn * 64 + y * 32, t);
      }
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        // (Ht first: the result's rows, which a lane holds four at a time, are then coordinates)
        acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh[y], al[0], acc[0][y], 0, 0, 0);
        acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh[y], al[1], acc[1][y], 0, 0, 0);
        acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bl[y], ah[0], acc[0][y], 0, 0, 0);
        acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bl[y], ah[1], acc[1][y], 0, 0, 0);
        acc[0][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh[y], ah[0], acc[0][y], 0, 0, 0);
        acc[1][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh[y], ah[1], acc[1][y], 0, 0, 0);
      }
    }
  }
  __syncthreads();                                        // the ring is idle: the output tile may reuse it

  // register r of lane l holds row 8*(r/4)+4*(l/32)+(r%4) (coordinate), column l%32 (channel): four
  // consecutive coordinates per 16-byte LDS store.  The tile leaves as C[part][walk tile][64 channel
  // slots][coordinate] (the walk's tiles are 64 channels, so this tile covers two of them), the layout
  // of W itself; rows past the end of the group repeat its last channel, which fills the slots the walk
  // reads for lanes it never stores.
  constexpr int kOutPitch = kBlk + 4;
  float (*out)[kOutPitch] = reinterpret_cast<float (*)[kOutPitch]>(&smem[0]);   // [channel][coordinate]
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[x][y][4 * r4 + e];
        *reinterpret_cast<f32x4*>(&out[wm * 64 + 32 * x + lane % 32][wn * 64 + 32 * y + 8 * r4 + 4 * (lane / 32)]) = v;
      }
  __syncthreads();
  const int n_walk = n_rt * G;
  for (int idx = tid; idx < kGemmRows * kBlk / 4; idx += 256) {
    const int r = idx / (kBlk / 4), i = 4 * (idx % (kBlk / 4));
    const int rt = 2 * gt + r / kRows;
    if (rt < n_rt) {
      float* dst = C + ((((int64_t)part * n_walk + k * n_rt + rt) * kRows + r % kRows) * kBlk + i);
      *reinterpret_cast<f32x4*>(dst) = *reinterpret_cast<const f32x4*>(&out[r][i]);
    }
  }
}

// The sequential walk through block `blk`: a workgroup of 4 waves per 64 channels of a group,
// FOUR LANES PER CHANNEL.  The block of W and What moves between global memory and LDS 16 bytes
// per lane; the block's 128 x 128 coefficients sit in LDS too.  The 128 targets of a
// channel live in LDS; the block is walked in four runs of 32 coordinates.  Inside a run every
// lane of the quad keeps 8 of the 32 targets in registers: the owner broadcasts the target of
// the current coordinate to its quad (DPP), every lane tries a quarter of the grid, two DPP
// exchanges settle the nearest point (lowest index among equals), and every lane corrects its
// own 8 targets.  The targets after the run are corrected when the run is over (32 changes at
// a time, on the fp32 matrix cores).  Channels past the end of the group repeat its
// last channel, and all four lanes of a quad store the same values, so no lane is ever masked.
// LV = 4, 8 or 16 bounds the number of grid points (the search is unrolled over it).
constexpr int kRun = 32;
constexpr int kQuadSwap1 = 0xB1, kQuadSwap2 = 0x4E;        // DPP quad_perm [1,0,3,2] and [2,3,0,1]
// (every lane of a quad permutation has a source lane, so bound_ctrl only spares the fill of the old value)
template <int CTRL>
__device__ inline float quad_dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ inline unsigned long long quad_key(float dist, int index) {
  return ((unsigned long long)__builtin_bit_cast(unsigned, dist) << 32) | (unsigned)index;
}
template <int CTRL>
__device__ inline int quad_dpp(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
// b[u] += the N parts p .. p + N - 1 of the partial sums, 4 coordinates of 8 channels two rows apart (src
// points at the thread's first one in part 0; a part is `part_stride` floats long): 8 N 16-byte loads in flight
template <int N>
__device__ __forceinline__ void add_parts(f32x4 (&b)[8], const float* __restrict__ src, int p, int64_t part_stride) {
  f32x4 t[N][8];
#pragma unroll
  for (int v = 0; v < N; ++v)
#pragma unroll
    for (int u = 0; u < 8; ++u) t[v][u] = *reinterpret_cast<const f32x4*>(src + (p + v) * part_stride + u * 2 * kBlk);
#pragma unroll
  for (int v = 0; v < N; ++v)
#pragma unroll
    for (int u = 0; u < 8; ++u) b[u] += t[v][u];
}
constexpr int kDeltaPitch = kBlk * 2 + 16;                              // bytes per channel of a delta half staged in LDS
constexpr int kWalkTw = 0;                                              // byte offsets of the walk's LDS arrays
constexpr int kWalkCur = kWalkTw + kBlk * (kRows + 1) * 4;
constexpr int kWalkCoef = kWalkCur + kBlk * (kRows + 1) * 4;
constexpr int kWalkCode = kWalkCoef + kBlk * kBlk * 4;
constexpr int kWalkEps = kWalkCode + kBlk * (kRows + 4);                // the changes made in the current run
constexpr int kWalkBytes = kWalkEps + kRun * (kRows + 1) * 4;
static_assert(kWalkEps % 4 == 0, "floats");
static_assert(2 * kRows * kDeltaPitch <= kWalkCode - kWalkCoef, "the staged delta halves fit where the coefficients were");
static_assert(kWalkCoef % 16 == 0, "the coefficient rows are read 16 bytes at a time");
template <int LV>
__device__ __forceinline__ void walk_body(char* smem, int tile, const float* __restrict__ C, int n_parts,
                                          const float* __restrict__ W, float* __restrict__ What,
                                          const float* __restrict__ codebook, int n_levels,
                                          const float* __restrict__ Cd, const unsigned short* __restrict__ Hth,
                                          const unsigned short* __restrict__ Htl, int64_t d_out, int64_t d,
                                          int64_t ld, int64_t ldp, int G, int n_rt, int blk, int next_blk,
                                          unsigned char* __restrict__ Q, unsigned short* __restrict__ Dh,
                                          unsigned short* __restrict__ Dl, float* __restrict__ E) {
  float (*tw)[kRows + 1] = reinterpret_cast<float (*)[kRows + 1]>(smem + kWalkTw);      // the targets
  float (*cur)[kRows + 1] = reinterpret_cast<float (*)[kRows + 1]>(smem + kWalkCur);    // the block of What, old values then new ones
  float (*coef)[kBlk] = reinterpret_cast<float (*)[kBlk]>(smem + kWalkCoef);            // coef[a][b] = Ht[i0 + b][i0 + a]
  unsigned char (*code)[kRows + 4] = reinterpret_cast<unsigned char (*)[kRows + 4]>(smem + kWalkCode);
  float (*eps)[kRows + 1] = reinterpret_cast<float (*)[kRows + 1]>(smem + kWalkEps);
  const int k = tile / n_rt, rt = tile % n_rt;
  const int64_t m = d_out / G;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int64_t j0 = (int64_t)k * m + (int64_t)rt * kRows, j_last = (int64_t)(k + 1) * m - 1;
  const int n_rows = (int)((j_last - j0 + 1) < kRows ? (j_last - j0 + 1) : kRows);
  const int64_t i0 = (int64_t)blk * kBlk;
  const int n_valid = (int)((d - i0) < kBlk ? (d - i0) : kBlk);   // coordinates of this block inside the matrix

  // The block's 128 x 128 coefficients go straight into LDS (64 KiB, 16 direct loads per wave), and the
  // rows of W and What into registers.
  {
    const float* src = Cd + (((int64_t)k * (ldp / kBlk) + blk) * kBlk) * kBlk;
    const unsigned dst = (unsigned)(uintptr_t)(lds_char_ptr)(smem + kWalkCoef);
    const int w_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
    for (int i = 0; i < 16; ++i) dma16(src + (w_u * 16 + i) * 256 + lane * 4, dst + (w_u * 16 + i) * 1024);
  }
  // the walk proper: channel ch of the tile, lane q of its quad, which tries levels q, q + 4, ...
  const int ch = 16 * wave + lane / 4, q = lane % 4;
  const int64_t j = ch < n_rows ? j0 + ch : j_last;
  float grid[LV / 4];
#pragma unroll
  for (int u = 0; u < LV / 4; ++u) {
    const int lvl = q + 4 * u;
    grid[u] = lvl < n_levels ? codebook[j * n_levels + lvl] : __builtin_inff();
  }

  // 16 bytes per lane: wave w moves rows 16 w .. 16 w + 15, two at a time, lane l the coordinates
  // 4 (l % 32) .. + 3 of row l / 32 of the pair.  Rows are 16-byte aligned and ld is a multiple of 4, so a
  // vector that starts inside the matrix ends inside the row; coordinates past the end count as zero.
  const int vc = 4 * (lane % 32);                           // first coordinate of this lane's vectors
  const bool vec_in = i0 + vc < d;
  f32x4 wreg[8], creg[8];                                   // W stays in registers for the write-back
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int r = 16 * wave + 2 * u + lane / 32;
    const int64_t jr = r < n_rows ? j0 + r : j_last;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    wreg[u] = vec_in ? *reinterpret_cast<const f32x4*>(W + jr * ld + i0 + vc) : zero;
    creg[u] = vec_in ? *reinterpret_cast<const f32x4*>(What + jr * ld + i0 + vc) : zero;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (i0 + vc + e >= d) {
        wreg[u][e] = 0.f;
        creg[u][e] = 0.f;
      }
  }

  // B0 = the sum of the parts in order (final since the previous launch), laid out like W and moved by
  // the same lanes; up to 32 16-byte loads in flight behind the ones above.
  f32x4 b0[8];
  {
    const int64_t part_stride = (int64_t)n_rt * G * kBlk * kRows;
    const float* src = C + ((int64_t)tile * kRows + 16 * wave + lane / 32) * kBlk + vc;
#pragma unroll
    for (int u = 0; u < 8; ++u) b0[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    int p = 0;
    for (; p + 4 <= n_parts; p += 4) add_parts<4>(b0, src, p, part_stride);
    if (p + 2 <= n_parts) {
      add_parts<2>(b0, src, p, part_stride);
      p += 2;
    }
    if (p < n_parts) add_parts<1>(b0, src, p, part_stride);
  }

#pragma unroll
  for (int u = 0; u < 8; ++u)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tw[vc + e][16 * wave + 2 * u + lane / 32] = wreg[u][e] - b0[u][e];     // the targets t[i] = w[i] - B0[i]
      cur[vc + e][16 * wave + 2 * u + lane / 32] = creg[u][e];
    }
  wait_vmcnt<0>();                                          // this wave's part of the coefficients has landed
  __syncthreads();
  // This block's share in the NEXT block's targets is computed at the end, from the new values still in
  // LDS; its other operand, rows 32 w .. 32 w + 31 of the next block of Ht restricted to this block's
  // columns (hi and lo), is fetched now and arrives during the walk.
  u32x4 fb[8][2];
  if (next_blk >= 0) {                                      // uniform
    const int64_t irow = (int64_t)next_blk * kBlk + 32 * wave + lane % 32;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int64_t off = ht_index(k, irow, i0 + 16 * t + 8 * (lane / 32), ldp);
      fb[t][0] = *reinterpret_cast<const u32x4*>(Hth + off);
      fb[t][1] = *reinterpret_cast<const u32x4*>(Htl + off);
    }
  }

  for (int c0 = 0; c0 < n_valid; c0 += kRun) {             // uniform
    // Coordinates past the end of the matrix (last block only) are walked like the others: their
    // coefficients are zero, so nothing they do reaches a real coordinate, and they are not stored.
    float own[8], was[kRun];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) own[kk] = tw[c0 + 8 * q + kk][ch];
#pragma unroll
    for (int ii = 0; ii < kRun; ++ii) was[ii] = cur[c0 + ii][ch];   // the old values, off the chain of decisions
    // the coefficients of a coordinate are read one coordinate ahead, before this one's LDS stores
    const f32x4* row0 = reinterpret_cast<const f32x4*>(&coef[c0][c0 + 8 * q]);   // Ht[c0 + 8q + kk][c0 + ii] over kk
    f32x4 n_lo = row0[0], n_hi = row0[1];
#pragma unroll
    for (int ii = 0; ii < kRun; ++ii) {
      const f32x4 c_lo = n_lo, c_hi = n_hi;
      if (ii + 1 < kRun) {
        const f32x4* row = reinterpret_cast<const f32x4*>(&coef[c0 + ii + 1][c0 + 8 * q]);
        n_lo = row[0];
        n_hi = row[1];
      }
      constexpr int kBroadcast[4] = {0x00, 0x55, 0xAA, 0xFF};
      float ti;                                             // target of coordinate c0 + ii: lane ii / 8 of the quad owns it
      switch (ii / 8) {
        case 0: ti = quad_dpp<kBroadcast[0]>(own[ii % 8]); break;
        case 1: ti = quad_dpp<kBroadcast[1]>(own[ii % 8]); break;
        case 2: ti = quad_dpp<kBroadcast[2]>(own[ii % 8]); break;
        default: ti = quad_dpp<kBroadcast[3]>(own[ii % 8]); break;
      }
      // this lane's quarter of the grid (levels q, q + 4, ...: increasing, so '<' keeps the lower index;
      // a level past the end of the grid holds +inf and is never nearer)
      float best = fabsf(grid[0] - ti), val = grid[0];
      int bq = q;
#pragma unroll
      for (int u = 1; u < LV / 4; ++u) {
        const float dist = fabsf(grid[u] - ti);
        const bool better = dist < best;
        best = better ? dist : best;
        val = better ? grid[u] : val;
        bq = better ? q + 4 * u : bq;
      }
      // settle it inside the quad: nearest point, lowest index among equally near ones.  Distances are
      // not negative, so their bit patterns order like the numbers, and (distance, index) compares as
      // one 64-bit key.
      {
        const float ob = quad_dpp<kQuadSwap1>(best), ov = quad_dpp<kQuadSwap1>(val);
        const int oq = quad_dpp<kQuadSwap1>(bq);
        const bool take = quad_key(ob, oq) < quad_key(best, bq);
        best = take ? ob : best;
        val = take ? ov : val;
        bq = take ? oq : bq;
      }
      {
        const float ob = quad_dpp<kQuadSwap2>(best), ov = quad_dpp<kQuadSwap2>(val);
        const int oq = quad_dpp<kQuadSwap2>(bq);
        const bool take = quad_key(ob, oq) < quad_key(best, bq);
        val = take ? ov : val;
        bq = take ? oq : bq;
      }
      const float e = val - was[ii];
      cur[c0 + ii][ch] = val;                               // all four lanes of the quad store the same value
      code[c0 + ii][ch] = (unsigned char)bq;
      eps[ii][ch] = e;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        own[kk] -= e * c_lo[kk];                            // (targets already used are corrected too: harmless)
        own[4 + kk] -= e * c_hi[kk];
      }
    }
    // The targets after the run, on the matrix cores (fp32 operands): for the wave's 16 channels
    //   t[ch][x] -= sum_ii eps[ch][ii] * coef[c0 + ii][x],   x = c0 + 32 .. , 16 coordinates at a time.
    // 16x16x4: lane l gives A[channel l % 16][ii = 4 s + l / 16] and B[ii = 4 s + l / 16][x = l % 16], and
    // holds the sums of channels 4 (l / 16) .. + 3 for coordinate l % 16.
    __syncthreads();                                        // the changes of the run are in LDS
    if (c0 + kRun < n_valid) {                              // uniform
      float a_frag[kRun / 4];
#pragma unroll
      for (int s = 0; s < kRun / 4; ++s) a_frag[s] = eps[4 * s + lane / 16][16 * wave + lane % 16];
      for (int c1 = c0 + kRun; c1 < n_valid; c1 += 16) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kRun / 4; ++s)
          acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a_frag[s], coef[c0 + 4 * s + lane / 16][c1 + lane % 16], acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) tw[c1 + lane % 16][16 * wave + 4 * (lane / 16) + r] -= acc[r];
      }
    }
    __syncthreads();                                        // the corrected targets, before the next run reads them
  }

  // Write the block back: What, the codes, and the split delta for the next blocks' GEMMs; the lanes keep
  // the rows and coordinates they loaded (W is still in their registers).  The delta halves of all 64
  // channel slots (slots past the end of the group repeat its last channel, as in the walk) are also left
  // in LDS, where the coefficients were: [channel][coordinate], rows of 272 bytes, hi then lo.
  unsigned char* dlt = reinterpret_cast<unsigned char*>(smem + kWalkCoef);
  const bool q_packed = Q && d % 4 == 0 && (reinterpret_cast<uintptr_t>(Q) & 3) == 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int r = 16 * wave + 2 * u + lane / 32;
    const int64_t jr = j0 + r, a = i0 + vc;
    f32x4 v;
    unsigned codes = 0;
    unsigned short h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = cur[vc + e][r];
      codes |= (unsigned)code[vc + e][r] << (8 * e);
      split_bf16(a + e < d ? v[e] - wreg[u][e] : 0.f, h[e], l[e]);
    }
    const u32x2 hv = {h[0] | ((unsigned)h[1] << 16), h[2] | ((unsigned)h[3] << 16)};
    const u32x2 lv = {l[0] | ((unsigned)l[1] << 16), l[2] | ((unsigned)l[3] << 16)};
    *reinterpret_cast<u32x2*>(dlt + r * kDeltaPitch + 2 * vc) = hv;
    *reinterpret_cast<u32x2*>(dlt + (kRows + r) * kDeltaPitch + 2 * vc) = lv;
    if ((r < n_rows) & vec_in) {
      if (a + 3 < d) {
        *reinterpret_cast<f32x4*>(What + jr * ld + a) = v;
      } else {
#pragma unroll
        for (int e = 0; e < 3; ++e)
          if (a + e < d) What[jr * ld + a + e] = v[e];
      }
      if (q_packed) {
        *reinterpret_cast<unsigned*>(Q + jr * d + a) = codes;
      } else if (Q) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (a + e < d) Q[jr * d + a + e] = (unsigned char)(codes >> (8 * e));
      }
      *reinterpret_cast<u32x2*>(Dh + delta_index(jr, a, d_out)) = hv;
      *reinterpret_cast<u32x2*>(Dl + delta_index(jr, a, d_out)) = lv;
    }
  }
  if (next_blk < 0) return;                                 // uniform: nothing follows this block

  // The share of this block in the targets of the next one (the GEMM beside this walk steps over this
  // block, whose values change meanwhile):
  //   E[j][i] = sum_{i' in blk} delta[j][i'] * Ht[next i0 + i][i'],   64 channels x 128 coordinates x 128,
  // from the same hi / lo halves that went to global memory, as one more part of the next block's sums.
  __syncthreads();
  f32x16 near[2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 16; ++r) near[x][r] = 0.f;
#pragma unroll
  for (int t = 0; t < 8; ++t)
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const unsigned char* arow = dlt + (32 * x + lane % 32) * kDeltaPitch + 2 * (16 * t + 8 * (lane / 32));
      const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(arow));
      const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(arow + kRows * kDeltaPitch));
      const bf16x8 bh = __builtin_bit_cast(bf16x8, fb[t][0]), bl = __builtin_bit_cast(bf16x8, fb[t][1]);
      near[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh, al, near[x], 0, 0, 0);
      near[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bl, ah, near[x], 0, 0, 0);
      near[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bh, ah, near[x], 0, 0, 0);
    }
  // register r of lane l holds coordinate 8*(r/4)+4*(l/32)+(r%4) of the wave's 32, channel l%32 of a block of 32
  float* dst = E + ((int64_t)tile * kRows + lane % 32) * kBlk + 32 * wave + 4 * (lane / 32);
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = near[x][4 * r4 + e];
      *reinterpret_cast<f32x4*>(dst + 32 * x * kBlk + 8 * r4) = v;
    }
}

// One launch per block: the first n_walk workgroups walk block `blk` (adding the n_in partial sums in
// Cin), the others compute the partial sums of block `next_blk` into parts 0 .. n_parts - 1 of Cout,
// stepping over the contraction elements of block `excl` (= blk, whose values change meanwhile; none
// if negative).  The walk supplies that block's share itself, as part n_parts of Cout (walk_next: the
// block it is for, negative if none follows).  The two halves share nothing but read-only data, so
// the GEMM for the next block hides behind the latency-bound walk of this one.
constexpr int kSmemBytes = (kWalkBytes > kGemmRing * kGemmStage ? kWalkBytes : kGemmRing * kGemmStage);
template <int LV>
__global__ __launch_bounds__(256) void cd_block_kernel(int n_walk, const float* __restrict__ Cin, int n_in, int n_parts,
                                                       const float* __restrict__ W, float* __restrict__ What,
                                                       const float* __restrict__ codebook, int n_levels,
                                                       const float* __restrict__ Cd,
                                                       const unsigned short* __restrict__ Hth,
                                                       const unsigned short* __restrict__ Htl, int64_t d_out,
                                                       int64_t d, int64_t ld, int64_t ldp, int G, int n_rt, int n_gt,
                                                       int blk, int walk_next, int next_blk, int excl,
                                                       unsigned char* __restrict__ Q,
                                                       unsigned short* __restrict__ Dh,
                                                       unsigned short* __restrict__ Dl, float* __restrict__ Cout,
                                                       int gemm_delay, int k_stages) {
  __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];
  if ((int)blockIdx.x < n_walk) {
    // (the same dealing for the walk: the tiles of a group, which share its coefficients, on as few XCDs as possible)
    const int tile = n_walk % 8 == 0 ? ((int)blockIdx.x % 8) * (n_walk / 8) + (int)blockIdx.x / 8 : (int)blockIdx.x;
    walk_body<LV>(smem, tile, Cin, n_in, W, What, codebook, n_levels, Cd, Hth, Htl, d_out, d, ld, ldp, G,
                  n_rt, blk, walk_next, Q, Dh, Dl, Cout + (int64_t)n_parts * n_walk * kBlk * kRows);
  } else {
    // The walk begins with a burst of loads (some 300 KiB per workgroup) and then hardly touches memory;
    // where the GEMM is the shorter of the two, it starts `gemm_delay` ticks of the 100 MHz clock late and
    // leaves the memory system to the walk for that burst.  (A bounded wait on a free-running clock.)
    if (gemm_delay > 0) {
      const uint64_t t0 = wall_clock64();
      while (wall_clock64() - t0 < (uint64_t)gemm_delay) __builtin_amdgcn_s_sleep(16);
    }
    // Workgroups are dealt to the 8 XCDs in turn (each with its own L2).  All row tiles of a part read the
    // same Ht tiles, so consecutive (part, tile) pairs are given to the same XCD: every XCD then fetches
    // about an eighth of Ht instead of all of it.
    int g = (int)blockIdx.x - n_walk;
    const int n_tiles = n_gt * G, n_gemm = (int)gridDim.x - n_walk;
    if (n_gemm % 8 == 0 && n_walk % 8 == 0) g = (g % 8) * (n_gemm / 8) + g / 8;
    gemm_far_body(smem, g % n_tiles, g / n_tiles, n_parts, Dh, Dl, Hth, Htl, d_out, ldp, G, n_gt, n_rt, next_blk, excl,
                  k_stages, Cout);
  }
}

struct Layout {
  int64_t ldp, n_blk;
  int n_rt, n_gt, n_parts;
  int gemm_delay;                                           // ticks of the 100 MHz clock the GEMM half starts late
  size_t ht_bytes, cdt_bytes, delta_bytes, c_bytes;
};
Layout make_layout(int64_t d_out, int64_t d_in, int G) {
  Layout L;
  L.n_blk = (d_in + kBlk - 1) / kBlk;
  L.ldp = L.n_blk * kBlk;
  const int64_t m = d_out / G;
  L.n_rt = (int)((m + kRows - 1) / kRows);
  L.n_gt = (int)((m + kGemmRows - 1) / kGemmRows);
  // enough GEMM workgroups to fill the compute units the walk leaves free, at least 128 contraction elements each
  const int64_t n_walk = (int64_t)L.n_rt * G, tiles = (int64_t)L.n_gt * G;
  const int64_t free_cus = n_walk < 192 ? 256 - n_walk : 64;
  int parts = (int)(free_cus / tiles);
  if (parts < 1) parts = 1;
  // Where the GEMM outlasts the walk by far (about 2 us per 64-deep stage and workgroup against some
  // 50 us of walk) and would occupy well under the whole chip, it is cut finer than the compute units
  // free at the start: the units the walk releases then pick up the rest.  (More parts also mean more
  // partial sums for the walk to add, so shapes that fill the chip anyway are left alone.)
  if (tiles * (L.ldp / 64) * 2 / free_cus > 80 && parts * tiles < 160) parts = (int)((512 + tiles - 1) / tiles);
  const int max_parts = (int)((L.ldp / 64 - 2) / 2);
  if (parts > max_parts) parts = max_parts;
  if (parts > 16) parts = 16;
  if (parts < 1) parts = 1;
  L.n_parts = parts;
  // Measured on MI355X: a walk takes about 31 us whatever the shape, 8 of them for its opening burst of
  // loads when it has the memory system to itself and twice that beside a GEMM in full swing; a GEMM
  // workgroup takes about 2.5 us plus 1 us per 32-deep stage.  A GEMM that would end well before the
  // walk therefore starts late by the difference (at most 9 us), which costs nothing and shortens the
  // walk; one that outlasts the walk starts at once.
  {
    const double stages = (double)(L.ldp / kGemmK - kBlkStages) / parts;
    double late_us = 31.0 - (2.5 + stages);
    late_us = late_us < 0.0 ? 0.0 : (late_us > 9.0 ? 9.0 : late_us);
    L.gemm_delay = (int)(late_us * 100.0);
  }
  auto up = [](size_t b) { return (b + 255) / 256 * 256; };
  L.ht_bytes = up((size_t)G * L.ldp * L.ldp * 2);
  L.cdt_bytes = up((size_t)G * L.n_blk * kBlk * kBlk * sizeof(float));
  L.delta_bytes = up((size_t)d_out * L.ldp * 2);
  // one of the two buffers that alternate: the GEMM's parts, and one more from the walk of the block before
  L.c_bytes = up((size_t)(L.n_parts + 1) * n_walk * kBlk * kRows * sizeof(float));
  return L;
}

}  // namespace

size_t cd_workspace(int64_t d_out, int64_t d_in, int G) {
  const Layout L = make_layout(d_out, d_in, G);
  return 2 * L.ht_bytes + L.cdt_bytes + 2 * L.delta_bytes + 2 * L.c_bytes;
}

namespace {
// The block loop shared by the two entry points.  ldlq = false: cyclic coordinate descent against H
// (What in: the current feasible weights).  ldlq = true: one pass of sequential rounding with the
// feedback coefficients of the factor R passed as H (What out only).
hipError_t run_assign(bool ldlq, const float* W, float* What, const float* codebook, int n_levels, int64_t d_out,
                      int64_t d_in, int64_t ld, const float* H, int G, int n_cycles, unsigned char* Q, void* ws,
                      bool prep_done, hipStream_t st) {
  const Layout L = make_layout(d_out, d_in, G);
  char* p = (char*)ws;
  unsigned short* Hth = (unsigned short*)p;                 // hi and lo halves interleaved per row and stage
  unsigned short* Htl = Hth + 32;
  p += 2 * L.ht_bytes;
  float* Cd = (float*)p;
  p += L.cdt_bytes;
  unsigned short* Dh = (unsigned short*)p;                  // hi and lo halves interleaved per channel and stage
  unsigned short* Dl = Dh + 32;
  p += 2 * L.delta_bytes;
  float* C = (float*)p;

  hipError_t e;
  const unsigned t64 = (unsigned)(L.ldp / 64);
  // (prep_done: an earlier call with the same H and this workspace has left the split coefficients in place)
  if (ldlq)
    ldlq_prep_kernel<<<dim3(t64, t64, (unsigned)G), dim3(256), 0, st>>>(H, d_in, L.ldp, Hth, Htl, Cd);
  else if (!prep_done)
    cd_prep_kernel<<<dim3(t64 * (t64 + 1) / 2, 1, (unsigned)G), dim3(256), 0, st>>>(H, d_in, L.ldp, Hth, Htl, Cd);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  {
    int64_t bx = (L.ldp + 255) / 256;
    if (bx > 64) bx = 64;
    if (ldlq)
      ldlq_init_kernel<<<dim3((unsigned)bx, (unsigned)d_out), dim3(256), 0, st>>>(W, What, d_in, ld, L.ldp, Dh, Dl);
    else
      cd_delta_kernel<<<dim3((unsigned)bx, (unsigned)d_out), dim3(256), 0, st>>>(W, What, d_in, ld, L.ldp, Dh, Dl);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  float* Cbuf[2] = {C, (float*)((char*)C + L.c_bytes)};
  const int gemm_delay = L.gemm_delay;
  const int n_walk = L.n_rt * G, n_gemm = L.n_gt * G * L.n_parts, n_blk = (int)L.n_blk;
  const int64_t total = (int64_t)n_cycles * n_blk;
#define GQ_LAUNCH_BLOCK(LV, GRID, NWALK, CIN, NIN, BLK, WNEXT, NEXT, EXCL, COUT)                                         \
  cd_block_kernel<LV><<<dim3((unsigned)(GRID)), dim3(256), 0, st>>>(NWALK, CIN, NIN, L.n_parts, W, What, codebook,       \
                                                                   n_levels, Cd, Hth, Htl, d_out, d_in, ld, L.ldp, G,   \
                                                                   L.n_rt, L.n_gt, BLK, WNEXT, NEXT, EXCL, Q, Dh, Dl,   \
                                                                   COUT, (NWALK) > 0 ? gemm_delay : 0,                  \
                                                                   ldlq ? kBlkStages * (NEXT) : (int)(L.ldp / kGemmK))
#define GQ_LAUNCH_ANY(GRID, NWALK, CIN, NIN, BLK, WNEXT, NEXT, EXCL, COUT)                                              \
  do {                                                                                                                  \
    if (n_levels <= 4) GQ_LAUNCH_BLOCK(4, GRID, NWALK, CIN, NIN, BLK, WNEXT, NEXT, EXCL, COUT);                         \
    else if (n_levels <= 8) GQ_LAUNCH_BLOCK(8, GRID, NWALK, CIN, NIN, BLK, WNEXT, NEXT, EXCL, COUT);                    \
    else GQ_LAUNCH_BLOCK(kMaxLevels, GRID, NWALK, CIN, NIN, BLK, WNEXT, NEXT, EXCL, COUT);                              \
  } while (0)
  // the partial sums of block 0 first, over the whole contraction (nothing changes meanwhile) ...
  GQ_LAUNCH_ANY(n_gemm, 0, Cbuf[1], 0, 0, -1, 0, -1, Cbuf[0]);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // ... then one launch per block: its walk, which ends with its own share in the next block's sums
  // (one more part), and beside it the other blocks' share in them
  for (int64_t t = 0; t < total; ++t) {
    const int blk = (int)(t % n_blk), next = (blk + 1) % n_blk;
    const bool more = t + 1 < total;
    GQ_LAUNCH_ANY(n_walk + (more ? n_gemm : 0), n_walk, Cbuf[t & 1], L.n_parts + (t > 0 ? 1 : 0), blk, more ? next : -1,
                  next, blk, Cbuf[(t + 1) & 1]);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
#undef GQ_LAUNCH_ANY
#undef GQ_LAUNCH_BLOCK
  return hipSuccess;
}
}  // namespace

hipError_t launch_cd_assign(const float* W, float* What, const float* codebook, int n_levels, int64_t d_out,
                            int64_t d_in, int64_t ld, const float* H, int G, int n_cycles, unsigned char* Q,
                            void* ws, bool prep_done, hipStream_t st) {
  return run_assign(false, W, What, codebook, n_levels, d_out, d_in, ld, H, G, n_cycles, Q, ws, prep_done, st);
}

hipError_t launch_ldlq_assign(const float* W, float* What, const float* codebook, int n_levels, int64_t d_out,
                              int64_t d_in, int64_t ld, const float* R, int G, unsigned char* Q, void* ws,
                              hipStream_t st) {
  return run_assign(true, W, What, codebook, n_levels, d_out, d_in, ld, R, G, 1, Q, ws, false, st);
}

}  // namespace gq
