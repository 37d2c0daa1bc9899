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

constexpr int kTile = 128;            // rows j and columns b per workgroup
constexpr int kKS = 16;               // contraction elements per LDS stage (one MFMA deep)
constexpr int kRowBytes = kKS * 2;    // a staged tile row: two 16-byte chunks
constexpr int kTileBytes = kTile * kRowBytes;       // 4 KiB
constexpr int kStageBytes = 4 * kTileBytes;         // {Dh, Dl, Hh, Hl}: 16 KiB
constexpr int kStages = 5;                          // ring depth: 80 KiB, two workgroups per CU
constexpr int kLoadsPerStage = kTileBytes / 1024;   // 1 KiB direct loads per wave and stage (wave w fills tile w)
constexpr int kTileElems = kTile * kKS;             // bf16 elements of one staged tile

// Element offset, inside a staged tile, of contraction element e (0..15) of row r (0..127): a row
// is two 16-byte chunks, and rows 8..15 of every 16 keep them swapped, so that the 16-byte
// fragment reads of 16 consecutive rows fall into 16 different bank groups.
__host__ __device__ inline int tile_pos(int r, int e) { return r * kKS + ((((e >> 3) ^ (r >> 3)) & 1) << 3) + (e & 7); }

__device__ inline void split_bf16(float x, unsigned short& hi, unsigned short& lo) {
  const __bf16 h = (__bf16)x;
  const __bf16 l = (__bf16)(x - (float)h);
  hi = __builtin_bit_cast(unsigned short, h);
  lo = __builtin_bit_cast(unsigned short, l);
}

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
#pragma unroll 4
  for (int i = 0; i < 32; ++i) {
    const int idx = t + 256 * i;
    const int r = idx / 64, ac = idx % 64;
    const int64_t j = j0 + r, a = a0 + ac;
    tile[r][ac] = (j < j_end && a < d) ? W[j * ld + a] - What[j * ld + a] : 0.f;
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
// stage st the contraction elements a = 16 st .. 16 st + 15, for st < 8 (tb + 1):
//   Hh/Hl[k][(tb * n_st + st) * kTileElems + tile_pos(r, e)] = hi/lo of H[k][a][b]  (a <= b),
// of H[k][b][a] below the diagonal of the diagonal 128-tile, 0 past d.  One workgroup turns a
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
  int ta, tb;
  tri_decode(blockIdx.x / 2, ta, tb);                       // 128-tiles, ta <= tb
  const int64_t a0 = (int64_t)ta * kTile + 64 * (blockIdx.x % 2), b0 = (int64_t)tb * kTile;
  const int t = threadIdx.x;
#pragma unroll 4
  for (int i = 0; i < 32; ++i) {
    const int idx = t + 256 * i;
    const int ar = idx / kTile, bc = idx % kTile;
    const int64_t a = a0 + ar, b = b0 + bc;
    float v = 0.f;
    if (a < d && b < d) v = a <= b ? Hk[a * d + b] : Hk[b * d + a];   // a > b only inside a diagonal tile
    tile[ar][bc] = v;
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

// Y tile [128 j][128 b] over a < (tb+1)*128 on bf16 MFMA with split operands, then the row dot.
//
// Staging.  The four operand tiles of a stage (128 rows x 16 contraction elements each, 4 KiB
// contiguous in the split arrays and already in LDS order) go from global memory straight into
// LDS (global_load_lds_dwordx4: wave w copies tile w with four 1 KiB loads), kStages - 1 stages
// ahead of their use, tracked by an explicit vmcnt wait and one workgroup barrier per stage.
__global__ __launch_bounds__(256, 2) void objective_mfma_kernel(const unsigned short* __restrict__ Dh,
                                                             const unsigned short* __restrict__ Dl,
                                                             const unsigned short* __restrict__ Hh,
                                                             const unsigned short* __restrict__ Hl,
                                                             const float* __restrict__ W, const float* __restrict__ What,
                                                             int64_t d_out, int64_t d, int64_t ld, int64_t ldp, int G,
                                                             int n_tb, int n_rb, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(1024))) char smem[kStages * kStageBytes];
  // the row-sum exchange at the end reuses the staging memory (after a barrier)
  float (*red)[kTile] = reinterpret_cast<float (*)[kTile]>(&smem[0]);

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

  const int tid = threadIdx.x;
  const int lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int wm = wave / 2, wn = wave % 2;

  // ---- this wave's share of the staging: tile `wave` of every stage, 16 bytes per lane -------
  const int64_t n_st = ldp / kKS;
  const unsigned short* gp[kLoadsPerStage];
  {
    const unsigned short* src =
        wave < 2 ? (wave == 0 ? Dh : Dl) + ((int64_t)k * n_rb + rb) * n_st * kTileElems
                 : (wave == 2 ? Hh : Hl) + (int64_t)k * ldp * ldp + (int64_t)tb * n_st * kTileElems;
#pragma unroll
    for (int i = 0; i < kLoadsPerStage; ++i) gp[i] = src + i * 512 + lane * 8;
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
  auto frag = [&](int slot, int t, int row0) -> bf16x8 {
    const u32x4 v = *reinterpret_cast<const u32x4*>(&smem[slot * kStageBytes + t * kTileBytes + row0 * kRowBytes + frag_off]);
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[x][y][r] = 0.f;

  // Fragments of one stage: rows of delta (hi, lo) and of the transposed H tile (hi, lo).
  struct Frags {
    bf16x8 ah[2], al[2], bh[2], bl[2];
  };
  auto read = [&](Frags& f, int slot) {
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      f.ah[x] = frag(slot, 0, wm * 64 + x * 32);
      f.al[x] = frag(slot, 1, wm * 64 + x * 32);
    }
#pragma unroll
    for (int y = 0; y < 2; ++y) {
      f.bh[y] = frag(slot, 2, wn * 64 + y * 32);
      f.bl[y] = frag(slot, 3, wn * 64 + y * 32);
    }
  };
  auto mma = [&](const Frags& f) {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.al[x], f.bh[y], acc[x][y], 0, 0, 0);
        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[x], f.bl[y], acc[x][y], 0, 0, 0);
        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.ah[x], f.bh[y], acc[x][y], 0, 0, 0);
      }
  };

  const int stages = (tb + 1) * (kTile / kKS);              // a multiple of 8, > kStages
  const int first_diag = tb * (kTile / kKS);
#pragma unroll
  for (int t = 0; t < kStages - 1; ++t) issue(t, true);
  int slot_next = 1, slot_fill = kStages - 1;               // ring slots of stage it + 1 and of stage it - 1

  // One step: the MFMAs of stage `it` run on fragments read during the previous step, while
  // the fragments of stage it + 1 are read and stage it + kStages - 1 is requested.  The step
  // is branch-free (past the end it reads a stale slot and requests the last stage again), so
  // the LDS reads of the next stage stay in flight behind the MFMAs.
  auto step = [&](const Frags& cur, Frags& nxt, int it) {
    wait_vmcnt<(kStages - 3) * kLoadsPerStage>();   // this wave's loads of stage it + 1 have landed
    // everyone's have; and everyone has issued the MFMAs of stage it - 1, so its slot is free
    __builtin_amdgcn_s_barrier();
    issue(slot_fill, it + kStages < stages);
    read(nxt, slot_next);
    __builtin_amdgcn_sched_barrier(0);              // keep the reads ahead of the MFMAs they overlap with
    mma(cur);
    __builtin_amdgcn_sched_barrier(0);
    slot_fill = slot_fill + 1 == kStages ? 0 : slot_fill + 1;
    slot_next = slot_next + 1 == kStages ? 0 : slot_next + 1;
  };

  Frags f0, f1;
  wait_vmcnt<(kStages - 2) * kLoadsPerStage>();
  __builtin_amdgcn_s_barrier();
  read(f0, 0);
  int it = 0;
  for (; it < first_diag; it += 2) {     // strictly-upper tiles
    step(f0, f1, it);
    step(f1, f0, it + 1);
  }
  if (tb > 0) {
    // they count twice (their mirror images are never visited)
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int y = 0; y < 2; ++y) acc[x][y] *= 2.f;
  }
  for (; it < stages; it += 2) {         // the diagonal tile
    step(f0, f1, it);
    step(f1, f0, it + 1);
  }
  wait_vmcnt<0>();   // the repeated requests of the last stage
  __syncthreads();   // the ring is idle: `red` may reuse it

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
  const int64_t n_rb = (d_out / G + kTile - 1) / kTile;
  L.delta_bytes = ((size_t)((int64_t)G * n_rb * kTile * L.ldp) * 2 + 255) / 256 * 256;
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
  const int64_t n_st = L.ldp / kKS;
  {
    split_delta_kernel<<<dim3((unsigned)(n_st / 4), (unsigned)(G * n_rb)), dim3(256), 0, st>>>(W, What, d_out, d_in, ld, G,
                                                                                              n_rb, n_st, Dh, Dl);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    split_h_kernel<<<dim3((unsigned)(2 * tri_count(n_tb)), (unsigned)G), dim3(256), 0, st>>>(H, d_in, L.ldp, n_st, Hh, Hl);
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
