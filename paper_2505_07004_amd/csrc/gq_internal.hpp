// Internal declarations shared by the translation units of libgq (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "gq.h"

namespace gq {

// ---- vector types used with the CDNA4 matrix-core builtins -----------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// ---- direct global->LDS loads (CDNA4) ---------------------------------------
typedef char __attribute__((address_space(3))) * lds_char_ptr;

// Direct global->LDS load: every active lane moves 16 bytes from its own global address to
// LDS address lds_base + 16*lane (lds_base is wave-uniform and travels in M0).  Tracked by vmcnt.
__device__ inline void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
// Same with 4 bytes per lane (LDS address lds_base + 4*lane).
__device__ inline void dma4(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
// The same two loads with the address split into a wave-uniform 64-bit base (scalar registers) and
// a 32-bit byte offset per lane: advancing the base costs scalar arithmetic only.
__device__ inline void dma16s(const void* sbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase) : "memory");
}
__device__ inline void dma4s(const void* sbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase) : "memory");
}
// fp32 as a sum of bf16 terms (round to nearest even each): two terms carry 16 mantissa bits, three
// carry all 24 (exact for every x whose exponent leaves room for the last term).
__device__ inline void split_bf16(float x, unsigned short& hi, unsigned short& lo) {
  const __bf16 h = (__bf16)x;
  const __bf16 l = (__bf16)(x - (float)h);
  hi = __builtin_bit_cast(unsigned short, h);
  lo = __builtin_bit_cast(unsigned short, l);
}
__device__ inline void split3_bf16(float x, unsigned short& hi, unsigned short& mid, unsigned short& lo) {
  const __bf16 h = (__bf16)x;
  const float r1 = x - (float)h;
  const __bf16 m = (__bf16)r1;
  const __bf16 l = (__bf16)(r1 - (float)m);
  hi = __builtin_bit_cast(unsigned short, h);
  mid = __builtin_bit_cast(unsigned short, m);
  lo = __builtin_bit_cast(unsigned short, l);
}

template <int N>
__device__ inline void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Number of tiles on or above the diagonal of a T x T tile grid.
__host__ __device__ inline int64_t tri_count(int64_t T) { return T * (T + 1) / 2; }

// Decode a linear index t in [0, tri_count(T)) into (i, j), i <= j, column-major over
// the upper triangle: column j holds rows 0..j, columns in increasing order.
__host__ __device__ inline void tri_decode(int64_t t, int& i, int& j) {
  // j = floor((sqrt(8t+1)-1)/2), fixed up for rounding.
  int64_t jj = (int64_t)((sqrt((double)(8 * t + 1)) - 1.0) * 0.5);
  while (jj * (jj + 1) / 2 > t) --jj;
  while ((jj + 1) * (jj + 2) / 2 <= t) ++jj;
  j = (int)jj;
  i = (int)(t - jj * (jj + 1) / 2);
}

// Order of the Gram kernel's tiles.  The upper triangle of a grid of NT tile columns (256 wide),
// tile column J holding R(J) = rpt * (J + 1) row blocks, is walked in bands of kTileBand tile
// columns; inside a band the row block is the slow index and the tile column the fast one, so a
// run of consecutive tiles (the workgroups resident on one XCD take such a run and share its
// panels through that XCD's L2) covers few distinct row blocks and few distinct tile columns.
// Measured at d = 4096, G = 4: bands of 2 fetch 26 % fewer bytes into L2 than single columns,
// bands of 4 fetch 70 % more.  Decodes t in [0, rpt * tri_count(NT)) into row block I and tile
// column J; the row blocks of the last tile column come last, in increasing order, so a
// truncated count drops exactly the row blocks past the end of a ragged matrix.
constexpr int kTileBand = 2;
__host__ __device__ inline void band_decode(int64_t t, int rpt, int64_t NT, int& I, int& J) {
  int dummy, j_col;
  tri_decode(t / rpt, dummy, j_col);                 // the tile column whose column-major range holds t
  const int64_t J0 = (int64_t)(j_col / kTileBand) * kTileBand;
  const int Kb = (int)((NT - J0) < kTileBand ? (NT - J0) : kTileBand);
  int64_t off = t - (int64_t)rpt * tri_count(J0);
  const int64_t R0 = (int64_t)rpt * (J0 + 1);        // row blocks that every tile column of the band has
  if (off < R0 * Kb) {
    I = (int)(off / Kb);
    J = (int)(J0 + off % Kb);
    return;
  }
  off -= R0 * Kb;
  for (int jj = 1; jj < Kb; ++jj) {                  // the staircase under the band's diagonal tiles
    const int w = Kb - jj;
    const int64_t seg = (int64_t)rpt * w;
    if (off < seg || jj == Kb - 1) {
      I = (int)(R0 + (int64_t)rpt * (jj - 1) + off / w);
      J = (int)(J0 + jj + off % w);
      return;
    }
    off -= seg;
  }
  I = 0;                                             // not reached for t in range
  J = (int)J0;
}

// Order of the wide bf16 Gram kernel's items (group counts divisible by 4): row blocks of 96 rows
// against tile columns of 256 columns.  Row block I (rows 96 I ..) meets tile column J on or above the
// diagonal iff 96 I < 256 (J + 1); rows_of_column counts those row blocks (NR = all row blocks of the
// matrix).  Items are walked in bands of two tile columns, row block slow, so that consecutive items
// (the workgroups resident on one XCD take such a run) share few row panels and few column panels.
constexpr int kWideRows = 96, kWideCols = 256;
// (`rows`: the height of a row block; 96 for four groups per workgroup, 192 when a workgroup takes two row
// blocks of two groups each)
__host__ __device__ inline int64_t wide_rows_of_column(int64_t J, int64_t NR, int64_t rows = kWideRows) {
  const int64_t c = (kWideCols * (J + 1) - 1) / rows + 1;
  return c < NR ? c : NR;
}
__host__ __device__ inline int64_t wide_tile_count(int64_t d, int64_t rows = kWideRows) {
  const int64_t NT = (d + kWideCols - 1) / kWideCols, NR = (d + rows - 1) / rows;
  int64_t t = 0;
  for (int64_t J = 0; J < NT; ++J) t += wide_rows_of_column(J, NR, rows);
  return t;
}
// Item t in [0, wide_tile_count(d)) -> row block I, tile column J.
__host__ __device__ inline void wide_decode(int64_t t, int64_t d, int& I, int& J, int64_t rows = kWideRows) {
  const int64_t NT = (d + kWideCols - 1) / kWideCols, NR = (d + rows - 1) / rows;
  for (int64_t J0 = 0; J0 < NT; J0 += 2) {
    const int64_t c0 = wide_rows_of_column(J0, NR, rows), c1 = (J0 + 1 < NT) ? wide_rows_of_column(J0 + 1, NR, rows) : 0;
    if (t < c0 + c1) {
      if (c1 == 0) {
        I = (int)t;
        J = (int)J0;
      } else if (t < 2 * c0) {             // both tile columns have this row block
        I = (int)(t / 2);
        J = (int)(J0 + t % 2);
      } else {                             // the staircase: only the second tile column reaches down here
        I = (int)(c0 + (t - 2 * c0));
        J = (int)(J0 + 1);
      }
      return;
    }
    t -= c0 + c1;
  }
  I = 0;                                   // not reached for t in range
  J = 0;
}

// ---- launchers (each validates nothing; the C ABI layer has done that) -----
hipError_t launch_group_weights(const void* dZ, gq_dtype dt, int64_t n, int64_t d_out, int64_t ld,
                                int G, float grad_scale, float* s, int64_t ld_s, hipStream_t st);

hipError_t launch_fisher_gram_f32(const float* X, int64_t n, int64_t d_in, int64_t ld, const float* s,
                                  int G, float* H, bool accumulate, hipStream_t st);

// n_dev (two-term calls only, may be null): device pointer to the number of leading rows of X that are in use;
// the rows from there to n are zero with zero weights, and the kernels leave their token steps out.
hipError_t launch_fisher_gram_bf16(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s,
                                   int G, float* H, bool accumulate, bool two_terms, void* ws, bool no_partials,
                                   hipStream_t st, const int* n_dev = nullptr);
// `no_partials`: ws holds only the repacked weights (fisher_gram_bf16_weights_bytes); every work item is then
// computed whole by one workgroup (no left-over runs, no second pass)
size_t fisher_gram_bf16_weights_bytes(int64_t n, int G);
size_t fisher_gram_bf16_wide_weights_bytes(int64_t n, int G);
size_t fisher_gram_bf16_workspace(int64_t n, int64_t d_in, int G);
// the wide kernel (96 x 256 blocks per wave; even group counts, one-term products, n >= 32): whether it can
// take such a call at all, and whether it is the one that runs (group counts not divisible by 4 need at
// least one whole round of work items)
bool fisher_gram_bf16_wide_applies(int64_t n, int G, bool two_terms);
bool fisher_gram_bf16_wide_chosen(int64_t n, int64_t d_in, int G, bool two_terms);
size_t fisher_gram_bf16_wide_workspace(int64_t n, int64_t d_in, int G);
hipError_t launch_fisher_gram_bf16_wide(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int64_t ld_s,
                                        int G, float* H, bool accumulate, void* ws, bool no_partials, hipStream_t st);

// GQ_HEAVY_TWO_TERMS: the tokens whose weight exceeds 16 times the mean weight of a group (at most
// heavy_capacity(n) of them, in token order) are taken out of the main call and run as a second, small call
// with the scaled operand in two bf16 terms.  The workspace is the plain one plus the gathered rows.
int64_t heavy_capacity(int64_t n);
size_t fisher_gram_heavy_workspace(int64_t n, int64_t d_in, int G);
hipError_t launch_fisher_gram_bf16_heavy(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                         float* H, bool accumulate, void* ws, hipStream_t st);
// The deferred form: a chunk call gathers its heavy rows into the caller's pool (pool_rows rows, a multiple of 32)
// and runs the main call only; the flush runs the two-term call over the rows in the pool, adding to H, and
// leaves the pool empty.
size_t fisher_gram_heavy_pool_bytes(int64_t d_in, int G, int64_t rows);
hipError_t launch_fisher_gram_bf16_heavy_deferred(const void* X, int64_t n, int64_t d_in, int64_t ld, const float* s, int G,
                                                  float* H, bool accumulate, void* ws, void* pool, int64_t pool_rows,
                                                  hipStream_t st);
hipError_t launch_fisher_gram_bf16_heavy_flush(void* pool, int64_t pool_rows, int64_t d_in, int G, float* H, void* ws,
                                               hipStream_t st);
// Relative speeds of the eight XCDs for the schedule of the wide Gram kernel (nullptr: all equal), a setting of
// the current device; and the speeds measured by the last plain one-term call that used workspace `ws`.
hipError_t fisher_gram_set_xcd_speeds(const float* a8);
hipError_t fisher_gram_measured_xcd_speeds(int64_t n, int64_t d_in, int G, const void* ws, float* a8);
hipError_t launch_zero_upper(float* H, int64_t d_in, int G, hipStream_t st);
hipError_t launch_mirror(float* H, int64_t d_in, int G, hipStream_t st);
hipError_t launch_damp_diagonal(float* H, int64_t d_in, int G, double damp_rel, double damp_abs, hipStream_t st);

hipError_t launch_objective(const float* W, const float* What, int64_t d_out, int64_t d_in, int64_t ld,
                            const float* H, int G, double* obj, float* obj_row, void* ws,
                            hipStream_t st);
size_t objective_workspace(int64_t d_out, int64_t d_in, int G);

hipError_t launch_cd_assign(const float* W, float* What, const float* codebook, int n_levels, int64_t d_out,
                            int64_t d_in, int64_t ld, const float* H, int G, int n_cycles, unsigned char* Q,
                            void* ws, bool prep_done, hipStream_t st);
size_t cd_workspace(int64_t d_out, int64_t d_in, int G);
hipError_t launch_ldlq_assign(const float* W, float* What, const float* codebook, int n_levels, int64_t d_out,
                              int64_t d_in, int64_t ld, const float* R, int G, unsigned char* Q, void* ws,
                              hipStream_t st);

hipError_t launch_damped_cholesky(const float* H, int64_t d, int G, double damp_rel, double damp_abs, bool reverse,
                                  float* F, int* info, void* ws, hipStream_t st);
size_t cholesky_workspace(int64_t d, int G);

hipError_t launch_lnq_codebook(const float* W, int64_t d_out, int64_t d_in, int64_t ld, const unsigned char* Q,
                               const float* H, int G, int n_levels, double lam, float* codebook, float* What,
                               void* ws, bool splits_done, hipStream_t st);
size_t lnq_codebook_workspace(int64_t d_out, int64_t d_in, int G, int n_levels);

}  // namespace gq
