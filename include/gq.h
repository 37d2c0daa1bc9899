/*
 * libgq — the computation GuidedQuant adds to layer-wise post-training
 * quantization, as hand-written HIP kernels for AMD MI355X (gfx950).
 *
 * For one linear layer with calibration input X[n, d_in] and output gradients
 * dZ[n, d_out], and G contiguous groups J_k of d_out/G output channels
 * (GuidedQuant, Algorithm 1, line 1):
 *
 *   gq_group_weights  s[i,k]  = c^2/|J_k| * sum_{j in J_k} dZ[i,j]^2      (Algorithm 1, line 2)
 *   gq_fisher_gram    H[k]   (+)= X^T Diag(s[:,k]) X                      (Algorithm 1, line 4)
 *   gq_fisher_mirror  H[k][b,a] = H[k][a,b]  for a < b                    (storage of the full square)
 *   gq_objective      obj[k]  = sum_{j in J_k} (w_j-what_j)^T H[k] (w_j-what_j)   (Eq. "ours2", Section 3.2)
 *   gq_cd_assign      cyclic coordinate descent on the assignments against H[k]   (Section 4.2, Eq. "cd_closed")
 *   gq_damped_cholesky  H[k] + eps I = L L^T (or R R^T, R upper)                     (Algorithm 2, line 1)
 *   gq_ldlq_assign    sequential rounding with error feedback (GPTQ / LDLQ) from a factor of H[k]
 *   gq_lnq_codebook   closed-form grids for fixed assignments against H[k]        (Section 4.2, Eq. "conti-sol")
 *   gq_lnq            grids and coordinate descent in alternation                 (Algorithm 2)
 *
 * Conventions shared by every call
 *   - Every data pointer is DEVICE memory on the current HIP device, allocated
 *     and owned by the caller.  The library never allocates, frees or keeps a
 *     pointer past the call.
 *   - All matrices are row-major.  `ld_*` is the distance between consecutive
 *     rows in ELEMENTS.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls validate their arguments on the host, enqueue kernels on that stream
 *     and return without synchronising; outputs are valid once the stream has
 *     been synchronised.
 *   - Return value: GQ_OK (0) or a negative gq_status.  On an argument error (every
 *     status except GQ_ERR_HIP) nothing has been enqueued and no output has been
 *     touched.  GQ_ERR_HIP reports a launch the runtime refused; kernels of the same
 *     call that were enqueued before it may still run, so the outputs are undefined.
 *   - Results are deterministic: identical arguments give bit-identical outputs
 *     (no floating-point atomics whose order can vary).
 *   - NaN/Inf in the inputs propagate; nothing is checked.
 */
#ifndef GQ_H_
#define GQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GQ_OK = 0,
  GQ_ERR_NULLPTR = -1,     /* a required pointer is NULL                                  */
  GQ_ERR_SHAPE = -2,       /* negative/zero size, G does not divide d_out, ld < width     */
  GQ_ERR_DTYPE = -3,       /* unknown gq_dtype                                            */
  GQ_ERR_ALIGN = -4,       /* base pointer or row pitch not aligned as documented         */
  GQ_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than *_workspace_bytes()          */
  GQ_ERR_HIP = -6,         /* a HIP runtime call or kernel launch failed                  */
  GQ_ERR_UNSUPPORTED = -7  /* valid request that this build does not implement            */
} gq_status;

typedef enum {
  GQ_F32 = 0,   /* IEEE binary32                                                        */
  GQ_BF16 = 1   /* bfloat16 (upper 16 bits of binary32)                                 */
} gq_dtype;

/* flags of gq_fisher_gram */
enum {
  GQ_ACCUMULATE = 1u << 0, /* H += ... ; without it the upper triangle of H is overwritten */
  GQ_MIRROR = 1u << 1,     /* after the update also fill the strictly lower triangle       */
  GQ_TWO_TERMS = 1u << 2,  /* GQ_BF16 only: carry the scaled operand as two bf16 terms     */
  GQ_HEAVY_TWO_TERMS = 1u << 3 /* GQ_BF16 only: two terms for the heaviest tokens only      */
};

/* Library version: major*10000 + minor*100 + patch. */
int gq_version(void);

/* Static, never-freed description of a gq_status value. */
const char* gq_status_string(int status);

/*
 * Averaged squared output gradients (Algorithm 1, line 2; the gradient scaling
 * constant of Section 3.2 is `grad_scale`, applied to dZ before squaring and
 * never undone; pass 1.0f for none).
 *
 *   dZ   [n, d_out]  device, dz_dtype GQ_F32 (GQ_BF16 also accepted), row pitch ld_dz elements
 *   s    [n, G]      device, fp32, dense (row pitch G)
 *   s[i,k] = grad_scale^2 / (d_out/G) * sum_{j = k*d_out/G}^{(k+1)*d_out/G - 1} dZ[i,j]^2
 *
 * n == 0 is a valid no-op.  Errors: GQ_ERR_SHAPE if n < 0, d_out <= 0, G <= 0,
 * d_out % G != 0 or ld_dz < d_out; GQ_ERR_ALIGN if dZ is not 16-byte aligned or
 * the row pitch in bytes is not a multiple of 16.
 */
int gq_group_weights(const void* dZ, gq_dtype dz_dtype, int64_t n, int64_t d_out, int64_t ld_dz,
                     int32_t G, float grad_scale, float* s, void* hip_stream);

/*
 * The same, written into G columns of a wider array: s[i*ld_s + k], k < G, ld_s >= G.
 * Linear layers that read the same input X (q/k/v, gate/up: the paper quantizes a block's
 * layers from one cached input) can put their weights side by side in one
 * [n, G_1 + G_2 + ...] array, each layer calling this with `s` pointing at its first
 * column, and then make ONE gq_fisher_gram call with G = G_1 + G_2 + ...: the result
 * H[G_1 + G_2 + ..., d_in, d_in] is the layers' group Hessians one after the other
 * (Algorithm 1, line 4, for every layer of the block in a single pass over X).
 * Additional error: GQ_ERR_SHAPE if ld_s < G.
 */
int gq_group_weights_strided(const void* dZ, gq_dtype dz_dtype, int64_t n, int64_t d_out, int64_t ld_dz,
                             int32_t G, float grad_scale, float* s, int64_t ld_s, void* hip_stream);

/*
 * Bytes of device workspace gq_fisher_gram needs for these sizes (may be 0).
 * Returns 0 for invalid arguments as well; gq_fisher_gram reports those.
 */
size_t gq_fisher_gram_workspace_bytes(gq_dtype x_dtype, int64_t n, int64_t d_in, int32_t G);

/*
 * Grouped Fisher/Hessian blocks (Algorithm 1, line 4), one token chunk at a time:
 *
 *   H[k][a,b] (+)= sum_{i<n} s[i,k] * X[i,a] * X[i,b]      for a <= b, k < G
 *
 *   X    [n, d_in]        device, x_dtype, row pitch ld_x elements; all n*ld_x elements must be
 *                         readable (whole 16-byte chunks are loaded, never past the pitch of a row)
 *   s    [n, G]           device fp32 (as written by gq_group_weights)
 *   H    [G, d_in, d_in]  device fp32, dense.  Only the upper triangle (incl.
 *                         diagonal) of each H[k] is read and written; the strictly
 *                         lower triangle is left untouched unless GQ_MIRROR is set,
 *                         in which case it is overwritten with the transpose and
 *                         H[k] is bit-exactly symmetric afterwards.
 *   flags  GQ_ACCUMULATE adds to the existing upper triangle (streaming over token
 *          chunks: first call without it, later calls with it).
 *   x_dtype selects the arithmetic: GQ_F32 -> fp32 matrix-core path (fp32 products,
 *          fp32 accumulation); GQ_BF16 -> bf16 matrix-core path: one operand is
 *          bf16_rne(s[i,k]*X[i,a]) (fp32 multiply, round to nearest even), the
 *          other the raw X[i,b]; fp32 accumulation.  The result is symmetric once
 *          mirrored, but positive semidefinite only up to that rounding (about
 *          5e-4 of its largest eigenvalue): damp accordingly before factoring it,
 *          or use GQ_TWO_TERMS or GQ_F32.
 *          GQ_TWO_TERMS (with GQ_BF16; ignored with GQ_F32): the scaled operand is
 *          carried as hi + lo, hi = bf16_rne(s*x), lo = bf16_rne(s*x - hi), two
 *          matrix-core products per pair: twice the work of the one-term path, every
 *          product exact to 2^-17, the result within about 1e-5 of the fp32 path and
 *          positive semidefinite to that level.
 *          GQ_HEAVY_TWO_TERMS (with GQ_BF16; ignored with GQ_F32 and when GQ_TWO_TERMS is
 *          set): the same sum, with two terms only where the rounding matters.  Token i is
 *          heavy if s[i,k] > 16 * mean_i s[i,k] for some k (mean over this call's n tokens);
 *          the first 32*ceil(n/2048) heavy tokens in token order are left out of the one-term
 *          pass and their rows run through a second, small two-term pass (further heavy
 *          tokens, if any, stay in the one-term pass).  With heavy-tailed token weights
 *          (squared gradients: Section 3.2) the rounding errors of those few tokens are what
 *          makes the one-term result indefinite; this mode costs a few per cent and, on the
 *          workloads measured, gives an H that a Cholesky factorization accepts with the
 *          usual small diagonal constant (Section 4.2).  Deterministic like the other modes.
 *   workspace  device buffer of at least gq_fisher_gram_workspace_bytes() bytes,
 *          256-byte aligned (may be NULL when that size is 0); contents are
 *          scratch.
 *
 * n == 0: valid; without GQ_ACCUMULATE the upper triangle is zero-filled.
 * Errors: GQ_ERR_SHAPE (n < 0, d_in <= 0, G <= 0, ld_x < d_in), GQ_ERR_DTYPE,
 * GQ_ERR_ALIGN (X or H not 16-byte aligned, or ld_x*sizeof(element) not a multiple
 * of 16), GQ_ERR_WORKSPACE, GQ_ERR_HIP.
 */
int gq_fisher_gram(const void* X, gq_dtype x_dtype, int64_t n, int64_t d_in, int64_t ld_x,
                   const float* s, int32_t G, float* H, uint32_t flags,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * GQ_HEAVY_TWO_TERMS for callers that feed the tokens in chunks (Algorithm 1, line 4, accumulated over
 * token chunks).  The two-term pass over a call's heaviest tokens adds to every entry of H, so with
 * gq_fisher_gram every chunk pays a read-modify-write of the whole H for a few dozen rows.  Here the
 * heavy rows of every chunk are gathered into a pool the caller keeps, and their pass runs once:
 *
 *   pool = device memory of gq_fisher_gram_heavy_pool_bytes(d_in, G, pool_rows) bytes, 256-byte aligned,
 *       filled with zero bytes ONCE before its first use; pool_rows (a multiple of 32, >= 32) is the
 *       number of token rows it takes.  The first 4 bytes hold the number of rows in use.
 *   gq_fisher_gram_heavy_deferred(...): gq_fisher_gram with GQ_BF16 and GQ_HEAVY_TWO_TERMS (the same
 *       selection rule, per call; flags: GQ_ACCUMULATE only), except that the heavy rows go to the
 *       pool instead of through their two-term pass.  Rows that the pool has no room for stay in the
 *       one-term pass, as rows beyond a call's capacity do.  workspace as for gq_fisher_gram.
 *   gq_fisher_gram_heavy_flush(...): adds the two-term products of the rows in the pool to H (upper
 *       triangle; GQ_MIRROR allowed, no other flag) and leaves the pool empty.  Call it after the last
 *       chunk, or whenever the pool may be full; an empty pool adds nothing.  workspace:
 *       gq_fisher_gram_workspace_bytes(GQ_BF16, pool_rows, d_in, G).
 *
 * H after the flush is the H of the same chunk calls made with gq_fisher_gram and GQ_HEAVY_TWO_TERMS up
 * to the order of the fp32 additions; identical arguments and pool contents give identical bits.
 * d_in and G must be the same in all calls on one pool between two flushes.  Calls on one pool must
 * not overlap.  Errors as gq_fisher_gram; GQ_ERR_SHAPE for a bad pool_rows.
 */
size_t gq_fisher_gram_heavy_pool_bytes(int64_t d_in, int32_t G, int64_t pool_rows);
int gq_fisher_gram_heavy_deferred(const void* X, gq_dtype x_dtype, int64_t n, int64_t d_in, int64_t ld_x, const float* s,
                                  int32_t G, float* H, uint32_t flags, void* workspace, size_t workspace_bytes,
                                  void* pool, int64_t pool_rows, void* hip_stream);
int gq_fisher_gram_heavy_flush(void* pool, int64_t pool_rows, int64_t d_in, int32_t G, float* H, uint32_t flags,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Schedule tuning of the bf16 Gram kernel (no passage of the paper: a property of the chip).  The eight
 * XCDs of one MI355X do not run the kernel at the same speed (shared power budget, silicon spread:
 * up to +-5 % around the mean, stable for a device), and the work items left over after the whole
 * rounds are cut into runs of equal COST.  With relative speeds set, the runs are cut so that all
 * workgroups finish at the same TIME instead (and calls with several rounds deal their whole items
 * to the XCDs in proportion to the speeds).
 *
 *   gq_fisher_gram_set_xcd_speeds(speeds): host pointer to 8 floats in [0.5, 2] (relative speed of
 *       XCD 0..7; only their ratios matter), or NULL for the default (all equal).  A setting of the
 *       current device for the rest of the process; used by every later GQ_BF16 gq_fisher_gram /
 *       gq_fisher_gram_noalloc call on it.  GQ_ERR_SHAPE for a value outside the range.
 *   gq_fisher_gram_measured_xcd_speeds(n, d_in, G, workspace, speeds): every plain one-term GQ_BF16
 *       call with G % 4 == 0 (or G % 2 == 0 and d_in large enough: two groups' items of 192 rows x 256
 *       columns, times up to three token segments, number at least 256) records, per workgroup, the time and the cost of its whole
 *       work items in its workspace; this call copies those records of the LAST such call with these
 *       sizes and this workspace to the host (it waits for the device) and writes the 8 relative
 *       speeds (mean 1) to the host array `speeds`.  The speeds are coupled through the chip's power
 *       budget (an XCD runs faster while others wait): measuring again under the tuned schedule and
 *       averaging with the setting, two or three times, gives a better setting than one measurement.
 *       GQ_ERR_UNSUPPORTED when such a call records nothing (other group counts, fewer than 256
 *       work items, no left-over items) or the records are empty.
 *
 * The speeds decide where the runs are cut, hence the rounding of the sums: results are bit-identical
 * for identical arguments and identical speeds, and within the documented tolerance for any speeds.
 */
int gq_fisher_gram_set_xcd_speeds(const float* speeds);
int gq_fisher_gram_measured_xcd_speeds(int64_t n, int64_t d_in, int32_t G, const void* workspace, float* speeds);

/*
 * gq_fisher_gram for callers that cannot allocate device memory and so cannot bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (minus the workspace), same arithmetic and same results up to the order of the fp32
 * additions over tokens (every tile of H is accumulated by one workgroup over all tokens; the
 * workspace version may split a tile's tokens between workgroups).  The scratch memory of the
 * call (the token weights repacked for the kernels) is a fixed device array inside the library,
 * gq_fisher_gram_noalloc_max_scratch_bytes() = 4 MiB per GPU, held until the process ends.
 * Nothing is allocated or freed by the call.
 *
 * Limit: GQ_BF16 needs 4 * G * (32 * ceil(n / 32) + 256) bytes of it (n = 65536 tokens with
 * G <= 15, for example); a larger call returns GQ_ERR_WORKSPACE and enqueues nothing.  GQ_F32 has
 * no limit.  All calls on one GPU share that GPU's array: calls that may run concurrently on one
 * GPU (different streams, different threads) race on it and must be serialised by the caller.
 * Other errors as gq_fisher_gram.
 */
size_t gq_fisher_gram_noalloc_max_scratch_bytes(void);
int gq_fisher_gram_noalloc(const void* X, gq_dtype x_dtype, int64_t n, int64_t d_in, int64_t ld_x,
                           const float* s, int32_t G, float* H, uint32_t flags, void* hip_stream);

/*
 * Fill the strictly lower triangle of every H[k] from its upper triangle, in
 * place: the paper caches its Hessians as full squares (the disk sizes of its
 * Table "cost_hess" are those of g dense d_in x d_in matrices per layer), and
 * the quantizers it feeds them to index them as such.  H [G, d_in, d_in] fp32;
 * bit-exactly symmetric afterwards.  Errors: GQ_ERR_SHAPE, GQ_ERR_NULLPTR,
 * GQ_ERR_ALIGN (H not 16-byte aligned).
 */
int gq_fisher_mirror(float* H, int64_t d_in, int32_t G, void* hip_stream);

/*
 * Damping of the group Hessians in place (Section 4.2: a small constant on the diagonal; the
 * users of H it names all damp it):  H[k][i,i] += damp_abs + damp_rel * mean_i H[k][i,i].
 * The same constant as gq_damped_cholesky applies internally; gq_cd_assign, gq_lnq_codebook
 * and gq_lnq take H as it is, so a caller who wants them to see the damped matrix calls this
 * first.  H [G, d_in, d_in] device fp32.  Errors: GQ_ERR_NULLPTR, GQ_ERR_SHAPE (d_in <= 0,
 * G <= 0, a constant negative or NaN).
 */
int gq_damp_diagonal(float* H, int64_t d_in, int32_t G, double damp_rel, double damp_abs, void* hip_stream);

/* Bytes of device workspace gq_objective needs (never 0 for valid sizes). */
size_t gq_objective_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G);

/*
 * GuidedQuant layer objective (Eq. "ours2", Section 3.2):
 *
 *   obj_row[j] = (W[j,:]-What[j,:])^T H[k(j)] (W[j,:]-What[j,:]),  k(j) = j / (d_out/G)
 *   obj[k]     = sum_{j in J_k} obj_row[j]
 *
 *   W, What  [d_out, d_in]    device fp32, row pitch ld_w elements; row j is output
 *                             channel j (the transpose of the paper's [d_in, d_out])
 *   H        [G, d_in, d_in]  device fp32; only the upper triangle (incl. diagonal)
 *                             of each H[k] is read (symmetry supplies the rest)
 *   obj      [G]              device fp64
 *   obj_row  [d_out]          device fp32, or NULL if not wanted
 *   workspace  at least gq_objective_workspace_bytes() bytes, 256-byte aligned
 *
 * Errors: GQ_ERR_NULLPTR, GQ_ERR_SHAPE (d_out <= 0, d_in <= 0, G <= 0,
 * d_out % G != 0, ld_w < d_in), GQ_ERR_ALIGN (W/What/H not 16-byte aligned or
 * ld_w*4 not a multiple of 16), GQ_ERR_WORKSPACE, GQ_ERR_HIP.
 */
int gq_objective(const float* W, const float* What, int64_t d_out, int64_t d_in, int64_t ld_w,
                 const float* H, int32_t G, double* obj, float* obj_row,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of device workspace gq_cd_assign needs (never 0 for valid sizes). */
size_t gq_cd_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G);

/*
 * The assignment step of layer-wise non-uniform quantization run against the group
 * Hessians (Section 4.2: Algorithm 2, lines 6-12, with the closed-form coordinate update
 * of Eq. "cd_closed"; coordinates are processed in blocks of 128 as in Algorithm 4).
 *
 * For cycle = 1..n_cycles, for i = 0..d_in-1 in this order, every output channel j
 * (group k = j / (d_out/G)) replaces What[j,i] by the point of its grid nearest to
 *
 *   t = W[j,i] - sum_{i' != i} H[k][i,i'] / H[k][i,i] * (What[j,i'] - W[j,i']),
 *
 * computed from the current What (coordinates < i already updated in this cycle).
 * Among equally near grid points the one with the lowest index wins.  The sums are
 * evaluated in fp32-grade arithmetic, so a target that lies within rounding distance
 * of the midpoint of two grid points may go to either of them.
 *
 *   W         [d_out, d_in]    device fp32, row pitch ld_w elements (row j = output channel j)
 *   What      [d_out, d_in]    device fp32, same pitch; in: the current quantized weights
 *                              (every entry a point of its channel's grid); out: the new ones
 *   codebook  [d_out, n_levels] device fp32, dense: the grid of every output channel,
 *                              1 <= n_levels <= 16, in any order
 *   H         [G, d_in, d_in]  device fp32 with positive diagonals; only the upper triangle
 *                              (incl. diagonal) of each H[k] is read
 *   Q         [d_out, d_in]    device bytes, dense, or NULL: the grid index chosen at the
 *                              last update of every coordinate
 *   workspace  at least gq_cd_workspace_bytes() bytes, 256-byte aligned
 *
 * n_cycles == 0 is a valid no-op.  Errors: GQ_ERR_NULLPTR, GQ_ERR_SHAPE (d_out <= 0,
 * d_in <= 0, G <= 0, d_out % G != 0, ld_w < d_in, n_cycles < 0, n_levels <= 0),
 * GQ_ERR_UNSUPPORTED (n_levels > 16, or d_out > 65535: the helper kernels put the channel
 * in the second grid dimension; the same limit holds for gq_ldlq_assign, gq_lnq_codebook
 * and gq_lnq), GQ_ERR_ALIGN (W/What/H not 16-byte aligned or
 * ld_w*4 not a multiple of 16), GQ_ERR_WORKSPACE, GQ_ERR_HIP.
 */
int gq_cd_assign(const float* W, float* What, const float* codebook, int32_t n_levels,
                 int64_t d_out, int64_t d_in, int64_t ld_w, const float* H, int32_t G,
                 int32_t n_cycles, uint8_t* Q,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* flags of gq_damped_cholesky */
enum {
  GQ_CHOL_REVERSE = 1u << 0 /* the upper triangular factor R, A = R R^T, instead of the lower L, A = L L^T */
};

/* Bytes of device workspace gq_damped_cholesky needs (0 for invalid sizes). */
size_t gq_cholesky_workspace_bytes(int64_t d_in, int32_t G);

/*
 * Cholesky factorization of the damped group Hessians (Algorithm 2, line 1; Section 4.2:
 * a small constant on the diagonal makes the matrix positive definite), in fp32:
 *
 *   A_k = H[k] + eps_k I,   eps_k = damp_abs + damp_rel * mean_i H[k][i,i]
 *   flags == 0:               A_k = L L^T,  F[k] = L lower triangular, zeros above the diagonal
 *   flags == GQ_CHOL_REVERSE: A_k = R R^T,  F[k] = R UPPER triangular, zeros below the diagonal
 *                             (the factorization taken from the last coordinate backwards; its
 *                             columns are the feedback coefficients gq_ldlq_assign needs)
 *
 *   H     [G, d_in, d_in]  device fp32, dense; only the upper triangle (incl. diagonal) is read
 *   F     [G, d_in, d_in]  device fp32, dense, every entry written; must not overlap H
 *   info  [G]              device int32 or NULL: 0, or 1 + the coordinate (in the order of
 *                          elimination: from the end for GQ_CHOL_REVERSE) of the first pivot
 *                          that was not positive; such a pivot is replaced by 1, so F stays
 *                          finite but is not a factor of A_k
 *   workspace  at least gq_cholesky_workspace_bytes() bytes, 256-byte aligned
 *
 * The paper leaves the constant open; the relative form is the convention of the GPTQ line
 * of work it cites (1 % of the mean diagonal).
 * Part of the work is enqueued on a second stream that the library keeps per device (created on
 * the first call: that call allocates a stream and three events) and is joined back into
 * `hip_stream` before the call returns; to the caller everything is ordered on `hip_stream`.
 * Errors: GQ_ERR_NULLPTR, GQ_ERR_SHAPE (d_in <= 0, G <= 0, a damping constant negative or
 * NaN, F == H), GQ_ERR_UNSUPPORTED (unknown flag), GQ_ERR_ALIGN (H or F not 16-byte aligned),
 * GQ_ERR_WORKSPACE, GQ_ERR_HIP.
 */
int gq_damped_cholesky(const float* H, int64_t d_in, int32_t G, double damp_rel, double damp_abs,
                       uint32_t flags, float* F, int32_t* info,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Sequential rounding with error feedback against the group Hessians: the GPTQ / LDLQ
 * quantizers the paper feeds its Hessians to (Appendix "Implementation Details for
 * Different Quantization Types"; the alternative assignment step of the LNQ ablation),
 * with a grid per output channel (a uniform grid is a special case).  From the UPPER
 * triangular factor R[k] of the damped matrix, H[k] + eps I = R[k] R[k]^T, for
 * i = 0..d_in-1 in this order every output channel j (group k = j / (d_out/G)) sets
 *
 *   What[j,i] = the grid point nearest to
 *               W[j,i] - sum_{i' < i} (What[j,i'] - W[j,i']) * R[k][i',i] / R[k][i,i].
 *
 * Ties go to the lowest grid index; the sums are evaluated in fp32-grade arithmetic as
 * in gq_cd_assign (same kernels, blocks of 128 coordinates), with the same caveat about
 * targets at a midpoint.
 *
 *   W         [d_out, d_in]     device fp32, row pitch ld_w elements
 *   What      [d_out, d_in]     device fp32, same pitch, written; must not overlap W
 *   codebook  [d_out, n_levels] device fp32, dense, 1 <= n_levels <= 16, any order
 *   R         [G, d_in, d_in]   device fp32, dense; only the upper triangle (incl. the
 *                               positive diagonal) is read
 *   Q         [d_out, d_in]     device bytes, dense, or NULL: the grid indices chosen
 *   workspace  at least gq_cd_workspace_bytes(d_out, d_in, G) bytes, 256-byte aligned
 *
 * Errors: as gq_cd_assign (no n_cycles); GQ_ERR_SHAPE also if What == W.
 */
int gq_ldlq_assign(const float* W, float* What, const float* codebook, int32_t n_levels,
                   int64_t d_out, int64_t d_in, int64_t ld_w, const float* R, int32_t G,
                   uint8_t* Q, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of device workspace gq_lnq_codebook needs (0 for invalid sizes). */
size_t gq_lnq_codebook_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G, int32_t n_levels);

/*
 * The codebook step of layer-wise non-uniform quantization run against the group
 * Hessians (Section 4.2: Algorithm 2, lines 4 and 14; the closed form of Eq. "conti-sol").
 * For fixed assignments Q, every output channel j (group k = j / (d_out/G)) gets the grid
 *
 *   codebook[j,:] = (P^T H[k] P + lam I)^-1 P^T H[k] W[j,:],   P[i,q] = 1 if Q[j,i] == q else 0,
 *
 * the minimiser of (W[j,:] - P c)^T H[k] (W[j,:] - P c) + lam |c|^2 over c.  P^T H[k] is
 * accumulated in fp32 from exact products (H enters as three bf16 terms), the n_levels x
 * n_levels system is solved in fp64 by Gaussian elimination with partial pivoting.  A grid
 * point no coordinate is assigned to gets the value 0 (lam > 0).
 *
 *   W         [d_out, d_in]     device fp32, row pitch ld_w elements (row j = output channel j)
 *   Q         [d_out, d_in]     device bytes, dense; every entry < n_levels
 *   H         [G, d_in, d_in]   device fp32; only the upper triangle (incl. diagonal) is read
 *   lam       >= 0              the paper's value is 1e-7
 *   codebook  [d_out, n_levels] device fp32, dense, written
 *   What      [d_out, d_in]     device fp32, pitch ld_w, or NULL: What[j,i] = codebook[j,Q[j,i]]
 *   workspace  at least gq_lnq_codebook_workspace_bytes() bytes, 256-byte aligned
 *
 * Errors: GQ_ERR_NULLPTR, GQ_ERR_SHAPE (d_out <= 0, d_in <= 0, G <= 0, d_out % G != 0,
 * ld_w < d_in, n_levels <= 0, lam < 0 or NaN), GQ_ERR_UNSUPPORTED (n_levels > 16),
 * GQ_ERR_ALIGN (W/What/H not 16-byte aligned or ld_w*4 not a multiple of 16),
 * GQ_ERR_WORKSPACE, GQ_ERR_HIP.  An entry of Q >= n_levels is not detected: its
 * coordinate is left out of every sum and its What is 0.
 */
int gq_lnq_codebook(const float* W, int64_t d_out, int64_t d_in, int64_t ld_w, const uint8_t* Q,
                    const float* H, int32_t G, int32_t n_levels, double lam,
                    float* codebook, float* What,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of device workspace gq_lnq needs (0 for invalid sizes). */
size_t gq_lnq_workspace_bytes(int64_t d_out, int64_t d_in, int32_t G, int32_t n_levels);

/*
 * Layer-wise non-uniform quantization against the group Hessians, the whole alternation of
 * Algorithm 2 (Section 4.2) in one call: starting from the assignments Q,
 *
 *   repeat n_iters times (T):  grids <- gq_lnq_codebook(Q);  What <- grids[Q];
 *                              Q, What <- n_cycles cycles (K) of gq_cd_assign
 *   finally:                   grids <- gq_lnq_codebook(Q);  What <- grids[Q]
 *
 * exactly as those two calls would do it (same kernels, same order).  The paper uses T = 2, K = 4
 * (T = 1 for the 70B models), lam = 1e-7.  By Prop. 4.1 no step increases the layer objective.
 *
 *   W         [d_out, d_in]     device fp32, row pitch ld_w elements
 *   What      [d_out, d_in]     device fp32, same pitch, written; must not overlap W
 *   Q         [d_out, d_in]     device bytes, dense; in: the initial assignments (every entry
 *                               < n_levels), out: the final ones
 *   codebook  [d_out, n_levels] device fp32, dense, written: the final grids
 *   H         [G, d_in, d_in]   device fp32 with positive diagonals; only the upper triangle is read
 *   workspace  at least gq_lnq_workspace_bytes() bytes, 256-byte aligned
 *
 * Errors: as gq_lnq_codebook and gq_cd_assign; GQ_ERR_SHAPE also if n_iters < 0 or What == W.
 */
int gq_lnq(const float* W, float* What, uint8_t* Q, float* codebook, int32_t n_levels,
           int64_t d_out, int64_t d_in, int64_t ld_w, const float* H, int32_t G,
           int32_t n_iters, int32_t n_cycles, double lam,
           void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GQ_H_ */
