/* rbgp.h -- C ABI of the MI355X (gfx950) RBGP4 sparse x dense product library.
 *
 * The library computes O = W_s x I, where the mask of W_s is the bipartite
 * graph product G_o (x) G_r (x) G_i (x) G_b of four biregular bipartite graphs
 * (Section 5, "RBGP4 sparsity pattern"): G_o and G_i sparse Ramanujan graphs,
 * G_r and G_b complete.  By Section 3 the biadjacency matrix of the product is
 * the Kronecker product of the factors' biadjacency matrices.  The mask is held
 * as the factors' adjacency lists only (Section 4, "Memory efficiency").
 *
 * Notation.  Factor i (0..3 = G_o, G_r, G_i, G_b) has rows[i] left vertices,
 * cols[i] right vertices and left degree row_deg[i]; its right degree is
 * rows[i]*row_deg[i]/cols[i].  M = prod rows, K = prod cols, rowdeg = prod
 * row_deg, nnz = M*rowdeg.  Row m = ((u0*rows[1]+u1)*rows[2]+u2)*rows[3]+u3
 * and column k = ((v0*cols[1]+v1)*cols[2]+v2)*cols[3]+v3 (last factor fastest).
 *
 * Canonical value order (the `data[rows][(1-sp)*cols]` array of the Appendix,
 * indexed as Algorithm 1 does): the kept values of row m are stored
 * contiguously, position t = ((j0*row_deg[1]+j1)*row_deg[2]+j2)*row_deg[3]+j3
 * holding column ((adj0[u0][j0]*cols[1]+adj1[u1][j1])*cols[2]+adj2[u2][j2])*cols[3]+adj3[u3][j3].
 * Adjacency lists ascend, so this is ascending-column order.
 *
 * Conventions.  Every function returns RBGP_OK (0) or a negative error code and
 * leaves its outputs untouched on error; no C++ exception crosses the boundary.
 * "host" pointers are ordinary process memory, "device" pointers are HIP device
 * memory of the current device.  The library never allocates or frees a buffer
 * the caller passes; it keeps small device-side copies of its own index tables
 * inside the mask object (created on first use on the current device, released
 * by rbgp_mask_free).  `hip_stream` is a hipStream_t passed as void* (NULL = the
 * default stream); device work is enqueued on it asynchronously unless stated.
 * One GPU: a mask object is bound to the device that is current on first use.
 * A mask object may be used from one host thread at a time.
 */
#ifndef RBGP_H_
#define RBGP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rbgp_mask rbgp_mask_t; /* opaque, host memory */

/* RBGP_F32: W, I, O fp32.  RBGP_BF16_F32ACC: W, I bfloat16, fp32 accumulation, O fp32.
 * RBGP_BF16: as RBGP_BF16_F32ACC, and rbgp_spmm / rbgp_conv3x3 round the fp32 sums to bfloat16
 * (nearest, ties to even) when they store O; everywhere else (packing, layouts, kernel choice,
 * rbgp_sddmm, whose dW stays fp32) the two bf16 modes are the same mode, and buffers packed for
 * one serve the other.  (The paper states no precision: Section 5.) */
enum { RBGP_F32 = 0, RBGP_BF16_F32ACC = 1, RBGP_BF16 = 2 };
typedef int rbgp_dtype_t; /* one of the three above; any other value is answered with RBGP_EINVAL */

enum {
  RBGP_OK = 0,
  RBGP_EINVAL = -1,        /* null pointer, non-positive size, density not 1/2^L, ... */
  RBGP_ENOMEM = -2,
  RBGP_ENOTRAMANUJAN = -3, /* no sample met the bound within max_tries */
  RBGP_ESHAPE = -4,        /* M, K, ld* do not match the mask */
  RBGP_EHIP = -5,          /* a HIP call failed (message via rbgp_last_hip_error) */
  RBGP_EUNSUPPORTED = -6,  /* requested kernel cannot run this mask / dtype */
  RBGP_EINTERNAL = -7,     /* rbgp_mask_check_tables found an inconsistent index table */
  RBGP_ETOOLARGE = -8      /* rbgp_sddmm_static: the problem needs more scratch memory than its fixed array holds */
};

/* per-factor result of the spectral test */
enum {
  RBGP_SPEC_OK = 0,
  RBGP_SPEC_COMPLETE = 1,
  RBGP_SPEC_DEGENERATE = 2,
  RBGP_SPEC_PRODUCT = 3   /* a factor made of several base graphs, each tested on its own (rbgp_make_mask_k) */
};

/* kernel families */
enum {
  RBGP_KERNEL_AUTO = 0,
  RBGP_KERNEL_GENERIC = 1,  /* plain FMA, any four-factor mask, canonical layout */
  RBGP_KERNEL_MFMA = 2,     /* RBGP4 masks: I tiles staged in LDS, MFMA on the dense blocks */
  RBGP_KERNEL_MFMA_REG = 3, /* RBGP4 masks: I rows streamed into registers and reused across a
                               cluster of tile rows, 16-row MFMA on the dense blocks */
  RBGP_KERNEL_MFMA_TILE = 4,/* bf16 modes only, never chosen by AUTO: every nonzero of G_o as a dense
                               block of W_s (zeros where the inner graphs have no edge), I staged in
                               LDS once per workgroup, 32-row MFMA.  Any inner graphs; needs
                               |G_r.U| |G_i.U| |G_b.U| = 32 and |G_r.V| |G_i.V| |G_b.V| <= 320.
                               rbgp_spmm then needs dev_I 16-byte aligned and ldI a multiple of 8,
                               rbgp_conv3x3 an image width that is a multiple of 8 (ESHAPE) */
  RBGP_KERNEL_MFMA_REG_FILLED = 5 /* the RBGP_KERNEL_MFMA_REG kernels on a superset of the mask, the packed buffer
                               storing a zero wherever the mask has no entry.  Either G_i filled in: all
                               |G_r.U| |G_i.U| |G_b.U| rows of a tile then share one column set (row repetition,
                               Section 5, bought with |G_i.V| / d_i times the products); for masks with few
                               rows per column set (|G_r.U| |G_b.U| <= 4, the slow rows of Table 3) and a
                               moderately sparse G_i.  Or G_o filled in (at least a quarter full): G_o (x) G_r
                               is then one tile column through all of K, walked in stages of up to 72 steps
                               instead of the few one tile holds, at |G_o.V| / d_o times the products.  The
                               library keeps the candidate it estimates cheaper; AUTO takes it where it
                               estimates it faster than the mask as given, never for masks whose G_b is the
                               nine taps of a 3x3 convolution (rbgp_conv3x3 does not run on it) */
};

/* tuning knobs (rbgp_mask_tune) */
enum {
  RBGP_TUNE_COLS_PER_LANE = 0,        /* MFMA: 1 or 2 */
  RBGP_TUNE_COLS_PER_WORKGROUP = 1,   /* MFMA: 64 or 128; MFMA_REG bf16: columns per wave, 64 or 128 */
  RBGP_TUNE_GROUPS_PER_WORKGROUP = 2, /* MFMA: a divisor of |G_i.U| */
  RBGP_TUNE_ROW_PAIRING = 3,          /* MFMA_REG fp32, masks whose rows repeat in groups of 5..8 (two tile
                                         rows per 16-row MFMA group): 1 = fixed pairs of tile rows, each wave
                                         walking the union of its pair's tiles; 2 = a wave owns one tile row
                                         and pairs it, tile by tile, with one of two partner rows that has
                                         the same tile (EUNSUPPORTED where that kernel does not apply: bf16,
                                         other group sizes, more than 32 tile rows, with RBGP_TUNE_K_SPLIT);
                                         default: 2 where it walks fewer tiles and N fills the chip */
  RBGP_TUNE_ROW_GROUPS = 4,           /* MFMA_REG: 16-row MFMA groups per wave, 1, 2 or 4 (each loaded row of I
                                         is reused by all of them).  bf16: any mask (larger clusters of tile
                                         rows).  fp32: only tile rows that have the very same tiles -- masks
                                         with more than 16 rows per column set, whose rows of G_r move into
                                         the tile-row index -- 2 for every stage size, 4 for stages of up to
                                         18 steps (else EUNSUPPORTED; a mask that fp32 runs regrouped, see
                                         rbgp_mask_reg_plan, has the tile rows of that factoring) */
  RBGP_TUNE_K_SPLIT = 5,              /* MFMA_REG: waves that share a column tile and split its
                                         nonzero tiles between them, 1, 2 or 4 (default: 1 unless N
                                         is too small to give every SIMD a wave) */
  RBGP_TUNE_COLUMN_TILES = 6,         /* MFMA_REG fp32, stages of up to 8 contraction steps, every tile row with
                                         the same number of tiles: column tiles (64 columns each) a wave takes
                                         one after the other, 1, 2, 4 or 8 (EUNSUPPORTED where the stage lists of
                                         that many tiles exceed 64 stages, for rbgp_conv3x3 and with a split) */
  RBGP_TUNE_REGISTER_SETS = 7,        /* MFMA_REG: 2 = two register sets (two stages of loads in flight per wave),
                                         1 = one set refilled in place, which lets more waves share a SIMD: fp32 with
                                         stages of 18 steps and more and one row group (two groups: 36 steps, or
                                         72 on the tap-grouped fused convolution), bf16 on 128-column tiles with
                                         stages of 36 or 72 steps and one or two row groups, of up to 36 steps
                                         and four groups (one tile row each), of 18 or 32 steps and two groups
                                         where a wave has one stage (EUNSUPPORTED elsewhere); default: 1 where
                                         it exists */
  RBGP_NUM_TUNE = 8
};

/* Device tables.  A mask keeps small index tables in device memory (adjacency lists, stage lists,
 * pack permutations; a few KB to a few hundred KB), built on first use: the first rbgp_pack /
 * rbgp_spmm / rbgp_conv3x3 / rbgp_sddmm call on a mask -- and the first after another kernel choice or
 * tuning value, with another convolution geometry, or, for rbgp_sddmm, with a larger N -- allocates
 * and uploads them (hipMalloc, synchronous copies).  Every later call with the same configuration
 * only launches kernels on `hip_stream`: it may be recorded into a HIP graph and replayed (make one
 * eager call first).  The tables belong to the mask and go with rbgp_mask_free.  All calls that use
 * one mask come from one thread at a time. */

/* Sample the four base graphs and build the mask (host only, no GPU call).
 * Appendix "Ramanujan Bipartite Graph Generation": a factor with row_deg < cols
 * is produced by L = log2(cols/row_deg) random 2-lifts of the complete bipartite
 * graph on (rows/2^L, cols/2^L) vertices and resampled until its second largest
 * singular value is <= sqrt(d_l-1)+sqrt(d_r-1) (Section 3), at most max_tries
 * times (<= 0 means 1000).  row_deg == cols means a complete factor.  A sparse
 * factor whose smaller degree is 1 cannot meet the bound; its first sample is
 * kept and reported RBGP_SPEC_DEGENERATE.  The random source is the counter
 * based SplitMix64 stream keyed by (seed, factor, attempt); equal arguments give
 * byte-identical masks.  *out is owned by the caller (rbgp_mask_free).
 * Errors: EINVAL (null, size <= 0, cols/row_deg not a power of two, rows not
 * divisible by it, M or K above 2^24), ENOTRAMANUJAN, ENOMEM. */
int rbgp_make_mask(const int32_t rows[4], const int32_t cols[4], const int32_t row_deg[4],
                   uint64_t seed, int32_t max_tries, rbgp_mask_t **out);

/* The general configuration of Section 5 ("RBGP4 sparsity pattern": a mask is configured by the
 * number of base graphs K and the type, sparse or complete, of each): `count` (1..16) base graphs
 * G_1 .. G_count, sampled like those of rbgp_make_mask (coin stream keyed by (seed, index of the base
 * graph, attempt)), whose product G_1 (x) ... (x) G_count is the mask.  roles[i] in 0..3, non-decreasing,
 * says which of the four factors G_o, G_r, G_i, G_b of the kernels' view base graph i belongs to: the
 * factor is the product of its base graphs (a role without any is the trivial graph on (1, 1) vertices),
 * which is again biregular, so the mask object, its canonical order (ascending column per row) and every
 * other entry point are those of a four-factor mask, and by associativity of the product the mask is
 * exactly G_1 (x) ... (x) G_count.  The MFMA kernel families need the factors of roles 1 and 3 complete:
 * where a role 1 or 3 is given a sparse base graph, the graphs of that role up to its last sparse one
 * join role 0 or 2 in the kernels' view (rbgp_mask_factor / rbgp_mask_spectrum report that view, the
 * mask, its canonical order and rbgp_mask_base do not change).  And where every base graph of role 2
 * is complete (all the sparsity in G_o), they join role 1 in that view: a complete G_i repeats rows
 * exactly as G_r does, and the kernels fill their row groups better from it.  The same holds for
 * rbgp_make_mask.
 * rbgp_mask_spectrum of a factor made of several base graphs reports the singular values of the
 * product (products of the base graphs' singular values), the bound of the product's degrees and
 * RBGP_SPEC_PRODUCT; rbgp_mask_base reports each base graph.  rbgp_make_mask(rows, cols, row_deg, ...)
 * is rbgp_make_mask_k(4, rows, cols, row_deg, {0, 1, 2, 3}, ...).  Errors as for rbgp_make_mask. */
int rbgp_make_mask_k(int32_t count, const int32_t *rows, const int32_t *cols, const int32_t *row_deg,
                     const int32_t *roles, uint64_t seed, int32_t max_tries, rbgp_mask_t **out);

/* Number of base graphs of the mask, and base graph i: sizes, left degree, role, a borrowed pointer to
 * its adjacency list (rows*deg int32, valid until mask_free) and its spectral data (any output
 * pointer may be NULL). */
int rbgp_mask_num_base(const rbgp_mask_t *mask);
int rbgp_mask_base(const rbgp_mask_t *mask, int i, int32_t *rows, int32_t *cols, int32_t *deg, int32_t *role,
                   const int32_t **adj, double *sigma1, double *sigma2, double *bound, int *status,
                   int *tries);

/* Release the mask and its device tables.  NULL is allowed. */
void rbgp_mask_free(rbgp_mask_t *mask);

/* Sizes of the product (any output pointer may be NULL). */
int rbgp_mask_shape(const rbgp_mask_t *mask, int64_t *M, int64_t *K, int64_t *rowdeg,
                    int64_t *coldeg, int64_t *nnz);

/* Factor i: sizes, left degree and a borrowed pointer to its adjacency list
 * (host, rows*deg int32, row-major, ascending per row; valid until mask_free). */
int rbgp_mask_factor(const rbgp_mask_t *mask, int i, int32_t *rows, int32_t *cols, int32_t *deg,
                     const int32_t **adj);

/* Spectral data of factor i: two largest singular values of its biadjacency
 * matrix (= lambda_1, lambda_2 of the graph), the Ramanujan bound, the status
 * (RBGP_SPEC_*) and the number of samples drawn (0 for a complete factor). */
int rbgp_mask_spectrum(const rbgp_mask_t *mask, int i, double *sigma1, double *sigma2,
                       double *bound, int *status, int *tries);

/* Column of every kept value in canonical order: out is caller-owned host
 * memory of M*rowdeg int32. */
int rbgp_mask_columns(const rbgp_mask_t *mask, int32_t *out);

/* Dense 0/1 mask, caller-owned host memory of M*K bytes (for tests). */
int rbgp_mask_dense(const rbgp_mask_t *mask, uint8_t *out);

/* Choose the kernel family used by rbgp_packed_bytes / rbgp_pack / rbgp_spmm for
 * this mask: AUTO (default: an MFMA family when the mask's shape is covered, else
 * GENERIC) or one family (EUNSUPPORTED if it does not cover the mask's shape; a
 * family that does not cover the dtype falls back to GENERIC, RBGP_KERNEL_MFMA_TILE
 * in fp32 mode to what AUTO would take).  Each family has its own packed layout:
 * changing it invalidates buffers packed before. */
int rbgp_mask_set_kernel(rbgp_mask_t *mask, int kernel);

/* Kernel family (never AUTO) that rbgp_pack / rbgp_spmm use for this dtype. */
int rbgp_mask_kernel(const rbgp_mask_t *mask, rbgp_dtype_t dtype);

/* Set one launch-shape knob (RBGP_TUNE_*) of this mask; 0 = library default.
 * Does not change the packed layout.  rbgp_spmm returns EUNSUPPORTED for a
 * combination that is not built. */
int rbgp_mask_tune(rbgp_mask_t *mask, int knob, int value);

/* Bytes of the device buffer that rbgp_pack fills (kernel layout incl. padding); 0 on error. */
size_t rbgp_packed_bytes(const rbgp_mask_t *mask, rbgp_dtype_t dtype);

/* The packed layout as a table (host only, no GPU call): out[p], for every element p of
 * the packed buffer (rbgp_packed_bytes() / element size entries, caller-owned host
 * memory), is the canonical index m*rowdeg + t of the kept value stored there, or -1
 * for padding (stored as zero).  Every kept value appears exactly once. */
int rbgp_pack_layout(const rbgp_mask_t *mask, rbgp_dtype_t dtype, int32_t *out);

/* Reorder the kept values from canonical order into the layout the SpMM kernel
 * reads, which stores the dense |G_r.U||G_b.U| x |G_b.V| blocks of one tile step
 * contiguously (the compact W tile that Algorithm 1 stages per step).
 * host_values: M*rowdeg elements of the dtype's input type (float or bf16 bits),
 * host memory, read before the call returns.  dev_packed: caller-owned device
 * buffer of rbgp_packed_bytes().  The permutation runs in a HIP kernel on
 * `hip_stream`; the call synchronises that stream before returning. */
int rbgp_pack(const rbgp_mask_t *mask, rbgp_dtype_t dtype, const void *host_values,
              void *dev_packed, void *hip_stream);

/* Same with the canonical values already in device memory (M*rowdeg elements);
 * asynchronous on `hip_stream`. */
int rbgp_pack_device(const rbgp_mask_t *mask, rbgp_dtype_t dtype, const void *dev_values,
                     void *dev_packed, void *hip_stream);

/* Backward products for training with the mask held fixed (Section 6: the masks are
 * predefined and do not change during training).  The paper times the forward product only;
 * these are its two gradients, computed without ever forming a dense M x K matrix.
 *
 * rbgp_mask_transpose: the mask of W_s^T.  The transpose of a product of biadjacency matrices
 * is the product of the transposed factors (Section 3), so it is again a four-factor mask
 * (G_o^T, G_r^T, G_i^T, G_b^T; adjacency lists = the co-adjacency lists of `mask`, ascending)
 * and every entry point above works on it with M and K exchanged; dI = W_s^T x dO is
 * rbgp_spmm on it.  Host only, no GPU call.  *out is independent of `mask` and owned by the
 * caller (rbgp_mask_free).  Errors: EINVAL, ENOMEM. */
int rbgp_mask_transpose(const rbgp_mask_t *mask, rbgp_mask_t **out);

/* out[s] (caller-owned host memory, nnz int32) = canonical index in `mask` (m * rowdeg + t) of
 * the kept value that has canonical index s in the transposed mask (k * coldeg + position of m
 * among the rows adjacent to column k, ascending). */
int rbgp_transpose_order(const rbgp_mask_t *mask, int32_t *out);

/* rbgp_pack / rbgp_pack_device for a mask made by rbgp_mask_transpose, with the values given in
 * the canonical order of the ORIGINAL mask (nnz elements): the same weights can be packed for the
 * forward product and for the backward data product without a reordering by the caller.
 * EINVAL for a mask that was not made by rbgp_mask_transpose (or rbgp_mask_conv3x3_transpose). */
int rbgp_pack_transposed(const rbgp_mask_t *mask_t, rbgp_dtype_t dtype, const void *host_values,
                         void *dev_packed, void *hip_stream);
int rbgp_pack_transposed_device(const rbgp_mask_t *mask_t, rbgp_dtype_t dtype, const void *dev_values,
                                void *dev_packed, void *hip_stream);

/* Gradient of the kept values: dW[m][t] = sum_n dO[m][n] * I[k][n] for the t-th kept column k
 * of row m -- the product dO x I^T sampled on the mask, nothing off the mask is computed.
 * dev_dO: M x N row-major, leading dimension ld_dO >= N; dev_I: K x N row-major, leading
 * dimension ldI >= N; both in the dtype's input type (fp32, or bf16 bits), 4-byte aligned
 * (bf16 with an odd leading dimension runs on the plain kernel).
 * dev_dW: nnz fp32 in canonical order, overwritten (N == 0 stores zeros).  RBGP4 masks that the
 * RBGP_KERNEL_MFMA_REG family covers run on MFMA kernels (unless the mask's kernel choice is
 * RBGP_KERNEL_GENERIC), every other mask on a plain kernel.  Sums over n are taken in a fixed
 * order: results are reproducible run to run.  Uses a partial-sum buffer that the library keeps
 * with the mask and grows as needed (a growing call synchronises the device): calls for one mask
 * must not overlap in time (put them on one stream).  Errors: ESHAPE
 * (sizes do not match the mask, leading dimension, alignment), EINVAL, EHIP.  Asynchronous on
 * `hip_stream`. */
int rbgp_sddmm(const rbgp_mask_t *mask, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N,
               const void *dev_dO, int64_t ld_dO, const void *dev_I, int64_t ldI, float *dev_dW,
               void *hip_stream);

/* rbgp_sddmm for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving or training loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same
 * results as rbgp_sddmm (bit for bit), but the call allocates and frees nothing on the device and
 * does not touch the mask's own device tables: the index tables and the partial sums of the kernels
 * live in one fixed array of 16.25 MiB (256 KiB of tables, 16 MiB of partial sums) that is part of
 * the library's code object on every GPU the library runs on, until the process ends.  The tables
 * reach it as kernel arguments (small launches on `hip_stream`), whenever the array holds another
 * mask's; the partial sums of a call overwrite those of the last.
 * Limits: RBGP_ETOOLARGE when the tables of the mask exceed 256 KiB or the call needs more than
 * 16 MiB of partial sums (partial sums = ceil(N / columns per workgroup) x nnz floats; the VGG19 and
 * WRN-40-4 layers of the paper need none to 1.2 MiB); at most 64 GPUs.
 * All calls on one GPU share the one array: calls that overlap in time on a GPU (two streams, two
 * threads) race on it, whatever masks they use; so does a call of this kind that overlaps one whose
 * tables it replaces.  Errors otherwise as rbgp_sddmm.  Asynchronous on `hip_stream`. */
int rbgp_sddmm_static(const rbgp_mask_t *mask, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N,
                      const void *dev_dO, int64_t ld_dO, const void *dev_I, int64_t ldI, float *dev_dW,
                      void *hip_stream);

/* O = W_s x I (Section 5, "GPU Implementation"; Algorithm 1 with C overwritten).
 * dev_I: K x N row-major with leading dimension ldI >= N elements (the lowered
 * convolution input, N = batch*H*W contiguous); dev_O: M x N row-major fp32 (bf16 bits
 * in RBGP_BF16 mode, 2-byte aligned) with leading dimension ldO >= N elements,
 * overwritten.  M and K must equal the mask's (ESHAPE otherwise).  N == 0 is a
 * no-op.  Buffers must not overlap.  The
 * RBGP_KERNEL_MFMA family needs dev_I 16-byte aligned and ldI a multiple of 4
 * (fp32) or 8 (bf16) elements, the RBGP_KERNEL_MFMA_REG family in bf16 mode dev_I
 * 8-byte aligned and ldI a multiple of 4 (64-column wave tiles), or 16-byte aligned
 * and ldI a multiple of 8 (128-column tiles, taken by default when both hold and N
 * is large enough); ESHAPE otherwise.  In bf16 mode it reads the last row of I up
 * to the next multiple of 4 (8) columns, inside the K x ldI array.  The other
 * cases take any alignment.  I and O may exceed 4 GiB; the RBGP_KERNEL_MFMA_REG
 * family returns EUNSUPPORTED when the rows of I that one of its stages spans
 * (at most |G_r.V| * |G_i.V| * |G_b.V|) times ldI reach 2 GiB.  dev_packed must have
 * been packed with the same kernel family and dtype.  Asynchronous on `hip_stream`. */
int rbgp_spmm(const rbgp_mask_t *mask, rbgp_dtype_t dtype, int64_t M, int64_t K, int64_t N,
              const void *dev_packed, const void *dev_I, int64_t ldI, void *dev_O, int64_t ldO,
              void *hip_stream);
/* Non-finite inputs.  The sum of Section 5 runs over the kept weights of a row only, and so does
 * RBGP_KERNEL_GENERIC: an infinity or NaN in a row of I reaches the outputs of the rows of W_s that keep
 * a weight in that column of the mask, nothing else.  The MFMA families fill their matrix-core groups
 * with zero weights where a stage is padded or (RBGP_KERNEL_MFMA_REG, RBGP_KERNEL_MFMA_TILE) a tile row
 * lacks a tile, and 0 x inf is NaN: with them a non-finite I[k][n] can turn any output of COLUMN n of O
 * (never another column) into NaN.  Finite I gives the same result on all families (to rounding). */

/* Fused 3x3 convolution (stride 1, zero padding 1): O = W_s x im2col(X) without the lowered
 * input ever being stored.  (The paper feeds its kernel batched activations lowered to a
 * matrix, Section 5 "GPU Implementation"; here the lowering is folded into the loads: the
 * nine taps are the columns of the complete factor G_b.)
 * The mask must have |G_b.V| = 9 complete, K = 9 * channels_in, M = channels_out.
 * dev_X: activations [channels_in][images][height + 2][width + 2] in the dtype's input type
 * (fp32, or bf16 bits), 4-byte aligned, with a border of one pixel that the caller keeps at
 * zero.  Row k = 9 * c + 3 * (dy + 1) + (dx + 1) of the lowered input is pixel (y + dy, x + dx)
 * of channel c; column n = (image * height + y) * width + x.  dev_O: M x N row-major fp32
 * (bf16 bits in RBGP_BF16 mode), N = images * height * width, leading dimension ldO >= N, overwritten.  dev_packed: as for
 * rbgp_spmm (same layout, same dtype).
 * Runs on the RBGP_KERNEL_MFMA_REG family (and, for masks set to it, on RBGP_KERNEL_MFMA_TILE):
 * EUNSUPPORTED for masks or kernel choices outside them; ESHAPE unless width is a multiple of 4
 * (8 on RBGP_KERNEL_MFMA_TILE) and the sizes match the mask.
 * Asynchronous on `hip_stream`. */
int rbgp_conv3x3(const rbgp_mask_t *mask, rbgp_dtype_t dtype, int64_t channels_out, int64_t channels_in,
                 int64_t images, int64_t height, int64_t width, const void *dev_packed, const void *dev_X,
                 void *dev_O, int64_t ldO, void *hip_stream);

/* Weight gradient of the fused 3x3 convolution: rbgp_sddmm with I = im2col(X) never stored, i.e.
 * dW[m][t] = sum_n dO[m][n] * X[c][image][y + dy][x + dx] for the kept column k = 9 * c + 3 * (dy + 1) + (dx + 1)
 * (same layouts and conventions as rbgp_conv3x3 and rbgp_sddmm: dev_X zero-padded
 * [channels_in][images][height + 2][width + 2], below 2 GiB; dev_dO M x N with N = images * height * width;
 * dev_dW nnz fp32 in canonical order).  Runs on the MFMA kernel of rbgp_sddmm only: EUNSUPPORTED for
 * masks outside the RBGP_KERNEL_MFMA_REG family or with |G_b.V| != 9 complete; ESHAPE unless width is
 * a multiple of 4 (fp32) or 8 (bf16) and the sizes match the mask.  Asynchronous on `hip_stream`. */
int rbgp_conv3x3_sddmm(const rbgp_mask_t *mask, rbgp_dtype_t dtype, int64_t channels_out, int64_t channels_in,
                       int64_t images, int64_t height, int64_t width, const void *dev_dO, int64_t ld_dO,
                       const void *dev_X, float *dev_dW, void *hip_stream);

/* Gradient of the fused 3x3 convolution with respect to its input.  With O = W_s x im2col(X), dX is
 * again a 3x3 convolution (stride 1, zero padding 1), of dO, whose weights W'[c][9 m + tap'] =
 * W_s[m][9 c + (8 - tap')] have the four-factor mask G_o^T (x) G_r^T (x) (G_i^T (x) J) (x) taps
 * (J complete on (1, |G_b.U|) vertices).  This call builds that mask (host only, as
 * rbgp_mask_transpose does for the plain product); then
 *   rbgp_pack_transposed(mask_x, dtype, values in the canonical order of `mask`, packed_x, stream)
 *   rbgp_conv3x3(mask_x, dtype, channels_in, channels_out, images, height, width, packed_x,
 *                dO zero-padded [channels_out][images][height + 2][width + 2], dX as a channels_in x N matrix, ...)
 * computes dX without the lowered gradient (9 x larger) ever being stored.  EUNSUPPORTED unless
 * |G_b.V| = 9 complete. */
int rbgp_mask_conv3x3_transpose(const rbgp_mask_t *mask, rbgp_mask_t **out);

/* For a mask made by rbgp_mask_transpose or rbgp_mask_conv3x3_transpose: out[s] (caller-owned host
 * memory, nnz int32) = canonical index, in the mask it was made from, of the kept value that has
 * canonical index s in this mask (what rbgp_pack_transposed applies).  EINVAL for other masks. */
int rbgp_mask_original_order(const rbgp_mask_t *derived, int32_t *out);

/* How the RBGP_KERNEL_MFMA_REG family walks this mask (host only; Section 5: G_o skips tiles, G_r and
 * G_b repeat rows).  info[0] = tile rows per 16-row MFMA group (0: the family does not cover the mask,
 * the rest is 0 too), [1] = stages per nonzero tile, [2] = contraction steps per stage (padded),
 * [3] = tile rows; fixed clusters of tile rows: [4] = clusters, [5] = longest stage list, [6] = sum of
 * the stage lists; tile-by-tile pairing (RBGP_TUNE_ROW_PAIRING = 2; all 0 where it does not apply):
 * [7] = quads of tile rows, [8] = most stages on one SIMD (two waves), [9] = sum of the stage lists,
 * [10] = longest stage list of a wave, [11] / [12] = distinct stages of I wanted by the first / the first
 * two stages of all waves together.  [13] = longest stage list on the mask with G_i filled in
 * (RBGP_KERNEL_MFMA_REG_FILLED; 0: not available for this mask).  Masks with more than 16 rows per column set and
 * a composite |G_b.U| (the transpose of a lowered 3x3 convolution): in fp32 the family runs on the same mask
 * factored as G_o (x) G_r (x) (G_i (x) J(q, 1)) (x) J(|G_b.U| / q, |G_b.V|), which fills more of the 16 rows of an
 * MFMA group; [14] = rows of a group in use there, [15] = its tile rows (0, 0: the mask runs as given).  Masks with
 * a complete G_o run (both dtypes) with G_o (x) G_r merged into one tile column, J(a_o, 1) (x) J(a_r, c_o c_r), where
 * that makes the stages longer and the walk cheaper; [14], [15] then describe that factoring. */
int rbgp_mask_reg_plan(const rbgp_mask_t *mask, int32_t info[16]);

/* Host-only self check of the index tables the RBGP_KERNEL_MFMA_REG kernels read for this mask: every
 * (tile row, nonzero tile, stage) is multiplied exactly once, by a stage whose rows of I are that
 * tile's and lie inside K, with a weight-fragment position inside the packed buffer; stage lists fit
 * their tables and end in sentinels.  RBGP_OK, or RBGP_EINTERNAL (a bug in the library). */
int rbgp_mask_check_tables(const rbgp_mask_t *mask);

/* Static description of an error code / of the last HIP failure in this thread. */
const char *rbgp_strerror(int code);
const char *rbgp_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RBGP_H_ */
