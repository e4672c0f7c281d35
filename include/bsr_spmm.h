/*
 * bsr_spmm -- block-sparse times dense product for AMD MI355X (gfx950).
 *
 *     Y = X * W^T        X dense (m, k), W block-sparse (n, k) in BSR, Y dense (m, n)
 *
 * The operation and the storage format are those of the paper's Background
 * section (the three arrays block_data / block_indices / index_pointer, W kept
 * as (n, k) so that a block-row of W produces a run of consecutive columns of
 * Y) and of the unnumbered equation in its Approaches section (X W_B^T = Y
 * with b_r | n and b_c | k):
 *
 *     block_data[p][a][c] = W[r*bs_r + a][block_indices[p]*bs_c + c]
 *         for p in [index_pointer[r], index_pointer[r+1])
 *     Y[i][r*bs_r + a]    = sum_p sum_c X[i][block_indices[p]*bs_c + c] * block_data[p][a][c]
 *
 * Conventions for every entry point
 *   - plain C ABI; every function returns a bsr_status, never throws or aborts;
 *   - "host" pointers are ordinary CPU memory, "device" pointers are GPU
 *     memory of the current HIP device; the library never allocates or frees
 *     device memory (the caller does, e.g. with PyTorch) and never takes
 *     ownership of a caller's buffer;
 *   - dense matrices are row-major and contiguous; index arrays are int32;
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream);
 *     device work is queued on it and the call returns without waiting.
 *
 * Debug mode.  A handle created while the environment variable BSR_SPMM_DEBUG is set to anything but "0"
 * re-checks, on the device and before every product (bsr_spmm, bsr_spmm_ex, bsr_spmm_static, bsr_sddmm),
 * the arrays every kernel address derives from: index_pointer and block_indices as they are in device
 * memory at that moment (BSR_ERR_INDPTR, BSR_ERR_INDEX) and the plan in the workspace
 * (BSR_ERR_WORKSPACE when it no longer holds what bsr_create() wrote).  On a failure nothing else is
 * launched.  The check waits for the stream (one extra launch, a 16-byte copy, a synchronisation), so
 * such a call is NOT asynchronous; it is skipped while the stream is being captured into a graph.
 */
#ifndef BSR_SPMM_H
#define BSR_SPMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element types of X, block_data and Y.  Accumulation is always fp32. */
typedef enum { BSR_F32 = 0, BSR_F16 = 1, BSR_BF16 = 2 } bsr_dtype;

typedef enum {
    BSR_OK = 0,
    BSR_ERR_NULL = 1,        /* a required pointer is NULL */
    BSR_ERR_SHAPE = 2,       /* negative size, bs_r <= 0, bs_c <= 0, bs_r !| n, bs_c !| k (Approaches: b_r | n, b_c | k),
                                or a size that does not fit the int32 index arithmetic */
    BSR_ERR_INDPTR = 3,      /* index_pointer[0] != 0, decreasing, or last entry != nnzb */
    BSR_ERR_INDEX = 4,       /* a block_indices entry outside [0, k/bs_c) */
    BSR_ERR_DTYPE = 5,       /* unknown dtype, or y_dtype neither the input type nor BSR_F32 */
    BSR_ERR_ALIGN = 6,       /* a device pointer is not 16-byte aligned */
    BSR_ERR_WORKSPACE = 7,   /* workspace smaller than bsr_workspace_size() reports, or the chosen kernel needs
                                scratch (bsr_scratch_size) that has not been lent with bsr_set_scratch */
    BSR_ERR_HIP = 8,         /* a HIP runtime call failed (launch, copy) */
    BSR_ERR_UNSUPPORTED = 9, /* the requested kernel path cannot handle this block shape */
    BSR_ERR_SCRATCH_LIMIT = 10 /* bsr_spmm_static(): the product needs more scratch than the library's built-in
                                  BSR_STATIC_SCRATCH_BYTES */
} bsr_status;

/* Which kernel family bsr_spmm_ex() uses. */
typedef enum {
    BSR_PATH_AUTO = 0,   /* the library's choice for this matrix and m */
    BSR_PATH_WAVE = 1,   /* wavefront-reduction kernels: lanes split the reduction inside and across the
                            stored blocks of a block-row, cross-lane sum at the end (the paper's
                            "parallelize within blocks" + "aggregate partial results", Sections 4.4.2-4.4.3);
                            any block shape */
    BSR_PATH_MFMA = 2    /* matrix-core kernels: one workgroup owns an (m-tile, block-row) tile of Y and walks
                            the stored blocks of the block-row (the tile-per-thread-block design of the paper's
                            "Utilizing shared memory" section, with run-time indices); block shapes listed at
                            bsr_spmm_ex() */
} bsr_path;

typedef struct bsr_matrix bsr_matrix;   /* opaque handle: shape, device pointers (not owned), plan */

/*
 * Structural check of a BSR pattern (Background: the three arrays).  HOST pointers.
 *   n, k        rows / columns of W;   bs_r, bs_c  block shape (bs_r | n, bs_c | k)
 *   nnzb        number of stored blocks
 *   index_pointer_host  n/bs_r + 1 entries: starts at 0, non-decreasing, ends at nnzb
 *   block_indices_host  nnzb entries in [0, k/bs_c); any order inside a block-row, duplicates allowed
 *                       (duplicates are summed, as the definition sums over stored blocks)
 * Returns BSR_OK or the first problem found (NULL, SHAPE, INDPTR, INDEX in that order).
 */
bsr_status bsr_validate(int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                        const int32_t* index_pointer_host, const int32_t* block_indices_host);

/*
 * Bytes of DEVICE workspace bsr_create() needs for its plan (block-row order and work lists).
 * Always > 0 and a multiple of 256.  Errors: NULL, SHAPE.
 */
bsr_status bsr_workspace_size(int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                              size_t* bytes);

/*
 * Build a handle for W.  Validates the pattern (as bsr_validate), bins the block-rows by
 * their number of stored blocks and orders them longest first (the paper's Discussion: rows
 * with very different block counts make equal-sized work units diverge), and copies that
 * plan into `workspace_dev` on `hip_stream` (asynchronous; the host staging copy is owned by
 * the handle).
 *   block_data_dev     DEVICE, nnzb*bs_r*bs_c elements of `dtype`, [nnzb][bs_r][bs_c] row-major
 *   block_indices_dev  DEVICE, nnzb int32          index_pointer_dev  DEVICE, n/bs_r+1 int32
 *   block_indices_host / index_pointer_host        HOST copies of the same two arrays, read during
 *                                                  this call only
 *   workspace_dev      DEVICE, at least bsr_workspace_size() bytes, 16-byte aligned
 * The four device buffers stay owned by the caller and must outlive the handle; their contents
 * (block values included) may change between products as long as the pattern does not.
 * nnzb == 0 is valid (Y becomes all zeros); then block_data_dev / block_indices_* may be NULL.
 * On error *out is set to NULL.
 */
bsr_status bsr_create(bsr_matrix** out, int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                      bsr_dtype dtype, const void* block_data_dev,
                      const int32_t* block_indices_dev, const int32_t* index_pointer_dev,
                      const int32_t* block_indices_host, const int32_t* index_pointer_host,
                      void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* Frees the handle's host memory only (after waiting for a plan upload that may still read it).
 * NULL is accepted. */
void bsr_destroy(bsr_matrix* W);

/*
 * Y[m][n] = X[m][k] * W^T  (Approaches, the equation; overwrite, not accumulate).
 *   X_dev   DEVICE, m*k elements of W's dtype, row-major      Y_dev  DEVICE, m*n elements of y_dtype
 *   y_dtype W's dtype or BSR_F32; the fp32 accumulator is rounded to nearest-even on store
 *   m       any value >= 0 (m == 0 returns BSR_OK without device work)
 * Every element of Y is written; columns of an empty block-row are exact zeros.  Asynchronous on
 * `hip_stream`; no hidden synchronisation.  A product may be queued on any stream: until the plan
 * upload that bsr_create() queued on its own stream has finished, products make their stream wait
 * for it (an event wait on the device, not on the host).  Products on one handle may run
 * concurrently (unless they use lent scratch, see bsr_set_scratch): some kernels read a per-m work
 * list that the first product of that m uploads into the workspace (the handle keeps the lists of
 * the 4 most recent values of m; other streams wait for that upload the same way).  With more than
 * 4 distinct m in flight at once on one handle a list may be replaced while an earlier product still
 * reads it: keep such products ordered on one stream.
 * NaN or Inf in X: kernels that fill their last, partial group of blocks with zero-valued dummy
 * blocks multiply those zeros by real entries of X (the thin-block kernels: by column 0 of X), so a
 * non-finite entry there can reach outputs it does not belong to.  Finite inputs are unaffected.
 * Errors: NULL, SHAPE (m < 0 or m*max(k,n) >= 2^31), DTYPE, ALIGN, HIP.
 */
bsr_status bsr_spmm(const bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev,
                    bsr_dtype y_dtype, void* hip_stream);

/*
 * Scratch.  Some kernels need device memory beyond X, W and Y for the duration of one product:
 * for thin blocks (bs_r = 16, bs_c = 1, fp32) one matrix-core path first writes a transposed copy of
 * X, m*k floats, so that the columns of X that the stored blocks select (Background: the block's
 * column index picks the part of X) become contiguous rows.  The library does not allocate it.
 *   bsr_scratch_size  bytes such a product with m rows would use (0 when no kernel for this W
 *                     needs scratch); multiple of 256.
 *   bsr_set_scratch   lends `bytes` of DEVICE memory (16-byte aligned) to the handle, or takes it
 *                     back with NULL.  The memory stays owned by the caller and must outlive its
 *                     use; products that use it must not overlap in time on one handle (they
 *                     share it), i.e. keep them on one stream.
 * A thin-block W whose block-rows store their blocks in non-decreasing block-column order (k a
 * multiple of 4, at most 64512) needs none: its product runs in one launch that gathers the columns
 * from rows of X staged in LDS, and is preferred unless the block-rows are dense (more than 80 blocks
 * per 1024 columns on average).  For any other thin-block W, without (enough) scratch BSR_PATH_AUTO
 * uses the wavefront-reduction kernels and BSR_PATH_MFMA returns BSR_ERR_WORKSPACE.
 */
bsr_status bsr_scratch_size(const bsr_matrix* W, int64_t m, size_t* bytes);
bsr_status bsr_set_scratch(bsr_matrix* W, void* scratch_dev, size_t bytes);

/*
 * As bsr_spmm() with the kernel family fixed.  BSR_PATH_MFMA needs bs_r and bs_c in {16, 32, 64};
 * or bs_r and bs_c in {8, 16} with n and k multiples of 16 (the blocks are grouped into 16x16
 * tiles); or the thin shape bs_c == 1 with bs_r == 16 and fp32; or its transpose, bs_r == 1 with bs_c == 16,
 * fp32, fp32 output and no block stored twice; otherwise BSR_ERR_UNSUPPORTED.
 * BSR_PATH_WAVE takes any shape.
 */
bsr_status bsr_spmm_ex(const bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev,
                       bsr_dtype y_dtype, bsr_path path, void* hip_stream);

/*
 * Plan-time tuning by timed trials ("Automatic parameter tuning": the paper picks its kernels'
 * parameters per input shape by running the candidates).  Runs the product for every candidate
 * kernel and setting the library has for this W, this m and this output type -- 2 warm-up and
 * `trials` timed launches each (trials < 1: 20), timed with events on `hip_stream` -- and remembers
 * the fastest in the handle: later bsr_spmm() / BSR_PATH_AUTO calls with the same m and y_dtype use
 * it.  Every candidate computes the same product, so Y_dev holds Y = X * W^T afterwards.
 *   X_dev, Y_dev  as for bsr_spmm(); their values do not change which kernel is fastest
 *   tried_out     (may be NULL) number of candidates that ran
 *   best_us_out   (may be NULL) microseconds per product of the one remembered
 * Waits for the stream (it is not asynchronous) and must not run concurrently with other calls on
 * the same handle.  Lend scratch first (bsr_set_scratch) if kernels that need it should compete.
 * Errors: as bsr_spmm(); on error nothing is remembered.
 */
bsr_status bsr_tune(bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev, bsr_dtype y_dtype,
                    int trials, void* hip_stream, int* tried_out, float* best_us_out);

/*
 * What bsr_tune() remembered for (m, y_dtype): settings_out = {kernel family (bsr_path), matrix-core
 * kernel variant (0 the library's choice, 1 direct, 2 k-split, 3 LDS tiles, 4 LDS stripe, 5 row groups for
 * the longest block-rows and LDS tiles for the others), wavefronts
 * per workgroup, tile setting, two per-variant settings}, 0 = the kernel's default; us_out (may be
 * NULL) its measured microseconds per product.  BSR_ERR_UNSUPPORTED if nothing is remembered.
 */
bsr_status bsr_tune_result(const bsr_matrix* W, int64_t m, bsr_dtype y_dtype, int32_t settings_out[6], float* us_out);

/* The path BSR_PATH_AUTO resolves to for this handle and m (never AUTO; what bsr_tune()
 * remembered is not consulted).  Errors: NULL. */
bsr_status bsr_query_path(const bsr_matrix* W, int64_t m, bsr_path* path_out);

/*
 * The sibling product Z = G * W (the gradient of the layer's input when Y = X * W^T is a sparse
 * layer's forward pass, the use the paper's Introduction names) is the same product with W^T in
 * place of W:  Z = G * (W^T)^T.  These two calls build W^T in the same storage format -- a (k, n)
 * matrix of bs_c x bs_r blocks -- from which bsr_create() makes a handle; then
 * bsr_spmm(handle of W^T, m, G, Z, ...) is the sibling product.
 *
 * bsr_transpose_pattern (HOST pointers): validates the pattern as bsr_validate and writes
 *   t_index_pointer_host  k/bs_c + 1 entries      t_block_indices_host  nnzb entries (block-rows of W)
 *   perm_host             nnzb entries: stored block q of W^T is the transpose of block perm[q] of W
 * The blocks of a block-row of W^T come by ascending block-row of W.
 *
 * bsr_transpose_values (DEVICE pointers, asynchronous on hip_stream):
 *   t_block_data[q][c][a] = block_data[perm[q]][a][c],  q in [0, nnzb)
 * t_block_data_dev has nnzb*bs_c*bs_r elements of `dtype`, caller-owned; call it again whenever
 * the values of W change.  Errors: NULL, SHAPE, DTYPE, INDPTR, INDEX, UNSUPPORTED (a block larger
 * than 64 KiB), HIP.
 */
bsr_status bsr_transpose_pattern(int64_t n, int64_t k, int32_t bs_r, int32_t bs_c, int64_t nnzb,
                                 const int32_t* index_pointer_host, const int32_t* block_indices_host,
                                 int32_t* t_index_pointer_host, int32_t* t_block_indices_host, int32_t* perm_host);
bsr_status bsr_transpose_values(bsr_dtype dtype, int32_t bs_r, int32_t bs_c, int64_t nnzb, const int32_t* perm_dev,
                                const void* block_data_dev, void* t_block_data_dev, void* hip_stream);

/*
 * The sampled sibling: the gradient of the stored blocks.  With Y = X * W^T a layer's forward pass
 * and G = dL/dY, Y is linear in block_data[p][a][c] with coefficient X[i][col*bs_c + c] in
 * Y[i][r*bs_r + a], so
 *     D[p][a][c] = sum over i of  G[i][r*bs_r + a] * X[i][block_indices[p]*bs_c + c]
 * for every stored block p of block-row r: the entries of G^T X at the positions W stores.
 *   G_dev   DEVICE, m*n elements of W's dtype, row-major     X_dev  DEVICE, m*k elements, row-major
 *   D_dev   DEVICE, nnzb*bs_r*bs_c elements of d_dtype (W's dtype or BSR_F32), the layout of
 *           block_data; every element is written; fp32 accumulation, rounded to nearest-even
 * Block shapes with bs_r, bs_c in {16, 32, 64} run on the matrix cores; blocks of 1, 2, 4, 8 or 16
 * rows and any width on a kernel that gives a lane one column of one block; any other shape on a plain
 * loop.  Thin blocks (16 x 1, fp32) with scratch lent for this m (bsr_scratch_size, bsr_set_scratch): X is
 * transposed into the scratch and a matrix-core kernel runs; the scratch is overwritten.
 * Asynchronous on hip_stream; reads W's pattern only, not its values.
 * Errors: NULL, SHAPE (m < 0 or m*max(k,n) >= 2^31), DTYPE, ALIGN, HIP.
 */
bsr_status bsr_sddmm(const bsr_matrix* W, int64_t m, const void* G_dev, const void* X_dev, void* D_dev,
                     bsr_dtype d_dtype, void* hip_stream);

/*
 * bsr_spmm() for callers that can neither allocate nor lend device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  (No passage of the paper defines this call; it is
 * the product of bsr_spmm_ex(..., BSR_PATH_MFMA, ...) for the one kernel family that needs per-call scratch.)
 * For thin blocks (bs_r = 16, bs_c = 1, fp32, y_dtype BSR_F32) the matrix-core path keeps a transposed copy
 * of X in scratch; here that scratch is an array of BSR_STATIC_SCRATCH_BYTES bytes inside the library's code
 * object instead of memory lent with bsr_set_scratch().  Every GPU the library is loaded on holds its own
 * copy of the array until the process ends; its address is looked up once per device (at bsr_create(), else
 * at the first call).  The call itself allocates and frees nothing, on the device or through any library.
 *   Arguments as bsr_spmm().  m >= 1 rows need bsr_scratch_size(W, m) bytes: beyond the built-in size the
 *   call returns BSR_ERR_SCRATCH_LIMIT and does no device work (256 x 4096: 4 MiB + 256 bytes).
 *   Any other block shape or output type: BSR_ERR_UNSUPPORTED (no other kernel needs per-call scratch; use
 *   bsr_spmm()).
 * All calls on one GPU share that GPU's array, whatever the handle or stream: calls that overlap in time on
 * one GPU race; keep them ordered on one stream.  The array keeps the last call's contents; nothing in it
 * has to start at zero (each call first overwrites every entry it later reads for rows below m).
 * Errors: as bsr_spmm(), plus SCRATCH_LIMIT and UNSUPPORTED.
 */
#define BSR_STATIC_SCRATCH_BYTES (8u << 20)
bsr_status bsr_spmm_static(const bsr_matrix* W, int64_t m, const void* X_dev, void* Y_dev,
                           bsr_dtype y_dtype, void* hip_stream);

/*
 * Measurement helper for the benchmark, not part of the product (no passage of the paper defines it): one
 * launch of a kernel that only issues independent matrix-core instructions of the given input type
 * (8 accumulator chains per wavefront, 32 wavefronts per CU, `iters` rounds, no memory traffic), so that
 * roofline fractions can be quoted against the rate this chip delivers as well as the published peak.
 *   sink_dev   DEVICE, 4 bytes, never written in practice     flops_out  HOST: the flops the launch performs
 * Asynchronous on hip_stream; time it with events.  Errors: NULL, SHAPE (iters outside [1, 2^20]), DTYPE, HIP.
 */
bsr_status bsr_probe_mfma(bsr_dtype dtype, int32_t iters, void* sink_dev, void* hip_stream, double* flops_out);

/* Static, human-readable text for a status code.  (Like bsr_workspace_size(), bsr_destroy(), bsr_query_path(),
 * bsr_scratch_size() and bsr_set_scratch(), a housekeeping call that no passage of the paper defines.) */
const char* bsr_status_string(bsr_status s);

#ifdef __cplusplus
}
#endif
#endif /* BSR_SPMM_H */
