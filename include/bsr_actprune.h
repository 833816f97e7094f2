/*
 * bsr_actprune.h -- C ABI of the structured-activation-pruning hot path for
 * AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the two halves of the
 * paper's block-sparse linear operator (Sec. III, Fig. 2):
 *   forward side : rank the fixed-size blocks of a saved activation matrix by
 *                  l2 magnitude, keep the best ones (Sec. IV) and store them in
 *                  Block Sparse Row format (Sec. II-A);
 *   backward side: the weight gradient dW = Xhat^T * dY computed directly from
 *                  that BSR tensor (Sec. III, "BSpMM").
 *
 * Conventions shared by every call
 *   - X is an [M x K] row-major matrix with leading dimension ldx (elements);
 *     blocks are br x bc; nbr = ceil(M/br), nbc = ceil(K/bc), nblocks =
 *     nbr*nbc; block (i,j) has the linear index i*nbc + j.  Blocks on a ragged
 *     edge cover only the valid elements; inside `values` their padding is +0.0.
 *   - dtype: BSR_F32 (IEEE binary32) or BSR_BF16 (bfloat16).  Indices are
 *     32-bit (Table II prices one index like one value); nblocks < 2^31.
 *   - Every pointer named below is a DEVICE pointer unless it says "host".  All
 *     buffers, the workspace included, are owned by the caller; the library
 *     never allocates or frees device memory and never synchronises.  Work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and the call
 *     returns at once.  Buffers must stay alive until that work has finished.
 *   - Pointers must be aligned to their element type; wider alignment (16 B,
 *     what any framework allocator gives) selects the vectorised kernels.
 *   - Return value: BSR_OK, or a negative BSR_ERR_* found on the host before
 *     anything was launched (nothing has been written then), or BSR_ERR_HIP if
 *     a launch failed (bsr_last_hip_error() holds the hipError_t).
 *   - Calls on different streams may run concurrently if their workspaces and
 *     outputs do not overlap.  The library keeps no state of its own besides a
 *     per-thread last-error value.
 */
#ifndef BSR_ACTPRUNE_H
#define BSR_ACTPRUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { BSR_F32 = 0, BSR_BF16 = 1 };

enum {
  BSR_OK = 0,
  BSR_ERR_NULL = -1,      /* a required pointer is NULL */
  BSR_ERR_SHAPE = -2,     /* negative / inconsistent / too large sizes */
  BSR_ERR_DTYPE = -3,     /* dtype is neither BSR_F32 nor BSR_BF16 */
  BSR_ERR_KEEP = -4,      /* keep outside [0,1] or NaN, or n_keep != bsr_keep_count range */
  BSR_ERR_WORKSPACE = -5, /* ws is NULL or smaller than bsr_workspace_bytes() */
  BSR_ERR_ALIGN = -6,     /* a pointer is not aligned to its element type */
  BSR_ERR_HIP = -7,       /* a HIP call failed; see bsr_last_hip_error() */
  BSR_ERR_LIMIT = -8      /* problem larger than the fixed capacity of an entry point that allocates nothing */
};

enum {
  BSR_OP_SCORE_SELECT = 0,
  BSR_OP_COMPRESS = 1,
  BSR_OP_DECOMPRESS = 2,
  BSR_OP_T_DENSE_MATMUL = 3,
  BSR_OP_AFFINE_SCALE_GRAD = 4
};

/* Host, pure.  Library version string. */
const char *bsr_version(void);

/* Host, pure.  Name of a BSR_ERR_* code. */
const char *bsr_error_string(int code);

/* Host.  hipError_t of the last failed HIP call on this thread (0 if none). */
int bsr_last_hip_error(void);

/*
 * Host, pure.  Number of blocks that survive pruning (Sec. IV: k = N*s blocks
 * are zeroed, s = 1 - keep): ceil(keep * nblocks) evaluated as one binary64
 * product, clamped to [0, nblocks].  Returns -1 if keep is outside [0,1] or NaN
 * or nblocks < 0.  Output buffers are sized from this value, so nothing is ever
 * read back from the device.
 */
int64_t bsr_keep_count(int64_t nblocks, double keep);

/*
 * Host, pure.  Bytes of one BSR-encoded matrix (Sec. II-A, Table II): n_keep
 * blocks of br*bc elements, one 4-byte column index per kept block, nbr+1
 * 4-byte row pointers.  Returns -1 on invalid arguments.
 */
int64_t bsr_storage_bytes(int64_t M, int64_t K, int br, int bc, int64_t n_keep,
                          int dtype);

/*
 * Host, pure.  Size in bytes of the device workspace `ws` that operation `op`
 * (BSR_OP_*) needs for the given problem; N is only used by
 * BSR_OP_T_DENSE_MATMUL.  The workspace needs no initialisation and holds
 * nothing of value between calls.  Returns 0 for invalid arguments (the
 * operation itself reports the error) and for operations that need none.
 */
size_t bsr_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, int br,
                           int bc, int dtype);

/*
 * Sec. IV, "Activation Pruning": score every block of X by its l2 magnitude
 * and select the blocks to keep.
 *   score[i*nbc+j] = sum of x^2 over the valid elements of block (i,j),
 *                    accumulated in binary64 (ranks like the l2 norm);
 *   keep_mask[b]   = 1 for the n_keep = bsr_keep_count(nblocks, keep) blocks of
 *                    highest score, 0 otherwise; equal scores are resolved
 *                    towards the lower linear block index; a NaN score ranks
 *                    above +inf.
 * X: [M x K] of dtype, leading dimension ldx >= K.  scores: [nblocks] binary64
 * or NULL (then they live only in the workspace).  keep_mask: [nblocks] bytes.
 * The whole matrix is one ranking group.  M == 0 or K == 0 is valid (nothing
 * is written).
 */
int bsr_score_select(const void *X, int dtype, int64_t M, int64_t K,
                     int64_t ldx, int br, int bc, double keep, double *scores,
                     uint8_t *keep_mask, void *ws, size_t ws_bytes,
                     void *stream);

/*
 * Host, pure.  Total number of kept blocks when the blocks are ranked in
 * groups of `group_rows` consecutive block-rows (Sec. IV: blocks are compared
 * only inside one activation of the mini-batch, so every activation keeps the
 * same number of blocks): the sum over the groups of
 * bsr_keep_count(blocks of the group, keep); the last group may have fewer
 * block-rows.  nbr, nbc = block-rows / block-columns of the matrix.  Returns -1
 * on invalid arguments (group_rows < 1, negative sizes, keep outside [0,1]).
 */
int64_t bsr_grouped_keep_count(int64_t nbr, int64_t nbc, int64_t group_rows,
                               double keep);

/*
 * Sec. IV, local ranking: like bsr_score_select, but the matrix is cut into
 * ranking groups of `group_rows` consecutive block-rows (for instance the
 * block-rows of one sample, or of a few samples when a sample's rows are not a
 * multiple of br) and every group keeps the bsr_keep_count(its blocks, keep)
 * best of its own blocks; ties go to the lower linear block index.  The mask
 * then holds bsr_grouped_keep_count(nbr, nbc, group_rows, keep) ones and feeds
 * bsr_compress unchanged.  group_rows >= nbr is the ungrouped selection.
 * Workspace: bsr_workspace_bytes(BSR_OP_SCORE_SELECT, ...).  Same argument
 * rules and error codes as bsr_score_select; group_rows < 1 -> BSR_ERR_SHAPE.
 */
int bsr_score_select_grouped(const void *X, int dtype, int64_t M, int64_t K,
                             int64_t ldx, int br, int bc, int64_t group_rows,
                             double keep, double *scores, uint8_t *keep_mask,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * For callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, outputs (bit for bit) and error codes as
 * bsr_score_select, without `ws`: the workspace is a fixed array of about
 * 10.3 MiB inside the library's code object, of which every GPU that the
 * library runs on holds its own copy until the process ends.  Limit: matrices
 * of at most bsr_score_select_static_max_blocks() = 524288 blocks; larger ones
 * return BSR_ERR_LIMIT before anything is launched.  No hipMalloc / hipFree, no
 * allocating library call.  All calls on one GPU share that GPU's array, which
 * keeps the contents of the last call (the kernels initialise what they read):
 * calls that overlap in time on one GPU -- different streams, or graphs replayed
 * concurrently -- race and give undefined masks; order them on one stream.
 * bsr_static_scratch_init() resolves the array's device address for the current
 * device ahead of time (the first call on a device does it otherwise); returns
 * BSR_OK or BSR_ERR_HIP.
 */
int64_t bsr_score_select_static_max_blocks(void);
int bsr_static_scratch_init(void);
int bsr_score_select_static(const void *X, int dtype, int64_t M, int64_t K,
                            int64_t ldx, int br, int bc, double keep,
                            double *scores, uint8_t *keep_mask, void *stream);

/*
 * Sec. III / Sec. II-A: conversion of the saved activation into BSR form.
 * From X and a keep mask with exactly n_keep ones build
 *   row_ptr [nbr+1] : running count of kept blocks per block-row (crow);
 *   col_idx [n_keep]: block-column of every kept block, block-row after
 *                     block-row, ascending inside a block-row (col);
 *   values  [n_keep*br*bc] of dtype: the kept blocks, bit copies of X,
 *                     row-major inside a block, +0.0 in edge padding.
 * If the mask holds a different number of ones than n_keep the result is
 * unspecified, but nothing is written outside the given buffers.
 * Workspace: bsr_workspace_bytes(BSR_OP_COMPRESS, ...), which is zero for most
 * shapes (then ws may be NULL); matrices of very many few-row blocks keep one
 * counter per workgroup there.
 */
int bsr_compress(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx,
                 int br, int bc, const uint8_t *keep_mask, int64_t n_keep,
                 int32_t *row_ptr, int32_t *col_idx, void *values, void *ws,
                 size_t ws_bytes, void *stream);

/*
 * Sec. II-A read backwards: X_out [M x K] (leading dimension ldx) receives the
 * kept blocks bit for bit and +0.0 everywhere else, i.e. mask (.) X.
 * row_ptr must be a valid BSR row pointer array for col_idx / values.
 */
int bsr_decompress(const int32_t *row_ptr, const int32_t *col_idx,
                   const void *values, int dtype, int64_t M, int64_t K,
                   int64_t ldx, int br, int bc, void *X_out, void *stream);

/*
 * Sec. III, Fig. 2 (the block-sparse product of the backward pass): weight
 * gradient of a linear layer from the pruned activation,
 *   dW[j*bc + c, n] (+)= sum over kept blocks (i,j), rows r of the block:
 *                          values[block][r][c] * dY[i*br + r, n].
 * dY: [M x N] of the same dtype as values, leading dimension lddy.  dW: [K x N]
 * binary32, leading dimension lddw; overwritten when accumulate == 0, added to
 * otherwise.  Accumulation is in binary32 on the matrix cores; bfloat16 products
 * are exact in binary32, binary32 products are rounded like any binary32
 * multiply-add.  This is X^T*dY; torch's nn.Linear.weight.grad is its transpose.
 * The contraction is split over block-rows; partial sums are reduced in a fixed
 * order, so results are reproducible run to run.
 * Block shapes 32x32, 64x64, 16x16 and 14x14 are multiplied as stored.  Any other
 * shape -- 1 x b row segments, b = K, rectangular blocks -- is first re-tiled into
 * 32x32 blocks inside the workspace; the workspace size reported for such a shape
 * includes that copy (about M*K elements).
 * col_idx may be in any order inside a block-row.
 * Non-finite dY: a 32x32 or 64x64 block that was pruned is never multiplied, so an
 * inf or NaN of dY reaches only the rows of dW that belong to kept blocks of its
 * block-row.  For every other block shape the kept blocks are multiplied inside
 * zero-filled 32-wide tiles, and a zero of the tile times inf is NaN: there the
 * rows of dW that belong to pruned blocks of that block-row may become NaN as
 * well (as they all do in a dense product with the masked matrix).  Columns of dW
 * other than the one of the non-finite value are never affected.
 */
int bsr_t_dense_matmul(const int32_t *row_ptr, const int32_t *col_idx,
                       const void *values, int dtype, int64_t M, int64_t K,
                       int br, int bc, const void *dY, int64_t N, int64_t lddy,
                       float *dW, int64_t lddw, int accumulate, void *ws,
                       size_t ws_bytes, void *stream);

/*
 * Several tensors per call (for instance the three pruned inputs of a residual
 * block, or those of all blocks): exactly the masks (and scores) that
 * bsr_score_select gives tensor by tensor, with a handful of kernel launches for
 * the whole batch instead of two to three per tensor -- selection is bound by
 * launch latency, not by work.  Every item is ranked on its own (Sec. IV: blocks
 * are compared inside one activation only).  `items` is a host array that is
 * read before the call returns; all tensors share `dtype`.  Workspace:
 * bsr_score_select_batched_workspace_bytes(items, n, dtype) (0 for invalid items).
 * Errors as for bsr_score_select, reported for the first offending item; nothing
 * is launched if any item is invalid.
 */
typedef struct bsr_select_item {
  const void *X;      /* device, [M x K], leading dimension ldx */
  int64_t M, K, ldx;
  int32_t br, bc;
  double keep;
  double *scores;     /* device, [nblocks], or NULL */
  uint8_t *keep_mask; /* device, [nblocks] */
} bsr_select_item;

size_t bsr_score_select_batched_workspace_bytes(const bsr_select_item *items,
                                                int n, int dtype);

int bsr_score_select_batched(const bsr_select_item *items, int n, int dtype,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * Sec. IV, local ranking, for several tensors per call: item i is ranked like
 * bsr_score_select_grouped with groups of group_rows[i] block-rows (same masks,
 * same keep counts per group), and tensors whose groups are of a similar size
 * share kernel launches.  Workspace and errors as for bsr_score_select_batched
 * (the same item type and the same workspace size); group_rows[i] < 1 is
 * BSR_ERR_SHAPE.  `items` and `group_rows` are host arrays, read before the call
 * returns.
 */
int bsr_score_select_grouped_batched(const bsr_select_item *items,
                                     const int64_t *group_rows, int n, int dtype,
                                     void *ws, size_t ws_bytes, void *stream);

/*
 * Several weight gradients per call (for instance those of all linear layers whose
 * pruned inputs are at hand): every item is one bsr_t_dense_matmul, but items of
 * the same block shape share kernel launches, so that the table build and the
 * write-out of one product overlap the main loop of another, and a product that
 * shares its launch splits its contraction into fewer parts (the other products
 * keep the GPU busy).  The sums are therefore added in another order than in the
 * single call: equal to rounding (same error bound), reproducible run to run, and
 * identical to the single call for a batch of one.
 * `items` is a host array, read before the call returns; all items share `dtype`;
 * outputs of different items must not overlap.  Workspace:
 * bsr_t_dense_matmul_batched_workspace_bytes(items, n, dtype) (0 for invalid
 * items).  Errors as for bsr_t_dense_matmul, for the first offending item; nothing
 * is launched if any item is invalid.
 */
typedef struct bsr_matmul_item {
  const int32_t *row_ptr;  /* device */
  const int32_t *col_idx;  /* device */
  const void *values;      /* device */
  int64_t M, K;
  int32_t br, bc;
  const void *dY;          /* device, [M x N], leading dimension lddy */
  int64_t N, lddy;
  float *dW;               /* device, [K x N], leading dimension lddw */
  int64_t lddw;
  int32_t accumulate;
} bsr_matmul_item;

size_t bsr_t_dense_matmul_batched_workspace_bytes(const bsr_matmul_item *items,
                                                  int n, int dtype);

int bsr_t_dense_matmul_batched(const bsr_matmul_item *items, int n, int dtype,
                               void *ws, size_t ws_bytes, void *stream);

/*
 * Several conversions per call: every item is one bsr_compress (Sec. III:
 * conversion of the activation to BSR) or one bsr_decompress (Sec. II-A read
 * backwards), with the same outputs bit for bit; tensors that take the same
 * kernel share launches, so a step over many small tensors costs a few launches
 * instead of one per tensor.  `items` is a host array, read before the call
 * returns; all items share `dtype`; outputs of different items must not overlap.
 * Workspace of bsr_compress_batched: bsr_compress_batched_workspace_bytes(items,
 * n, dtype), the sum of what bsr_compress needs per item (0 for the shapes that
 * need none, and for invalid items).  Errors as for the single calls, for the
 * first offending item; nothing is launched if any item is invalid.
 */
typedef struct bsr_compress_item {
  const void *X;            /* device, [M x K], leading dimension ldx */
  int64_t M, K, ldx;
  int32_t br, bc;
  const uint8_t *keep_mask; /* device, [nblocks] */
  int64_t n_keep;
  int32_t *row_ptr;         /* device, [nbr + 1] */
  int32_t *col_idx;         /* device, [n_keep] */
  void *values;             /* device, [n_keep x br x bc] */
} bsr_compress_item;

size_t bsr_compress_batched_workspace_bytes(const bsr_compress_item *items,
                                            int n, int dtype);

int bsr_compress_batched(const bsr_compress_item *items, int n, int dtype,
                         void *ws, size_t ws_bytes, void *stream);

typedef struct bsr_decompress_item {
  const int32_t *row_ptr;   /* device */
  const int32_t *col_idx;   /* device */
  const void *values;       /* device */
  int64_t M, K, ldx;
  int32_t br, bc;
  void *X_out;              /* device, [M x K], leading dimension ldx */
} bsr_decompress_item;

int bsr_decompress_batched(const bsr_decompress_item *items, int n, int dtype,
                           void *stream);

/*
 * Sec. VI (outlook) names a block-sparse version of ResMLP's affine scaling
 * layer, y[m,k] = alpha[k] * x[m,k] + beta[k].  Of its backward pass only the
 * scale gradient needs the saved input; from the pruned input in BSR form:
 *   dalpha[j*bc + c] (+)= sum over kept blocks (i,j), rows r of the block:
 *                          values[block][r][c] * dY[i*br + r, j*bc + c].
 * dY: [M x K] of the same dtype as values, leading dimension lddy (the layer's
 * output gradient has the shape of its input).  dalpha: [K] binary32,
 * overwritten when accumulate == 0, added to otherwise.  Products and sums in
 * binary32, in a fixed order (reproducible run to run).  Pruned blocks are not
 * read.  Workspace: bsr_workspace_bytes(BSR_OP_AFFINE_SCALE_GRAD, M, K, 0, ...).
 * Errors as for bsr_t_dense_matmul.
 */
int bsr_affine_scale_grad(const int32_t *row_ptr, const int32_t *col_idx,
                          const void *values, int dtype, int64_t M, int64_t K,
                          int br, int bc, const void *dY, int64_t lddy,
                          float *dalpha, int accumulate, void *ws,
                          size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BSR_ACTPRUNE_H */
