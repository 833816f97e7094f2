/*
 * oracle.c -- plain CPU reference for structured activation pruning.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition of what the GPU library computes.  It shares no code, header,
 * table or helper with the HIP path and is never called by it: only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg load it.
 *
 * What it follows (paper sections):
 *   - Sec. IV "Activation Pruning": every fixed-size block of an activation
 *     matrix is ranked by its l2 norm and the k = N*s lowest-ranked blocks are
 *     forced to zero (N blocks, sparsity s).  We rank by the sum of squares
 *     (same order as the norm, no sqrt that could merge distinct keys) and keep
 *     n_keep = ceil(keep * N) blocks with keep = 1 - s; equal scores are
 *     resolved towards the lowest linear block index.
 *   - Sec. II-A "Sparse data structures": Block Sparse Row layout.  crow (here
 *     row_ptr) holds the running count of kept blocks per block-row, its last
 *     entry being the total; col (here col_idx) holds the block-column of each
 *     kept block, row after row; values holds the blocks themselves.
 *   - Sec. III "Block Sparse Operators", Fig. 2: the weight gradient of a
 *     linear layer is computed from the pruned, saved input activation:
 *     dW = Xhat^T * dY with Xhat the masked activation.
 *
 * Conventions: X is [M x K] row-major with leading dimension ldx (elements);
 * blocks are br x bc; nbr = ceil(M/br), nbc = ceil(K/bc); block (i,j) has the
 * linear index i*nbc + j.  Edge blocks of a ragged matrix cover only the valid
 * elements; their padding is +0.0 inside `values`.  Element types: 0 = IEEE
 * binary32, 1 = bfloat16 (upper half of a binary32, passed as uint16_t).  All
 * floating-point arithmetic is binary64; every input converts to binary64
 * exactly, and so does every product of two inputs.
 *
 * Pins (tests marked "not gpu"): scores against exact summation and closed
 * forms; selection against brute-force subset enumeration, the keep-count rule
 * and the tie rule; BSR against the format's invariants and PyTorch's own BSR
 * conversion; round trip against mask*X bytewise; dW against a float64 matrix
 * product of the masked matrix, linearity over blocks and keep = 1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

static size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4u : 2u; }

/* Exact conversion of one stored element to binary64. */
static double load_elem(const void *base, int dtype, int64_t idx) {
  if (dtype == ORACLE_F32) return (double)((const float *)base)[idx];
  uint32_t w = (uint32_t)((const uint16_t *)base)[idx] << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* Sec. IV: k = N*s blocks are pruned; the kept count is its complement,
 * fixed here as ceil(keep*N) evaluated as one binary64 product.  Returns -1
 * for keep outside [0,1] (NaN included). */
int64_t oracle_keep_count(int64_t nblocks, double keep) {
  if (!(keep >= 0.0 && keep <= 1.0) || nblocks < 0) return -1;
  double v = ceil(keep * (double)nblocks);
  int64_t n = (int64_t)v;
  if (n < 0) n = 0;
  if (n > nblocks) n = nblocks;
  return n;
}

/* Sec. IV: l2 magnitude of every block; stored as the sum of squares. */
void oracle_block_scores(const void *X, int dtype, int64_t M, int64_t K,
                         int64_t ldx, int br, int bc, double *scores) {
  int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < nbr; ++i) {
    for (int64_t j = 0; j < nbc; ++j) {
      double acc = 0.0;
      for (int64_t m = i * br; m < (i + 1) * br && m < M; ++m)
        for (int64_t k = j * bc; k < (j + 1) * bc && k < K; ++k) {
          double x = load_elem(X, dtype, m * ldx + k);
          acc += x * x;
        }
      scores[i * nbc + j] = acc;
    }
  }
}

/* Ranking key: the bit pattern of a non-negative binary64 orders like its
 * value; every NaN becomes one quiet-NaN pattern that ranks above +inf, so a
 * block holding a NaN is kept and stays visible downstream. */
static uint64_t rank_key(double s) {
  uint64_t u;
  if (s != s) return UINT64_C(0x7FF8000000000000);
  memcpy(&u, &s, sizeof u);
  return u;
}

/* 1 if block a ranks strictly before block b: higher score first, then the
 * lower linear index. */
static int ranks_before(const uint64_t *key, int64_t a, int64_t b) {
  if (key[a] != key[b]) return key[a] > key[b];
  return a < b;
}

static void merge_sort(int64_t *idx, int64_t *tmp, int64_t lo, int64_t hi,
                       const uint64_t *key) {
  if (hi - lo < 2) return;
  int64_t mid = lo + (hi - lo) / 2;
  merge_sort(idx, tmp, lo, mid, key);
  merge_sort(idx, tmp, mid, hi, key);
  int64_t a = lo, b = mid, o = lo;
  while (a < mid && b < hi)
    tmp[o++] = ranks_before(key, idx[b], idx[a]) ? idx[b++] : idx[a++];
  while (a < mid) tmp[o++] = idx[a++];
  while (b < hi) tmp[o++] = idx[b++];
  memcpy(idx + lo, tmp + lo, (size_t)(hi - lo) * sizeof *idx);
}

/* Sec. IV: rank all blocks, keep the n_keep best.  Full stable sort of the
 * block indices by (score descending, index ascending); the first n_keep
 * entries of the sorted list are the kept blocks.  Returns 0, or -1 when out
 * of memory. */
int oracle_select(const double *scores, int64_t nblocks, int64_t n_keep,
                  uint8_t *mask) {
  memset(mask, 0, (size_t)nblocks);
  if (nblocks == 0) return 0;
  uint64_t *key = malloc((size_t)nblocks * sizeof *key);
  int64_t *idx = malloc((size_t)nblocks * sizeof *idx);
  int64_t *tmp = malloc((size_t)nblocks * sizeof *tmp);
  if (!key || !idx || !tmp) {
    free(key); free(idx); free(tmp);
    return -1;
  }
  for (int64_t b = 0; b < nblocks; ++b) {
    key[b] = rank_key(scores[b]);
    idx[b] = b;
  }
  merge_sort(idx, tmp, 0, nblocks, key);
  for (int64_t r = 0; r < n_keep && r < nblocks; ++r) mask[idx[r]] = 1;
  free(key); free(idx); free(tmp);
  return 0;
}

/* Sec. IV, locality of the selection: the paper ranks the blocks of each
 * activation of the mini-batch on their own, not the whole batch at once.  Here
 * a ranking group is `group_rows` consecutive block-rows (the block-rows of one
 * sample, or of a few samples); every group keeps the
 * ceil(keep * blocks of the group) best of its own blocks, ties to the lowest
 * linear index as everywhere.  The last group may have fewer block-rows.
 * Returns the total number of kept blocks, -1 when out of memory, -2 for a bad
 * argument. */
int64_t oracle_select_grouped(const double *scores, int64_t nbr, int64_t nbc,
                              int64_t group_rows, double keep, uint8_t *mask) {
  if (group_rows <= 0 || nbr < 0 || nbc < 0) return -2;
  int64_t total = 0;
  for (int64_t i0 = 0; i0 < nbr; i0 += group_rows) {
    int64_t rows = nbr - i0 < group_rows ? nbr - i0 : group_rows;
    int64_t blocks = rows * nbc;
    int64_t n_keep = oracle_keep_count(blocks, keep);
    if (n_keep < 0) return -2;
    if (oracle_select(scores + i0 * nbc, blocks, n_keep, mask + i0 * nbc) != 0)
      return -1;
    total += n_keep;
  }
  return total;
}

/* Sec. III: the selected (lowest) blocks are forced to zero.  Xhat gets the
 * bits of X inside kept blocks and +0.0 elsewhere. */
void oracle_mask_dense(const void *X, int dtype, int64_t M, int64_t K,
                       int64_t ldx, int br, int bc, const uint8_t *mask,
                       void *Xhat, int64_t ldxhat) {
  int64_t nbc = ceil_div(K, bc);
  size_t e = elem_size(dtype);
  for (int64_t m = 0; m < M; ++m)
    for (int64_t k = 0; k < K; ++k) {
      char *dst = (char *)Xhat + (size_t)(m * ldxhat + k) * e;
      if (mask[(m / br) * nbc + k / bc])
        memcpy(dst, (const char *)X + (size_t)(m * ldx + k) * e, e);
      else
        memset(dst, 0, e);
    }
}

/* Sec. II-A: encode the kept blocks of X as BSR.  row_ptr has nbr+1 entries,
 * col_idx one entry per kept block, values br*bc elements per kept block
 * (row-major inside the block, padding of edge blocks = +0.0). */
void oracle_bsr_from_mask(const void *X, int dtype, int64_t M, int64_t K,
                          int64_t ldx, int br, int bc, const uint8_t *mask,
                          int32_t *row_ptr, int32_t *col_idx, void *values) {
  int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  size_t e = elem_size(dtype);
  int64_t p = 0;
  row_ptr[0] = 0;
  for (int64_t i = 0; i < nbr; ++i) {
    for (int64_t j = 0; j < nbc; ++j) {
      if (!mask[i * nbc + j]) continue;
      col_idx[p] = (int32_t)j;
      for (int r = 0; r < br; ++r)
        for (int c = 0; c < bc; ++c) {
          int64_t m = i * br + r, k = j * bc + c;
          char *dst = (char *)values + (size_t)((p * br + r) * bc + c) * e;
          if (m < M && k < K)
            memcpy(dst, (const char *)X + (size_t)(m * ldx + k) * e, e);
          else
            memset(dst, 0, e);
        }
      ++p;
    }
    row_ptr[i + 1] = (int32_t)p;
  }
}

/* Sec. II-A read the other way: rebuild the dense [M x K] matrix. */
void oracle_bsr_to_dense(const int32_t *row_ptr, const int32_t *col_idx,
                         const void *values, int dtype, int64_t M, int64_t K,
                         int64_t ldout, int br, int bc, void *Xout) {
  int64_t nbr = ceil_div(M, br);
  size_t e = elem_size(dtype);
  for (int64_t m = 0; m < M; ++m)
    memset((char *)Xout + (size_t)(m * ldout) * e, 0, (size_t)K * e);
  for (int64_t i = 0; i < nbr; ++i)
    for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
      int64_t j = col_idx[p];
      for (int r = 0; r < br; ++r)
        for (int c = 0; c < bc; ++c) {
          int64_t m = i * br + r, k = j * bc + c;
          if (m < M && k < K)
            memcpy((char *)Xout + (size_t)(m * ldout + k) * e,
                   (const char *)values + (size_t)((p * br + r) * bc + c) * e,
                   e);
        }
    }
}

/* Sec. III / Fig. 2: one entry of the weight gradient,
 * dW[k,n] = sum_m Xhat[m,k] * dY[m,n], accumulated in binary64 with m
 * ascending. */
double oracle_dw_entry(const void *Xhat, const void *dY, int dtype, int64_t M,
                       int64_t ldx, int64_t lddy, int64_t k, int64_t n) {
  double acc = 0.0;
  for (int64_t m = 0; m < M; ++m)
    acc += load_elem(Xhat, dtype, m * ldx + k) * load_elem(dY, dtype, m * lddy + n);
  return acc;
}

/* Whole weight gradient dW [K x N] (leading dimension N), the naive triple
 * loop over the masked dense activation. */
void oracle_dw(const void *Xhat, const void *dY, int dtype, int64_t M,
               int64_t K, int64_t ldx, int64_t N, int64_t lddy, double *dW) {
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < K; ++k)
    for (int64_t n = 0; n < N; ++n)
      dW[k * N + n] = oracle_dw_entry(Xhat, dY, dtype, M, ldx, lddy, k, n);
}

/* Sec. VI (outlook): the block-sparse version of ResMLP's affine scaling layer,
 * y[m,k] = alpha[k] * x[m,k] + beta[k].  Of its backward pass only the scale
 * gradient depends on the saved (pruned) input:
 *   dalpha[k] = sum_m Xhat[m,k] * dY[m,k],
 * accumulated in binary64 with m ascending (dbeta = sum_m dY[m,k] and
 * dx = alpha * dy never see X). */
void oracle_affine_dscale(const void *Xhat, const void *dY, int dtype, int64_t M,
                          int64_t K, int64_t ldx, int64_t lddy, double *dalpha) {
  for (int64_t k = 0; k < K; ++k) {
    double acc = 0.0;
    for (int64_t m = 0; m < M; ++m)
      acc += load_elem(Xhat, dtype, m * ldx + k) * load_elem(dY, dtype, m * lddy + k);
    dalpha[k] = acc;
  }
}

/* Sec. II-A, Table II: bytes of one BSR-encoded matrix with 4-byte indices:
 * the kept blocks, one column index per kept block, nbr+1 row pointers. */
int64_t oracle_bsr_bytes(int64_t n_keep, int64_t nbr, int br, int bc,
                         int elem_bytes) {
  return n_keep * (int64_t)br * bc * elem_bytes + 4 * n_keep + 4 * (nbr + 1);
}
