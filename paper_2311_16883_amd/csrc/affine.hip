// Scale gradient of the block-sparse affine layer (paper Sec. VI names a block-sparse
// version of ResMLP's affine scaling layer y = alpha * x + beta; of its backward pass
// only dalpha[k] = sum_m X[m,k] * dY[m,k] needs the saved input):
//   dalpha[j*bc + c] = sum over kept blocks (i,j), rows r: values[block][r][c] * dY[i*br + r, j*bc + c].
// HBM-bound: the kept values and the matching half of dY are read once.
//
// A workgroup owns a range of block-rows (one split of the sum) and 256 consecutive
// column vectors.  As in the BSR -> dense kernel an LDS table maps block-column ->
// stored block (built for eight block-rows at a time, whose entries are one index
// range), lanes run along the matrix row, the four waves take every fourth row with
// four rows' loads in flight; a lane keeps binary32 sums for its (up to kAffVecs) vectors of columns and
// adds rows top to bottom.  Waves, then splits, are added in a fixed order, so the
// result is reproducible bit for bit.  Pruned blocks are never touched.
#include "common.h"

namespace bsr {

namespace {

constexpr int kAffVecs = 1;                      // column vectors per lane
constexpr int kAffSplits = 512;                  // splits of the sum over block-rows, at most
constexpr int kAffRows = 8;                      // block-rows whose tables are built together
constexpr int kAffCols = 64 * kAffVecs;          // block-columns a workgroup's vectors can fall into, at most

template <typename T, int V>
__global__ __launch_bounds__(256) void affine_dscale_kernel(
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, const T *__restrict__ values,
    const T *__restrict__ dY, int64_t M, int64_t K, int64_t lddy, int br, int bc, int64_t nbr, int64_t nbc,
    int64_t rows_per_split, float *__restrict__ partial) {
  __shared__ int32_t slot[kAffRows * kAffCols];
  __shared__ int32_t rp[kAffRows + 1];
  __shared__ float red[4][64 * kAffVecs][V];
  const int t = threadIdx.x, lane = t & 63, rg = t >> 6;
  // this workgroup's columns: 64 * kAffVecs consecutive vectors of the matrix row, whatever
  // block-columns they fall into (at most that many, since a block row has at least one vector)
  const int vpb = bc / V;                                  // vectors per block row
  const int64_t w0 = (int64_t)blockIdx.x * (64 * kAffVecs);
  const int64_t vr = K / V;                                // vectors per matrix row
  const int64_t j0 = w0 / vpb;
  int64_t j1 = (w0 + 64 * kAffVecs - 1) / vpb;
  if (j1 > nbc - 1) j1 = nbc - 1;
  const int ncols = (int)(j1 - j0 + 1);
  int cu[kAffVecs], vu[kAffVecs];
  float acc[kAffVecs][V];
#pragma unroll
  for (int u = 0; u < kAffVecs; ++u) {
    const int64_t w = w0 + lane + 64 * u;
    const int64_t j = w / vpb;
    cu[u] = w < vr ? (int)(j - j0) : -1;
    vu[u] = (int)(w - j * vpb);
#pragma unroll
    for (int q = 0; q < V; ++q) acc[u][q] = 0.0f;
  }
  const int64_t i_lo = (int64_t)blockIdx.y * rows_per_split;
  const int64_t i_hi = (i_lo + rows_per_split) < nbr ? (i_lo + rows_per_split) : nbr;
  const int64_t block_elems = (int64_t)br * bc;
  constexpr int kInFlight = 4;
  for (int64_t ib = i_lo; ib < i_hi; ib += kAffRows) {
    // block-column -> stored block for kAffRows block-rows at once: their entries are one index range
    const int nb = (int)((i_hi - ib) < kAffRows ? (i_hi - ib) : kAffRows);
    if (t <= nb) rp[t] = row_ptr[ib + t];
    for (int c = t; c < nb * ncols; c += 256) slot[c] = -1;
    __syncthreads();
    const int64_t P0 = rp[0], P1 = rp[nb];
    for (int64_t p = P0 + t; p < P1; p += 256) {
      int b = 0;
      while (b + 1 < nb && p >= rp[b + 1]) ++b;
      const int64_t j = col_idx[p];
      if (j >= j0 && j < j0 + ncols) slot[b * ncols + (int)(j - j0)] = (int32_t)p;
    }
    __syncthreads();
    for (int b = 0; b < nb; ++b) {
      const int64_t i = ib + b;
      const int rows = (int)((M - i * br) < br ? (M - i * br) : br);
      const T *yrow = dY + i * br * lddy + w0 * V;
#pragma unroll
      for (int u = 0; u < kAffVecs; ++u) {
        if (cu[u] < 0) continue;
        const int32_t p = slot[b * ncols + cu[u]];
        if (p < 0) continue;
        const T *xs = values + (int64_t)p * block_elems + (int64_t)vu[u] * V;
        const T *ys = yrow + (int64_t)(lane + 64 * u) * V;
        for (int r0 = rg; r0 < rows; r0 += 4 * kInFlight) {
          Vec<T, V> xv[kInFlight], yv[kInFlight];
#pragma unroll
          for (int k = 0; k < kInFlight; ++k) {
            const int r = r0 + 4 * k;
            if (r < rows) {
              xv[k] = *reinterpret_cast<const Vec<T, V> *>(xs + (int64_t)r * bc);
              yv[k] = *reinterpret_cast<const Vec<T, V> *>(ys + (int64_t)r * lddy);
            }
          }
#pragma unroll
          for (int k = 0; k < kInFlight; ++k) {
            if (r0 + 4 * k < rows) {
#pragma unroll
              for (int q = 0; q < V; ++q)
                acc[u][q] = fmaf(elem_to_float<T>(xv[k].e[q]), elem_to_float<T>(yv[k].e[q]), acc[u][q]);
            }
          }
        }
      }
    }
    __syncthreads();
  }
  // waves in a fixed order, then out: partial[split][column]
#pragma unroll
  for (int u = 0; u < kAffVecs; ++u)
#pragma unroll
    for (int q = 0; q < V; ++q) red[rg][lane + 64 * u][q] = acc[u][q];
  __syncthreads();
  for (int w = t; w < 64 * kAffVecs; w += 256) {
    const int64_t col = (w0 + w) * V;
    if (w0 + w >= vr) continue;
#pragma unroll
    for (int q = 0; q < V; ++q)
      partial[(int64_t)blockIdx.y * K + col + q] = ((red[0][w][q] + red[1][w][q]) + red[2][w][q]) + red[3][w][q];
  }
}

// dalpha[k] = (accumulate ? dalpha[k] : 0) + sum over splits of partial[split][k]: one wave per
// column, lane l adds splits l, l + 64, ... in ascending order, then the lanes are added
// in a fixed butterfly order (reproducible).  The output is tiny (K values) and the
// number of splits large, so the parallelism has to come from the splits.
__global__ __launch_bounds__(256) void affine_reduce_kernel(const float *__restrict__ partial, int splits,
                                                            int64_t K, float *__restrict__ dalpha,
                                                            int accumulate) {
  const int lane = threadIdx.x & 63;
  const int64_t k = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (k >= K) return;
  float sum = 0.0f;
#pragma unroll 8
  for (int sp = lane; sp < splits; sp += 64) sum += partial[(int64_t)sp * K + k];
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) sum += __shfl_xor(sum, d, 64);
  if (lane == 0) dalpha[k] = accumulate ? dalpha[k] + sum : sum;
}

struct AffinePlan {
  int v;                 // elements per vector
  int64_t gx, splits, rows_per_split;
};

// Shape-only part of the plan (the vector width also depends on pointers and strides).
void affine_split(int64_t nbr, int64_t gx, int64_t *splits, int64_t *rows_per_split) {
  int64_t s = 2048 / (gx > 0 ? gx : 1);
  if (s > kAffSplits) s = kAffSplits;
  if (s > nbr) s = nbr;
  if (s < 1) s = 1;
  *rows_per_split = ceil_div(nbr, s);
  *splits = ceil_div(nbr, *rows_per_split);
}

}  // namespace

size_t affine_ws_bytes(int64_t M, int64_t K, int br, int bc) {
  if (M <= 0 || K <= 0) return 0;
  // room for the largest number of splits the launcher ever picks
  const int64_t nbr = ceil_div(M, br);
  int64_t splits = nbr < kAffSplits ? nbr : kAffSplits;
  (void)bc;
  return align_up((size_t)splits * K * sizeof(float), 256);
}

int launch_affine_dscale(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype, int64_t M,
                         int64_t K, int br, int bc, const void *dY, int64_t lddy, float *dalpha, int accumulate,
                         void *ws, hipStream_t s) {
  const int e = elem_bytes(dtype);
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  AffinePlan p;
  p.v = pick_vector(16 / e, e, bc, K, lddy, dY, values);
  p.gx = ceil_div(K / p.v, 64 * kAffVecs);
  affine_split(nbr, p.gx, &p.splits, &p.rows_per_split);
  float *partial = static_cast<float *>(ws);
  const dim3 grid((unsigned)p.gx, (unsigned)p.splits);
#define BSR_AFFINE(T, V)                                                                                     \
  hipLaunchKernelGGL((affine_dscale_kernel<T, V>), grid, dim3(256), 0, s, row_ptr, col_idx,                  \
                     static_cast<const T *>(values), static_cast<const T *>(dY), M, K, lddy, br, bc, nbr,    \
                     nbc, p.rows_per_split, partial)
  if (dtype == BSR_F32) {
    switch (p.v) {
      case 4: BSR_AFFINE(float, 4); break;
      case 2: BSR_AFFINE(float, 2); break;
      default: BSR_AFFINE(float, 1); break;
    }
  } else {
    switch (p.v) {
      case 8: BSR_AFFINE(uint16_t, 8); break;
      case 4: BSR_AFFINE(uint16_t, 4); break;
      case 2: BSR_AFFINE(uint16_t, 2); break;
      default: BSR_AFFINE(uint16_t, 1); break;
    }
  }
#undef BSR_AFFINE
  const int rc = check_launch();
  if (rc != BSR_OK) return rc;
  hipLaunchKernelGGL(affine_reduce_kernel, dim3((unsigned)ceil_div(K, 4)), dim3(256), 0, s, partial,
                     (int)p.splits, K, dalpha, accumulate);
  return check_launch();
}

}  // namespace bsr
