// Weight gradient from a BSR activation, any block shape (paper Sec. III, Fig. 2:
// dW = Xhat^T * dY, "BSpMM").  Plain binary32 FMA path: used for block shapes
// and element types the matrix-core kernel does not cover.
//
// A workgroup owns a 64 x 64 tile of dW and a contiguous range of block-rows
// (split of the contraction).  Per block-row it looks up which block-columns of
// its tile are kept (LDS table), stages 16 rows of the kept blocks (zeros where
// pruned) and of dY in LDS and accumulates 4 x 4 outputs per thread.  Block-rows
// without a kept block in the tile are skipped.  With more than one split the
// partial tiles go to the workspace and are summed in a fixed order afterwards.
#include "common.h"

namespace bsr {

namespace {

constexpr int TK = 64, TN = 64, RM = 16;

template <typename T>
__global__ __launch_bounds__(256) void dw_generic_kernel(
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const T *__restrict__ values, int64_t M, int64_t K, int br, int bc, int64_t nbr, int64_t nbc,
    const T *__restrict__ dY, int64_t N, int64_t lddy, float *__restrict__ out, int64_t ldo,
    int64_t split_stride, int64_t rows_per_split, int accumulate) {
  __shared__ float A[RM][TK];
  __shared__ float B[RM][TN];
  __shared__ int32_t slot[TK];

  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  const int64_t k0 = (int64_t)blockIdx.x * TK, n0 = (int64_t)blockIdx.y * TN;
  const int64_t i_begin = (int64_t)blockIdx.z * rows_per_split;
  const int64_t i_end = (i_begin + rows_per_split) < nbr ? (i_begin + rows_per_split) : nbr;
  const int64_t jfirst = k0 / bc;
  int64_t jlast = (k0 + TK - 1) / bc;
  if (jlast > nbc - 1) jlast = nbc - 1;
  const int ncol = (int)(jlast - jfirst + 1);

  float acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

  for (int64_t i = i_begin; i < i_end; ++i) {
    if (t < ncol) slot[t] = -1;
    __syncthreads();
    const int64_t p0 = row_ptr[i], p1 = row_ptr[i + 1];
    int hit = 0;
    for (int64_t p = p0 + t; p < p1; p += 256) {
      const int64_t j = col_idx[p];
      if (j >= jfirst && j <= jlast) {
        slot[j - jfirst] = (int32_t)p;
        hit = 1;
      }
    }
    if (!__syncthreads_or(hit)) continue;

    for (int r0 = 0; r0 < br; r0 += RM) {
      for (int e = t; e < RM * TK; e += 256) {
        const int rr = e / TK, kk = e % TK;
        const int64_t k = k0 + kk;
        const int r = r0 + rr;
        float v = 0.f;
        if (k < K && r < br) {
          const int64_t j = k / bc;
          const int32_t p = slot[j - jfirst];
          if (p >= 0) v = elem_to_float<T>(values[((int64_t)p * br + r) * bc + (k - j * bc)]);
        }
        A[rr][kk] = v;
      }
      for (int e = t; e < RM * TN; e += 256) {
        const int rr = e / TN, nn = e % TN;
        const int64_t m = i * br + r0 + rr, n = n0 + nn;
        float v = 0.f;
        if (r0 + rr < br && m < M && n < N) v = elem_to_float<T>(dY[m * lddy + n]);
        B[rr][nn] = v;
      }
      __syncthreads();
#pragma unroll
      for (int rr = 0; rr < RM; ++rr) {
        float a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          a[u] = A[rr][ty * 4 + u];
          b[u] = B[rr][tx * 4 + u];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int w = 0; w < 4; ++w) acc[u][w] = fmaf(a[u], b[w], acc[u][w]);
      }
      __syncthreads();
    }
  }

  float *o = out + (int64_t)blockIdx.z * split_stride;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t k = k0 + ty * 4 + u;
    if (k >= K) continue;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int64_t n = n0 + tx * 4 + w;
      if (n >= N) continue;
      float *dst = o + k * ldo + n;
      *dst = accumulate ? *dst + acc[u][w] : acc[u][w];
    }
  }
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial,
                                                            int splits, int64_t K, int64_t N,
                                                            float *__restrict__ dW, int64_t lddw,
                                                            int accumulate) {
  const int64_t total = K * N;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total;
       e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t k = e / N, n = e % N;
    float s = accumulate ? dW[k * lddw + n] : 0.f;
    for (int sp = 0; sp < splits; ++sp) s += partial[(int64_t)sp * total + e];
    dW[k * lddw + n] = s;
  }
}

// Same sum, four columns per thread (N, lddw and the pointers allow 16-byte access).
__global__ __launch_bounds__(256) void splitk_reduce4_kernel(const float4 *__restrict__ partial,
                                                             int splits, int64_t K, int64_t N4,
                                                             float *__restrict__ dW, int64_t lddw,
                                                             int accumulate) {
  const int64_t total4 = K * N4;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < total4;
       e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t k = e / N4, n4 = e % N4;
    float4 *dst = reinterpret_cast<float4 *>(dW + k * lddw) + n4;
    float4 s = accumulate ? *dst : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int sp = 0; sp < splits; ++sp) {
      const float4 v = partial[(int64_t)sp * total4 + e];
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *dst = s;
  }
}

// The same sums for several tensors in one launch (item = tensor, found from the prefix of
// workgroup counts); per element the order of the additions is that of the kernels above.
struct ReduceBatch {
  ReduceJob it[kReduceBatchMax];
  uint32_t wg_begin[kReduceBatchMax + 1];
};

__global__ __launch_bounds__(256) void splitk_reduce_batched_kernel(ReduceBatch b, int n) {
  int i = 0;
  while (i + 1 < n && blockIdx.x >= b.wg_begin[i + 1]) ++i;
  const ReduceJob &it = b.it[i];
  const int64_t wg = blockIdx.x - b.wg_begin[i], wgs = b.wg_begin[i + 1] - b.wg_begin[i];
  const bool vec = it.N % 4 == 0 && it.lddw % 4 == 0 && (uintptr_t)it.dW % 16 == 0 && (uintptr_t)it.partial % 16 == 0;
  if (vec) {
    const int64_t N4 = it.N / 4, total4 = it.K * N4;
    const float4 *partial = reinterpret_cast<const float4 *>(it.partial);
    for (int64_t e = wg * 256 + threadIdx.x; e < total4; e += wgs * 256) {
      const int64_t k = e / N4, n4 = e % N4;
      float4 *dst = reinterpret_cast<float4 *>(it.dW + k * it.lddw) + n4;
      float4 s = it.accumulate ? *dst : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
      for (int sp = 0; sp < it.splits; ++sp) {
        const float4 v = partial[(int64_t)sp * total4 + e];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      *dst = s;
    }
  } else {
    const int64_t total = it.K * it.N;
    for (int64_t e = wg * 256 + threadIdx.x; e < total; e += wgs * 256) {
      const int64_t k = e / it.N, c = e % it.N;
      float s = it.accumulate ? it.dW[k * it.lddw + c] : 0.f;
      for (int sp = 0; sp < it.splits; ++sp) s += it.partial[(int64_t)sp * total + e];
      it.dW[k * it.lddw + c] = s;
    }
  }
}

int generic_splits(int64_t M, int64_t K, int64_t N, int br) {
  const int64_t nbr = ceil_div(M, br);
  const int64_t tiles = ceil_div(K, TK) * ceil_div(N, TN);
  int64_t s = 2048 / (tiles > 0 ? tiles : 1);
  if (s < 1) s = 1;
  if (s > nbr) s = nbr;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  return (int)s;
}

}  // namespace

int launch_splitk_reduce(const float *partial, int splits, int64_t K, int64_t N, float *dW,
                         int64_t lddw, int accumulate, hipStream_t s) {
  const int64_t total = K * N;
  if (total == 0) return BSR_OK;
  if (N % 4 == 0 && lddw % 4 == 0 && (uintptr_t)dW % 16 == 0 && (uintptr_t)partial % 16 == 0) {
    const int64_t blocks = ceil_div(total / 4, 256);
    hipLaunchKernelGGL(splitk_reduce4_kernel, dim3((unsigned)(blocks < 8192 ? blocks : 8192)),
                       dim3(256), 0, s, reinterpret_cast<const float4 *>(partial), splits, K, N / 4,
                       dW, lddw, accumulate);
    return check_launch();
  }
  const int64_t blocks = ceil_div(total, 256);
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(256),
                     0, s, partial, splits, K, N, dW, lddw, accumulate);
  return check_launch();
}

int launch_splitk_reduce_batched(const ReduceJob *jobs, int n, hipStream_t s) {
  for (int i0 = 0; i0 < n; i0 += kReduceBatchMax) {
    const int m = n - i0 < kReduceBatchMax ? n - i0 : kReduceBatchMax;
    ReduceBatch b;
    uint32_t wgs = 0;
    for (int i = 0; i < m; ++i) {
      b.it[i] = jobs[i0 + i];
      b.wg_begin[i] = wgs;
      const int64_t blocks = ceil_div(ceil_div(jobs[i0 + i].K * jobs[i0 + i].N, 4), 256);
      wgs += (uint32_t)(blocks < 1 ? 1 : (blocks < 2048 ? blocks : 2048));
    }
    b.wg_begin[m] = wgs;
    hipLaunchKernelGGL(splitk_reduce_batched_kernel, dim3(wgs), dim3(256), 0, s, b, m);
    const int rc = check_launch();
    if (rc != BSR_OK) return rc;
  }
  return BSR_OK;
}

size_t dw_generic_ws_bytes(int64_t M, int64_t K, int64_t N, int br, int bc) {
  (void)bc;
  const int s = generic_splits(M, K, N, br);
  return s > 1 ? (size_t)s * (size_t)K * (size_t)N * sizeof(float) : 0;
}

int launch_dw_generic(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype,
                      int64_t M, int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy,
                      float *dW, int64_t lddw, int accumulate, void *ws, size_t ws_bytes,
                      hipStream_t s) {
  if (K == 0 || N == 0) return BSR_OK;
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  const int splits = generic_splits(M, K, N, br);
  if (splits > 1 && (ws == nullptr || ws_bytes < dw_generic_ws_bytes(M, K, N, br, bc)))
    return BSR_ERR_WORKSPACE;
  const int64_t rps = nbr > 0 ? ceil_div(nbr, splits) : 1;
  float *out = splits > 1 ? static_cast<float *>(ws) : dW;
  const int64_t ldo = splits > 1 ? N : lddw;
  const int64_t stride = splits > 1 ? K * N : 0;
  const int acc_direct = splits > 1 ? 0 : accumulate;
  dim3 grid((unsigned)ceil_div(K, TK), (unsigned)ceil_div(N, TN), (unsigned)splits);
  if (dtype == BSR_F32)
    hipLaunchKernelGGL((dw_generic_kernel<float>), grid, dim3(256), 0, s, row_ptr, col_idx,
                       static_cast<const float *>(values), M, K, br, bc, nbr, nbc,
                       static_cast<const float *>(dY), N, lddy, out, ldo, stride, rps, acc_direct);
  else
    hipLaunchKernelGGL((dw_generic_kernel<uint16_t>), grid, dim3(256), 0, s, row_ptr, col_idx,
                       static_cast<const uint16_t *>(values), M, K, br, bc, nbr, nbc,
                       static_cast<const uint16_t *>(dY), N, lddy, out, ldo, stride, rps, acc_direct);
  int rc = check_launch();
  if (rc != BSR_OK || splits == 1) return rc;
  return launch_splitk_reduce(out, splits, K, N, dW, lddw, accumulate, s);
}

}  // namespace bsr
