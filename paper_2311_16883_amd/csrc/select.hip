// Top-k block selection (paper Sec. IV: the k lowest-ranked blocks are pruned).
//
// Exact selection of the n_keep best blocks in the total order
//   (score descending, linear block index ascending)
// without sorting everything and without a host round trip.  Every block gets
// a unique 96-bit rank value
//   C = key * 2^32 + (nblocks - 1 - index),
// where key is the bit pattern of its non-negative binary64 score (orders like
// the value; any NaN becomes one quiet-NaN pattern above +inf).  "Best" means
// largest C.  The kernel finds the n_keep-th largest C by a most-significant-
// digit-first radix select with 12-bit digits: a histogram of the current
// digit over the blocks that still match the chosen prefix, a suffix scan to
// find the digit that holds the n_keep-th element, repeat.  As soon as the
// matching set fits in LDS it is ranked there exactly by counting, which also
// settles ties through the index part of C.  All arithmetic is integer, so the
// result is the same on every run.
#include "common.h"

namespace bsr {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kDigitBits = 12;
constexpr int kBins = 1 << kDigitBits;
constexpr int kCap = 1024;                 // candidates ranked in LDS

typedef unsigned __int128 u128;

__device__ __forceinline__ uint64_t score_key(double s) {
  if (s != s) return 0x7FF8000000000000ull;
  return (uint64_t)__double_as_longlong(s);
}

__device__ __forceinline__ u128 rank_value(uint64_t key, uint32_t inv_idx) {
  return ((u128)key << 32) | (u128)inv_idx;
}

// Exclusive prefix sum over the kSelThreads threads of the block.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot,
                                                         uint32_t *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int w = 0; w < kSelThreads / 64; ++w) {
    const uint32_t x = wave_tot[w];
    if (w < wave) base += x;
    tot += x;
  }
  __syncthreads();
  *total = tot;
  return base + incl - v;
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(const double *__restrict__ scores,
                                                             int64_t nblocks, int64_t n_keep,
                                                             uint8_t *__restrict__ mask) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint64_t ckey[kCap];
  __shared__ uint32_t cidx[kCap];
  __shared__ uint32_t wave_tot[kSelThreads / 64];
  __shared__ uint32_t sh_digit, sh_above, sh_count, sh_n;

  const int t = threadIdx.x;
  const uint32_t nb = (uint32_t)nblocks;

  u128 prefix = 0;          // the top 12*level bits every candidate shares
  int level = 0;
  uint32_t want = (uint32_t)n_keep;   // how many of the candidates are kept
  uint32_t n_cand = nb;

  while (n_cand > (uint32_t)kCap) {   // level < kDigits: distinct C leave <= 1 candidate after all digits
    for (int b = t; b < kBins; b += kSelThreads) hist[b] = 0;
    __syncthreads();
    const int shift_prefix = 96 - kDigitBits * level;
    const int shift_digit = shift_prefix - kDigitBits;
    for (uint32_t b = t; b < nb; b += kSelThreads) {
      const u128 c = rank_value(score_key(scores[b]), nb - 1 - b);
      if (level == 0 || (c >> shift_prefix) == prefix)
        atomicAdd(&hist[(uint32_t)(c >> shift_digit) & (kBins - 1)], 1u);
    }
    __syncthreads();
    // thread t owns the bins kBins-1-4t ... kBins-4-4t (descending digits)
    uint32_t h[4], own = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      h[u] = hist[kBins - 1 - (4 * t + u)];
      own += h[u];
    }
    uint32_t total;
    uint32_t above = block_exclusive_scan(own, wave_tot, &total);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (above < want && want <= above + h[u]) {
        sh_digit = (uint32_t)(kBins - 1 - (4 * t + u));
        sh_above = above;
        sh_count = h[u];
      }
      above += h[u];
    }
    __syncthreads();
    prefix = (prefix << kDigitBits) | (u128)sh_digit;
    want -= sh_above;
    n_cand = sh_count;
    ++level;
    __syncthreads();
  }

  // Everything above the prefix is kept, everything below is pruned, the
  // candidates that match it go to LDS.
  if (t == 0) sh_n = 0;
  __syncthreads();
  const int shift_prefix = 96 - kDigitBits * level;
  for (uint32_t b = t; b < nb; b += kSelThreads) {
    const uint64_t key = score_key(scores[b]);
    bool inside = true;
    if (level > 0) {
      const u128 top = rank_value(key, nb - 1 - b) >> shift_prefix;
      if (top != prefix) {
        inside = false;
        mask[b] = top > prefix ? 1 : 0;
      }
    }
    if (inside) {
      const uint32_t pos = atomicAdd(&sh_n, 1u);
      ckey[pos] = key;
      cidx[pos] = b;
    }
  }
  __syncthreads();
  const uint32_t n = sh_n;
  if ((uint32_t)t < n) {
    const uint64_t key = ckey[t];
    const uint32_t idx = cidx[t];
    uint32_t better = 0;   // candidates that rank strictly before this one
    for (uint32_t o = 0; o < n; ++o) {
      const uint64_t ok = ckey[o];
      better += (ok > key || (ok == key && cidx[o] < idx)) ? 1u : 0u;
    }
    mask[idx] = better < want ? 1 : 0;
  }
}

__global__ void fill_u8_kernel(uint8_t *p, int64_t n, uint8_t v) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    p[i] = v;
}

}  // namespace

int launch_select(const double *scores, int64_t nblocks, int64_t n_keep, uint8_t *keep_mask,
                  hipStream_t s) {
  if (nblocks == 0) return BSR_OK;
  if (n_keep <= 0 || n_keep >= nblocks) {
    const int grid = (int)(ceil_div(nblocks, 256) < 1024 ? ceil_div(nblocks, 256) : 1024);
    hipLaunchKernelGGL(fill_u8_kernel, dim3(grid), dim3(256), 0, s, keep_mask, nblocks,
                       (uint8_t)(n_keep > 0 ? 1 : 0));
    return check_launch();
  }
  hipLaunchKernelGGL(select_kernel, dim3(1), dim3(kSelThreads), 0, s, scores, nblocks, n_keep,
                     keep_mask);
  return check_launch();
}

}  // namespace bsr
