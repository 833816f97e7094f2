// Top-k block selection (paper Sec. IV: the k lowest-ranked blocks are pruned).
//
// Exact selection of the n_keep best blocks in the total order
//   (score descending, linear block index ascending)
// without sorting everything and without a host round trip.  key is the bit
// pattern of the non-negative binary64 score (orders like the value; any NaN
// becomes one quiet-NaN pattern above +inf), so all arithmetic is integer and
// the result is the same on every run.
//
// Building blocks.  radix_select: one workgroup, most-significant-digit-first
// radix select (12-bit digits) on the 96-bit rank value
// C = key * 2^32 + (nblocks-1-index): histogram of the current digit over the
// elements that still match the chosen prefix, suffix scan for the digit holding
// the n_keep-th element, repeat; once the matching set fits in LDS it is ranked
// exactly by counting, which settles ties through the index part of C.  It works
// for any input and is the fallback of bracketed_select, which is much faster
// when the caller can bracket the threshold's key (see there).
//
// Small inputs (<= 12288 blocks) and per-group selection: one workgroup per
// ranking group, bracketed_select between the group's smallest and largest key.
//
// Large inputs: two grid-wide passes and a one-workgroup finish, three launches.
//   pass 1  every workgroup draws the same small sample, takes from it two order
//           statistics lo <= hi that bracket the rank of the threshold, and
//           counts its slice of the keys into 256 buckets: bucket 0 below lo, the
//           last bucket above hi, equal-width buckets in between (any monotone
//           bucketing keeps the selection exact; a good bracket only makes the
//           threshold bucket small).  Each workgroup stores its own counts: no
//           atomics, nothing to clear.
//   pass 2  every workgroup adds up the counts, finds the bucket that holds the
//           n_keep-th largest key, keeps the buckets above it, prunes the ones
//           below and appends the keys inside it to a candidate list (one atomic
//           per workgroup).
//   finish  one workgroup stages the candidates in LDS and selects among them
//           exactly, with the bucket's key range as a bracket: 32-bit codes linear
//           in the key, one 8-bit radix pass as a rule, then a ranking of the
//           handful that share the threshold's code through lane reads.  The
//           general radix select remains the fallback when a bracket misses or
//           too many keys are equal.
#include "common.h"

namespace bsr {

namespace {

constexpr int kDigitBits = 12;
constexpr int kBins = 1 << kDigitBits;
constexpr int kCap = 1024;       // candidates ranked in LDS
constexpr int kSample = 256;
constexpr int kGridThreads = 256;
constexpr int kBuckets = 256;    // buckets of the grid-wide passes (one per thread)
constexpr int kStage = 1024;     // candidates the last workgroup stages in LDS

typedef unsigned __int128 u128;

__device__ __forceinline__ uint64_t score_key(double s) {
  if (s != s) return 0x7FF8000000000000ull;
  return (uint64_t)__double_as_longlong(s);
}

__device__ __forceinline__ u128 rank_value(uint64_t key, uint32_t inv_idx) {
  return ((u128)key << 32) | (u128)inv_idx;
}

// Where the elements to select from live: all scores, or a candidate list.
struct AllScores {
  const double *scores;
  __device__ __forceinline__ uint64_t key(uint32_t e) const { return score_key(scores[e]); }
  __device__ __forceinline__ uint32_t idx(uint32_t e) const { return e; }
};
struct Candidates {
  const uint64_t *keys;
  const uint32_t *idxs;
  __device__ __forceinline__ uint64_t key(uint32_t e) const { return keys[e]; }
  __device__ __forceinline__ uint32_t idx(uint32_t e) const { return idxs[e]; }
};

struct SelectShared {
  uint32_t hist[kBins];
  uint64_t ckey[kCap];
  uint32_t cidx[kCap];
  uint32_t wave_tot[16];
  uint32_t digit, above, count, n;
};

// Exclusive prefix sum over the THREADS threads of the block.
template <int THREADS>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *wave_tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  __syncthreads();
  return base + incl - v;
}

template <int THREADS>
__device__ __forceinline__ void rank_candidates(SelectShared &sh, uint32_t m, uint32_t want,
                                                uint8_t *__restrict__ mask);

// One workgroup marks the `want` best of the n elements of `src` in mask
// (1 = kept, 0 = pruned); every element of src gets its byte written.
template <int THREADS, typename Source>
__device__ void radix_select(const Source &src, uint32_t n, uint32_t want, uint32_t nblocks,
                             uint8_t *__restrict__ mask, SelectShared &sh) {
  const int t = threadIdx.x;
  constexpr int kPerThread = kBins / THREADS;
  u128 prefix = 0;          // the top 12*level bits every candidate shares
  int level = 0;
  uint32_t n_cand = n;

  while (n_cand > (uint32_t)kCap) {   // distinct C: at most one candidate is left after all 8 digits
    for (int b = t; b < kBins; b += THREADS) sh.hist[b] = 0;
    __syncthreads();
    const int shift_prefix = 96 - kDigitBits * level;
    const int shift_digit = shift_prefix - kDigitBits;
    for (uint32_t e = t; e < n; e += THREADS) {
      const u128 c = rank_value(src.key(e), nblocks - 1 - src.idx(e));
      if (level == 0 || (c >> shift_prefix) == prefix)
        atomicAdd(&sh.hist[(uint32_t)(c >> shift_digit) & (kBins - 1)], 1u);
    }
    __syncthreads();
    // thread t owns kPerThread bins, descending digits
    uint32_t h[kPerThread], own = 0;
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
      h[u] = sh.hist[kBins - 1 - (kPerThread * t + u)];
      own += h[u];
    }
    uint32_t above = block_exclusive_scan<THREADS>(own, sh.wave_tot);
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
      if (above < want && want <= above + h[u]) {
        sh.digit = (uint32_t)(kBins - 1 - (kPerThread * t + u));
        sh.above = above;
        sh.count = h[u];
      }
      above += h[u];
    }
    __syncthreads();
    prefix = (prefix << kDigitBits) | (u128)sh.digit;
    want -= sh.above;
    n_cand = sh.count;
    ++level;
    __syncthreads();
  }

  // Everything above the prefix is kept, everything below pruned, the
  // candidates that match it are ranked in LDS.
  if (t == 0) sh.n = 0;
  __syncthreads();
  const int shift_prefix = 96 - kDigitBits * level;
  for (uint32_t e = t; e < n; e += THREADS) {
    const uint64_t key = src.key(e);
    const uint32_t idx = src.idx(e);
    bool inside = true;
    if (level > 0) {
      const u128 top = rank_value(key, nblocks - 1 - idx) >> shift_prefix;
      if (top != prefix) {
        inside = false;
        mask[idx] = top > prefix ? 1 : 0;
      }
    }
    if (inside) {
      const uint32_t pos = atomicAdd(&sh.n, 1u);
      sh.ckey[pos] = key;
      sh.cidx[pos] = idx;
    }
  }
  __syncthreads();
  rank_candidates<THREADS>(sh, sh.n, want, mask);
}

// Selection with a bracket.  The caller knows (or hopes) that the want-th best
// of the n elements of `src` has its key inside [lo, hi].  Keys above hi are only
// counted; keys inside get a 32-bit code, 1 + ((key - lo) >> shift), that stays
// in registers (KPT per thread, n <= KPT * THREADS) for the radix passes that
// find the code of the threshold: the codes spread evenly over the bracket, so
// usually one 12-bit pass with next to no bin shared.  key -> code is monotone, so
// a larger (smaller) code than the threshold's means kept (pruned) for certain;
// the few elements that share the threshold's code are ranked exactly on their
// full keys and indices.  If the bracket misses the threshold or more than kCap
// elements share its code (e.g. very many all-zero blocks), the general radix
// select takes over.  Every element of src gets its mask byte written.
struct BracketShared {
  uint32_t wave_cnt[2][16];
};

// Exact ranking of the m candidates listed in sh.ckey / sh.cidx: the `want` best
// in (key descending, index ascending) order are kept.  Up to 64 candidates sit
// one per lane of the first wave and are compared through lane reads (no LDS
// round trip per comparison); longer lists (many equal keys) go through LDS.
template <int THREADS>
__device__ __forceinline__ void rank_candidates(SelectShared &sh, uint32_t m, uint32_t want,
                                                uint8_t *__restrict__ mask) {
  const int t = threadIdx.x;
  if (m <= 64u) {
    if (t < 64) {
      const bool live = (uint32_t)t < m;
      const uint64_t k = live ? sh.ckey[t] : 0ull;
      const uint32_t idx = live ? sh.cidx[t] : 0u;
      const uint32_t klo = (uint32_t)k, khi = (uint32_t)(k >> 32);
      uint32_t better = 0;   // candidates that rank strictly before this one
      for (uint32_t o = 0; o < m; ++o) {
        const uint64_t ok = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)khi, (int)o) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)klo, (int)o);
        const uint32_t oidx = (uint32_t)__builtin_amdgcn_readlane((int)idx, (int)o);
        better += (ok > k || (ok == k && oidx < idx)) ? 1u : 0u;
      }
      if (live) mask[idx] = better < want ? 1 : 0;
    }
    return;
  }
  if (m <= (uint32_t)THREADS) {
    // the m x m comparisons are spread over all threads: `parts` threads share one
    // candidate, each counts over its own range of opponents
    const uint32_t parts = (uint32_t)THREADS / m, chunk = (m + parts - 1) / parts;
    for (uint32_t c = t; c < m; c += THREADS) sh.hist[c] = 0;
    __syncthreads();
    const uint32_t c = (uint32_t)t % m, part = (uint32_t)t / m;
    if (part < parts) {
      const uint64_t k = sh.ckey[c];
      const uint32_t idx = sh.cidx[c];
      const uint32_t o0 = part * chunk, o1 = (o0 + chunk) < m ? (o0 + chunk) : m;
      uint32_t better = 0;
#pragma unroll 4
      for (uint32_t o = o0; o < o1; ++o) {
        const uint64_t ok = sh.ckey[o];
        better += (ok > k || (ok == k && sh.cidx[o] < idx)) ? 1u : 0u;
      }
      if (better) atomicAdd(&sh.hist[c], better);
    }
    __syncthreads();
    if ((uint32_t)t < m) mask[sh.cidx[t]] = sh.hist[t] < want ? 1 : 0;
    return;
  }
  for (uint32_t c = t; c < m; c += THREADS) {
    const uint64_t k = sh.ckey[c];
    const uint32_t idx = sh.cidx[c];
    uint32_t better = 0;
#pragma unroll 8
    for (uint32_t o = 0; o < m; ++o) {
      const uint64_t ok = sh.ckey[o];
      better += (ok > k || (ok == k && sh.cidx[o] < idx)) ? 1u : 0u;
    }
    mask[idx] = better < want ? 1 : 0;
  }
}

// DB = bits per radix pass: the pass costs one histogram of 2^DB bins (zeroed,
// filled, scanned by THREADS threads), so small workgroups take small digits.
template <int THREADS, int KPT, int DB, typename Source>
__device__ void bracketed_select(const Source &src, uint32_t n, uint32_t want_total, uint64_t lo, uint64_t hi,
                                 uint32_t nblocks, uint8_t *__restrict__ mask, SelectShared &sh,
                                 BracketShared &bs) {
  constexpr int kLocalBins = 1 << DB;
  constexpr int kPerThread = kLocalBins / THREADS;
  static_assert(kPerThread >= 1 && kLocalBins <= kBins, "one bin per thread at least");
  constexpr uint32_t kAbove = 0xFFFFFFFFu, kBelow = 0u;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  // element i of this thread is number t + i * THREADS of src; the first cnt exist
  const int cnt = (uint32_t)t < n ? (int)((n - 1u - (uint32_t)t) / THREADS) + 1 : 0;
  const uint64_t range = hi - lo;
  // smallest shift with 1 + (range >> shift) <= 0xFFFFFFFE
  int shift = range == 0 ? 0 : 64 - __clzll((long long)range);          // bit length of range
  shift = shift > 31 ? shift - 31 : 0;

  uint32_t code[KPT];
  uint32_t n_above = 0, n_inside = 0;
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    const uint32_t e = (uint32_t)(t + i * THREADS);
    const uint64_t key = src.key(e < n ? e : 0u);
    uint32_t c = 1u + (uint32_t)((key - lo) >> shift);
    c = key > hi ? kAbove : (key < lo ? kBelow : c);
    if (i >= cnt) c = kBelow;
    n_above += c == kAbove ? 1u : 0u;
    n_inside += (c != kAbove && c != kBelow) ? 1u : 0u;
    code[i] = c;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    n_above += __shfl_xor(n_above, d, 64);
    n_inside += __shfl_xor(n_inside, d, 64);
  }
  if (lane == 0) { bs.wave_cnt[0][wave] = n_above; bs.wave_cnt[1][wave] = n_inside; }
  __syncthreads();
  n_above = 0;
  n_inside = 0;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) { n_above += bs.wave_cnt[0][w]; n_inside += bs.wave_cnt[1][w]; }

  // bits [ctop, 32) of the threshold's code are settled and equal cprefix
  int ctop = 32;
  uint32_t cprefix = 0, want = want_total - n_above, n_cand = n_inside;
  const bool bracketed = want_total > n_above && want <= n_inside;
  while (bracketed && n_cand > 64u && ctop > 0) {
    const int dshift = ctop > DB ? ctop - DB : 0;
    const uint32_t dmask = (1u << (ctop - dshift)) - 1u;
    for (int b = t; b < kLocalBins; b += THREADS) sh.hist[b] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      const uint32_t c = code[i];
      if (c != kAbove && c != kBelow && (ctop == 32 || (c >> ctop) == cprefix))
        atomicAdd(&sh.hist[(c >> dshift) & dmask], 1u);
    }
    __syncthreads();
    uint32_t h[kPerThread], own = 0;
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
      h[u] = sh.hist[kLocalBins - 1 - (kPerThread * t + u)];
      own += h[u];
    }
    uint32_t above = block_exclusive_scan<THREADS>(own, sh.wave_tot);
#pragma unroll
    for (int u = 0; u < kPerThread; ++u) {
      if (above < want && want <= above + h[u]) {
        sh.digit = (uint32_t)(kLocalBins - 1 - (kPerThread * t + u));
        sh.above = above;
        sh.count = h[u];
      }
      above += h[u];
    }
    __syncthreads();
    cprefix = ctop == 32 ? sh.digit : ((cprefix << (ctop - dshift)) | sh.digit);
    want -= sh.above;
    n_cand = sh.count;
    ctop = dshift;
    __syncthreads();
  }
  if (!bracketed || n_cand > (uint32_t)kCap) {
    radix_select<THREADS>(src, n, want_total, nblocks, mask, sh);
    return;
  }

  // larger code: kept; smaller: pruned; equal: ranked exactly on the full keys
  if (t == 0) sh.n = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    if (i < cnt) {
      const uint32_t e = (uint32_t)(t + i * THREADS);
      const uint32_t c = code[i];
      const bool inside = c != kAbove && c != kBelow;
      // with no pass run (ctop == 32) every element inside the bracket is a candidate
      const uint32_t chi = ctop == 32 ? 0u : c >> ctop;
      if (inside && chi == cprefix) {
        const uint32_t pos = atomicAdd(&sh.n, 1u);
        sh.ckey[pos] = src.key(e);
        sh.cidx[pos] = src.idx(e);
      } else {
        mask[src.idx(e)] = (c == kAbove || (inside && chi > cprefix)) ? 1 : 0;
      }
    }
  }
  __syncthreads();
  rank_candidates<THREADS>(sh, sh.n, want, mask);
}

// Per-group selection (paper Sec. IV: blocks are only compared inside one
// activation of the mini-batch): a ranking group is `group_blocks` consecutive
// blocks in linear order (whole block-rows); workgroup g selects inside group g
// with indices local to the group.  The group's smallest and largest key serve
// as the bracket of bracketed_select: codes linear in the key, a radix pass or
// two, exact ranking of what shares the threshold's code.  The last group may be
// shorter (last_blocks, keeping n_keep_last).
// One workgroup selects the `want` best of the n scores at `scores` into gmask.
template <int THREADS, int KPT, int DB>
__device__ __forceinline__ void select_one_group(const double *__restrict__ scores, uint32_t n, uint32_t want,
                                                 uint8_t *__restrict__ gmask) {
  __shared__ SelectShared sh;
  __shared__ BracketShared bs;
  __shared__ uint64_t wave_min[THREADS / 64], wave_max[THREADS / 64];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  if (want == 0 || want >= n) {
    for (uint32_t e = t; e < n; e += THREADS) gmask[e] = want > 0 ? 1 : 0;
    return;
  }
  AllScores src{scores};
  uint64_t mn = ~0ull, mx = 0ull;
#pragma unroll
  for (int i = 0; i < KPT; ++i) {
    const uint32_t e = (uint32_t)(t + i * THREADS);
    if (e < n) {
      const uint64_t k = src.key(e);
      mn = k < mn ? k : mn;
      mx = k > mx ? k : mx;
    }
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const uint64_t a = __shfl_xor(mn, d, 64), b = __shfl_xor(mx, d, 64);
    mn = a < mn ? a : mn;
    mx = b > mx ? b : mx;
  }
  if (lane == 0) { wave_min[wave] = mn; wave_max[wave] = mx; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) {
    mn = wave_min[w] < mn ? wave_min[w] : mn;
    mx = wave_max[w] > mx ? wave_max[w] : mx;
  }
  bracketed_select<THREADS, KPT, DB>(src, n, want, mn, mx, n, gmask, sh, bs);
}

template <int THREADS, int KPT, int DB>
__global__ __launch_bounds__(THREADS) void select_groups_kernel(
    const double *__restrict__ scores, uint32_t group_blocks, uint32_t n_keep_group, uint32_t last_blocks,
    uint32_t n_keep_last, uint8_t *__restrict__ mask) {
  const bool last = blockIdx.x == gridDim.x - 1;
  const size_t off = (size_t)blockIdx.x * group_blocks;
  select_one_group<THREADS, KPT, DB>(scores + off, last ? last_blocks : group_blocks,
                                     last ? n_keep_last : n_keep_group, mask + off);
}

// Per-group selection of several tensors in one launch: tensor k owns the workgroups
// [wg_begin_k, wg_begin_k + groups_k), one workgroup per group.
constexpr int kGroupBatchMax = 24;
struct GroupItem {
  const double *scores;
  uint8_t *mask;
  uint32_t group_blocks, n_keep_group, last_blocks, n_keep_last, groups, wg_begin;
};
struct GroupBatch {
  GroupItem it[kGroupBatchMax];
};
template <int THREADS, int KPT, int DB>
__global__ __launch_bounds__(THREADS) void select_groups_batched_kernel(GroupBatch b, int n) {
  int k = 0;
  while (k + 1 < n && blockIdx.x >= b.it[k + 1].wg_begin) ++k;
  const GroupItem &it = b.it[k];
  const uint32_t g = blockIdx.x - it.wg_begin;
  const bool last = g == it.groups - 1;
  const size_t off = (size_t)g * it.group_blocks;
  select_one_group<THREADS, KPT, DB>(it.scores + off, last ? it.last_blocks : it.group_blocks,
                                     last ? it.n_keep_last : it.n_keep_group, it.mask + off);
}

// Control block shared by the two grid-wide passes (lives in the workspace;
// written by workgroup 0 of pass 1).
struct SelectCtrl {
  uint32_t n_cand, shift;
  uint64_t lo, hi;
};

__device__ __forceinline__ uint32_t bucket_of(uint64_t key, uint64_t lo, uint64_t hi, uint32_t shift) {
  if (key < lo) return 0u;
  if (key > hi) return (uint32_t)kBuckets - 1u;
  return 1u + (uint32_t)((key - lo) >> shift);
}

// NS = sample size: 64 (ranked inside one wave through lane reads, no LDS round
// trips) or kSample = 256 (ranked through LDS; a tighter bracket for very large
// inputs, where the threshold bucket must still fit the candidate ranking).
template <int NS>
__device__ __forceinline__ void select_count_body(
    const double *__restrict__ scores, uint32_t nblocks, uint32_t n_keep, uint32_t per_wg,
    uint32_t *__restrict__ counts, SelectCtrl *__restrict__ ctrl, uint32_t wg) {
  __shared__ uint32_t hist[kBuckets];
  __shared__ uint64_t sample[kSample];
  __shared__ uint64_t bracket[2];
  const int t = threadIdx.x;
  constexpr int kKeys = 4;                        // keys per thread held in registers (per_wg <= 1024)

  // this workgroup's slice (loads in flight while the sample is ranked)
  const uint32_t e0 = wg * per_wg;
  const uint32_t e1 = (e0 + per_wg) < nblocks ? (e0 + per_wg) : nblocks;
  double raw[kKeys];
#pragma unroll
  for (int i = 0; i < kKeys; ++i) {
    const uint32_t e = e0 + t + i * kGridThreads;
    raw[i] = scores[e < e1 ? e : e0];
  }

  // the same sample in every workgroup: NS evenly spaced keys
  uint64_t mine = 0;
  if (t < NS) mine = score_key(scores[(uint64_t)t * nblocks / NS]);
  hist[t] = 0;
  const double frac = 1.0 - (double)n_keep / (double)nblocks;       // threshold's quantile from below
  const int pos = (int)(frac * NS);
  const int delta = 3 + (int)(3.5 * sqrt(NS * frac * (1.0 - frac)));
  const int rlo = pos - delta < 0 ? 0 : pos - delta;
  const int rhi = pos + delta > NS - 1 ? NS - 1 : pos + delta;
  if (NS == 64) {
    if (t < 64) {
      // ascending rank of my sample key (ties by position) from the other lanes' keys
      int rank = 0;
      const uint32_t mlo = (uint32_t)mine, mhi = (uint32_t)(mine >> 32);
#pragma unroll 16
      for (int o = 0; o < 64; ++o) {
        const uint64_t k = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mhi, o) << 32) |
                           (uint32_t)__builtin_amdgcn_readlane((int)mlo, o);
        rank += (k < mine || (k == mine && o < t)) ? 1 : 0;
      }
      // the two order statistics around the threshold's expected position
      if (rank == rlo) bracket[0] = mine;
      if (rank == rhi) bracket[1] = mine;
    }
  } else {
    sample[t] = mine;
    __syncthreads();
    int rank = 0;
#pragma unroll 16
    for (int o = 0; o < NS; ++o) {
      const uint64_t k = sample[o];
      rank += (k < mine || (k == mine && o < t)) ? 1 : 0;
    }
    if (rank == rlo) bracket[0] = mine;
    if (rank == rhi) bracket[1] = mine;
  }
  __syncthreads();
  const uint64_t lo = bracket[0], hi = bracket[1];
  const uint64_t range = hi - lo;
  // smallest shift with (range >> shift) <= kBuckets - 3
  uint32_t shift = range == 0 ? 0u : (uint32_t)(64 - __clzll((long long)range));   // bit length of range
  shift = shift > 8 ? shift - 8 : 0u;
  if ((range >> shift) > (uint64_t)(kBuckets - 3)) ++shift;
  if (wg == 0 && t == 0) {
    ctrl->n_cand = 0;
    ctrl->shift = shift;
    ctrl->lo = lo;
    ctrl->hi = hi;
  }
#pragma unroll
  for (int i = 0; i < kKeys; ++i)
    if (e0 + t + i * kGridThreads < e1) atomicAdd(&hist[bucket_of(score_key(raw[i]), lo, hi, shift)], 1u);
  // longer slices (more than 256 K blocks): eight loads in flight per round
  for (uint32_t eb = e0 + t + kKeys * kGridThreads; eb < e1; eb += 8 * kGridThreads) {
    double more[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t e = eb + i * kGridThreads;
      more[i] = scores[e < e1 ? e : e0];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (eb + i * kGridThreads < e1) atomicAdd(&hist[bucket_of(score_key(more[i]), lo, hi, shift)], 1u);
  }
  __syncthreads();
  counts[wg * kBuckets + t] = hist[t];
}

template <int NS>
__global__ __launch_bounds__(kGridThreads) void select_count_kernel(
    const double *__restrict__ scores, uint32_t nblocks, uint32_t n_keep, uint32_t per_wg,
    uint32_t *__restrict__ counts, SelectCtrl *__restrict__ ctrl) {
  select_count_body<NS>(scores, nblocks, n_keep, per_wg, counts, ctrl, blockIdx.x);
}

// MODE 1: classification only; MODE 2: only the selection among the candidates, by one
// workgroup of a later launch.  (One kernel in which the last workgroup to finish, found by an
// atomic ticket, does the selection needs a release fence in every workgroup -- an L2 write-back
// on this GPU -- which costs more than the second launch.)
template <int MODE>
__device__ __forceinline__ void select_classify_body(
    const double *__restrict__ scores, uint32_t nblocks, uint32_t n_keep, uint32_t per_wg,
    const uint32_t *__restrict__ counts, SelectCtrl *__restrict__ ctrl,
    uint64_t *__restrict__ cand_key, uint32_t *__restrict__ cand_idx, uint8_t *__restrict__ mask,
    uint32_t wg, uint32_t nwgs) {
  __shared__ SelectShared sh;
  __shared__ BracketShared bs;
  __shared__ uint32_t wg_cand, wg_base;
  const int t = threadIdx.x;
  const uint32_t shift = ctrl->shift;
  const uint64_t lo = ctrl->lo, hi = ctrl->hi;
  constexpr int kKeys = 4;                        // keys per thread loaded up front (per_wg <= 1024 as a rule)

  const uint32_t e0 = wg * per_wg;
  const uint32_t e1 = (e0 + per_wg) < nblocks ? (e0 + per_wg) : nblocks;
  double raw[kKeys];
  if constexpr (MODE != 2) {
#pragma unroll
    for (int i = 0; i < kKeys; ++i) {
      const uint32_t e = e0 + t + i * kGridThreads;
      raw[i] = scores[e < e1 ? e : e0];
    }
  }
  if (t == 0) wg_cand = 0;

  // the bucket that holds the n_keep-th largest key (same answer in every workgroup):
  // thread t owns bucket kBuckets-1-t, the scan runs from the top
  uint32_t own = 0;
  for (uint32_t w0 = 0; w0 < nwgs; w0 += 64) {       // 64 independent loads in flight per round
    uint32_t part[64];
#pragma unroll
    for (uint32_t w = 0; w < 64; ++w)
      part[w] = w0 + w < nwgs ? counts[(w0 + w) * kBuckets + (kBuckets - 1 - t)] : 0u;
#pragma unroll
    for (uint32_t w = 0; w < 64; ++w) own += part[w];
  }
  const uint32_t above_me = block_exclusive_scan<kGridThreads>(own, sh.wave_tot);
  if (above_me < n_keep && n_keep <= above_me + own) {
    sh.digit = (uint32_t)(kBuckets - 1 - t);
    sh.above = above_me;
  }
  __syncthreads();
  const uint32_t bucket = sh.digit, above = sh.above;
  __syncthreads();

  if constexpr (MODE != 2) {
  // other buckets: mask bytes; the threshold's bucket: this workgroup's candidates
  // go to LDS first, so the global list takes one atomic per workgroup
  auto classify = [&](uint32_t e, uint64_t key) {
    const uint32_t b = bucket_of(key, lo, hi, shift);
    if (b != bucket) {
      mask[e] = b > bucket ? 1 : 0;
    } else {
      const uint32_t pos = atomicAdd(&wg_cand, 1u);
      if (pos < (uint32_t)kCap) {
        sh.ckey[pos] = key;
        sh.cidx[pos] = e;
      } else {                                   // more than the LDS list holds: straight to the global list
        const uint32_t g = atomicAdd(&ctrl->n_cand, 1u);
        cand_key[g] = key;
        cand_idx[g] = e;
      }
    }
  };
#pragma unroll
  for (int i = 0; i < kKeys; ++i) {
    const uint32_t e = e0 + t + i * kGridThreads;
    if (e < e1) classify(e, score_key(raw[i]));
  }
  for (uint32_t eb = e0 + t + kKeys * kGridThreads; eb < e1; eb += 8 * kGridThreads) {
    double more[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t e = eb + i * kGridThreads;
      more[i] = scores[e < e1 ? e : e0];
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (eb + i * kGridThreads < e1) classify(eb + i * kGridThreads, score_key(more[i]));
  }
  __syncthreads();
  const uint32_t mine = wg_cand < (uint32_t)kCap ? wg_cand : (uint32_t)kCap;
  if (t == 0 && mine > 0) wg_base = atomicAdd(&ctrl->n_cand, mine);
  __syncthreads();
  for (uint32_t c = t; c < mine; c += kGridThreads) {
    cand_key[wg_base + c] = sh.ckey[c];
    cand_idx[wg_base + c] = sh.cidx[c];
  }
  }
  if constexpr (MODE == 1) return;

  // the candidates all lie in the threshold bucket's key range,
  // which serves as the bracket of their exact selection
  const uint32_t n = __hip_atomic_load(&ctrl->n_cand, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  Candidates src{cand_key, cand_idx};
  uint64_t blo, bhi;
  if (bucket == 0) {
    blo = 0;
    bhi = lo - 1;                  // (bucket 0 is empty if lo == 0: never the threshold's)
  } else if (bucket == (uint32_t)kBuckets - 1) {
    blo = hi + 1;
    bhi = ~0ull;
  } else {
    blo = lo + ((uint64_t)(bucket - 1) << shift);
    bhi = blo + ((1ull << shift) - 1ull);
    if (bhi > hi) bhi = hi;
  }
  if (n <= (uint32_t)kStage) {
    // one trip to memory: the candidates move to LDS and are selected from there
    __shared__ uint64_t skey[kStage];
    __shared__ uint32_t sidx[kStage];
    for (uint32_t c = t; c < n; c += kGridThreads) {
      skey[c] = cand_key[c];
      sidx[c] = cand_idx[c];
    }
    __syncthreads();
    Candidates staged{skey, sidx};
    bracketed_select<kGridThreads, kStage / kGridThreads, 8>(staged, n, n_keep - above, blo, bhi, nblocks, mask, sh, bs);
  } else {
    radix_select<kGridThreads>(src, n, n_keep - above, nblocks, mask, sh);
  }
}

// ---- several independent selections per launch (one per tensor of a batch) ----
// The kernels above with blockIdx.y (grid-wide passes) or blockIdx.x (one workgroup
// per selection) naming the selection; its parameters come from the kernel
// arguments.  Selection is bound by launch and fence latency, not by work, so a
// batch costs about as much as one selection.
constexpr int kBatchMax = 40;
struct SelectItem {
  const double *scores;
  uint8_t *mask;
  uint32_t nblocks, n_keep, per_wg, wgs;
  uint32_t *counts;
  SelectCtrl *ctrl;
  uint64_t *cand_key;
  uint32_t *cand_idx;
};
struct SelectBatch {
  SelectItem it[kBatchMax];
};

template <int NS>
__global__ __launch_bounds__(kGridThreads) void select_count_batched_kernel(SelectBatch b) {
  const SelectItem &it = b.it[blockIdx.y];
  if (blockIdx.x >= it.wgs) return;
  select_count_body<NS>(it.scores, it.nblocks, it.n_keep, it.per_wg, it.counts, it.ctrl, blockIdx.x);
}

__global__ __launch_bounds__(kGridThreads) void select_classify_batched_kernel(SelectBatch b) {
  const SelectItem &it = b.it[blockIdx.y];
  if (blockIdx.x >= it.wgs) return;
  select_classify_body<1>(it.scores, it.nblocks, it.n_keep, it.per_wg, it.counts, it.ctrl, it.cand_key,
                          it.cand_idx, it.mask, blockIdx.x, it.wgs);
}

__global__ __launch_bounds__(kGridThreads) void select_finish_batched_kernel(SelectBatch b) {
  const SelectItem &it = b.it[blockIdx.x];
  select_classify_body<2>(it.scores, it.nblocks, it.n_keep, it.per_wg, it.counts, it.ctrl, it.cand_key,
                          it.cand_idx, it.mask, 0u, it.wgs);
}

template <int THREADS, int KPT, int DB>
__global__ __launch_bounds__(THREADS) void select_small_batched_kernel(SelectBatch b) {
  const SelectItem &it = b.it[blockIdx.x];
  select_one_group<THREADS, KPT, DB>(it.scores, it.nblocks, it.n_keep, it.mask);
}

__global__ void fill_u8_kernel(uint8_t *p, int64_t n, uint8_t v) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    p[i] = v;
}

constexpr int64_t kSmallLimit = 12288;     // one workgroup (up to 12 keys per thread)
constexpr int64_t kRideAlong = 4096;       // smallest tensor that the grid-wide passes of a batched call take along

constexpr int kMaxGridWgs = 256;

struct SelectPlan {
  size_t counts_off, ctrl_off, key_off, idx_off, total;
};

SelectPlan select_plan(int64_t nblocks) {
  SelectPlan p;
  p.counts_off = 0;
  p.ctrl_off = align_up((size_t)kMaxGridWgs * kBuckets * sizeof(uint32_t), 256);
  p.key_off = p.ctrl_off + align_up(sizeof(SelectCtrl), 256);
  p.idx_off = p.key_off + align_up((size_t)nblocks * sizeof(uint64_t), 256);
  p.total = p.idx_off + align_up((size_t)nblocks * sizeof(uint32_t), 256);
  return p;
}

}  // namespace

// (tensors of more than kRideAlong blocks may join the grid-wide passes of a batched call)
size_t select_ws_bytes(int64_t nblocks) {
  return nblocks > kRideAlong ? select_plan(nblocks).total : 0;
}

int launch_select(const double *scores, int64_t nblocks, int64_t n_keep, uint8_t *keep_mask, void *ws,
                  hipStream_t s) {
  if (nblocks == 0) return BSR_OK;
  if (n_keep <= 0 || n_keep >= nblocks) {
    const int grid = (int)(ceil_div(nblocks, 256) < 1024 ? ceil_div(nblocks, 256) : 1024);
    hipLaunchKernelGGL(fill_u8_kernel, dim3(grid), dim3(256), 0, s, keep_mask, nblocks,
                       (uint8_t)(n_keep > 0 ? 1 : 0));
    return check_launch();
  }
  if (nblocks <= kSmallLimit) {
    // one workgroup: the per-group kernel with a single group
    if (nblocks <= 1024)
      hipLaunchKernelGGL((select_groups_kernel<256, 4, 8>), dim3(1), dim3(256), 0, s, scores, (uint32_t)nblocks,
                         (uint32_t)n_keep, (uint32_t)nblocks, (uint32_t)n_keep, keep_mask);
    else if (nblocks <= 8192)
      hipLaunchKernelGGL((select_groups_kernel<1024, 8, kDigitBits>), dim3(1), dim3(1024), 0, s, scores,
                         (uint32_t)nblocks, (uint32_t)n_keep, (uint32_t)nblocks, (uint32_t)n_keep, keep_mask);
    else
      hipLaunchKernelGGL((select_groups_kernel<1024, 12, kDigitBits>), dim3(1), dim3(1024), 0, s, scores,
                         (uint32_t)nblocks, (uint32_t)n_keep, (uint32_t)nblocks, (uint32_t)n_keep, keep_mask);
    return check_launch();
  }
  const SelectPlan p = select_plan(nblocks);
  char *base = static_cast<char *>(ws);
  uint32_t *counts = reinterpret_cast<uint32_t *>(base + p.counts_off);
  SelectCtrl *ctrl = reinterpret_cast<SelectCtrl *>(base + p.ctrl_off);
  uint64_t *cand_key = reinterpret_cast<uint64_t *>(base + p.key_off);
  uint32_t *cand_idx = reinterpret_cast<uint32_t *>(base + p.idx_off);
  int64_t wgs = ceil_div(nblocks, 1024);
  if (wgs > kMaxGridWgs) wgs = kMaxGridWgs;
  const uint32_t per_wg = (uint32_t)ceil_div(nblocks, wgs);
  if (nblocks <= 262144)
    hipLaunchKernelGGL(select_count_kernel<64>, dim3((unsigned)wgs), dim3(kGridThreads), 0, s, scores,
                       (uint32_t)nblocks, (uint32_t)n_keep, per_wg, counts, ctrl);
  else
    hipLaunchKernelGGL(select_count_kernel<kSample>, dim3((unsigned)wgs), dim3(kGridThreads), 0, s, scores,
                       (uint32_t)nblocks, (uint32_t)n_keep, per_wg, counts, ctrl);
  int rc = check_launch();
  if (rc != BSR_OK) return rc;
  // Classification and the selection among the candidates as two launches: one more launch costs
  // less than the release fence of every workgroup that finding the last one to finish takes.
  SelectBatch b;
  b.it[0] = SelectItem{scores, keep_mask, (uint32_t)nblocks, (uint32_t)n_keep, per_wg, (uint32_t)wgs, counts, ctrl,
                       cand_key, cand_idx};
  hipLaunchKernelGGL(select_classify_batched_kernel, dim3((unsigned)wgs, 1), dim3(kGridThreads), 0, s, b);
  rc = check_launch();
  if (rc != BSR_OK) return rc;
  hipLaunchKernelGGL(select_finish_batched_kernel, dim3(1), dim3(kGridThreads), 0, s, b);
  return check_launch();
}

int launch_select_grouped(const double *scores, int64_t nbr, int64_t nbc, int64_t group_rows,
                          int64_t n_keep_group, int64_t n_keep_last, uint8_t *keep_mask, void *ws,
                          hipStream_t s) {
  if (nbr == 0 || nbc == 0) return BSR_OK;
  const int64_t groups = ceil_div(nbr, group_rows);
  const int64_t group_blocks = group_rows * nbc;
  const int64_t last_blocks = (nbr - (groups - 1) * group_rows) * nbc;
  if (groups == 1) return launch_select(scores, last_blocks, n_keep_last, keep_mask, ws, s);
  if (group_blocks > kSmallLimit) {
    // large groups: the grid-wide selection, one group after the other on the stream
    for (int64_t g = 0; g < groups; ++g) {
      const bool last = g == groups - 1;
      const int rc = launch_select(scores + g * group_blocks, last ? last_blocks : group_blocks,
                                   last ? n_keep_last : n_keep_group, keep_mask + g * group_blocks, ws, s);
      if (rc != BSR_OK) return rc;
    }
    return BSR_OK;
  }
  if (group_blocks <= 1024)
    hipLaunchKernelGGL((select_groups_kernel<256, 4, 8>), dim3((unsigned)groups), dim3(256), 0, s, scores,
                       (uint32_t)group_blocks, (uint32_t)n_keep_group, (uint32_t)last_blocks,
                       (uint32_t)n_keep_last, keep_mask);
  else if (group_blocks <= 8192)
    hipLaunchKernelGGL((select_groups_kernel<1024, 8, kDigitBits>), dim3((unsigned)groups), dim3(1024), 0, s,
                       scores, (uint32_t)group_blocks, (uint32_t)n_keep_group, (uint32_t)last_blocks,
                       (uint32_t)n_keep_last, keep_mask);
  else
    hipLaunchKernelGGL((select_groups_kernel<1024, 12, kDigitBits>), dim3((unsigned)groups), dim3(1024), 0, s,
                       scores, (uint32_t)group_blocks, (uint32_t)n_keep_group, (uint32_t)last_blocks,
                       (uint32_t)n_keep_last, keep_mask);
  return check_launch();
}

int launch_select_batched(const SelectJob *jobs, int n, hipStream_t s) {
  // classes: 0 one workgroup <= 1024 blocks, 1 <= 8192, 2 <= 12288, 3 grid-wide with the
  // 64-key sample, 4 grid-wide with the 256-key sample; everything else goes one by one.
  // The launches of the classes run one after the other and each is bound by latency, not
  // work: when the grid-wide passes run anyway, mid-sized tensors join them instead of
  // having a launch of one-workgroup selections of their own.
  bool grid_wide_runs = false;
  for (int i = 0; i < n; ++i)
    if (jobs[i].nblocks > kSmallLimit && jobs[i].nblocks <= 262144 && jobs[i].n_keep > 0 &&
        jobs[i].n_keep < jobs[i].nblocks)
      grid_wide_runs = true;
  for (int cls = 0; cls < 5; ++cls) {
    SelectBatch b;
    int m = 0;
    uint32_t max_wgs = 0;
    auto flush = [&]() -> int {
      if (m == 0) return BSR_OK;
      switch (cls) {
        case 0:
          hipLaunchKernelGGL((select_small_batched_kernel<256, 4, 8>), dim3(m), dim3(256), 0, s, b);
          break;
        case 1:
          hipLaunchKernelGGL((select_small_batched_kernel<1024, 8, kDigitBits>), dim3(m), dim3(1024), 0, s, b);
          break;
        case 2:
          hipLaunchKernelGGL((select_small_batched_kernel<1024, 12, kDigitBits>), dim3(m), dim3(1024), 0, s, b);
          break;
        default:
          if (cls == 3)
            hipLaunchKernelGGL(select_count_batched_kernel<64>, dim3(max_wgs, m), dim3(kGridThreads), 0, s, b);
          else
            hipLaunchKernelGGL(select_count_batched_kernel<kSample>, dim3(max_wgs, m), dim3(kGridThreads), 0, s, b);
          {
            const int rc = check_launch();
            if (rc != BSR_OK) return rc;
          }
          hipLaunchKernelGGL(select_classify_batched_kernel, dim3(max_wgs, m), dim3(kGridThreads), 0, s, b);
          {
            const int rc = check_launch();
            if (rc != BSR_OK) return rc;
          }
          hipLaunchKernelGGL(select_finish_batched_kernel, dim3(m), dim3(kGridThreads), 0, s, b);
          break;
      }
      m = 0;
      max_wgs = 0;
      return check_launch();
    };
    for (int i = 0; i < n; ++i) {
      const SelectJob &j = jobs[i];
      if (j.nblocks == 0) continue;
      const bool degenerate = j.n_keep <= 0 || j.n_keep >= j.nblocks;
      int c;
      if (degenerate) c = -1;
      else if (j.nblocks <= 1024) c = 0;
      else if (grid_wide_runs && j.nblocks > kRideAlong) c = 3;
      else if (j.nblocks <= 8192) c = 1;
      else if (j.nblocks <= kSmallLimit) c = 2;
      else if (j.nblocks <= 262144) c = 3;
      else c = 4;
      if (c == -1) {
        if (cls == 0) {                                      // all kept / none kept: a fill, once
          const int rc = launch_select(j.scores, j.nblocks, j.n_keep, j.mask, j.ws, s);
          if (rc != BSR_OK) return rc;
        }
        continue;
      }
      if (c != cls) continue;
      SelectItem &it = b.it[m];
      it.scores = j.scores;
      it.mask = j.mask;
      it.nblocks = (uint32_t)j.nblocks;
      it.n_keep = (uint32_t)j.n_keep;
      it.per_wg = 0;
      it.wgs = 1;
      it.counts = nullptr;
      it.ctrl = nullptr;
      it.cand_key = nullptr;
      it.cand_idx = nullptr;
      if (cls >= 3) {
        const SelectPlan p = select_plan(j.nblocks);
        char *base = static_cast<char *>(j.ws);
        it.counts = reinterpret_cast<uint32_t *>(base + p.counts_off);
        it.ctrl = reinterpret_cast<SelectCtrl *>(base + p.ctrl_off);
        it.cand_key = reinterpret_cast<uint64_t *>(base + p.key_off);
        it.cand_idx = reinterpret_cast<uint32_t *>(base + p.idx_off);
        int64_t wgs = ceil_div(j.nblocks, 1024);
        if (wgs > kMaxGridWgs) wgs = kMaxGridWgs;
        it.wgs = (uint32_t)wgs;
        it.per_wg = (uint32_t)ceil_div(j.nblocks, wgs);
        if (it.wgs > max_wgs) max_wgs = it.wgs;
      }
      if (++m == kBatchMax) {
        const int rc = flush();
        if (rc != BSR_OK) return rc;
      }
    }
    const int rc = flush();
    if (rc != BSR_OK) return rc;
  }
  return BSR_OK;
}

int launch_select_grouped_batched(const GroupedSelectJob *jobs, int n, hipStream_t s) {
  // classes by blocks per group: 0 <= 1024, 1 <= 8192, 2 <= kSmallLimit (one workgroup per group, the
  // tensors of a class share launches); a tensor of one group or of larger groups goes on its own
  for (int cls = 0; cls < 3; ++cls) {
    GroupBatch b;
    int m = 0;
    uint32_t wgs = 0;
    auto flush = [&]() -> int {
      if (m == 0) return BSR_OK;
      if (cls == 0)
        hipLaunchKernelGGL((select_groups_batched_kernel<256, 4, 8>), dim3(wgs), dim3(256), 0, s, b, m);
      else if (cls == 1)
        hipLaunchKernelGGL((select_groups_batched_kernel<1024, 8, kDigitBits>), dim3(wgs), dim3(1024), 0, s, b, m);
      else
        hipLaunchKernelGGL((select_groups_batched_kernel<1024, 12, kDigitBits>), dim3(wgs), dim3(1024), 0, s, b, m);
      m = 0;
      wgs = 0;
      return check_launch();
    };
    for (int i = 0; i < n; ++i) {
      const GroupedSelectJob &j = jobs[i];
      if (j.nbr == 0 || j.nbc == 0) continue;
      const int64_t groups = ceil_div(j.nbr, j.group_rows);
      const int64_t group_blocks = j.group_rows * j.nbc;
      const int c = groups == 1 || group_blocks > kSmallLimit ? -1 : (group_blocks <= 1024 ? 0 : (group_blocks <= 8192 ? 1 : 2));
      if (c == -1) {
        if (cls == 0) {
          const int rc = launch_select_grouped(j.scores, j.nbr, j.nbc, j.group_rows, j.n_keep_group, j.n_keep_last,
                                               j.mask, j.ws, s);
          if (rc != BSR_OK) return rc;
        }
        continue;
      }
      if (c != cls) continue;
      GroupItem &it = b.it[m];
      it.scores = j.scores;
      it.mask = j.mask;
      it.group_blocks = (uint32_t)group_blocks;
      it.n_keep_group = (uint32_t)j.n_keep_group;
      it.last_blocks = (uint32_t)((j.nbr - (groups - 1) * j.group_rows) * j.nbc);
      it.n_keep_last = (uint32_t)j.n_keep_last;
      it.groups = (uint32_t)groups;
      it.wg_begin = wgs;
      wgs += (uint32_t)groups;
      if (++m == kGroupBatchMax) {
        const int rc = flush();
        if (rc != BSR_OK) return rc;
      }
    }
    const int rc = flush();
    if (rc != BSR_OK) return rc;
  }
  return BSR_OK;
}

}  // namespace bsr
