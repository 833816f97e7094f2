// Dense -> BSR conversion and its inverse (paper Sec. II-A: crow / col / values;
// Sec. III: the saved activation is kept in that format).
//
//   index build : exclusive prefix sum of the keep mask in linear block order
//                 -> row_ptr (crow) and col_idx (col), one launch;
//   pack        : bit copy of the kept blocks into `values` (HBM-bound gather);
//   decompress  : BSR -> dense, pruned positions become +0.0.
// All three are pure data movement / integer work and are bit-exact.
#include <vector>

#include "common.h"

namespace bsr {

namespace {

constexpr int kIdxThreads = 256;

__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t x) {
  // bit 7 of every byte that is not zero
  return __popc((((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u);
}

// Workgroup w owns the linear block range [w*per_wg, (w+1)*per_wg).  It first
// counts the kept blocks in front of its range (every workgroup re-reads the
// mask prefix from L2: at most a few hundred KB, no second launch, no atomics),
// then scans its own range: thread t owns a contiguous chunk.
__global__ __launch_bounds__(kIdxThreads) void index_build_kernel(
    const uint8_t *__restrict__ mask, int64_t nblocks, int64_t nbr, int64_t nbc, int64_t n_keep,
    int64_t per_wg, int32_t *__restrict__ row_ptr, int32_t *__restrict__ col_idx) {
  __shared__ uint32_t wave_tot[kIdxThreads / 64];
  __shared__ uint32_t sh_prefix;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t lo = (int64_t)blockIdx.x * per_wg;
  const int64_t hi = (lo + per_wg) < nblocks ? (lo + per_wg) : nblocks;

  // ---- kept blocks in [0, lo) ----
  uint32_t cnt = 0;
  {
    const uintptr_t addr = reinterpret_cast<uintptr_t>(mask);
    int64_t head = (int64_t)((16 - (addr & 15)) & 15);
    if (head > lo) head = lo;
    const int64_t nvec = (lo - head) / 16;
    const int64_t tail0 = head + nvec * 16;
    if (t < head) cnt += mask[t] ? 1u : 0u;
    const uint4 *v = reinterpret_cast<const uint4 *>(mask + head);
    for (int64_t e = t; e < nvec; e += kIdxThreads) {
      const uint4 x = v[e];
      cnt += nonzero_bytes(x.x) + nonzero_bytes(x.y) + nonzero_bytes(x.z) + nonzero_bytes(x.w);
    }
    if (tail0 + t < lo) cnt += mask[tail0 + t] ? 1u : 0u;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
  if (lane == 0) wave_tot[wave] = cnt;
  __syncthreads();
  if (t == 0) {
    uint32_t p = 0;
    for (int w = 0; w < kIdxThreads / 64; ++w) p += wave_tot[w];
    sh_prefix = p;
  }
  __syncthreads();
  const uint32_t prefix = sh_prefix;
  __syncthreads();

  // ---- own range ----
  const int64_t chunk = ceil_div(per_wg, kIdxThreads);
  const int64_t b0 = lo + (int64_t)t * chunk;
  const int64_t b1 = (b0 + chunk) < hi ? (b0 + chunk) : hi;
  uint32_t mine = 0;
  for (int64_t b = b0; b < b1; ++b) mine += mask[b] ? 1u : 0u;
  uint32_t incl = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t o = __shfl_up(incl, d, 64);
    if (lane >= d) incl += o;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = prefix;
  for (int w = 0; w < wave; ++w) base += wave_tot[w];
  int64_t run = (int64_t)base + incl - mine;   // kept blocks before b0
  if (b0 < b1) {
    int64_t i = b0 / nbc, j = b0 % nbc;
    for (int64_t b = b0; b < b1; ++b) {
      if (j == 0) row_ptr[i] = (int32_t)run;
      if (mask[b]) {
        if (run < n_keep) col_idx[run] = (int32_t)j;
        ++run;
      }
      if (++j == nbc) { j = 0; ++i; }
    }
    if (b1 == nblocks) row_ptr[nbr] = (int32_t)run;
  }
}

__global__ void zero_row_ptr_kernel(int32_t *row_ptr, int64_t n) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * blockDim.x)
    row_ptr[i] = 0;
}

// Vector of VB bytes copied as a unit.
template <int VB> struct BytesOf;
template <> struct BytesOf<2> { typedef uint16_t type; };
template <> struct BytesOf<4> { typedef uint32_t type; };
template <> struct BytesOf<8> { typedef uint2 type; };
template <> struct BytesOf<16> { typedef uint4 type; };

template <int VB> __device__ __forceinline__ typename BytesOf<VB>::type zero_bytes();
template <> __device__ __forceinline__ uint16_t zero_bytes<2>() { return 0; }
template <> __device__ __forceinline__ uint32_t zero_bytes<4>() { return 0; }
template <> __device__ __forceinline__ uint2 zero_bytes<8>() { return make_uint2(0, 0); }
template <> __device__ __forceinline__ uint4 zero_bytes<16>() { return make_uint4(0, 0, 0, 0); }

// Gather: one workgroup per block-row (grid-stride), threads over
// (kept block, row, vector).  rowb / ldb / kb are in bytes.
template <int VB>
__global__ __launch_bounds__(256) void pack_kernel(
    const uint8_t *__restrict__ X, int64_t M, int64_t kb, int64_t ldb, int br, int64_t bcb,
    int64_t nbr, const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    int64_t n_keep, uint8_t *__restrict__ values) {
  typedef typename BytesOf<VB>::type V;
  const int vpb = (int)(bcb / VB);
  for (int64_t i = blockIdx.x; i < nbr; i += gridDim.x) {
    int64_t p0 = row_ptr[i], p1 = row_ptr[i + 1];
    if (p1 > n_keep) p1 = n_keep;
    const int64_t work = (p1 - p0) * br * vpb;
    for (int64_t f = threadIdx.x; f < work; f += blockDim.x) {
      const int v = (int)(f % vpb);
      const int r = (int)((f / vpb) % br);
      const int64_t q = f / ((int64_t)vpb * br);
      const int64_t j = col_idx[p0 + q];
      const int64_t m = i * br + r;
      const int64_t cb = j * bcb + (int64_t)v * VB;
      V val = zero_bytes<VB>();
      if (m < M && cb < kb) val = *reinterpret_cast<const V *>(X + m * ldb + cb);
      *reinterpret_cast<V *>(values + ((p0 + q) * br + r) * bcb + (int64_t)v * VB) = val;
    }
  }
}

constexpr int kFusedCols = 4096;   // block-columns per block-row the fused kernel can list in LDS

// Kept blocks in mask[0, n): 16-byte loads, every thread returns the total.
__device__ __forceinline__ uint32_t count_kept_prefix(const uint8_t *__restrict__ mask, int64_t n,
                                                      uint32_t *wave_tot, uint32_t *total) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  uint32_t cnt = 0;
  const uintptr_t addr = reinterpret_cast<uintptr_t>(mask);
  int64_t head = (int64_t)((16 - (addr & 15)) & 15);
  if (head > n) head = n;
  const int64_t nvec = (n - head) / 16;
  const int64_t tail0 = head + nvec * 16;
  if (t < head) cnt += mask[t] ? 1u : 0u;
  const uint4 *v = reinterpret_cast<const uint4 *>(mask + head);
#pragma unroll 4
  for (int64_t e = t; e < nvec; e += 256) {
    const uint4 x = v[e];
    cnt += nonzero_bytes(x.x) + nonzero_bytes(x.y) + nonzero_bytes(x.z) + nonzero_bytes(x.w);
  }
  if (tail0 + t < n) cnt += mask[tail0 + t] ? 1u : 0u;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
  if (lane == 0) wave_tot[wave] = cnt;
  __syncthreads();
  if (t == 0) *total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
  __syncthreads();
  const uint32_t r = *total;
  __syncthreads();
  return r;
}

// Mask -> BSR in one launch: workgroup i owns block-row i.  It counts the kept
// blocks in front of its row (the mask prefix comes from L2: a few dozen KB), lists
// the row's kept block-columns (row_ptr / col_idx and an LDS copy), then copies the
// kept blocks.  Thread -> (row, vector) inside a block is fixed up front, so the
// copy loops do no division.  Positions at or beyond n_keep are never written.
// What one tensor's launch needs (kernel arguments; an array of these for several tensors per
// launch).  kb, ldb, bcb: row length, row pitch and block row length in bytes.
struct CompressArgs {
  const uint8_t *mask, *X;
  int32_t *row_ptr, *col_idx;
  uint8_t *values;
  int64_t M, kb, ldb, bcb, nbr, nbc, n_keep;
  int br;
  uint32_t wg_begin;       // first workgroup of this tensor in a launch of several
  int have_row_ptr;        // row_ptr was written by row_ptr_batched_kernel: nothing to count here
};

// i = block-row (the workgroup's number among those of its tensor)
template <int VB>
__device__ __forceinline__ void compress_body(const CompressArgs &a, const int64_t i) {
  typedef typename BytesOf<VB>::type V;
  const uint8_t *__restrict__ mask = a.mask;
  const uint8_t *__restrict__ X = a.X;
  int32_t *__restrict__ row_ptr = a.row_ptr;
  int32_t *__restrict__ col_idx = a.col_idx;
  uint8_t *__restrict__ values = a.values;
  const int64_t M = a.M, kb = a.kb, ldb = a.ldb, bcb = a.bcb, nbr = a.nbr, nbc = a.nbc, n_keep = a.n_keep;
  const int br = a.br;
  __shared__ uint32_t wave_tot[4];
  __shared__ uint32_t total;
  __shared__ int32_t kept_j[kFusedCols];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const uint32_t prefix = a.have_row_ptr ? (uint32_t)row_ptr[i] : count_kept_prefix(mask, i * nbc, wave_tot, &total);

  // ---- this row's kept block-columns, in order ----
  uint32_t row_kept = 0;
  const uint8_t *mrow = mask + i * nbc;
  for (int64_t c0 = 0; c0 < nbc; c0 += 256) {
    const int64_t j = c0 + t;
    const bool flag = j < nbc && mrow[j] != 0;
    const unsigned long long ball = __ballot(flag);
    if (lane == 0) wave_tot[wave] = (uint32_t)__popcll(ball);
    __syncthreads();
    uint32_t before = row_kept;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    const uint32_t pos = before + (uint32_t)__popcll(ball & ((1ull << lane) - 1ull));
    if (flag) {
      kept_j[pos] = (int32_t)j;
      if ((int64_t)prefix + pos < n_keep) col_idx[prefix + pos] = (int32_t)j;
    }
    row_kept += wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    __syncthreads();
  }
  if (t == 0 && !a.have_row_ptr) {
    row_ptr[i] = (int32_t)prefix;
    if (i == nbr - 1) row_ptr[nbr] = (int32_t)(prefix + row_kept);
  }
  int64_t nk = row_kept;                                   // blocks of this row that have a place in `values`
  if ((int64_t)prefix + nk > n_keep) nk = n_keep > (int64_t)prefix ? n_keep - prefix : 0;
  if (nk == 0) return;

  // ---- copy ----
  const int vpb = (int)(bcb / VB);
  const int S = br * vpb;                                  // vectors per block
  const uint8_t *xrow = X + i * br * ldb;
  uint8_t *vrow = values + (int64_t)prefix * S * VB;
  const int64_t rows_left = M - i * br;
  auto copy = [&](int q, int r, int v, int e) {
    const int64_t cb = (int64_t)kept_j[q] * bcb + (int64_t)v * VB;
    V val = zero_bytes<VB>();
    if (r < rows_left && cb < kb) val = *reinterpret_cast<const V *>(xrow + (int64_t)r * ldb + cb);
    store_stream(reinterpret_cast<V *>(vrow + ((int64_t)q * S + e) * VB), val);
  };
  if (S <= 256) {
    const int G = 256 / S, g = t / S, e = t - g * S;      // G blocks per pass
    if (g < G) {
      const int r = e / vpb, v = e - r * vpb;
#pragma unroll 4
      for (int q = g; q < (int)nk; q += G) copy(q, r, v, e);
    }
  } else {
    for (int e = t; e < S; e += 256) {
      const int r = e / vpb, v = e - r * vpb;
#pragma unroll 4
      for (int q = 0; q < (int)nk; ++q) copy(q, r, v, e);
    }
  }
}

template <int VB>
__global__ __launch_bounds__(256) void compress_kernel(CompressArgs a) {
  compress_body<VB>(a, blockIdx.x);
}

// Several tensors per launch: tensor k owns the workgroups [wg_begin_k, wg_begin_{k+1}).
constexpr int kPackBatchMax = 24;
struct CompressBatch {
  CompressArgs it[kPackBatchMax];
};
template <int VB>
__global__ __launch_bounds__(256) void compress_batched_kernel(CompressBatch b, int n) {
  int k = 0;
  while (k + 1 < n && blockIdx.x >= b.it[k + 1].wg_begin) ++k;
  compress_body<VB>(b.it[k], blockIdx.x - b.it[k].wg_begin);
}

constexpr int kMapCols = 1024;   // block-columns per workgroup in decompress

// Scatter: a workgroup owns block-row i and a chunk of kMapCols block-columns;
// an LDS table maps block-column -> position in `values` (or -1 = pruned).  The
// 64 lanes of a wave run along the matrix row (1 KB stores), the four waves take
// every fourth row; a lane looks its vector's block up once and then walks down
// the rows with all loads of a batch in flight: no division in the copy loop.
struct DecompressArgs {
  const int32_t *row_ptr, *col_idx;
  const uint8_t *values;
  uint8_t *X_out;
  int64_t M, kb, ldb, bcb, nbr, nbc;
  int br;
  uint32_t gx, gy;         // the tensor's grid: chunks of block-columns x workgroups striding over block-rows
  uint32_t wg_begin;       // first workgroup of this tensor in a launch of several
};

// bx, by: the workgroup's place in its tensor's gx x gy grid
template <int VB>
__device__ __forceinline__ void decompress_body(const DecompressArgs &a, const uint32_t bx, const uint32_t by) {
  typedef typename BytesOf<VB>::type V;
  const int32_t *__restrict__ row_ptr = a.row_ptr;
  const int32_t *__restrict__ col_idx = a.col_idx;
  const uint8_t *__restrict__ values = a.values;
  uint8_t *__restrict__ X_out = a.X_out;
  const int64_t M = a.M, kb = a.kb, ldb = a.ldb, bcb = a.bcb, nbr = a.nbr, nbc = a.nbc;
  const int br = a.br;
  __shared__ int32_t slot[kMapCols];
  const int t = threadIdx.x, lane = t & 63, rg = t >> 6;
  const int64_t j0 = (int64_t)bx * kMapCols;
  const int ncols = (int)((nbc - j0) < kMapCols ? (nbc - j0) : kMapCols);
  const int vpb = (int)(bcb / VB);
  const int vrow = ncols * vpb;                            // vectors per matrix row in the chunk
  const int64_t block_bytes = (int64_t)br * bcb;
  constexpr int kInFlight = 8;
  for (int64_t i = by; i < nbr; i += a.gy) {
    for (int c = t; c < ncols; c += 256) slot[c] = -1;
    __syncthreads();
    const int64_t p0 = row_ptr[i], p1 = row_ptr[i + 1];
    for (int64_t p = p0 + t; p < p1; p += 256) {
      const int64_t j = col_idx[p];
      if (j >= j0 && j < j0 + ncols) slot[j - j0] = (int32_t)p;
    }
    __syncthreads();
    const int rows = (int)((M - i * br) < br ? (M - i * br) : br);
    uint8_t *orow = X_out + i * br * ldb + j0 * bcb;
    for (int w = lane; w < vrow; w += 64) {
      const int c = w / vpb, v = w - c * vpb;
      const int64_t cb = (int64_t)c * bcb + (int64_t)v * VB;      // byte column inside the chunk
      if (j0 * bcb + cb >= kb) continue;
      const int32_t p = slot[c];
      const uint8_t *src = values + (int64_t)(p < 0 ? 0 : p) * block_bytes + (int64_t)v * VB;
      for (int r0 = rg; r0 < rows; r0 += 4 * kInFlight) {
        V val[kInFlight];
#pragma unroll
        for (int b = 0; b < kInFlight; ++b) {
          const int r = r0 + 4 * b;
          val[b] = zero_bytes<VB>();
          if (p >= 0 && r < rows) val[b] = *reinterpret_cast<const V *>(src + (int64_t)r * bcb);
        }
#pragma unroll
        for (int b = 0; b < kInFlight; ++b) {
          const int r = r0 + 4 * b;
          if (r < rows) store_stream(reinterpret_cast<V *>(orow + (int64_t)r * ldb + cb), val[b]);
        }
      }
    }
    __syncthreads();
  }
}

template <int VB>
__global__ __launch_bounds__(256) void decompress_kernel(DecompressArgs a) {
  decompress_body<VB>(a, blockIdx.x, blockIdx.y);
}

struct DecompressBatch {
  DecompressArgs it[kPackBatchMax];
};
template <int VB>
__global__ __launch_bounds__(256) void decompress_batched_kernel(DecompressBatch b, int n) {
  int k = 0;
  while (k + 1 < n && blockIdx.x >= b.it[k + 1].wg_begin) ++k;
  const uint32_t local = blockIdx.x - b.it[k].wg_begin;
  decompress_body<VB>(b.it[k], local % b.it[k].gx, local / b.it[k].gx);
}

// ---- narrow blocks: whole block-rows staged in LDS ----
//
// A workgroup owns g.rb consecutive block-rows, whose matrix rows are one contiguous
// span of memory.  The dense side is moved with wide linear accesses (every byte of
// a cache line used by one instruction), the BSR side as one contiguous run of
// 32-bit words (the kept blocks of consecutive block-rows follow each other in
// `values`), and the re-ordering between the two happens in LDS.  Word w of the run
// belongs to kept block q = w / blk_words, row r and word c of that row; base[q] is
// the block's first word in the span, lim[q] its valid rows and words (ragged edges).
// LDS layout: span | base | lim, sized by the launcher.

__device__ __forceinline__ void span_decode(const SpanGeom &g, uint32_t w, uint32_t *q, uint32_t *r, uint32_t *c) {
  *q = span_div(w, (uint32_t)g.blk_words, g.magic_blk);
  const uint32_t rem = w - *q * (uint32_t)g.blk_words;
  *r = span_div(rem, (uint32_t)g.seg_words, g.magic_seg);
  *c = rem - *r * (uint32_t)g.seg_words;
}

__device__ __forceinline__ uint32_t span_lim(const SpanGeom &g, int rows, uint32_t b, uint32_t j) {
  const int rv = rows - (int)b * g.br < g.br ? rows - (int)b * g.br : g.br;
  const int cv = g.row_words - (int)j * g.seg_words < g.seg_words ? g.row_words - (int)j * g.seg_words : g.seg_words;
  return ((uint32_t)rv << 16) | (uint32_t)cv;
}

// BSR side of a workgroup: word w of the run comes from the span (0 outside the matrix)
__device__ __forceinline__ void span_write_run(const SpanGeom &g, const uint32_t *span, const uint32_t *base,
                                               const uint32_t *lim, uint32_t total_w, uint32_t *__restrict__ out) {
#pragma unroll 4
  for (uint32_t w = threadIdx.x; w < total_w; w += 256) {
    uint32_t q, r, c;
    span_decode(g, w, &q, &r, &c);
    const uint32_t l = lim[q];
    uint32_t val = 0;
    if (r < (l >> 16) && c < (l & 0xFFFFu)) val = span[base[q] + r * g.row_words + c];
    store_stream(out + w, val);
  }
}

inline size_t span_lds_words(const SpanGeom &g) { return align_up((size_t)g.rb * g.br * g.row_words, 4); }

// Kept blocks of every workgroup's mask range (per_wg = rb * nbc <= kSpanList bytes): one wave per range.
__global__ __launch_bounds__(256) void span_count_kernel(const uint8_t *__restrict__ mask, int64_t nblocks,
                                                         int per_wg, int64_t wgs, uint32_t *__restrict__ wg_kept) {
  const int lane = threadIdx.x & 63;
  const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= wgs) return;
  const int64_t e0 = w * per_wg;
  const int n = (int)((nblocks - e0) < per_wg ? (nblocks - e0) : per_wg);
  uint32_t cnt = 0;
#pragma unroll 4
  for (int e = lane; e < n; e += 64) cnt += mask[e0 + e] != 0 ? 1u : 0u;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
  if (lane == 0) wg_kept[w] = cnt;
}

// row_ptr of several tensors in one launch, one workgroup of 1024 threads per tensor: the mask is
// read front to back, 16 blocks per thread and pass, with a running count of the kept blocks in
// front of every block (lane exchanges inside a wave, the waves' totals through LDS); the thread
// that holds the first block of a block-row writes that row's entry.  With row_ptr at hand the
// conversion kernels need not count the mask in front of their rows (every workgroup on its own,
// out of L2: more bytes than the tensor itself for narrow blocks).
constexpr int kRowPtrThreads = 1024;
constexpr int kRowPtrBatchMax = 40;
constexpr int64_t kRowPtrMaxBlocks = int64_t(1) << 22;     // one workgroup reads the whole mask
struct RowPtrItem {
  const uint8_t *mask;
  int32_t *row_ptr;
  int64_t nbr, nbc;
};
struct RowPtrBatch {
  RowPtrItem it[kRowPtrBatchMax];
};
__global__ __launch_bounds__(kRowPtrThreads) void row_ptr_batched_kernel(RowPtrBatch b) {
  const RowPtrItem &it = b.it[blockIdx.x];
  const uint8_t *__restrict__ mask = it.mask;
  int32_t *__restrict__ row_ptr = it.row_ptr;
  const uint32_t nbc = (uint32_t)it.nbc;
  const uint32_t nblocks = (uint32_t)(it.nbr * it.nbc);
  constexpr int kPer = 16;                                  // blocks per thread and pass
  __shared__ uint32_t wave_tot[2][kRowPtrThreads / 64];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  uint32_t base = 0;                                        // kept blocks in front of this pass
  const bool aligned = reinterpret_cast<uintptr_t>(mask) % 16 == 0;
  int phase = 0;
  for (uint32_t e0 = 0; e0 < nblocks; e0 += kPer * kRowPtrThreads, phase ^= 1) {
    const uint32_t first = e0 + (uint32_t)t * kPer;
    uint8_t f[kPer];
    if (aligned && first + kPer <= nblocks) {
      const uint4 v = *reinterpret_cast<const uint4 *>(mask + first);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < kPer; ++k) f[k] = (uint8_t)(w[k >> 2] >> (8 * (k & 3)));
    } else {
#pragma unroll
      for (int k = 0; k < kPer; ++k) f[k] = first + k < nblocks ? mask[first + k] : (uint8_t)0;
    }
    uint32_t mine = 0;
#pragma unroll
    for (int k = 0; k < kPer; ++k) mine += f[k] != 0 ? 1u : 0u;
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[phase][wave] = incl;
    __syncthreads();
    uint32_t before = base, all = 0;
#pragma unroll
    for (int w = 0; w < kRowPtrThreads / 64; ++w) {
      if (w < wave) before += wave_tot[phase][w];
      all += wave_tot[phase][w];
    }
    uint32_t run = before + incl - mine;
    if (first < nblocks) {
      uint32_t r = first / nbc, c = first - r * nbc;        // block-row and column of the thread's first block
#pragma unroll
      for (int k = 0; k < kPer; ++k) {
        if (first + k < nblocks) {
          if (c == 0) row_ptr[r] = (int32_t)run;
          run += f[k] != 0 ? 1u : 0u;
          if (++c == nbc) { c = 0; ++r; }
        }
      }
    }
    base += all;
  }
  if (t == 0) row_ptr[it.nbr] = (int32_t)base;
}

struct CompressSpanArgs {
  const uint8_t *mask, *X;
  const uint32_t *wg_kept;  // kept blocks of every workgroup's mask range, or null (see span_count_kernel)
  int32_t *row_ptr, *col_idx;
  uint32_t *values;
  int64_t M, nbr, n_keep;
  SpanGeom g;
  uint32_t span_words;
  uint32_t wg_begin;        // first workgroup of this tensor in a launch of several
  int have_row_ptr;         // row_ptr was written by row_ptr_batched_kernel: nothing to count here
};

// wg = the workgroup's number among those of its tensor
template <int VB>
__device__ __forceinline__ void compress_span_body(const CompressSpanArgs &a, const uint32_t wg) {
  typedef typename BytesOf<VB>::type V;
  constexpr int kVecs = kSpanBytes / VB / 256;
  const uint8_t *__restrict__ mask = a.mask;
  const uint8_t *__restrict__ X = a.X;
  const uint32_t *__restrict__ wg_kept = a.wg_kept;
  int32_t *__restrict__ row_ptr = a.row_ptr;
  int32_t *__restrict__ col_idx = a.col_idx;
  uint32_t *__restrict__ values = a.values;
  const int64_t M = a.M, nbr = a.nbr, n_keep = a.n_keep;
  const SpanGeom &g = a.g;
  const size_t span_words = a.span_words;
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  uint32_t *span = lds, *base = lds + span_words, *lim = base + g.rb * g.nbc;
  __shared__ uint32_t wave_tot[4];
  __shared__ uint32_t total;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t i0 = (int64_t)wg * g.rb;
  const int nb = (int)((nbr - i0) < g.rb ? (nbr - i0) : g.rb);
  const int64_t m0 = i0 * g.br;
  const int rows = (int)((M - m0) < (int64_t)nb * g.br ? (M - m0) : (int64_t)nb * g.br);
  const int nvec = rows * g.row_words * 4 / VB;
  // the span's loads go out first: the mask work below hides their latency
  const V *src = reinterpret_cast<const V *>(X + m0 * g.row_words * 4);
  V reg[kVecs];
#pragma unroll
  for (int k = 0; k < kVecs; ++k) {
    reg[k] = zero_bytes<VB>();
    if (t + 256 * k < nvec) reg[k] = src[t + 256 * k];
  }
  // kept blocks in front of this workgroup: from the mask itself, or from the per-workgroup
  // counts of span_count_kernel when the mask is too long to re-read in every workgroup
  uint32_t prefix;
  if (a.have_row_ptr) {
    prefix = (uint32_t)row_ptr[i0];
  } else if (wg_kept == nullptr) {
    prefix = count_kept_prefix(mask, i0 * g.nbc, wave_tot, &total);
  } else {
    uint32_t cnt = 0;
    for (uint32_t w = t; w < wg; w += 256) cnt += wg_kept[w];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) cnt += __shfl_xor(cnt, d, 64);
    if (lane == 0) wave_tot[wave] = cnt;
    __syncthreads();
    prefix = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    __syncthreads();
  }

  // ---- kept blocks of these block-rows, in order ----
  const int nblk = nb * g.nbc;
  const uint8_t *mrow = mask + i0 * g.nbc;
  uint32_t kept = 0;
  for (int c0 = 0; c0 < nblk; c0 += 256) {
    const int idx = c0 + t;
    const bool flag = idx < nblk && mrow[idx] != 0;
    const unsigned long long ball = __ballot(flag);
    if (lane == 0) wave_tot[wave] = (uint32_t)__popcll(ball);
    __syncthreads();
    uint32_t before = kept;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    const uint32_t pos = before + (uint32_t)__popcll(ball & ((1ull << lane) - 1ull));
    if (idx < nblk) {
      const uint32_t b = span_div((uint32_t)idx, (uint32_t)g.nbc, g.magic_nbc), j = (uint32_t)idx - b * g.nbc;
      if (j == 0 && !a.have_row_ptr) row_ptr[i0 + b] = (int32_t)(prefix + pos);
      if (flag) {
        base[pos] = b * g.br * g.row_words + j * g.seg_words;
        lim[pos] = span_lim(g, rows, b, j);
        if ((int64_t)prefix + pos < n_keep) col_idx[prefix + pos] = (int32_t)j;
      }
    }
    kept += wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    __syncthreads();
  }
  if (t == 0 && i0 + nb == nbr && !a.have_row_ptr) row_ptr[nbr] = (int32_t)(prefix + kept);
  V *sv = reinterpret_cast<V *>(span);
#pragma unroll
  for (int k = 0; k < kVecs; ++k)
    if (t + 256 * k < nvec) sv[t + 256 * k] = reg[k];
  __syncthreads();
  int64_t nk = kept;                                       // blocks that have a place in `values`
  if ((int64_t)prefix + nk > n_keep) nk = n_keep > (int64_t)prefix ? n_keep - prefix : 0;
  span_write_run(g, span, base, lim, (uint32_t)nk * (uint32_t)g.blk_words, values + (int64_t)prefix * g.blk_words);
}

template <int VB>
__global__ __launch_bounds__(256) void compress_span_kernel(CompressSpanArgs a) {
  compress_span_body<VB>(a, blockIdx.x);
}

struct CompressSpanBatch {
  CompressSpanArgs it[kPackBatchMax];
};
template <int VB>
__global__ __launch_bounds__(256) void compress_span_batched_kernel(CompressSpanBatch b, int n) {
  int k = 0;
  while (k + 1 < n && blockIdx.x >= b.it[k + 1].wg_begin) ++k;
  compress_span_body<VB>(b.it[k], blockIdx.x - b.it[k].wg_begin);
}

struct DecompressSpanArgs {
  const int32_t *row_ptr, *col_idx;
  const uint32_t *values;
  uint8_t *X_out;
  int64_t M, nbr;
  SpanGeom g;
  uint32_t span_words;
  uint32_t wg_begin;        // first workgroup of this tensor in a launch of several
};

template <int VB>
__device__ __forceinline__ void decompress_span_body(const DecompressSpanArgs &a, const uint32_t wg) {
  typedef typename BytesOf<VB>::type V;
  constexpr int kVecs = kSpanBytes / VB / 256;
  constexpr int kWords = kSpanBytes / 4 / 256;
  const int32_t *__restrict__ row_ptr = a.row_ptr;
  const int32_t *__restrict__ col_idx = a.col_idx;
  const uint32_t *__restrict__ values = a.values;
  uint8_t *__restrict__ X_out = a.X_out;
  const int64_t M = a.M, nbr = a.nbr;
  const SpanGeom &g = a.g;
  const size_t span_words = a.span_words;
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  uint32_t *span = lds, *base = lds + span_words, *lim = base + g.rb * g.nbc;
  __shared__ int32_t rp[kSpanRows + 2];
  const int t = threadIdx.x;
  const int64_t i0 = (int64_t)wg * g.rb;
  const int nb = (int)((nbr - i0) < g.rb ? (nbr - i0) : g.rb);
  const int64_t m0 = i0 * g.br;
  const int rows = (int)((M - m0) < (int64_t)nb * g.br ? (M - m0) : (int64_t)nb * g.br);
  const int nvec = rows * g.row_words * 4 / VB;
  if (t <= nb) rp[t] = row_ptr[i0 + t];
  __syncthreads();
  const int64_t p0 = rp[0];
  int nk = rp[nb] - rp[0];
  if (nk < 0) nk = 0;
  if (nk > nb * g.nbc) nk = nb * g.nbc;                    // a well-formed row_ptr never exceeds this
  // the kept blocks of these block-rows: one contiguous run, all loads in flight
  const uint32_t total_w = (uint32_t)nk * (uint32_t)g.blk_words;
  const uint32_t *vsrc = values + p0 * g.blk_words;
  uint32_t reg[kWords];
#pragma unroll
  for (int k = 0; k < kWords; ++k) {
    reg[k] = 0;
    if ((uint32_t)(t + 256 * k) < total_w) reg[k] = vsrc[t + 256 * k];
  }
  uint4 *s4 = reinterpret_cast<uint4 *>(span);
  for (int v = t; v < (rows * g.row_words + 3) / 4; v += 256) s4[v] = make_uint4(0, 0, 0, 0);
  for (int q = t; q < nk; q += 256) {
    const int64_t p = p0 + q;
    uint32_t b = 0;
    while ((int)b + 1 < nb && p >= rp[b + 1]) ++b;
    const int32_t j = col_idx[p];
    const bool ok = j >= 0 && j < g.nbc;
    base[q] = ok ? b * g.br * g.row_words + (uint32_t)j * g.seg_words : 0u;
    lim[q] = ok ? span_lim(g, rows, b, (uint32_t)j) : 0u;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kWords; ++k) {
    const uint32_t w = (uint32_t)(t + 256 * k);
    if (w < total_w) {
      uint32_t q, r, c;
      span_decode(g, w, &q, &r, &c);
      const uint32_t l = lim[q];
      if (r < (l >> 16) && c < (l & 0xFFFFu)) span[base[q] + r * g.row_words + c] = reg[k];
    }
  }
  __syncthreads();
  const V *sv = reinterpret_cast<const V *>(span);
  V *dst = reinterpret_cast<V *>(X_out + m0 * g.row_words * 4);
#pragma unroll
  for (int k = 0; k < kVecs; ++k)
    if (t + 256 * k < nvec) store_stream(dst + t + 256 * k, sv[t + 256 * k]);
}

template <int VB>
__global__ __launch_bounds__(256) void decompress_span_kernel(DecompressSpanArgs a) {
  decompress_span_body<VB>(a, blockIdx.x);
}

struct DecompressSpanBatch {
  DecompressSpanArgs it[kPackBatchMax];
};
template <int VB>
__global__ __launch_bounds__(256) void decompress_span_batched_kernel(DecompressSpanBatch b, int n) {
  int k = 0;
  while (k + 1 < n && blockIdx.x >= b.it[k + 1].wg_begin) ++k;
  decompress_span_body<VB>(b.it[k], blockIdx.x - b.it[k].wg_begin);
}

// Widest byte vector that divides every extent and alignment involved.
int pick_bytes(int esize, int bc, int64_t K, int64_t ld, const void *a, const void *b) {
  int vb = 16;
  while (vb > esize) {
    const bool ok = ((int64_t)bc * esize) % vb == 0 && (K * esize) % vb == 0 && (ld * esize) % vb == 0 &&
                    (uintptr_t)a % vb == 0 && (uintptr_t)b % vb == 0;
    if (ok) break;
    vb >>= 1;
  }
  return vb;
}

}  // namespace

bool span_geometry(int dtype, int64_t M, int64_t K, int64_t ld, int br, int bc, const void *p0,
                   const void *p1, SpanGeom *g) {
  const int e = elem_bytes(dtype);
  if (M <= 0 || K <= 0 || ld != K) return false;
  const int64_t rowb = K * e, segb = (int64_t)bc * e;
  if (rowb % 4 != 0 || segb % 4 != 0) return false;
  // blocks of 8 or more rows whose rows take 16-byte vectors are served by the direct kernels
  if (segb % 16 == 0 && rowb % 16 == 0 && br >= 8) return false;
  if ((uintptr_t)p0 % 16 != 0 || (uintptr_t)p1 % 16 != 0) return false;
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  // a block-row padded to whole blocks must fit the span (bounds the BSR run of a workgroup as well)
  const int64_t brow_bytes = (int64_t)br * nbc * segb;
  if (brow_bytes > kSpanBytes || nbc > kSpanList) return false;
  int64_t rb = kSpanBytes / brow_bytes;
  if (rb > kSpanRows) rb = kSpanRows;
  if (rb > kSpanList / nbc) rb = kSpanList / nbc;
  if (rb > nbr) rb = nbr;
  g->rb = (int)rb;
  g->br = br;
  g->nbc = (int)nbc;
  g->row_words = (int)(rowb / 4);
  g->seg_words = (int)(segb / 4);
  g->blk_words = br * g->seg_words;
  g->vb = rowb % 16 == 0 ? 16 : rowb % 8 == 0 ? 8 : 4;
  auto magic = [](uint32_t d) { return (uint32_t)(((uint64_t(1) << 32) + d - 1) / d); };
  g->magic_blk = magic((uint32_t)g->blk_words);
  g->magic_seg = magic((uint32_t)g->seg_words);
  g->magic_nbc = magic((uint32_t)g->nbc);
  g->magic_br = magic((uint32_t)br);
  return true;
}

int launch_index_build(const uint8_t *keep_mask, int64_t nbr, int64_t nbc, int64_t n_keep,
                       int32_t *row_ptr, int32_t *col_idx, hipStream_t s) {
  const int64_t nblocks = nbr * nbc;
  if (nblocks == 0) {
    hipLaunchKernelGGL(zero_row_ptr_kernel, dim3(1), dim3(64), 0, s, row_ptr, nbr + 1);
    return check_launch();
  }
  int64_t wgs = ceil_div(nblocks, 2048);
  if (wgs > 128) wgs = 128;
  const int64_t per_wg = ceil_div(nblocks, wgs);
  hipLaunchKernelGGL(index_build_kernel, dim3((unsigned)wgs), dim3(kIdxThreads), 0, s, keep_mask,
                     nblocks, nbr, nbc, n_keep, per_wg, row_ptr, col_idx);
  return check_launch();
}

int launch_pack(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                const int32_t *row_ptr, const int32_t *col_idx, int64_t n_keep, void *values,
                hipStream_t s) {
  if (n_keep == 0 || M == 0 || K == 0) return BSR_OK;
  const int e = elem_bytes(dtype);
  const int64_t nbr = ceil_div(M, br);
  const int vb = pick_bytes(e, bc, K, ldx, X, values);
  const unsigned grid = (unsigned)(nbr < 8192 ? nbr : 8192);
  const uint8_t *x = static_cast<const uint8_t *>(X);
  uint8_t *v = static_cast<uint8_t *>(values);
#define BSR_PACK(VB)                                                                             \
  hipLaunchKernelGGL((pack_kernel<VB>), dim3(grid), dim3(256), 0, s, x, M, K * e, ldx * e, br,  \
                     (int64_t)bc * e, nbr, row_ptr, col_idx, n_keep, v)
  switch (vb) {
    case 16: BSR_PACK(16); break;
    case 8: BSR_PACK(8); break;
    case 4: BSR_PACK(4); break;
    default: BSR_PACK(2); break;
  }
#undef BSR_PACK
  return check_launch();
}

size_t compress_ws_bytes(int dtype, int64_t M, int64_t K, int br, int bc) {
  SpanGeom g;
  if (!span_geometry(dtype, M, K, K, br, bc, nullptr, nullptr, &g)) return 0;
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  const int64_t wgs = ceil_div(nbr, g.rb);
  if (wgs * (nbr * nbc / 2) <= (int64_t(64) << 20)) return 0;      // every workgroup re-counts the mask prefix
  return align_up((size_t)wgs * sizeof(uint32_t), 256);
}

namespace {

// How one tensor is converted: the kernel family, its vector width and its arguments.
enum { kPackSpan = 0, kPackDirect = 1, kPackOther = 2 };
struct CompressPlan {
  int path, vb;
  bool count_first;          // span path: a first launch counts every workgroup's kept blocks
  unsigned wgs;
  size_t lds;
  CompressArgs direct;
  CompressSpanArgs span;
};

CompressPlan plan_compress(const CompressJob &j, int dtype) {
  CompressPlan p{};
  const int64_t nbr = ceil_div(j.M, j.br), nbc = ceil_div(j.K, j.bc);
  const int e = elem_bytes(dtype);
  SpanGeom g;
  if (nbr > 0 && nbc > 0 && (uintptr_t)j.values % 4 == 0 &&
      span_geometry(dtype, j.M, j.K, j.ldx, j.br, j.bc, j.X, nullptr, &g)) {
    p.path = kPackSpan;
    p.vb = g.vb;
    const size_t span_words = span_lds_words(g);
    p.lds = (span_words + 2 * (size_t)g.rb * g.nbc) * 4;
    p.wgs = (unsigned)ceil_div(nbr, g.rb);
    // one launch if re-counting the mask prefix in every workgroup stays cheap (bytes out of
    // L2); else a first launch counts every workgroup's kept blocks into the workspace
    p.count_first = compress_ws_bytes(dtype, j.M, j.K, j.br, j.bc) != 0;
    p.span = CompressSpanArgs{j.keep_mask, static_cast<const uint8_t *>(j.X),
                              p.count_first ? static_cast<const uint32_t *>(j.ws) : nullptr, j.row_ptr, j.col_idx,
                              static_cast<uint32_t *>(j.values), j.M, nbr, j.n_keep, g, (uint32_t)span_words, 0u, 0};
    return p;
  }
  // one fused launch when a block-row's columns fit its LDS list and re-reading the
  // mask prefix in every workgroup stays cheap (nbr * nblocks / 2 bytes out of L2)
  const bool fused = nbr > 0 && nbc > 0 && nbc <= kFusedCols && nbr <= 65535 &&
                     nbr * nbr * nbc <= (int64_t(1) << 31);
  if (!fused) {
    p.path = kPackOther;
    return p;
  }
  p.path = kPackDirect;
  p.vb = pick_bytes(e, j.bc, j.K, j.ldx, j.X, j.values);
  p.wgs = (unsigned)nbr;
  p.direct = CompressArgs{j.keep_mask, static_cast<const uint8_t *>(j.X), j.row_ptr, j.col_idx,
                          static_cast<uint8_t *>(j.values), j.M, j.K * e, j.ldx * e, (int64_t)j.bc * e, nbr, nbc,
                          j.n_keep, j.br, 0u, 0};
  return p;
}

struct DecompressPlan {
  int path, vb;
  unsigned wgs;
  size_t lds;
  DecompressArgs direct;
  DecompressSpanArgs span;
};

DecompressPlan plan_decompress(const DecompressJob &j, int dtype) {
  DecompressPlan p{};
  const int e = elem_bytes(dtype);
  const int64_t nbr = ceil_div(j.M, j.br), nbc = ceil_div(j.K, j.bc);
  SpanGeom g;
  if ((uintptr_t)j.values % 4 == 0 && span_geometry(dtype, j.M, j.K, j.ldx, j.br, j.bc, j.X_out, nullptr, &g)) {
    p.path = kPackSpan;
    p.vb = g.vb;
    const size_t span_words = span_lds_words(g);
    p.lds = (span_words + 2 * (size_t)g.rb * g.nbc) * 4;
    p.wgs = (unsigned)ceil_div(nbr, g.rb);
    p.span = DecompressSpanArgs{j.row_ptr, j.col_idx, static_cast<const uint32_t *>(j.values),
                                static_cast<uint8_t *>(j.X_out), j.M, nbr, g, (uint32_t)span_words, 0u};
    return p;
  }
  p.path = kPackDirect;
  p.vb = pick_bytes(e, j.bc, j.K, j.ldx, j.X_out, j.values);
  const unsigned gx = (unsigned)ceil_div(nbc, kMapCols);
  int64_t gy = nbr;
  if (gy > 16384) gy = 16384;
  p.wgs = gx * (unsigned)gy;
  p.direct = DecompressArgs{j.row_ptr, j.col_idx, static_cast<const uint8_t *>(j.values),
                            static_cast<uint8_t *>(j.X_out), j.M, j.K * e, j.ldx * e, (int64_t)j.bc * e, nbr, nbc,
                            j.br, gx, (uint32_t)gy, 0u};
  return p;
}

}  // namespace

int launch_compress(const uint8_t *keep_mask, const void *X, int dtype, int64_t M, int64_t K, int64_t ldx,
                    int br, int bc, int64_t n_keep, int32_t *row_ptr, int32_t *col_idx, void *values,
                    void *ws, hipStream_t s) {
  const CompressJob job{keep_mask, X, M, K, ldx, br, bc, n_keep, row_ptr, col_idx, values, ws};
  const CompressPlan p = plan_compress(job, dtype);
  if (p.path == kPackSpan) {
    if (p.count_first) {
      const SpanGeom &g = p.span.g;
      hipLaunchKernelGGL(span_count_kernel, dim3((unsigned)ceil_div((int64_t)p.wgs, 4)), dim3(256), 0, s, keep_mask,
                         p.span.nbr * g.nbc, g.rb * g.nbc, (int64_t)p.wgs, static_cast<uint32_t *>(ws));
      const int rc = check_launch();
      if (rc != BSR_OK) return rc;
    }
#define BSR_COMPRESS_SPAN(VB) \
  hipLaunchKernelGGL((compress_span_kernel<VB>), dim3(p.wgs), dim3(256), p.lds, s, p.span)
    switch (p.vb) {
      case 16: BSR_COMPRESS_SPAN(16); break;
      case 8: BSR_COMPRESS_SPAN(8); break;
      default: BSR_COMPRESS_SPAN(4); break;
    }
#undef BSR_COMPRESS_SPAN
    return check_launch();
  }
  if (p.path == kPackOther) {
    const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
    int rc = launch_index_build(keep_mask, nbr, nbc, n_keep, row_ptr, col_idx, s);
    if (rc != BSR_OK) return rc;
    return launch_pack(X, dtype, M, K, ldx, br, bc, row_ptr, col_idx, n_keep, values, s);
  }
#define BSR_COMPRESS(VB) hipLaunchKernelGGL((compress_kernel<VB>), dim3(p.wgs), dim3(256), 0, s, p.direct)
  switch (p.vb) {
    case 16: BSR_COMPRESS(16); break;
    case 8: BSR_COMPRESS(8); break;
    case 4: BSR_COMPRESS(4); break;
    default: BSR_COMPRESS(2); break;
  }
#undef BSR_COMPRESS
  return check_launch();
}

int launch_decompress(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype,
                      int64_t M, int64_t K, int64_t ldx, int br, int bc, void *X_out, hipStream_t s) {
  if (M == 0 || K == 0) return BSR_OK;
  const DecompressJob job{row_ptr, col_idx, values, M, K, ldx, br, bc, X_out};
  const DecompressPlan p = plan_decompress(job, dtype);
  if (p.path == kPackSpan) {
#define BSR_UNPACK_SPAN(VB) \
  hipLaunchKernelGGL((decompress_span_kernel<VB>), dim3(p.wgs), dim3(256), p.lds, s, p.span)
    switch (p.vb) {
      case 16: BSR_UNPACK_SPAN(16); break;
      case 8: BSR_UNPACK_SPAN(8); break;
      default: BSR_UNPACK_SPAN(4); break;
    }
#undef BSR_UNPACK_SPAN
    return check_launch();
  }
#define BSR_UNPACK(VB) \
  hipLaunchKernelGGL((decompress_kernel<VB>), dim3(p.direct.gx, p.direct.gy), dim3(256), 0, s, p.direct)
  switch (p.vb) {
    case 16: BSR_UNPACK(16); break;
    case 8: BSR_UNPACK(8); break;
    case 4: BSR_UNPACK(4); break;
    default: BSR_UNPACK(2); break;
  }
#undef BSR_UNPACK
  return check_launch();
}

// Several tensors per call: the tensors that take the same kernel (family and vector width) share
// launches, kPackBatchMax per launch; a tensor that needs more than one launch of its own (counting
// pass, separate index build) goes through the single-tensor path.  The results are those of the
// single-tensor calls (bit copies either way).
int launch_compress_batched(const CompressJob *jobs, int n, int dtype, hipStream_t s) {
  static const int kVbs[4] = {16, 8, 4, 2};
  std::vector<CompressPlan> plans((size_t)n);
  for (int i = 0; i < n; ++i) plans[(size_t)i] = plan_compress(jobs[i], dtype);
  // with several tensors in the call one more launch costs little next to what it saves: row_ptr of
  // every tensor first, one workgroup per tensor
  if (n >= 2) {
    RowPtrBatch rb;
    int m = 0;
    auto flush_rows = [&]() -> int {
      if (m == 0) return BSR_OK;
      hipLaunchKernelGGL(row_ptr_batched_kernel, dim3(m), dim3(kRowPtrThreads), 0, s, rb);
      m = 0;
      return check_launch();
    };
    for (int i = 0; i < n; ++i) {
      CompressPlan &p = plans[(size_t)i];
      const CompressJob &j = jobs[i];
      const int64_t nbr = ceil_div(j.M, j.br), nbc = ceil_div(j.K, j.bc);
      if (p.path == kPackOther || p.wgs == 0 || nbr * nbc > kRowPtrMaxBlocks) continue;
      rb.it[m] = RowPtrItem{j.keep_mask, j.row_ptr, nbr, nbc};
      if (p.path == kPackSpan) {
        p.span.have_row_ptr = 1;
        p.span.wg_kept = nullptr;
        p.count_first = false;
      } else {
        p.direct.have_row_ptr = 1;
      }
      if (++m == kRowPtrBatchMax) {
        const int rc = flush_rows();
        if (rc != BSR_OK) return rc;
      }
    }
    const int rc = flush_rows();
    if (rc != BSR_OK) return rc;
  }
  for (int path = kPackSpan; path <= kPackDirect; ++path) {
    for (int vi = 0; vi < 4; ++vi) {
      const int vb = kVbs[vi];
      CompressBatch db;
      CompressSpanBatch sb;
      int m = 0;
      uint32_t total = 0;
      size_t lds = 0;
      auto flush = [&]() -> int {
        if (m == 0) return BSR_OK;
        if (path == kPackSpan) {
          switch (vb) {
            case 16: hipLaunchKernelGGL((compress_span_batched_kernel<16>), dim3(total), dim3(256), lds, s, sb, m); break;
            case 8: hipLaunchKernelGGL((compress_span_batched_kernel<8>), dim3(total), dim3(256), lds, s, sb, m); break;
            default: hipLaunchKernelGGL((compress_span_batched_kernel<4>), dim3(total), dim3(256), lds, s, sb, m); break;
          }
        } else {
          switch (vb) {
            case 16: hipLaunchKernelGGL((compress_batched_kernel<16>), dim3(total), dim3(256), 0, s, db, m); break;
            case 8: hipLaunchKernelGGL((compress_batched_kernel<8>), dim3(total), dim3(256), 0, s, db, m); break;
            case 4: hipLaunchKernelGGL((compress_batched_kernel<4>), dim3(total), dim3(256), 0, s, db, m); break;
            default: hipLaunchKernelGGL((compress_batched_kernel<2>), dim3(total), dim3(256), 0, s, db, m); break;
          }
        }
        m = 0;
        total = 0;
        lds = 0;
        return check_launch();
      };
      for (int i = 0; i < n; ++i) {
        const CompressPlan &p = plans[(size_t)i];
        if (p.path != path || p.vb != vb || p.count_first || p.wgs == 0) continue;
        if (path == kPackSpan) {
          sb.it[m] = p.span;
          sb.it[m].wg_begin = total;
          if (p.lds > lds) lds = p.lds;
        } else {
          db.it[m] = p.direct;
          db.it[m].wg_begin = total;
        }
        total += p.wgs;
        if (++m == kPackBatchMax) {
          const int rc = flush();
          if (rc != BSR_OK) return rc;
        }
      }
      const int rc = flush();
      if (rc != BSR_OK) return rc;
    }
  }
  for (int i = 0; i < n; ++i) {
    const CompressPlan &p = plans[(size_t)i];
    const CompressJob &j = jobs[i];
    if (p.path == kPackOther || (p.path == kPackSpan && p.count_first)) {
      const int rc = launch_compress(j.keep_mask, j.X, dtype, j.M, j.K, j.ldx, j.br, j.bc, j.n_keep, j.row_ptr,
                                     j.col_idx, j.values, j.ws, s);
      if (rc != BSR_OK) return rc;
    }
  }
  return BSR_OK;
}

int launch_decompress_batched(const DecompressJob *jobs, int n, int dtype, hipStream_t s) {
  static const int kVbs[4] = {16, 8, 4, 2};
  std::vector<DecompressPlan> plans((size_t)n);
  for (int i = 0; i < n; ++i) plans[(size_t)i] = plan_decompress(jobs[i], dtype);
  for (int path = kPackSpan; path <= kPackDirect; ++path) {
    for (int vi = 0; vi < 4; ++vi) {
      const int vb = kVbs[vi];
      DecompressBatch db;
      DecompressSpanBatch sb;
      int m = 0;
      uint32_t total = 0;
      size_t lds = 0;
      auto flush = [&]() -> int {
        if (m == 0) return BSR_OK;
        if (path == kPackSpan) {
          switch (vb) {
            case 16: hipLaunchKernelGGL((decompress_span_batched_kernel<16>), dim3(total), dim3(256), lds, s, sb, m); break;
            case 8: hipLaunchKernelGGL((decompress_span_batched_kernel<8>), dim3(total), dim3(256), lds, s, sb, m); break;
            default: hipLaunchKernelGGL((decompress_span_batched_kernel<4>), dim3(total), dim3(256), lds, s, sb, m); break;
          }
        } else {
          switch (vb) {
            case 16: hipLaunchKernelGGL((decompress_batched_kernel<16>), dim3(total), dim3(256), 0, s, db, m); break;
            case 8: hipLaunchKernelGGL((decompress_batched_kernel<8>), dim3(total), dim3(256), 0, s, db, m); break;
            case 4: hipLaunchKernelGGL((decompress_batched_kernel<4>), dim3(total), dim3(256), 0, s, db, m); break;
            default: hipLaunchKernelGGL((decompress_batched_kernel<2>), dim3(total), dim3(256), 0, s, db, m); break;
          }
        }
        m = 0;
        total = 0;
        lds = 0;
        return check_launch();
      };
      for (int i = 0; i < n; ++i) {
        const DecompressPlan &p = plans[(size_t)i];
        if (jobs[i].M == 0 || jobs[i].K == 0 || p.path != path || p.vb != vb || p.wgs == 0) continue;
        if (path == kPackSpan) {
          sb.it[m] = p.span;
          sb.it[m].wg_begin = total;
          if (p.lds > lds) lds = p.lds;
        } else {
          db.it[m] = p.direct;
          db.it[m].wg_begin = total;
        }
        total += p.wgs;
        if (++m == kPackBatchMax) {
          const int rc = flush();
          if (rc != BSR_OK) return rc;
        }
      }
      const int rc = flush();
      if (rc != BSR_OK) return rc;
    }
  }
  return BSR_OK;
}

}  // namespace bsr
