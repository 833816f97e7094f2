// Block scoring (paper Sec. IV: blocks are ranked by their l2 magnitude).
//
// score[i*nbc + j] = sum of x^2 over the valid elements of block (i,j), in
// binary64.  One streaming read of X: HBM-bound.  A workgroup owns `RB`
// consecutive block-rows and a chunk of `jc` block-columns; consecutive lanes
// read consecutive vectors of one matrix row (coalesced), row groups stride over
// the rows, and the partial sums meet in LDS where one lane per block adds them
// in a fixed order (reproducible bit for bit, no atomics).
#include "common.h"

namespace bsr {

namespace {

constexpr int kScoreThreads = 256;

struct ScoreGeom {
  int jc;    // block-columns per workgroup
  int vpbt;  // lanes across one block row (= min(vectors per block row, 256))
  int vct;   // lanes across the chunk (= jc * vpbt)
  int gb;    // row groups per block-row
  int rb;    // block-rows handled per pass
  int nchunks;
  int direct;  // 1: score_direct_body, one lane per vector column of a block-row; nchunks = its workgroups
};

// bx, by, gy: the workgroup's place in its tensor's (chunks x passes) grid.  Threads beyond
// g.vct * g.gb * g.rb (a batched launch runs every tensor with 256) find no row group and idle.
template <typename T, int V>
__device__ __forceinline__ void score_body(
    const T *__restrict__ X, int64_t M, int64_t K, int64_t ldx, int br, int bc, int64_t nbr,
    int64_t nbc, const ScoreGeom &g, double *__restrict__ scores, uint32_t bx, uint32_t by, uint32_t gy) {
  __shared__ double part[kScoreThreads];
  const int t = threadIdx.x;
  const int lane_col = t % g.vct;          // vector column inside the chunk
  const int grp = t / g.vct;               // row group
  const int ib = grp / g.gb;               // block-row of this pass
  const int gr = grp % g.gb;               // row group inside the block-row
  const int jj = lane_col / g.vpbt;        // block-column inside the chunk
  const int vpb = bc / V;                  // vectors per block row
  const int64_t j = (int64_t)bx * g.jc + jj;
  const int64_t col0 = j * bc;

  for (int64_t pass = by; pass * g.rb < nbr; pass += gy) {
    const int64_t i = pass * g.rb + ib;
    double acc = 0.0;
    if (ib < g.rb && i < nbr && j < nbc) {
      const int64_t m0 = i * br;
      const int rows = (int)((M - m0) < br ? (M - m0) : br);
      for (int u = lane_col % g.vpbt; u < vpb; u += g.vpbt) {
        const int64_t col = col0 + (int64_t)u * V;
        if (col >= K) break;
        const T *p = X + m0 * ldx + col;
        // kInFlight loads are issued before the first of them is consumed (the
        // kernel is bound by memory latency, not arithmetic); the order of the
        // additions stays r ascending, whatever the batching
        constexpr int kInFlight = 8;
        for (int r0 = gr; r0 < rows; r0 += kInFlight * g.gb) {
          Vec<T, V> v[kInFlight];
#pragma unroll
          for (int b = 0; b < kInFlight; ++b) {
            const int r = r0 + b * g.gb;
            if (r < rows) v[b] = *reinterpret_cast<const Vec<T, V> *>(p + (int64_t)r * ldx);
          }
#pragma unroll
          for (int b = 0; b < kInFlight; ++b) {
            if (r0 + b * g.gb < rows) {
#pragma unroll
              for (int q = 0; q < V; ++q) {
                const double x = (double)elem_to_float<T>(v[b].e[q]);
                acc = fma(x, x, acc);
              }
            }
          }
        }
      }
    }
    part[t] = acc;
    __syncthreads();
    // one lane per (block-row, block-column) of this pass adds the partials
    if (t < g.rb * g.jc) {
      const int oib = t / g.jc, ojj = t % g.jc;
      const int64_t oi = pass * g.rb + oib, oj = (int64_t)bx * g.jc + ojj;
      if (oi < nbr && oj < nbc) {
        double s = 0.0;
        for (int a = 0; a < g.gb; ++a)
          for (int u = 0; u < g.vpbt; ++u) s += part[(oib * g.gb + a) * g.vct + ojj * g.vpbt + u];
        scores[oi * nbc + oj] = s;
      }
    }
    __syncthreads();
  }
}

// Large matrices: bc / V * rs lanes own a block -- lane (part, u) reads vector u of the rows
// part, part + rs, ... of the block, eight loads on their way at a time (consecutive lanes
// read consecutive vectors of a matrix row, whole 64-byte pieces or more) -- and add their sums
// with a butterfly of lane exchanges in a fixed order.  No LDS, no barrier, every lane busy.
// rs (a power of two, g.gb) is chosen so that the tensor has enough lanes for the chip.
// wg = index of the workgroup among the ceil(nbr * nbc * (bc / V) * rs / 256) of its tensor.
template <typename T, int V>
__device__ __forceinline__ void score_direct_body(
    const T *__restrict__ X, int64_t M, int64_t K, int64_t ldx, int br, int bc, int64_t nbr,
    int64_t nbc, int rs, double *__restrict__ scores, uint32_t wg) {
  const uint32_t vpb = (uint32_t)(bc / V);                 // lanes across a block row: a power of two
  const uint32_t lpb = vpb * (uint32_t)rs;                 // lanes per block: a power of two, at most 64
  const uint32_t per_row = (uint32_t)nbc * lpb;            // lanes per block-row
  const uint32_t gid = wg * (uint32_t)kScoreThreads + threadIdx.x;
  const uint32_t i = gid / per_row, c = gid - i * per_row;
  const uint32_t j = c / lpb, within = c & (lpb - 1), part = within / vpb, u = within & (vpb - 1);
  const int64_t col = (int64_t)j * bc + (int64_t)u * V;
  const bool live = (int64_t)i < nbr && col < K;
  const int64_t m0 = (int64_t)i * br;
  const int rows = live ? (int)((M - m0) < br ? (M - m0) : br) : 0;
  const T *p = X + m0 * ldx + col;
  double acc0 = 0.0, acc1 = 0.0;                           // even and odd elements of the vectors
  // (eight, not more: with sixteen the registers they need leave room for three waves per SIMD only,
  // and a workgroup has nothing in flight while it adds up)
  constexpr int kInFlight = 8;
  for (int r0 = (int)part; r0 < rows; r0 += kInFlight * rs) {
    Vec<T, V> v[kInFlight];
#pragma unroll
    for (int b = 0; b < kInFlight; ++b)
      if (r0 + b * rs < rows) v[b] = load_stream(reinterpret_cast<const Vec<T, V> *>(p + (int64_t)(r0 + b * rs) * ldx));
#pragma unroll
    for (int b = 0; b < kInFlight; ++b) {
      if (r0 + b * rs < rows) {
#pragma unroll
        for (int q = 0; q < V; ++q) {
          const double x = (double)elem_to_float<T>(v[b].e[q]);
          if (q & 1) acc1 = fma(x, x, acc1);
          else acc0 = fma(x, x, acc0);
        }
      }
    }
  }
  double sum = acc0 + acc1;
  for (uint32_t o = 1; o < lpb; o <<= 1) sum += __shfl_xor(sum, (int)o);
  if (live && within == 0) scores[(int64_t)i * nbc + j] = sum;
}

template <typename T, int V>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(
    const T *__restrict__ X, int64_t M, int64_t K, int64_t ldx, int br, int bc, int64_t nbr,
    int64_t nbc, ScoreGeom g, double *__restrict__ scores) {
  if (g.direct) score_direct_body<T, V>(X, M, K, ldx, br, bc, nbr, nbc, g.gb, scores, blockIdx.x);
  else score_body<T, V>(X, M, K, ldx, br, bc, nbr, nbc, g, scores, blockIdx.x, blockIdx.y, gridDim.y);
}

// Several tensors per launch: workgroup w belongs to the tensor whose range of
// workgroups holds w; the tensors' parameters come with the kernel arguments.
constexpr int kScoreBatchMax = 24;
struct ScoreItem {
  const void *X;
  double *scores;
  int64_t M, K, ldx, nbr, nbc;
  int br, bc;
  ScoreGeom g;
  uint32_t wg_begin, gy;
};
struct ScoreBatch {
  ScoreItem it[kScoreBatchMax];
};

template <typename T, int V>
__global__ __launch_bounds__(kScoreThreads) void score_batched_kernel(ScoreBatch b, int n) {
  int i = 0;
  while (i + 1 < n && blockIdx.x >= b.it[i + 1].wg_begin) ++i;
  const ScoreItem &it = b.it[i];
  const uint32_t local = blockIdx.x - it.wg_begin;
  if (it.g.direct) {
    score_direct_body<T, V>(static_cast<const T *>(it.X), it.M, it.K, it.ldx, it.br, it.bc, it.nbr, it.nbc, it.g.gb, it.scores,
                            local);
    return;
  }
  score_body<T, V>(static_cast<const T *>(it.X), it.M, it.K, it.ldx, it.br, it.bc, it.nbr, it.nbc, it.g, it.scores,
                   local % (uint32_t)it.g.nchunks, local / (uint32_t)it.g.nchunks, it.gy);
}

// Narrow blocks (rows shorter than a 16-byte vector, e.g. 14x14 patches) and blocks
// of few rows (1 x b row segments) on contiguous matrix rows: a workgroup reads the rows of g.rb block-rows as one
// linear span into LDS, then a thread per (matrix row, block-column, piece of 32
// elements) adds that piece's squares left to right, and a thread per block adds
// the pieces row by row.  LDS layout: span | partial sums (binary64).
template <typename T, typename V>
__device__ __forceinline__ void score_span_body(const uint8_t *__restrict__ X, int64_t M, int64_t K, int bc,
                                                int64_t nbr, const SpanGeom &g, size_t span_words, int pieces,
                                                uint32_t magic_pieces, double *__restrict__ scores,
                                                uint32_t wg) {
  constexpr int kVecs = kSpanBytes / (int)sizeof(V) / 256;
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  double *part = reinterpret_cast<double *>(lds + span_words);
  const int t = threadIdx.x;
  const int64_t i0 = (int64_t)wg * g.rb;
  const int nb = (int)((nbr - i0) < g.rb ? (nbr - i0) : g.rb);
  const int64_t m0 = i0 * g.br;
  const int rows = (int)((M - m0) < (int64_t)nb * g.br ? (M - m0) : (int64_t)nb * g.br);
  const int nvec = rows * g.row_words * 4 / (int)sizeof(V);
  const V *src = reinterpret_cast<const V *>(X + m0 * g.row_words * 4);
  V reg[kVecs];
#pragma unroll
  for (int k = 0; k < kVecs; ++k)
    if (t + 256 * k < nvec) reg[k] = src[t + 256 * k];
  V *sv = reinterpret_cast<V *>(lds);
#pragma unroll
  for (int k = 0; k < kVecs; ++k)
    if (t + 256 * k < nvec) sv[t + 256 * k] = reg[k];
  __syncthreads();
  const T *sp = reinterpret_cast<const T *>(lds);
  const int kk = (int)K;
  // a row segment is summed in pieces of 32 elements (`pieces` per segment)
  for (int pc = t; pc < rows * g.nbc * pieces; pc += 256) {
    const uint32_t pair = span_div((uint32_t)pc, (uint32_t)pieces, magic_pieces), sub = (uint32_t)pc - pair * pieces;
    const uint32_t row = span_div(pair, (uint32_t)g.nbc, g.magic_nbc), j = pair - row * g.nbc;
    const int c0 = (int)j * bc + (int)sub * 32;
    int c1 = c0 + 32 < (int)(j + 1) * bc ? c0 + 32 : (int)(j + 1) * bc;
    if (c1 > kk) c1 = kk;
    const T *p = sp + (int)row * kk;
    double acc = 0.0;
    for (int c = c0; c < c1; ++c) {
      const double x = (double)elem_to_float<T>(p[c]);
      acc = fma(x, x, acc);
    }
    part[pc] = acc;
  }
  __syncthreads();
  for (int bj = t; bj < nb * g.nbc; bj += 256) {
    const uint32_t b = span_div((uint32_t)bj, (uint32_t)g.nbc, g.magic_nbc), j = (uint32_t)bj - b * g.nbc;
    const int r1 = rows - (int)b * g.br < g.br ? rows - (int)b * g.br : g.br;
    double sum = 0.0;
    for (int r = 0; r < r1; ++r)
      for (int u = 0; u < pieces; ++u) sum += part[(((int)b * g.br + r) * g.nbc + (int)j) * pieces + u];
    scores[(i0 + b) * g.nbc + j] = sum;
  }
}

template <typename T, typename V>
__global__ __launch_bounds__(256) void score_span_kernel(const uint8_t *__restrict__ X, int64_t M, int64_t K,
                                                         int bc, int64_t nbr, SpanGeom g, size_t span_words,
                                                         int pieces, uint32_t magic_pieces,
                                                         double *__restrict__ scores) {
  score_span_body<T, V>(X, M, K, bc, nbr, g, span_words, pieces, magic_pieces, scores, blockIdx.x);
}

struct SpanScoreItem {
  const uint8_t *X;
  double *scores;
  int64_t M, K, nbr;
  SpanGeom g;
  uint32_t span_words, magic_pieces;
  int bc, pieces;
  uint32_t wg_begin;
};
struct SpanScoreBatch {
  SpanScoreItem it[kScoreBatchMax];
};

template <typename T, typename V>
__global__ __launch_bounds__(256) void score_span_batched_kernel(SpanScoreBatch b, int n) {
  int i = 0;
  while (i + 1 < n && blockIdx.x >= b.it[i + 1].wg_begin) ++i;
  const SpanScoreItem &it = b.it[i];
  score_span_body<T, V>(it.X, it.M, it.K, it.bc, it.nbr, it.g, it.span_words, it.pieces, it.magic_pieces, it.scores,
                        blockIdx.x - it.wg_begin);
}

// Few-row blocks whose row segments are whole 16-byte vectors (1 x b row segments):
// the same span of g.rb block-rows, but every lane keeps its vectors in registers
// and only their sums of squares go to LDS; a thread per block then adds the
// vectors of its segments left to right, row by row.
template <typename T>
__global__ __launch_bounds__(256) void score_rows_kernel(const uint8_t *__restrict__ X, int64_t M, int bc,
                                                         int64_t nbr, SpanGeom g, double *__restrict__ scores) {
  constexpr int VE = 16 / (int)sizeof(T);
  constexpr int kVecs = kSpanBytes / 16 / 256;
  __shared__ double part[kSpanBytes / 16];
  const int t = threadIdx.x;
  const int64_t i0 = (int64_t)blockIdx.x * g.rb;
  const int nb = (int)((nbr - i0) < g.rb ? (nbr - i0) : g.rb);
  const int64_t m0 = i0 * g.br;
  const int rows = (int)((M - m0) < (int64_t)nb * g.br ? (M - m0) : (int64_t)nb * g.br);
  const int rv = g.row_words / 4;                        // vectors per matrix row
  const int nvec = rows * rv;
  const Vec<T, VE> *src = reinterpret_cast<const Vec<T, VE> *>(X + m0 * g.row_words * 4);
  Vec<T, VE> reg[kVecs];
#pragma unroll
  for (int k = 0; k < kVecs; ++k)
    if (t + 256 * k < nvec) reg[k] = src[t + 256 * k];
#pragma unroll
  for (int k = 0; k < kVecs; ++k) {
    if (t + 256 * k < nvec) {
      double acc = 0.0;
#pragma unroll
      for (int q = 0; q < VE; ++q) {
        const double x = (double)elem_to_float<T>(reg[k].e[q]);
        acc = fma(x, x, acc);
      }
      part[t + 256 * k] = acc;
    }
  }
  __syncthreads();
  const int vps = bc / VE;                               // vectors per row segment
  for (int bj = t; bj < nb * g.nbc; bj += 256) {
    const uint32_t b = span_div((uint32_t)bj, (uint32_t)g.nbc, g.magic_nbc), j = (uint32_t)bj - b * g.nbc;
    const int r1 = rows - (int)b * g.br < g.br ? rows - (int)b * g.br : g.br;
    const int u1 = rv - (int)j * vps < vps ? rv - (int)j * vps : vps;       // ragged last block-column
    double sum = 0.0;
    for (int r = 0; r < r1; ++r)
      for (int u = 0; u < u1; ++u) sum += part[((int)b * g.br + r) * rv + (int)j * vps + u];
    scores[(i0 + b) * g.nbc + j] = sum;
  }
}

template <typename T>
int run_score_span(const void *X, int64_t M, int64_t K, int bc, const SpanGeom &g, double *scores,
                   hipStream_t s) {
  const int64_t nbr = ceil_div(M, g.br);
  if (g.vb == 16 && g.seg_words % 4 == 0) {
    hipLaunchKernelGGL((score_rows_kernel<T>), dim3((unsigned)ceil_div(nbr, g.rb)), dim3(256), 0, s,
                       static_cast<const uint8_t *>(X), M, bc, nbr, g, scores);
    return check_launch();
  }
  const size_t span_words = align_up((size_t)g.rb * g.br * g.row_words, 4);
  const int pieces = (bc + 31) / 32;
  const uint32_t magic_pieces = (uint32_t)(((uint64_t(1) << 32) + pieces - 1) / pieces);
  const size_t lds = span_words * 4 + (size_t)g.rb * g.br * g.nbc * pieces * sizeof(double);
  const dim3 grid((unsigned)ceil_div(nbr, g.rb));
  const uint8_t *x = static_cast<const uint8_t *>(X);
  switch (g.vb) {
    case 16:
      hipLaunchKernelGGL((score_span_kernel<T, uint4>), grid, dim3(256), lds, s, x, M, K, bc, nbr, g, span_words, pieces, magic_pieces, scores);
      break;
    case 8:
      hipLaunchKernelGGL((score_span_kernel<T, uint2>), grid, dim3(256), lds, s, x, M, K, bc, nbr, g, span_words, pieces, magic_pieces, scores);
      break;
    default:
      hipLaunchKernelGGL((score_span_kernel<T, uint32_t>), grid, dim3(256), lds, s, x, M, K, bc, nbr, g, span_words, pieces, magic_pieces, scores);
      break;
  }
  return check_launch();
}

// Launch geometry of score_kernel for vectors of V elements; *gy = passes of the grid.
ScoreGeom score_geometry(int V, int64_t M, int64_t K, int br, int bc, int64_t *gy_out) {
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  ScoreGeom g;
  const int vpb = bc / V;
  g.direct = 0;
  // large matrices take the direct body: rs lanes share a vector column of a block so that the
  // tensor has at least 64 Ki lanes, and every lane still has a few rows
  if (vpb >= 1 && vpb <= 64 && (vpb & (vpb - 1)) == 0 && vpb * V == bc) {
    int rs = 1;
    while (nbr * nbc * vpb * rs < 65536 && vpb * rs * 2 <= 64 && rs * 2 * 4 <= br) rs *= 2;
    const int64_t lanes = nbr * nbc * vpb * rs;
    if (lanes >= 16384 && lanes < (int64_t(1) << 31)) {
      g.direct = 1;
      g.jc = g.vpbt = g.vct = g.rb = 1;
      g.gb = rs;
      g.nchunks = (int)ceil_div(lanes, (int64_t)kScoreThreads);
      *gy_out = 1;
      return g;
    }
  }
  g.vpbt = vpb < kScoreThreads ? vpb : kScoreThreads;
  // about one wave across the chunk (a 1 KB row segment per load instruction), the
  // other waves of the workgroup as row groups: many workgroups, few rows per
  // thread, so that all of a thread's loads are in flight at once
  // (a matrix row of at most two waves stays in one piece)
  g.jc = g.vpbt >= 64 ? 1 : 64 / g.vpbt;
  if (nbc * g.vpbt <= 128 || g.jc > nbc) g.jc = (int)nbc;
  g.vct = g.jc * g.vpbt;
  const int groups = kScoreThreads / g.vct;      // >= 1
  g.gb = groups < br ? groups : br;
  g.rb = groups / g.gb;
  if (g.rb > nbr) g.rb = (int)nbr;
  g.nchunks = (int)ceil_div(nbc, g.jc);
  const int64_t passes = ceil_div(nbr, g.rb);
  // enough workgroups to fill 256 CUs several times over, bounded so that a
  // workgroup of a very tall matrix loops instead of flooding the dispatcher
  int64_t gy = passes;
  const int64_t cap = ceil_div(16384, g.nchunks);
  if (gy > cap) gy = cap;
  if (gy > 65535) gy = 65535;
  *gy_out = gy;
  return g;
}

template <typename T, int V>
int run_score(const void *X, int64_t M, int64_t K, int64_t ldx, int br, int bc, double *scores,
              hipStream_t s) {
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  int64_t gy;
  const ScoreGeom g = score_geometry(V, M, K, br, bc, &gy);
  dim3 grid((unsigned)g.nchunks, (unsigned)gy, 1);
  hipLaunchKernelGGL((score_kernel<T, V>), grid, dim3(g.direct ? kScoreThreads : g.vct * g.gb * g.rb), 0, s,
                     static_cast<const T *>(X), M, K, ldx, br, bc, nbr, nbc, g, scores);
  return check_launch();
}

// Which kernel scores a tensor: 0 = score_kernel with vectors of `key` elements,
// 1 = score_span_kernel with `key`-byte accesses, 2 = score_rows_kernel.
int score_kind(int dtype, const void *X, int64_t M, int64_t K, int64_t ldx, int br, int bc, SpanGeom *g, int *key) {
  if (span_geometry(dtype, M, K, ldx, br, bc, X, nullptr, g) &&
      (int64_t)g->rb * br * g->nbc * ((bc + 31) / 32) <= 6144) {
    *key = g->vb;
    return (g->vb == 16 && g->seg_words % 4 == 0) ? 2 : 1;
  }
  *key = dtype == BSR_F32 ? pick_vector(4, 4, bc, K, ldx, X) : pick_vector(8, 2, bc, K, ldx, X);
  return 0;
}

template <typename T>
int launch_generic_batch(const ScoreBatch &b, int n, uint32_t wgs, int v, hipStream_t s) {
  const dim3 grid(wgs), block(kScoreThreads);
  if (sizeof(T) == 4) {
    switch (v) {
      case 4: hipLaunchKernelGGL((score_batched_kernel<float, 4>), grid, block, 0, s, b, n); break;
      case 2: hipLaunchKernelGGL((score_batched_kernel<float, 2>), grid, block, 0, s, b, n); break;
      default: hipLaunchKernelGGL((score_batched_kernel<float, 1>), grid, block, 0, s, b, n); break;
    }
  } else {
    switch (v) {
      case 8: hipLaunchKernelGGL((score_batched_kernel<uint16_t, 8>), grid, block, 0, s, b, n); break;
      case 4: hipLaunchKernelGGL((score_batched_kernel<uint16_t, 4>), grid, block, 0, s, b, n); break;
      case 2: hipLaunchKernelGGL((score_batched_kernel<uint16_t, 2>), grid, block, 0, s, b, n); break;
      default: hipLaunchKernelGGL((score_batched_kernel<uint16_t, 1>), grid, block, 0, s, b, n); break;
    }
  }
  return check_launch();
}

template <typename T>
int launch_span_batch(const SpanScoreBatch &b, int n, uint32_t wgs, size_t lds, int vb, hipStream_t s) {
  const dim3 grid(wgs), block(256);
  switch (vb) {
    case 16: hipLaunchKernelGGL((score_span_batched_kernel<T, uint4>), grid, block, lds, s, b, n); break;
    case 8: hipLaunchKernelGGL((score_span_batched_kernel<T, uint2>), grid, block, lds, s, b, n); break;
    default: hipLaunchKernelGGL((score_span_batched_kernel<T, uint32_t>), grid, block, lds, s, b, n); break;
  }
  return check_launch();
}

}  // namespace

int launch_score(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                 double *scores, hipStream_t s) {
  if (M == 0 || K == 0) return BSR_OK;
  SpanGeom g;
  // partial sums in LDS: at most 48 KB of binary64 beside the span
  if (span_geometry(dtype, M, K, ldx, br, bc, X, nullptr, &g) &&
      (int64_t)g.rb * br * g.nbc * ((bc + 31) / 32) <= 6144)
    return dtype == BSR_F32 ? run_score_span<float>(X, M, K, bc, g, scores, s)
                            : run_score_span<uint16_t>(X, M, K, bc, g, scores, s);
  if (dtype == BSR_F32) {
    switch (pick_vector(4, 4, bc, K, ldx, X)) {
      case 4: return run_score<float, 4>(X, M, K, ldx, br, bc, scores, s);
      case 2: return run_score<float, 2>(X, M, K, ldx, br, bc, scores, s);
      default: return run_score<float, 1>(X, M, K, ldx, br, bc, scores, s);
    }
  }
  switch (pick_vector(8, 2, bc, K, ldx, X)) {
    case 8: return run_score<uint16_t, 8>(X, M, K, ldx, br, bc, scores, s);
    case 4: return run_score<uint16_t, 4>(X, M, K, ldx, br, bc, scores, s);
    case 2: return run_score<uint16_t, 2>(X, M, K, ldx, br, bc, scores, s);
    default: return run_score<uint16_t, 1>(X, M, K, ldx, br, bc, scores, s);
  }
}

int launch_score_batched(const ScoreJob *jobs, int n, int dtype, hipStream_t s) {
  // tensors that take the same kernel instance share launches of up to kScoreBatchMax tensors
  static const int kKeys[2][4] = {{8, 4, 2, 1}, {16, 8, 4, 0}};
  for (int kind = 0; kind < 2; ++kind) {
    for (int ki = 0; ki < 4; ++ki) {
      const int want_key = kKeys[kind][ki];
      if (want_key == 0) continue;
      ScoreBatch gb;
      SpanScoreBatch sb;
      int m = 0;
      uint32_t wgs = 0;
      size_t lds = 0;
      auto flush = [&]() -> int {
        if (m == 0) return BSR_OK;
        int rc;
        if (kind == 0)
          rc = dtype == BSR_F32 ? launch_generic_batch<float>(gb, m, wgs, want_key, s)
                                : launch_generic_batch<uint16_t>(gb, m, wgs, want_key, s);
        else
          rc = dtype == BSR_F32 ? launch_span_batch<float>(sb, m, wgs, lds, want_key, s)
                                : launch_span_batch<uint16_t>(sb, m, wgs, lds, want_key, s);
        m = 0;
        wgs = 0;
        lds = 0;
        return rc;
      };
      for (int i = 0; i < n; ++i) {
        const ScoreJob &j = jobs[i];
        if (j.M == 0 || j.K == 0) continue;
        SpanGeom g;
        int key;
        const int k = score_kind(dtype, j.X, j.M, j.K, j.ldx, j.br, j.bc, &g, &key);
        if (k == 2) {                                        // register-resident row segments: one by one
          if (kind == 0 && ki == 0) {
            const int rc = launch_score(j.X, dtype, j.M, j.K, j.ldx, j.br, j.bc, j.scores, s);
            if (rc != BSR_OK) return rc;
          }
          continue;
        }
        if (k != kind || key != want_key) continue;
        const int64_t nbr = ceil_div(j.M, j.br), nbc = ceil_div(j.K, j.bc);
        if (kind == 0) {
          ScoreItem &it = gb.it[m];
          int64_t gy;
          it.g = score_geometry(key, j.M, j.K, j.br, j.bc, &gy);
          it.X = j.X;
          it.scores = j.scores;
          it.M = j.M; it.K = j.K; it.ldx = j.ldx; it.nbr = nbr; it.nbc = nbc;
          it.br = j.br; it.bc = j.bc;
          it.wg_begin = wgs;
          it.gy = (uint32_t)gy;
          wgs += (uint32_t)(it.g.nchunks * gy);
        } else {
          SpanScoreItem &it = sb.it[m];
          it.g = g;
          it.X = static_cast<const uint8_t *>(j.X);
          it.scores = j.scores;
          it.M = j.M; it.K = j.K; it.nbr = nbr;
          it.bc = j.bc;
          it.pieces = (j.bc + 31) / 32;
          it.magic_pieces = (uint32_t)(((uint64_t(1) << 32) + it.pieces - 1) / it.pieces);
          it.span_words = (uint32_t)align_up((size_t)g.rb * g.br * g.row_words, 4);
          const size_t need = (size_t)it.span_words * 4 + (size_t)g.rb * g.br * g.nbc * it.pieces * sizeof(double);
          if (need > lds) lds = need;
          it.wg_begin = wgs;
          wgs += (uint32_t)ceil_div(nbr, g.rb);
        }
        if (++m == kScoreBatchMax) {
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
