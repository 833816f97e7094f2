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
};

template <typename T, int V>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(
    const T *__restrict__ X, int64_t M, int64_t K, int64_t ldx, int br, int bc, int64_t nbr,
    int64_t nbc, ScoreGeom g, double *__restrict__ scores) {
  __shared__ double part[kScoreThreads];
  const int t = threadIdx.x;
  const int lane_col = t % g.vct;          // vector column inside the chunk
  const int grp = t / g.vct;               // row group
  const int ib = grp / g.gb;               // block-row of this pass
  const int gr = grp % g.gb;               // row group inside the block-row
  const int jj = lane_col / g.vpbt;        // block-column inside the chunk
  const int vpb = bc / V;                  // vectors per block row
  const int64_t j = (int64_t)blockIdx.x * g.jc + jj;
  const int64_t col0 = j * bc;

  for (int64_t pass = blockIdx.y; pass * g.rb < nbr; pass += gridDim.y) {
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
      const int64_t oi = pass * g.rb + oib, oj = (int64_t)blockIdx.x * g.jc + ojj;
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

template <typename T, int V>
int run_score(const void *X, int64_t M, int64_t K, int64_t ldx, int br, int bc, double *scores,
              hipStream_t s) {
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  ScoreGeom g;
  const int vpb = bc / V;
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
  dim3 grid((unsigned)g.nchunks, (unsigned)gy, 1);
  hipLaunchKernelGGL((score_kernel<T, V>), grid, dim3(g.vct * g.gb * g.rb), 0, s,
                     static_cast<const T *>(X), M, K, ldx, br, bc, nbr, nbc, g, scores);
  return check_launch();
}

}  // namespace

int launch_score(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                 double *scores, hipStream_t s) {
  if (M == 0 || K == 0) return BSR_OK;
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

}  // namespace bsr
