// C ABI of libbsr_actprune: argument validation on the host, then kernel
// launches on the caller's stream.  See include/bsr_actprune.h for the contract
// of every entry point.
#include <cmath>
#include <vector>

#include "common.h"

namespace bsr {

static thread_local int g_last_hip_error = 0;

void set_hip_error(int e) { g_last_hip_error = e; }

int check_launch() {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return BSR_OK;
  g_last_hip_error = (int)e;
  return BSR_ERR_HIP;
}

namespace {

constexpr int64_t kMaxBlocks = (int64_t(1) << 31) - 1;
constexpr int kMaxBlockDim = 1 << 16;

struct Geometry {
  int64_t nbr, nbc, nblocks;
};

// Shared shape checks.  ld is the leading dimension of the dense matrix.
int check_shape(int dtype, int64_t M, int64_t K, int64_t ld, int br, int bc, Geometry *g) {
  if (dtype != BSR_F32 && dtype != BSR_BF16) return BSR_ERR_DTYPE;
  if (M < 0 || K < 0 || br < 1 || bc < 1 || br > kMaxBlockDim || bc > kMaxBlockDim) return BSR_ERR_SHAPE;
  if (ld < K) return BSR_ERR_SHAPE;
  if (M > (int64_t(1) << 40) || K > (int64_t(1) << 40) || ld > (int64_t(1) << 40)) return BSR_ERR_SHAPE;
  g->nbr = ceil_div(M, br);
  g->nbc = ceil_div(K, bc);
  if (g->nbr > kMaxBlocks || g->nbc > kMaxBlocks) return BSR_ERR_SHAPE;
  if (g->nbc != 0 && g->nbr > kMaxBlocks / g->nbc) return BSR_ERR_SHAPE;
  g->nblocks = g->nbr * g->nbc;
  if ((double)M * (double)ld * 4.0 > 9.0e18) return BSR_ERR_SHAPE;
  return BSR_OK;
}

bool misaligned(const void *p, size_t a) { return p != nullptr && (uintptr_t)p % a != 0; }

size_t scores_bytes(int64_t nblocks) { return align_up((size_t)nblocks * sizeof(double), 256); }

size_t score_select_ws(int64_t nblocks) { return scores_bytes(nblocks) + select_ws_bytes(nblocks); }

// How well a product suits the wide-tile kernel: its tiles of 384 x 128 times the ways its
// contraction can be split, i.e. the workgroups it can keep busy.  A call takes the wide
// kernel when that reaches half the compute units.
int64_t wide_parallelism(int64_t M, int64_t K, int64_t N, int br) {
  const int64_t nbr = ceil_div(M, br);
  return ceil_div(K, 384) * ceil_div(N, 128) * (nbr < 16 ? nbr : 16);
}

// Small square blocks and a small weight matrix (the cross-patch layers) in a batched call: the kernel whose
// workgroups own all of dW, once the contraction is long enough to split over a few of them.  (A product on
// its own would need so many splits to fill the GPU that the narrow-tile kernel is the faster one.)
bool use_narrow(int dtype, int br, int bc, const void *values, const void *dY, int64_t M, int64_t K, int64_t N,
                int64_t lddy) {
  return dw_narrow_supported(dtype, br, bc, values, dY, M, K, N, lddy) && ceil_div(M, br) >= 16;
}

bool use_wide_single(int dtype, int br, int bc, const void *values, const void *dY, int64_t M, int64_t K, int64_t N,
                     int64_t lddy) {
  return dw_wide_supported(dtype, br, bc, values, dY, M, K, N, lddy) && wide_parallelism(M, K, N, br) >= 128;
}

}  // namespace
}  // namespace bsr

using namespace bsr;

extern "C" {

const char *bsr_version(void) { return "bsr_actprune 0.1 (gfx950)"; }

const char *bsr_error_string(int code) {
  switch (code) {
    case BSR_OK: return "BSR_OK";
    case BSR_ERR_NULL: return "BSR_ERR_NULL";
    case BSR_ERR_SHAPE: return "BSR_ERR_SHAPE";
    case BSR_ERR_DTYPE: return "BSR_ERR_DTYPE";
    case BSR_ERR_KEEP: return "BSR_ERR_KEEP";
    case BSR_ERR_WORKSPACE: return "BSR_ERR_WORKSPACE";
    case BSR_ERR_ALIGN: return "BSR_ERR_ALIGN";
    case BSR_ERR_HIP: return "BSR_ERR_HIP";
    case BSR_ERR_LIMIT: return "BSR_ERR_LIMIT";
    default: return "BSR_ERR_UNKNOWN";
  }
}

int bsr_last_hip_error(void) { return g_last_hip_error; }

int64_t bsr_keep_count(int64_t nblocks, double keep) {
  if (nblocks < 0 || !(keep >= 0.0 && keep <= 1.0)) return -1;
  const double v = std::ceil(keep * (double)nblocks);
  int64_t n = (int64_t)v;
  if (n < 0) n = 0;
  if (n > nblocks) n = nblocks;
  return n;
}

int64_t bsr_storage_bytes(int64_t M, int64_t K, int br, int bc, int64_t n_keep, int dtype) {
  Geometry g;
  if (check_shape(dtype, M, K, K, br, bc, &g) != BSR_OK) return -1;
  if (n_keep < 0 || n_keep > g.nblocks) return -1;
  return n_keep * (int64_t)br * bc * elem_bytes(dtype) + 4 * n_keep + 4 * (g.nbr + 1);
}

size_t bsr_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, int br, int bc, int dtype) {
  Geometry g;
  if (check_shape(dtype, M, K, K, br, bc, &g) != BSR_OK) return 0;
  switch (op) {
    case BSR_OP_SCORE_SELECT: return score_select_ws(g.nblocks);
    case BSR_OP_COMPRESS: return compress_ws_bytes(dtype, M, K, br, bc);
    case BSR_OP_DECOMPRESS: return 0;
    case BSR_OP_T_DENSE_MATMUL:
      if (N < 0) return 0;
      {
        size_t a = dw_generic_ws_bytes(M, K, N, br, bc);
        if (dw_mfma_supported(dtype, br, bc, nullptr, M, K, N, N)) {
          size_t b = dw_mfma_ws_bytes(dtype, M, K, N, br, bc);
          if (dw_wide_supported(dtype, br, bc, nullptr, nullptr, M, K, N, N)) {
            const size_t c = dw_wide_ws_bytes(M, K, N, br);
            if (c > b) b = c;
          }
          if (b > a) a = b;
        } else if (dw_reblock_supported(dtype, br, bc, M, K, N, N)) {
          const size_t b = dw_reblock_ws_bytes(dtype, M, K, N);
          if (b > a) a = b;
        }
        if (dw_narrow_supported(dtype, br, bc, nullptr, nullptr, M, K, N, N)) {
          const size_t b = dw_narrow_ws_bytes(M, K, N, br);
          if (b > a) a = b;
        }
        return align_up(a, 256);
      }
    case BSR_OP_AFFINE_SCALE_GRAD: return affine_ws_bytes(M, K, br, bc);
    default: return 0;
  }
}

int bsr_score_select(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                     double keep, double *scores, uint8_t *keep_mask, void *ws, size_t ws_bytes,
                     void *stream) {
  Geometry g;
  int rc = check_shape(dtype, M, K, ldx, br, bc, &g);
  if (rc != BSR_OK) return rc;
  const int64_t n_keep = bsr_keep_count(g.nblocks, keep);
  if (n_keep < 0) return BSR_ERR_KEEP;
  if (g.nblocks == 0) return BSR_OK;
  if (X == nullptr || keep_mask == nullptr) return BSR_ERR_NULL;
  if (misaligned(X, elem_bytes(dtype)) || misaligned(scores, 8) || misaligned(ws, 16)) return BSR_ERR_ALIGN;
  const size_t need = score_select_ws(g.nblocks);
  if (ws == nullptr || ws_bytes < need) return BSR_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  double *sc = scores != nullptr ? scores : static_cast<double *>(ws);
  rc = launch_score(X, dtype, M, K, ldx, br, bc, sc, s);
  if (rc != BSR_OK) return rc;
  return launch_select(sc, g.nblocks, n_keep, keep_mask, static_cast<char *>(ws) + scores_bytes(g.nblocks), s);
}

int64_t bsr_grouped_keep_count(int64_t nbr, int64_t nbc, int64_t group_rows, double keep) {
  if (nbr < 0 || nbc < 0 || group_rows < 1 || !(keep >= 0.0 && keep <= 1.0)) return -1;
  if (nbr == 0 || nbc == 0) return 0;
  const int64_t groups = (nbr + group_rows - 1) / group_rows;
  const int64_t last_rows = nbr - (groups - 1) * group_rows;
  const int64_t full = groups > 1 ? bsr_keep_count(group_rows * nbc, keep) : 0;
  return (groups - 1) * full + bsr_keep_count(last_rows * nbc, keep);
}

int bsr_score_select_grouped(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                             int64_t group_rows, double keep, double *scores, uint8_t *keep_mask,
                             void *ws, size_t ws_bytes, void *stream) {
  Geometry g;
  int rc = check_shape(dtype, M, K, ldx, br, bc, &g);
  if (rc != BSR_OK) return rc;
  if (group_rows < 1) return BSR_ERR_SHAPE;
  if (!(keep >= 0.0 && keep <= 1.0)) return BSR_ERR_KEEP;
  if (g.nblocks == 0) return BSR_OK;
  if (X == nullptr || keep_mask == nullptr) return BSR_ERR_NULL;
  if (misaligned(X, elem_bytes(dtype)) || misaligned(scores, 8) || misaligned(ws, 16)) return BSR_ERR_ALIGN;
  const size_t need = score_select_ws(g.nblocks);
  if (ws == nullptr || ws_bytes < need) return BSR_ERR_WORKSPACE;
  if (group_rows > g.nbr) group_rows = g.nbr;
  const int64_t groups = (g.nbr + group_rows - 1) / group_rows;
  const int64_t last_rows = g.nbr - (groups - 1) * group_rows;
  const int64_t n_keep_group = bsr_keep_count(group_rows * g.nbc, keep);
  const int64_t n_keep_last = bsr_keep_count(last_rows * g.nbc, keep);
  hipStream_t s = static_cast<hipStream_t>(stream);
  double *sc = scores != nullptr ? scores : static_cast<double *>(ws);
  rc = launch_score(X, dtype, M, K, ldx, br, bc, sc, s);
  if (rc != BSR_OK) return rc;
  return launch_select_grouped(sc, g.nbr, g.nbc, group_rows, n_keep_group, n_keep_last, keep_mask,
                               static_cast<char *>(ws) + scores_bytes(g.nblocks), s);
}

int bsr_compress(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                 const uint8_t *keep_mask, int64_t n_keep, int32_t *row_ptr, int32_t *col_idx,
                 void *values, void *ws, size_t ws_bytes, void *stream) {
  Geometry g;
  int rc = check_shape(dtype, M, K, ldx, br, bc, &g);
  if (rc != BSR_OK) return rc;
  if (n_keep < 0 || n_keep > g.nblocks) return BSR_ERR_KEEP;
  const size_t need = compress_ws_bytes(dtype, M, K, br, bc);
  if (need > 0 && (ws == nullptr || ws_bytes < need)) return BSR_ERR_WORKSPACE;
  if (need > 0 && misaligned(ws, 16)) return BSR_ERR_ALIGN;
  if (row_ptr == nullptr) return BSR_ERR_NULL;
  if (g.nblocks > 0 && (X == nullptr || keep_mask == nullptr)) return BSR_ERR_NULL;
  if (n_keep > 0 && (col_idx == nullptr || values == nullptr)) return BSR_ERR_NULL;
  if (misaligned(X, elem_bytes(dtype)) || misaligned(values, elem_bytes(dtype)) ||
      misaligned(row_ptr, 4) || misaligned(col_idx, 4))
    return BSR_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  return launch_compress(keep_mask, X, dtype, M, K, ldx, br, bc, n_keep, row_ptr, col_idx, values, ws, s);
}

int bsr_decompress(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype,
                   int64_t M, int64_t K, int64_t ldx, int br, int bc, void *X_out, void *stream) {
  Geometry g;
  int rc = check_shape(dtype, M, K, ldx, br, bc, &g);
  if (rc != BSR_OK) return rc;
  if (g.nblocks == 0) return BSR_OK;
  if (row_ptr == nullptr || X_out == nullptr) return BSR_ERR_NULL;
  if (misaligned(X_out, elem_bytes(dtype)) || misaligned(values, elem_bytes(dtype)) ||
      misaligned(row_ptr, 4) || misaligned(col_idx, 4))
    return BSR_ERR_ALIGN;
  return launch_decompress(row_ptr, col_idx, values, dtype, M, K, ldx, br, bc, X_out,
                           static_cast<hipStream_t>(stream));
}

int bsr_t_dense_matmul(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype,
                       int64_t M, int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy,
                       float *dW, int64_t lddw, int accumulate, void *ws, size_t ws_bytes,
                       void *stream) {
  Geometry g;
  int rc = check_shape(dtype, M, K, K, br, bc, &g);
  if (rc != BSR_OK) return rc;
  if (N < 0 || lddy < N || lddw < N || N > (int64_t(1) << 40)) return BSR_ERR_SHAPE;
  if (K == 0 || N == 0) return BSR_OK;
  if (dW == nullptr || row_ptr == nullptr) return BSR_ERR_NULL;
  if (M > 0 && dY == nullptr) return BSR_ERR_NULL;
  if (misaligned(values, elem_bytes(dtype)) || misaligned(dY, elem_bytes(dtype)) ||
      misaligned(dW, 4) || misaligned(row_ptr, 4) || misaligned(col_idx, 4) || misaligned(ws, 16))
    return BSR_ERR_ALIGN;
  const size_t need = bsr_workspace_bytes(BSR_OP_T_DENSE_MATMUL, M, K, N, br, bc, dtype);
  if (need > 0 && (ws == nullptr || ws_bytes < need)) return BSR_ERR_WORKSPACE;
  if (use_wide_single(dtype, br, bc, values, dY, M, K, N, lddy)) {
    const DwJob job{row_ptr, col_idx, values, M, K, br, bc, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes};
    return launch_dw_wide(job, static_cast<hipStream_t>(stream));
  }
  if (dw_mfma_supported(dtype, br, bc, values, M, K, N, lddy))
    return launch_dw_mfma(dtype, row_ptr, col_idx, values, M, K, br, bc, dY, N, lddy, dW, lddw, accumulate,
                          ws, ws_bytes, static_cast<hipStream_t>(stream));
  // other block shapes: re-tiled into 32x32 blocks for the matrix-core kernel, unless the
  // problem is so small that the single launch of the general kernel is the faster way
  if (M * K > 65536 && dw_reblock_supported(dtype, br, bc, M, K, N, lddy) &&
      ws_bytes >= dw_reblock_ws_bytes(dtype, M, K, N))
    return launch_dw_reblocked(dtype, row_ptr, col_idx, values, M, K, br, bc, dY, N, lddy, dW, lddw,
                               accumulate, ws, ws_bytes, static_cast<hipStream_t>(stream));
  return launch_dw_generic(row_ptr, col_idx, values, dtype, M, K, br, bc, dY, N, lddy, dW, lddw,
                           accumulate, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int bsr_affine_scale_grad(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype,
                          int64_t M, int64_t K, int br, int bc, const void *dY, int64_t lddy, float *dalpha,
                          int accumulate, void *ws, size_t ws_bytes, void *stream) {
  Geometry g;
  int rc = check_shape(dtype, M, K, K, br, bc, &g);
  if (rc != BSR_OK) return rc;
  if (lddy < K) return BSR_ERR_SHAPE;
  if (K == 0) return BSR_OK;
  if (dalpha == nullptr || row_ptr == nullptr) return BSR_ERR_NULL;
  if (M > 0 && dY == nullptr) return BSR_ERR_NULL;
  if (misaligned(values, elem_bytes(dtype)) || misaligned(dY, elem_bytes(dtype)) || misaligned(dalpha, 4) ||
      misaligned(row_ptr, 4) || misaligned(col_idx, 4) || misaligned(ws, 16))
    return BSR_ERR_ALIGN;
  const size_t need = bsr_workspace_bytes(BSR_OP_AFFINE_SCALE_GRAD, M, K, 0, br, bc, dtype);
  if (need > 0 && (ws == nullptr || ws_bytes < need)) return BSR_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (M == 0) return launch_splitk_reduce(nullptr, 0, 1, K, dalpha, K, accumulate, s);
  return launch_affine_dscale(row_ptr, col_idx, values, dtype, M, K, br, bc, dY, lddy, dalpha, accumulate, ws, s);
}

size_t bsr_score_select_batched_workspace_bytes(const bsr_select_item *items, int n, int dtype) {
  if (items == nullptr || n <= 0) return 0;
  size_t total = 0;
  for (int i = 0; i < n; ++i) {
    Geometry g;
    const bsr_select_item &it = items[i];
    if (check_shape(dtype, it.M, it.K, it.ldx, it.br, it.bc, &g) != BSR_OK) return 0;
    total += align_up(score_select_ws(g.nblocks), 256);
  }
  return total;
}

int bsr_score_select_batched(const bsr_select_item *items, int n, int dtype, void *ws, size_t ws_bytes,
                             void *stream) {
  if (n < 0) return BSR_ERR_SHAPE;
  if (n == 0) return BSR_OK;
  if (items == nullptr) return BSR_ERR_NULL;
  std::vector<ScoreJob> score_jobs;
  std::vector<SelectJob> select_jobs;
  score_jobs.reserve(n);
  select_jobs.reserve(n);
  if (misaligned(ws, 16)) return BSR_ERR_ALIGN;
  size_t off = 0;
  for (int i = 0; i < n; ++i) {
    const bsr_select_item &it = items[i];
    Geometry g;
    const int rc = check_shape(dtype, it.M, it.K, it.ldx, it.br, it.bc, &g);
    if (rc != BSR_OK) return rc;
    const int64_t n_keep = bsr_keep_count(g.nblocks, it.keep);
    if (n_keep < 0) return BSR_ERR_KEEP;
    if (g.nblocks == 0) continue;
    if (it.X == nullptr || it.keep_mask == nullptr) return BSR_ERR_NULL;
    if (misaligned(it.X, elem_bytes(dtype)) || misaligned(it.scores, 8)) return BSR_ERR_ALIGN;
    const size_t need = align_up(score_select_ws(g.nblocks), 256);
    if (ws == nullptr || off + need > ws_bytes) return BSR_ERR_WORKSPACE;
    char *base = static_cast<char *>(ws) + off;
    off += need;
    double *sc = it.scores != nullptr ? it.scores : reinterpret_cast<double *>(base);
    score_jobs.push_back(ScoreJob{it.X, it.M, it.K, it.ldx, it.br, it.bc, sc});
    select_jobs.push_back(SelectJob{sc, g.nblocks, n_keep, it.keep_mask, base + scores_bytes(g.nblocks)});
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int rc = launch_score_batched(score_jobs.data(), (int)score_jobs.size(), dtype, s);
  if (rc != BSR_OK) return rc;
  return launch_select_batched(select_jobs.data(), (int)select_jobs.size(), s);
}

int bsr_score_select_grouped_batched(const bsr_select_item *items, const int64_t *group_rows, int n, int dtype,
                                     void *ws, size_t ws_bytes, void *stream) {
  if (n < 0) return BSR_ERR_SHAPE;
  if (n == 0) return BSR_OK;
  if (items == nullptr || group_rows == nullptr) return BSR_ERR_NULL;
  if (misaligned(ws, 16)) return BSR_ERR_ALIGN;
  std::vector<ScoreJob> score_jobs;
  std::vector<GroupedSelectJob> select_jobs;
  score_jobs.reserve(n);
  select_jobs.reserve(n);
  size_t off = 0;
  for (int i = 0; i < n; ++i) {
    const bsr_select_item &it = items[i];
    Geometry g;
    const int rc = check_shape(dtype, it.M, it.K, it.ldx, it.br, it.bc, &g);
    if (rc != BSR_OK) return rc;
    if (group_rows[i] < 1) return BSR_ERR_SHAPE;
    if (!(it.keep >= 0.0 && it.keep <= 1.0)) return BSR_ERR_KEEP;
    if (g.nblocks == 0) continue;
    if (it.X == nullptr || it.keep_mask == nullptr) return BSR_ERR_NULL;
    if (misaligned(it.X, elem_bytes(dtype)) || misaligned(it.scores, 8)) return BSR_ERR_ALIGN;
    const size_t need = align_up(score_select_ws(g.nblocks), 256);
    if (ws == nullptr || off + need > ws_bytes) return BSR_ERR_WORKSPACE;
    char *base = static_cast<char *>(ws) + off;
    off += need;
    double *sc = it.scores != nullptr ? it.scores : reinterpret_cast<double *>(base);
    const int64_t rows = group_rows[i] > g.nbr ? g.nbr : group_rows[i];
    const int64_t groups = (g.nbr + rows - 1) / rows;
    const int64_t last_rows = g.nbr - (groups - 1) * rows;
    score_jobs.push_back(ScoreJob{it.X, it.M, it.K, it.ldx, it.br, it.bc, sc});
    select_jobs.push_back(GroupedSelectJob{sc, g.nbr, g.nbc, rows, bsr_keep_count(rows * g.nbc, it.keep),
                                           bsr_keep_count(last_rows * g.nbc, it.keep), it.keep_mask,
                                           base + scores_bytes(g.nblocks)});
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int rc = launch_score_batched(score_jobs.data(), (int)score_jobs.size(), dtype, s);
  if (rc != BSR_OK) return rc;
  return launch_select_grouped_batched(select_jobs.data(), (int)select_jobs.size(), s);
}

size_t bsr_t_dense_matmul_batched_workspace_bytes(const bsr_matmul_item *items, int n, int dtype) {
  if (items == nullptr || n <= 0) return 0;
  size_t total = 0;
  for (int i = 0; i < n; ++i) {
    const bsr_matmul_item &it = items[i];
    Geometry g;
    if (check_shape(dtype, it.M, it.K, it.K, it.br, it.bc, &g) != BSR_OK || it.N < 0) return 0;
    total += align_up(bsr_workspace_bytes(BSR_OP_T_DENSE_MATMUL, it.M, it.K, it.N, it.br, it.bc, dtype), 256);
  }
  return total;
}

int bsr_t_dense_matmul_batched(const bsr_matmul_item *items, int n, int dtype, void *ws, size_t ws_bytes,
                               void *stream) {
  if (n < 0) return BSR_ERR_SHAPE;
  if (n == 0) return BSR_OK;
  if (items == nullptr) return BSR_ERR_NULL;
  if (misaligned(ws, 16)) return BSR_ERR_ALIGN;
  std::vector<DwJob> batch, single, wide, narrow;
  batch.reserve(n);
  int64_t wide_par = 0;
  size_t off = 0;
  for (int i = 0; i < n; ++i) {
    const bsr_matmul_item &it = items[i];
    Geometry g;
    const int rc = check_shape(dtype, it.M, it.K, it.K, it.br, it.bc, &g);
    if (rc != BSR_OK) return rc;
    if (it.N < 0 || it.lddy < it.N || it.lddw < it.N || it.N > (int64_t(1) << 40)) return BSR_ERR_SHAPE;
    if (it.K == 0 || it.N == 0) continue;
    if (it.dW == nullptr || it.row_ptr == nullptr) return BSR_ERR_NULL;
    if (it.M > 0 && it.dY == nullptr) return BSR_ERR_NULL;
    if (misaligned(it.values, elem_bytes(dtype)) || misaligned(it.dY, elem_bytes(dtype)) || misaligned(it.dW, 4) ||
        misaligned(it.row_ptr, 4) || misaligned(it.col_idx, 4))
      return BSR_ERR_ALIGN;
    const size_t need = align_up(bsr_workspace_bytes(BSR_OP_T_DENSE_MATMUL, it.M, it.K, it.N, it.br, it.bc, dtype), 256);
    if (need > 0 && (ws == nullptr || off + need > ws_bytes)) return BSR_ERR_WORKSPACE;
    const DwJob job{it.row_ptr, it.col_idx, it.values, it.M, it.K, it.br, it.bc, it.dY, it.N, it.lddy, it.dW,
                    it.lddw, it.accumulate, need > 0 ? static_cast<char *>(ws) + off : nullptr, need};
    off += need;
    if (n > 1 && use_narrow(dtype, it.br, it.bc, it.values, it.dY, it.M, it.K, it.N, it.lddy)) {
      narrow.push_back(job);
    } else if (dw_wide_supported(dtype, it.br, it.bc, it.values, it.dY, it.M, it.K, it.N, it.lddy)) {
      wide.push_back(job);
      wide_par += wide_parallelism(it.M, it.K, it.N, it.br);
    } else if (dw_mfma_supported(dtype, it.br, it.bc, it.values, it.M, it.K, it.N, it.lddy)) {
      batch.push_back(job);
    } else {
      single.push_back(job);
    }
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // too few tiles to fill the GPU even with a deep split: the narrow-tile kernel suits those better
  if (!wide.empty() && wide_par < 128) {
    batch.insert(batch.end(), wide.begin(), wide.end());
    wide.clear();
  }
  // the partial tiles of both kinds of products are added up by one launch behind the two kernels
  std::vector<ReduceJob> reductions;
  int rc = launch_dw_wide_batched(wide.data(), (int)wide.size(), s, &reductions);
  if (rc == BSR_OK) rc = launch_dw_narrow_batched(narrow.data(), (int)narrow.size(), s, &reductions);
  if (rc == BSR_OK && !reductions.empty()) rc = launch_splitk_reduce_batched(reductions.data(), (int)reductions.size(), s);
  if (rc == BSR_OK) rc = launch_dw_mfma_batched(dtype, batch.data(), (int)batch.size(), s);
  for (size_t i = 0; rc == BSR_OK && i < single.size(); ++i) {
    const DwJob &j = single[i];
    rc = bsr_t_dense_matmul(j.row_ptr, j.col_idx, j.values, dtype, j.M, j.K, j.br, j.bc, j.dY, j.N, j.lddy, j.dW,
                            j.lddw, j.accumulate, j.ws, j.ws_bytes, stream);
  }
  return rc;
}

size_t bsr_compress_batched_workspace_bytes(const bsr_compress_item *items, int n, int dtype) {
  if (items == nullptr || n <= 0) return 0;
  size_t total = 0;
  for (int i = 0; i < n; ++i) {
    const bsr_compress_item &it = items[i];
    Geometry g;
    if (check_shape(dtype, it.M, it.K, it.ldx, it.br, it.bc, &g) != BSR_OK) return 0;
    total += align_up(compress_ws_bytes(dtype, it.M, it.K, it.br, it.bc), 256);
  }
  return total;
}

int bsr_compress_batched(const bsr_compress_item *items, int n, int dtype, void *ws, size_t ws_bytes,
                         void *stream) {
  if (n < 0) return BSR_ERR_SHAPE;
  if (n == 0) return BSR_OK;
  if (items == nullptr) return BSR_ERR_NULL;
  if (misaligned(ws, 16)) return BSR_ERR_ALIGN;
  std::vector<CompressJob> jobs;
  jobs.reserve((size_t)n);
  size_t off = 0;
  for (int i = 0; i < n; ++i) {
    const bsr_compress_item &it = items[i];
    Geometry g;
    const int rc = check_shape(dtype, it.M, it.K, it.ldx, it.br, it.bc, &g);
    if (rc != BSR_OK) return rc;
    if (it.n_keep < 0 || it.n_keep > g.nblocks) return BSR_ERR_KEEP;
    const size_t need = align_up(compress_ws_bytes(dtype, it.M, it.K, it.br, it.bc), 256);
    if (need > 0 && (ws == nullptr || off + need > ws_bytes)) return BSR_ERR_WORKSPACE;
    if (it.row_ptr == nullptr) return BSR_ERR_NULL;
    if (g.nblocks > 0 && (it.X == nullptr || it.keep_mask == nullptr)) return BSR_ERR_NULL;
    if (it.n_keep > 0 && (it.col_idx == nullptr || it.values == nullptr)) return BSR_ERR_NULL;
    if (misaligned(it.X, elem_bytes(dtype)) || misaligned(it.values, elem_bytes(dtype)) ||
        misaligned(it.row_ptr, 4) || misaligned(it.col_idx, 4))
      return BSR_ERR_ALIGN;
    jobs.push_back(CompressJob{it.keep_mask, it.X, it.M, it.K, it.ldx, it.br, it.bc, it.n_keep, it.row_ptr,
                               it.col_idx, it.values, need > 0 ? static_cast<char *>(ws) + off : nullptr});
    off += need;
  }
  return launch_compress_batched(jobs.data(), (int)jobs.size(), dtype, static_cast<hipStream_t>(stream));
}

int bsr_decompress_batched(const bsr_decompress_item *items, int n, int dtype, void *stream) {
  if (n < 0) return BSR_ERR_SHAPE;
  if (n == 0) return BSR_OK;
  if (items == nullptr) return BSR_ERR_NULL;
  std::vector<DecompressJob> jobs;
  jobs.reserve((size_t)n);
  for (int i = 0; i < n; ++i) {
    const bsr_decompress_item &it = items[i];
    Geometry g;
    const int rc = check_shape(dtype, it.M, it.K, it.ldx, it.br, it.bc, &g);
    if (rc != BSR_OK) return rc;
    if (g.nblocks == 0) continue;
    if (it.row_ptr == nullptr || it.X_out == nullptr) return BSR_ERR_NULL;
    if (misaligned(it.X_out, elem_bytes(dtype)) || misaligned(it.values, elem_bytes(dtype)) ||
        misaligned(it.row_ptr, 4) || misaligned(it.col_idx, 4))
      return BSR_ERR_ALIGN;
    jobs.push_back(DecompressJob{it.row_ptr, it.col_idx, it.values, it.M, it.K, it.ldx, it.br, it.bc, it.X_out});
  }
  return launch_decompress_batched(jobs.data(), (int)jobs.size(), dtype, static_cast<hipStream_t>(stream));
}

}  // extern "C"
