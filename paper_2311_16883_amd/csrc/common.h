// Internal declarations shared by the HIP translation units of libbsr_actprune.
// Nothing here is part of the C ABI (see include/bsr_actprune.h).
#pragma once

#include <hip/hip_runtime.h>

#include <vector>
#include <stddef.h>
#include <stdint.h>

#include "bsr_actprune.h"

namespace bsr {

__host__ __device__ static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static inline int elem_bytes(int dtype) { return dtype == BSR_F32 ? 4 : 2; }

// Largest power-of-two vector width (in elements, at most max_v) such that
// every vector access stays inside one block row and is naturally aligned.
static inline int pick_vector(int max_v, int esize, int64_t bc, int64_t K, int64_t ld,
                              const void *p0, const void *p1 = nullptr) {
  int v = max_v;
  while (v > 1) {
    uintptr_t a = (uintptr_t)v * (uintptr_t)esize;
    bool ok = bc % v == 0 && K % v == 0 && ld % v == 0 && (uintptr_t)p0 % a == 0 &&
              (p1 == nullptr || (uintptr_t)p1 % a == 0);
    if (ok) break;
    v >>= 1;
  }
  return v;
}

// Records hipGetLastError() after a launch; returns BSR_OK or BSR_ERR_HIP.
int check_launch();
void set_hip_error(int e);

// ---- launchers (one per kernel family); all enqueue on `s` and return ----

// score.hip: scores[i*nbc+j] = sum of squares of block (i,j), binary64.
int launch_score(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                 double *scores, hipStream_t s);

// several tensors scored with as few launches as their shapes allow
struct ScoreJob {
  const void *X;
  int64_t M, K, ldx;
  int br, bc;
  double *scores;
};
int launch_score_batched(const ScoreJob *jobs, int n, int dtype, hipStream_t s);

// select.hip: keep_mask = 1 for the n_keep best (score desc, index asc).
size_t select_ws_bytes(int64_t nblocks);
int launch_select(const double *scores, int64_t nblocks, int64_t n_keep, uint8_t *keep_mask, void *ws,
                  hipStream_t s);

// several independent selections with as few launches as their sizes allow
struct SelectJob {
  const double *scores;
  int64_t nblocks, n_keep;
  uint8_t *mask;
  void *ws;            // select_ws_bytes(nblocks) bytes of its own
};
int launch_select_batched(const SelectJob *jobs, int n, hipStream_t s);

// per-group selection: groups of group_rows block-rows, n_keep_group kept per full group
int launch_select_grouped(const double *scores, int64_t nbr, int64_t nbc, int64_t group_rows,
                          int64_t n_keep_group, int64_t n_keep_last, uint8_t *keep_mask, void *ws,
                          hipStream_t s);

// ... of several tensors, those with groups of a similar size sharing launches
struct GroupedSelectJob {
  const double *scores;
  int64_t nbr, nbc, group_rows, n_keep_group, n_keep_last;
  uint8_t *mask;
  void *ws;            // select_ws_bytes(nbr * nbc) bytes of its own
};
int launch_select_grouped_batched(const GroupedSelectJob *jobs, int n, hipStream_t s);

// pack.hip
int launch_index_build(const uint8_t *keep_mask, int64_t nbr, int64_t nbc, int64_t n_keep,
                       int32_t *row_ptr, int32_t *col_idx, hipStream_t s);
int launch_pack(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                const int32_t *row_ptr, const int32_t *col_idx, int64_t n_keep, void *values,
                hipStream_t s);
// mask -> row_ptr, col_idx, values (one fused launch when the shape allows it)
size_t compress_ws_bytes(int dtype, int64_t M, int64_t K, int br, int bc);
int launch_compress(const uint8_t *keep_mask, const void *X, int dtype, int64_t M, int64_t K, int64_t ldx,
                    int br, int bc, int64_t n_keep, int32_t *row_ptr, int32_t *col_idx, void *values,
                    void *ws, hipStream_t s);
int launch_decompress(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype,
                      int64_t M, int64_t K, int64_t ldx, int br, int bc, void *X_out, hipStream_t s);

// Several tensors per call (see launch_compress_batched in pack.hip).
struct CompressJob {
  const uint8_t *keep_mask;
  const void *X;
  int64_t M, K, ldx;
  int br, bc;
  int64_t n_keep;
  int32_t *row_ptr, *col_idx;
  void *values;
  void *ws;                // this tensor's workspace (compress_ws_bytes), may be null when none is needed
};
struct DecompressJob {
  const int32_t *row_ptr, *col_idx;
  const void *values;
  int64_t M, K, ldx;
  int br, bc;
  void *X_out;
};
int launch_compress_batched(const CompressJob *jobs, int n, int dtype, hipStream_t s);
int launch_decompress_batched(const DecompressJob *jobs, int n, int dtype, hipStream_t s);

// dw_generic.hip: any block shape, binary32 FMA.
size_t dw_generic_ws_bytes(int64_t M, int64_t K, int64_t N, int br, int bc);
int launch_dw_generic(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype,
                      int64_t M, int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy,
                      float *dW, int64_t lddw, int accumulate, void *ws, size_t ws_bytes,
                      hipStream_t s);

// dw_mfma.hip: bfloat16 and binary32 on the matrix cores, block shapes 32x32, 64x64, 16x16, 14x14.
bool dw_mfma_supported(int dtype, int br, int bc, const void *values, int64_t M, int64_t K, int64_t N,
                       int64_t lddy);
size_t dw_mfma_ws_bytes(int dtype, int64_t M, int64_t K, int64_t N, int br, int bc);
int launch_dw_mfma(int dtype, const int32_t *row_ptr, const int32_t *col_idx, const void *values, int64_t M,
                   int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy, float *dW,
                   int64_t lddw, int accumulate, void *ws, size_t ws_bytes, hipStream_t s);

// reblock.hip: any block shape re-tiled into 32x32 blocks in the workspace, then dw_mfma.
bool dw_reblock_supported(int dtype, int br, int bc, int64_t M, int64_t K, int64_t N, int64_t lddy);
size_t dw_reblock_ws_bytes(int dtype, int64_t M, int64_t K, int64_t N);
int launch_dw_reblocked(int dtype, const int32_t *row_ptr, const int32_t *col_idx, const void *values, int64_t M,
                        int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy, float *dW,
                        int64_t lddw, int accumulate, void *ws, size_t ws_bytes, hipStream_t s);

// affine.hip: dalpha[k] = sum over kept blocks of values * dY at the same position.
size_t affine_ws_bytes(int64_t M, int64_t K, int br, int bc);
int launch_affine_dscale(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int dtype, int64_t M,
                         int64_t K, int br, int bc, const void *dY, int64_t lddy, float *dalpha, int accumulate,
                         void *ws, hipStream_t s);

// dw_generic.hip: dW = (accumulate ? dW : 0) + sum_s partial[s], s ascending.
int launch_splitk_reduce(const float *partial, int splits, int64_t K, int64_t N, float *dW,
                         int64_t lddw, int accumulate, hipStream_t s);

// Geometry of the kernels that stage whole block-rows in LDS (score.hip, pack.hip).
// They serve blocks whose rows are narrower than a 16-byte vector (14x14 patches:
// 28-byte rows) and blocks of few rows (1 x b row segments: a block-row is too
// little work for a workgroup) when the matrix rows are contiguous (ld == K), so
// that the rows of `rb` consecutive block-rows form one contiguous span that is
// read or written with wide linear accesses and re-ordered through LDS.  Sizes are
// in 32-bit words.
constexpr int kSpanBytes = 16384;   // LDS span of one workgroup
constexpr int kSpanList = 1024;     // kept blocks one workgroup can list
constexpr int kSpanRows = 32;       // block-rows one workgroup can take
struct SpanGeom {
  int rb;          // block-rows per workgroup
  int br;          // rows per block
  int nbc;         // block-columns
  int row_words;   // K * e / 4
  int seg_words;   // bc * e / 4
  int blk_words;   // br * seg_words
  int vb;          // bytes per linear access (16, 8 or 4): divides the row pitch
  uint32_t magic_blk, magic_seg, magic_nbc, magic_br;   // see span_div
};
// True (and *g filled) when the shape qualifies; p0 / p1 are the dense matrices
// involved (16-byte alignment needed), either may be null.
bool span_geometry(int dtype, int64_t M, int64_t K, int64_t ld, int br, int bc, const void *p0,
                   const void *p1, SpanGeom *g);

// Several reductions / several dW products per launch.
constexpr int kReduceBatchMax = 24;
struct ReduceJob {
  const float *partial;
  float *dW;
  int64_t K, N, lddw;
  int splits, accumulate;
};
int launch_splitk_reduce_batched(const ReduceJob *jobs, int n, hipStream_t s);

struct DwJob {
  const int32_t *row_ptr, *col_idx;
  const void *values;
  int64_t M, K;
  int br, bc;
  const void *dY;
  int64_t N, lddy;
  float *dW;
  int64_t lddw;
  int accumulate;
  void *ws;
  size_t ws_bytes;
};
// dw_mfma.hip: the jobs (all of block shapes and sizes dw_mfma_supported accepts, none with
// K == 0 or N == 0) with as few launches as their kernel instances allow.
int launch_dw_mfma_batched(int dtype, const DwJob *jobs, int n, hipStream_t s);

// dw_wide.hip: bfloat16, 32x32 / 64x64 blocks, 384-row tiles fed by global -> LDS copies.
// dw_narrow.hip: bfloat16, small square blocks, a weight matrix of at most 224 x 224: one workgroup owns all of dW
bool dw_narrow_supported(int dtype, int br, int bc, const void *values, const void *dY, int64_t M, int64_t K,
                         int64_t N, int64_t lddy);
size_t dw_narrow_ws_bytes(int64_t M, int64_t K, int64_t N, int br);
// `later`: when not null, the reductions of the products that were split are appended there instead of
// being launched: the caller launches them (launch_splitk_reduce_batched) once its other kernels are queued.
int launch_dw_narrow_batched(const DwJob *jobs, int n, hipStream_t s, std::vector<ReduceJob> *later = nullptr);
bool dw_wide_supported(int dtype, int br, int bc, const void *values, const void *dY, int64_t M, int64_t K,
                       int64_t N, int64_t lddy);
size_t dw_wide_ws_bytes(int64_t M, int64_t K, int64_t N, int br);
int launch_dw_wide(const DwJob &j, hipStream_t s);
int launch_dw_wide_batched(const DwJob *jobs, int n, hipStream_t s, std::vector<ReduceJob> *later = nullptr);

// ---- device helpers ----

// w / d for w * d < 2^32, with magic = ceil(2^32 / d) (d == 1 has no 32-bit magic)
__device__ __forceinline__ uint32_t span_div(uint32_t w, uint32_t d, uint32_t magic) {
  return d == 1 ? w : __umulhi(w, magic);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) {
  return __uint_as_float((uint32_t)h << 16);
}

template <typename T>
__device__ __forceinline__ float elem_to_float(T v);
template <>
__device__ __forceinline__ float elem_to_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ float elem_to_float<uint16_t>(uint16_t v) { return bf16_bits_to_float(v); }

template <typename T, int V>
struct alignas(sizeof(T) * V) Vec {
  T e[V];
};

// Loads and stores of data that the kernel touches once (the streaming side of the HBM-bound
// kernels): non-temporal accesses, which leave the caches to what is read again.  V is any
// trivially copyable type of 2, 4, 8 or 16 bytes at its natural alignment.
template <typename V>
__device__ __forceinline__ V load_stream(const V *p) {
  typedef uint32_t __attribute__((ext_vector_type(4))) w4;
  typedef uint32_t __attribute__((ext_vector_type(2))) w2;
  static_assert(sizeof(V) == 16 || sizeof(V) == 8 || sizeof(V) == 4 || sizeof(V) == 2, "2, 4, 8 or 16 bytes");
  if constexpr (sizeof(V) == 16) return __builtin_bit_cast(V, __builtin_nontemporal_load(reinterpret_cast<const w4 *>(p)));
  else if constexpr (sizeof(V) == 8) return __builtin_bit_cast(V, __builtin_nontemporal_load(reinterpret_cast<const w2 *>(p)));
  else if constexpr (sizeof(V) == 4) return __builtin_bit_cast(V, __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p)));
  else return __builtin_bit_cast(V, __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(p)));
}
template <typename V>
__device__ __forceinline__ void store_stream(V *p, const V &v) {
  typedef uint32_t __attribute__((ext_vector_type(4))) w4;
  typedef uint32_t __attribute__((ext_vector_type(2))) w2;
  static_assert(sizeof(V) == 16 || sizeof(V) == 8 || sizeof(V) == 4 || sizeof(V) == 2, "2, 4, 8 or 16 bytes");
  if constexpr (sizeof(V) == 16) __builtin_nontemporal_store(__builtin_bit_cast(w4, v), reinterpret_cast<w4 *>(p));
  else if constexpr (sizeof(V) == 8) __builtin_nontemporal_store(__builtin_bit_cast(w2, v), reinterpret_cast<w2 *>(p));
  else if constexpr (sizeof(V) == 4) __builtin_nontemporal_store(__builtin_bit_cast(uint32_t, v), reinterpret_cast<uint32_t *>(p));
  else __builtin_nontemporal_store(__builtin_bit_cast(uint16_t, v), reinterpret_cast<uint16_t *>(p));
}

}  // namespace bsr
