// Weight gradient from a BSR activation on the matrix cores (paper Sec. III,
// Fig. 2: dW = Xhat^T * dY, "BSpMM"), bfloat16 inputs, binary32 accumulation.
//
// Both operands are stored with the contraction index m (activation rows) as
// the slow axis -- a kept block is [r][c] with c = output row of dW, dY is
// [m][n] -- while v_mfma_f32_32x32x16_bf16 wants every lane to hold 8
// consecutive contraction elements.  Tiles therefore go to LDS in their natural
// row-major order and the fragments come back through ds_read_b64_tr_b16, which
// transposes 4 x 16 sub-tiles across 16 lanes.
//
// Work decomposition.  A workgroup (4 waves, 2 x 2) owns a KT x NT tile of dW
// and a contiguous range of block-rows (split of the contraction).  At start it
// turns the BSR row segments that cross its tile into one (bit mask, first
// position) pair per block-row in LDS; after that the main loop reads no index
// from global memory.  The loop walks stages of MS activation rows: the kept
// blocks of the stage are copied into a dense LDS tile (zeros where a pruned
// block shares a 32-wide matrix-core tile with a kept one), dY rows next to it,
// and every 16-row x 32-column piece of the activation tile that holds no kept
// block is skipped by a wave-uniform branch -- the sparsity is exploited at
// matrix-core granularity.  Global loads of stage s+1 are in flight (held in
// registers) while stage s is multiplied.  With more than one split the partial
// tiles go to the workspace and a second kernel adds them in a fixed order.
#include "common.h"

namespace bsr {

namespace {

typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(16))) float v16f;

constexpr int kThreads = 256;
constexpr int kMaxRowsPerSplit = 1024;   // block-rows whose tile index fits in LDS

template <int BYTES> struct Chunk;
template <> struct Chunk<16> { typedef uint4 type; };
template <> struct Chunk<8> { typedef uint2 type; };
template <> struct Chunk<4> { typedef uint32_t type; };
template <> struct Chunk<2> { typedef uint16_t type; };

template <int BYTES> __device__ __forceinline__ typename Chunk<BYTES>::type chunk_zero();
template <> __device__ __forceinline__ uint4 chunk_zero<16>() { return make_uint4(0, 0, 0, 0); }
template <> __device__ __forceinline__ uint2 chunk_zero<8>() { return make_uint2(0, 0); }
template <> __device__ __forceinline__ uint32_t chunk_zero<4>() { return 0u; }
template <> __device__ __forceinline__ uint16_t chunk_zero<2>() { return 0; }

// 8 contraction elements x 16 rows/columns for this lane's 16-lane group,
// transposed out of a row-major LDS tile (two 4 x 16 sub-tiles).
__device__ __forceinline__ v8bf read_fragment(const uint16_t *tile, int ld, int row0, int col0) {
  const int l = threadIdx.x & 63, g = l >> 4, L = l & 15;
  const int row = row0 + 8 * (g >> 1) + (L >> 2);
  const int col = col0 + 16 * (g & 1) + 4 * (L & 3);
  const uint16_t *p = tile + row * ld + col;
  typedef v4s __attribute__((address_space(3))) * lds_v4s;
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * ld));
  v8s r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return __builtin_bit_cast(v8bf, r);
}

template <int BR, int BC, int MS, int KT, int NT, int VB>
struct Geo {
  static constexpr int R = MS / BR;                       // block-rows per stage
  static constexpr int ROWS = R * BR;                     // rows of a stage that carry data
  static constexpr bool KALIGNED = (KT % BC == 0);
  static constexpr int JT = KALIGNED ? KT / BC : KT / BC + 2;   // block-columns that can cross a tile
  static constexpr bool SKIP_ONLY = (BC % 32 == 0) && (BR % 16 == 0) && KALIGNED;  // no zero fill needed
  static constexpr int VA = (BC % 8 == 0) ? 8 : ((BC % 4 == 0) ? 4 : ((BC % 2 == 0) ? 2 : 1));
  static constexpr int VPB = BR * BC / VA;                // vectors per block
  static constexpr int NA = (R * JT * VPB + kThreads - 1) / kThreads;
  static constexpr int NB = (ROWS * (NT / VB) + kThreads - 1) / kThreads;
  static constexpr int LDA = KT + 16, LDB = NT + 16;      // padded LDS rows (elements)
  static constexpr int KSUB = KT / 32, NSUB = NT / 32, MSUB = MS / 16;
  static_assert(MS % 16 == 0 && KT % 64 == 0 && NT % 64 == 0 && R >= 1, "tile shape");
  static_assert(JT <= 32, "tile index is a 32-bit mask");
  static_assert(NA <= 16, "2 state bits per staged vector");
};

template <int BR, int BC, int MS, int KT, int NT, int VB>
__global__ __launch_bounds__(kThreads) void dw_mfma_kernel(
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const uint16_t *__restrict__ values, const uint16_t *__restrict__ dY, float *__restrict__ out,
    int64_t M, int64_t K, int64_t N, int64_t lddy, int64_t ldo, int64_t split_stride, int64_t nbr,
    int64_t nbc, int64_t stages_per_split, int accumulate) {
  typedef Geo<BR, BC, MS, KT, NT, VB> G;
  typedef typename Chunk<G::VA * 2>::type AVec;
  typedef typename Chunk<VB * 2>::type BVec;

  __shared__ __attribute__((aligned(16))) uint16_t sA[MS * G::LDA];
  __shared__ __attribute__((aligned(16))) uint16_t sB[MS * G::LDB];
  __shared__ uint32_t sMask[kMaxRowsPerSplit];
  __shared__ int32_t sBase[kMaxRowsPerSplit];
  __shared__ uint32_t sAct[2][G::MSUB];

  const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
  const int wk = wave >> 1, wn = wave & 1;
  const int64_t k0 = (int64_t)blockIdx.x * KT, n0 = (int64_t)blockIdx.y * NT;
  const int64_t total_stages = ceil_div(nbr, G::R);
  const int64_t s_begin = (int64_t)blockIdx.z * stages_per_split;
  int64_t s_end = s_begin + stages_per_split;
  if (s_end > total_stages) s_end = total_stages;
  const int64_t i_begin = s_begin * G::R;
  const int nrows = (int)((s_end - s_begin) * G::R);       // block-rows of this split (may run past nbr)
  const int64_t jfirst = k0 / BC;
  int64_t jlast = (k0 + KT - 1) / BC;
  if (jlast > nbc - 1) jlast = nbc - 1;
  const int jt = (int)(jlast - jfirst + 1);

  // ---- tile index: per block-row, which block-columns of the tile are kept ----
  for (int e = t; e < MS * G::LDA / 2; e += kThreads) reinterpret_cast<uint32_t *>(sA)[e] = 0u;
  for (int e = t; e < MS * G::LDB / 2; e += kThreads) reinterpret_cast<uint32_t *>(sB)[e] = 0u;
  if (t < 2 * G::MSUB) (&sAct[0][0])[t] = 0u;
  for (int rr = t; rr < nrows; rr += kThreads) {
    const int64_t i = i_begin + rr;
    uint32_t mask = 0;
    int32_t base = 0;
    if (i < nbr) {
      const int32_t p0 = row_ptr[i], p1 = row_ptr[i + 1];
      bool first = true;
      for (int32_t p = p0; p < p1; ++p) {
        const int64_t j = col_idx[p];
        if (j >= jfirst && j <= jlast) {
          if (first) { base = p; first = false; }
          mask |= 1u << (int)(j - jfirst);
        }
      }
    }
    sMask[rr] = mask;
    sBase[rr] = base;
  }
  __syncthreads();

  AVec ra[G::NA];
  uint32_t ra_state = 0;     // 2 bits per vector: 0 = leave LDS alone, 1 = data, 2 = zeros
  BVec rb[G::NB];

  auto prefetch = [&](int64_t s) {
    const int rr0 = (int)((s - s_begin) * G::R);
    ra_state = 0;
#pragma unroll
    for (int it = 0; it < G::NA; ++it) {
      const int v = t + it * kThreads;
      const int slot = v / G::VPB, off = v % G::VPB;
      const int rbk = slot / G::JT, jl = slot % G::JT;
      ra[it] = chunk_zero<G::VA * 2>();
      if (slot < G::R * G::JT && jl < jt) {
        const uint32_t mask = sMask[rr0 + rbk];
        if ((mask >> jl) & 1u) {
          const int64_t p = (int64_t)sBase[rr0 + rbk] + __popc(mask & ((1u << jl) - 1u));
          ra[it] = *reinterpret_cast<const AVec *>(values + p * (BR * BC) + (int64_t)off * G::VA);
          ra_state |= 1u << (2 * it);
        } else if (!G::SKIP_ONLY) {
          ra_state |= 2u << (2 * it);
        }
      }
    }
    const int64_t m0 = (i_begin + rr0) * BR;
#pragma unroll
    for (int it = 0; it < G::NB; ++it) {
      const int v = t + it * kThreads;
      const int r = v / (NT / VB), c = (v % (NT / VB)) * VB;
      rb[it] = chunk_zero<VB * 2>();
      if (r < G::ROWS && m0 + r < M && n0 + c < N)
        rb[it] = *reinterpret_cast<const BVec *>(dY + (m0 + r) * lddy + n0 + c);
    }
  };

  auto stage_to_lds = [&](int64_t s) {
    const int rr0 = (int)((s - s_begin) * G::R);
    const int par = (int)(s & 1);
#pragma unroll
    for (int it = 0; it < G::NA; ++it) {
      const uint32_t st = (ra_state >> (2 * it)) & 3u;
      if (st == 0) continue;
      const int v = t + it * kThreads;
      const int slot = v / G::VPB, off = v % G::VPB;
      const int rbk = slot / G::JT, jl = slot % G::JT;
      const int r = (off * G::VA) / BC, c = (off * G::VA) % BC;
      const int col = (int)((jfirst + jl) * BC - k0) + c;
      if (col < 0 || col + G::VA > KT) continue;
      *reinterpret_cast<AVec *>(&sA[(rbk * BR + r) * G::LDA + col]) = ra[it];
    }
#pragma unroll
    for (int it = 0; it < G::NB; ++it) {
      const int v = t + it * kThreads;
      const int r = v / (NT / VB), c = (v % (NT / VB)) * VB;
      if (r < G::ROWS) *reinterpret_cast<BVec *>(&sB[r * G::LDB + c]) = rb[it];
    }
    // which 16-row x 32-column pieces of the activation tile hold a kept block
    if (t < G::R * G::JT) {
      const int rbk = t / G::JT, jl = t % G::JT;
      if (jl < jt && ((sMask[rr0 + rbk] >> jl) & 1u)) {
        int c0 = (int)((jfirst + jl) * BC - k0), c1 = c0 + BC - 1;
        if (c0 < 0) c0 = 0;
        if (c1 > KT - 1) c1 = KT - 1;
        if (c0 <= c1) {
          const uint32_t bits = ((2u << (c1 >> 5)) - 1u) & ~((1u << (c0 >> 5)) - 1u);
          for (int ms = (rbk * BR) >> 4; ms <= (rbk * BR + BR - 1) >> 4; ++ms) atomicOr(&sAct[par][ms], bits);
        }
      }
    }
    if (t < G::MSUB) sAct[par ^ 1][t] = 0u;
  };

  v16f acc[2][2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[u][w][r] = 0.f;

  static_assert(KT == 128 && NT == 128, "2 x 2 waves of 64 x 64");

  if (s_begin < s_end) prefetch(s_begin);
  for (int64_t s = s_begin; s < s_end; ++s) {
    stage_to_lds(s);
    __syncthreads();
    if (s + 1 < s_end) prefetch(s + 1);
    const int par = (int)(s & 1);
#pragma unroll
    for (int ms = 0; ms < G::MSUB; ++ms) {
      const uint32_t act = (uint32_t)__builtin_amdgcn_readfirstlane((int)sAct[par][ms]);
      const uint32_t mine = (act >> (2 * wk)) & 3u;
      if (mine == 0) continue;
      const v8bf b0 = read_fragment(sB, G::LDB, ms * 16, (2 * wn) * 32);
      const v8bf b1 = read_fragment(sB, G::LDB, ms * 16, (2 * wn + 1) * 32);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (!((mine >> u) & 1u)) continue;
        const v8bf a = read_fragment(sA, G::LDA, ms * 16, (2 * wk + u) * 32);
        acc[u][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b0, acc[u][0], 0, 0, 0);
        acc[u][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b1, acc[u][1], 0, 0, 0);
      }
    }
    __syncthreads();
  }

  float *o = out + (int64_t)blockIdx.z * split_stride;
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int w = 0; w < 2; ++w)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t k = k0 + (2 * wk + u) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int64_t n = n0 + (2 * wn + w) * 32 + (lane & 31);
        if (k < K && n < N) {
          float *dst = o + k * ldo + n;
          *dst = accumulate ? *dst + acc[u][w][r] : acc[u][w][r];
        }
      }
}

struct Plan {
  int splits;
  int64_t stages_per_split;
};

template <int BR, int MS>
Plan make_plan(int64_t M, int64_t K, int64_t N) {
  constexpr int R = MS / BR;
  const int64_t nbr = ceil_div(M, BR);
  const int64_t stages = ceil_div(nbr, R);
  const int64_t tiles = ceil_div(K, 128) * ceil_div(N, 128);
  int64_t s = 1024 / (tiles > 0 ? tiles : 1);
  if (s > stages) s = stages;
  if (s < 1) s = 1;
  int64_t sps = stages > 0 ? ceil_div(stages, s) : 1;
  if (sps * R > kMaxRowsPerSplit) sps = kMaxRowsPerSplit / R;
  s = stages > 0 ? ceil_div(stages, sps) : 1;
  Plan p;
  p.splits = (int)s;
  p.stages_per_split = sps;
  return p;
}

template <int BR, int BC, int MS>
int run(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int64_t M, int64_t K,
        const void *dY, int64_t N, int64_t lddy, float *dW, int64_t lddw, int accumulate, void *ws,
        size_t ws_bytes, hipStream_t s) {
  const Plan p = make_plan<BR, MS>(M, K, N);
  const size_t need = p.splits > 1 ? (size_t)p.splits * K * N * sizeof(float) : 0;
  if (need > 0 && (ws == nullptr || ws_bytes < need)) return BSR_ERR_WORKSPACE;
  const int64_t nbr = ceil_div(M, BR), nbc = ceil_div(K, BC);
  float *out = p.splits > 1 ? static_cast<float *>(ws) : dW;
  const int64_t ldo = p.splits > 1 ? N : lddw;
  const int64_t stride = p.splits > 1 ? K * N : 0;
  const int acc_direct = p.splits > 1 ? 0 : accumulate;
  dim3 grid((unsigned)ceil_div(K, 128), (unsigned)ceil_div(N, 128), (unsigned)p.splits);
  const uint16_t *v = static_cast<const uint16_t *>(values);
  const uint16_t *y = static_cast<const uint16_t *>(dY);
  int vb = 8;
  while (vb > 1 && (N % vb != 0 || lddy % vb != 0 || (uintptr_t)dY % (2 * vb) != 0)) vb >>= 1;
#define BSR_DW_LAUNCH(VB)                                                                         \
  hipLaunchKernelGGL((dw_mfma_kernel<BR, BC, MS, 128, 128, VB>), grid, dim3(kThreads), 0, s,       \
                     row_ptr, col_idx, v, y, out, M, K, N, lddy, ldo, stride, nbr, nbc,            \
                     p.stages_per_split, acc_direct)
  if (vb == 8) BSR_DW_LAUNCH(8);
  else if (vb == 4) BSR_DW_LAUNCH(4);
  else if (vb == 2) BSR_DW_LAUNCH(2);
  else BSR_DW_LAUNCH(1);
#undef BSR_DW_LAUNCH
  int rc = check_launch();
  if (rc != BSR_OK || p.splits == 1) return rc;
  return launch_splitk_reduce(out, p.splits, K, N, dW, lddw, accumulate, s);
}

template <int BR, int MS>
size_t ws_for(int64_t M, int64_t K, int64_t N) {
  const Plan p = make_plan<BR, MS>(M, K, N);
  return p.splits > 1 ? (size_t)p.splits * K * N * sizeof(float) : 0;
}

}  // namespace

bool dw_mfma_supported(int dtype, int br, int bc, const void *values) {
  if (dtype != BSR_BF16) return false;
  if ((uintptr_t)values % 16 != 0) return false;
  return (br == 32 && bc == 32) || (br == 64 && bc == 64) || (br == 16 && bc == 16) ||
         (br == 14 && bc == 14);
}

size_t dw_mfma_ws_bytes(int64_t M, int64_t K, int64_t N, int br, int bc) {
  (void)bc;
  switch (br) {
    case 32: return ws_for<32, 32>(M, K, N);
    case 64: return ws_for<64, 64>(M, K, N);
    case 16: return ws_for<16, 32>(M, K, N);
    case 14: return ws_for<14, 32>(M, K, N);
    default: return 0;
  }
}

int launch_dw_mfma(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int64_t M,
                   int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy, float *dW,
                   int64_t lddw, int accumulate, void *ws, size_t ws_bytes, hipStream_t s) {
  if (K == 0 || N == 0) return BSR_OK;
  if (br == 32 && bc == 32)
    return run<32, 32, 32>(row_ptr, col_idx, values, M, K, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes, s);
  if (br == 64 && bc == 64)
    return run<64, 64, 64>(row_ptr, col_idx, values, M, K, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes, s);
  if (br == 16 && bc == 16)
    return run<16, 16, 32>(row_ptr, col_idx, values, M, K, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes, s);
  if (br == 14 && bc == 14)
    return run<14, 14, 32>(row_ptr, col_idx, values, M, K, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes, s);
  return BSR_ERR_SHAPE;
}

}  // namespace bsr
