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
#include <cstdlib>

#include "common.h"

namespace bsr {

namespace {

typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(16))) float v16f;

constexpr int kMaxRowsPerSplit = 512;   // block-rows whose tile index fits in LDS

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

template <int BYTES> struct Chunk;
template <> struct Chunk<16> { typedef u32x4 type; };
template <> struct Chunk<8> { typedef u32x2 type; };
template <> struct Chunk<4> { typedef uint32_t type; };
template <> struct Chunk<2> { typedef uint16_t type; };

constexpr uint32_t kOutOfRange = 0xFFFFFFFFu;   // buffer offset that reads as zero, touches no memory

// Untyped buffer resource over [base, base + bytes): loads at offsets beyond
// `bytes` return zero without a memory access, which predicates a load without
// a branch (the compiler can then count outstanding loads exactly).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// off = per-lane byte offset (range-checked against the descriptor), soff =
// wave-uniform byte offset added to the address.
template <int BYTES>
__device__ __forceinline__ typename Chunk<BYTES>::type buffer_load(__amdgpu_buffer_rsrc_t r, uint32_t off,
                                                                   uint32_t soff = 0);
template <> __device__ __forceinline__ u32x4 buffer_load<16>(__amdgpu_buffer_rsrc_t r, uint32_t off, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, off, soff, 0);
}
template <> __device__ __forceinline__ u32x2 buffer_load<8>(__amdgpu_buffer_rsrc_t r, uint32_t off, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b64(r, off, soff, 0);
}
template <> __device__ __forceinline__ uint32_t buffer_load<4>(__amdgpu_buffer_rsrc_t r, uint32_t off, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b32(r, off, soff, 0);
}
template <> __device__ __forceinline__ uint16_t buffer_load<2>(__amdgpu_buffer_rsrc_t r, uint32_t off, uint32_t soff) {
  return __builtin_amdgcn_raw_buffer_load_b16(r, off, soff, 0);
}

// 8 contraction elements x 16 rows/columns for this lane's 16-lane group,
// transposed out of a row-major LDS tile (two 4 x 16 sub-tiles).  `p` already
// points at this lane's first sub-tile (see lane_fragment_offset).
__device__ __forceinline__ v8bf read_fragment(const uint16_t *p, int ld) {
  typedef v4s __attribute__((address_space(3))) * lds_v4s;
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * ld));
  v8s r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return __builtin_bit_cast(v8bf, r);
}

// LDS tiles are 128 elements (256 bytes, all 64 banks) wide and unpadded.  The
// transposing read fetches four consecutive rows per 16-lane group, which
// would all hit the same banks; so the 32-byte chunk index of every element
// is XOR-ed with twice the row's low two bits: four consecutive rows of one
// chunk, and of the neighbouring chunk read by the next lane group, then land
// on eight different bank groups.
constexpr int kLd = 128;
__device__ __forceinline__ int swizzled(int row, int col) {
  return row * kLd + ((((col >> 4) ^ ((row & 3) << 1)) << 4) | (col & 15));
}

// Element offset of this lane's part of the 16-row x 32-column fragment whose
// top-left corner is (0, col0): lanes 0-15 / 16-31 take columns 0-15 / 16-31 of
// rows 0-7, lanes 32-63 the same columns of rows 8-15.  Adding a multiple of
// 4 rows keeps the swizzle valid.
__device__ __forceinline__ int lane_fragment_offset(int col0) {
  const int l = threadIdx.x & 63, g = l >> 4, L = l & 15;
  return swizzled(8 * (g >> 1) + (L >> 2), col0 + 16 * (g & 1) + 4 * (L & 3));
}

#ifdef BSR_DW_PROFILE
__device__ unsigned long long g_prof[4096][8];
__device__ unsigned long long g_trace[4][64][6];
#define PROF_T(x) const unsigned long long x = __builtin_readcyclecounter()
#else
#define PROF_T(x)
#endif

constexpr int KT = 128, NT = 128;   // dW tile of one workgroup: 2 x WN waves, 64 x (128 / WN) each

template <int BR, int BC, int MS, int VB, int WN>
struct Geo {
  static constexpr int THREADS = 128 * WN;                // 2 x WN waves
  static constexpr int NTW = NT / (32 * WN);               // 32-column pieces of dW per wave along N
  static constexpr int R = MS / BR;                       // block-rows per stage
  static constexpr int ROWS = R * BR;                     // rows of a stage that carry data
  static constexpr bool KALIGNED = (KT % BC == 0);
  static constexpr int JT = KALIGNED ? KT / BC : KT / BC + 2;   // block-columns that can cross a tile
  // every 16 x 32 piece of the activation tile lies inside one block: pruned
  // blocks are skipped outright and their LDS content is never read
  static constexpr bool SKIP_ONLY = (BC % 32 == 0) && (BR % 16 == 0) && KALIGNED;
  static constexpr int VA = (BC % 8 == 0) ? 8 : ((BC % 4 == 0) ? 4 : ((BC % 2 == 0) ? 2 : 1));
  static constexpr int VPB = BR * BC / VA;                // vectors per block
  static constexpr int NA = (R * JT * VPB + THREADS - 1) / THREADS;
  static constexpr int NB = (ROWS * (NT / VB) + THREADS - 1) / THREADS;
  static constexpr int LDA = kLd, LDB = kLd;             // LDS rows (elements), swizzled not padded
  static constexpr int MSUB = MS / 16;
  // a wave-wide activation load (64 vectors) never straddles two blocks: the keep
  // decision and the block address are wave-uniform and live in scalar registers
  static constexpr bool UNIFORM_A = (VPB % 64 == 0);
  static constexpr int STAGE_WORDS = (MS * LDA + MS * LDB) / 2;   // 32-bit words of one stage (A tile, B tile)
  static_assert(MS % 16 == 0 && R >= 1 && MSUB <= 8, "stage shape");
  static_assert(JT <= 32, "tile index is a 32-bit mask");
};

// D = stages whose global loads are in flight (register ring), D even.
// WN = waves along N (2: 64 x 64 per wave, 4: 64 x 32 per wave and twice the waves).
template <int BR, int BC, int MS, int VB, int D, int WN>
__global__ __launch_bounds__(128 * WN) void dw_mfma_kernel(
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
    const uint16_t *__restrict__ values, const uint16_t *__restrict__ dY, float *__restrict__ out,
    int64_t M, int64_t K, int64_t N, int64_t lddy, int64_t ldo, int64_t split_stride, int64_t nbr,
    int64_t nbc, int64_t stages_per_split, int accumulate, int tiles_k, int tiles_n, int splits,
    int xcd_map, uint32_t values_bytes, uint32_t dy_bytes) {
  typedef Geo<BR, BC, MS, VB, WN> G;
  constexpr int kThreads = G::THREADS;
  typedef typename Chunk<G::VA * 2>::type AVec;
  typedef typename Chunk<VB * 2>::type BVec;
  static_assert(D % 2 == 0, "ring depth and LDS double buffer stay in phase");

  // Workgroup ids are dealt to the 8 XCDs round-robin (id % 8).  All tiles of one
  // split of the contraction read the same activation rows and dY rows, so the
  // (split, tile) work items are numbered split-major and XCD x takes the x-th
  // contiguous eighth of them: each XCD then works on (parts of) at most a few
  // neighbouring splits, whose operands it fetches into its L2 once, and every
  // XCD gets the same number of workgroups.  Only performance depends on the
  // dispatch order assumption, never correctness.
  const int tiles = tiles_k * tiles_n;
  const int items = tiles * splits;
  int item;
  if (xcd_map) {
    const int per_xcd = (items + 7) / 8;
    item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd) return;
  } else {
    item = blockIdx.x;
  }
  if (item >= items) return;
  const int split = item / tiles, tile = item % tiles;
  const int tile_x = tile % tiles_k, tile_y = tile / tiles_k;

  // two stage buffers (A tile then B tile each); before the main loop the
  // same memory holds the column indices of this split
  __shared__ __attribute__((aligned(16))) uint32_t sStage[2 * G::STAGE_WORDS + kThreads * 4];   // + one 16-byte dump slot per thread
  __shared__ uint32_t sMask[kMaxRowsPerSplit];
  __shared__ int32_t sBase[kMaxRowsPerSplit + 1];
  __shared__ uint32_t sAct[3][8];

  // the wave index lives in a scalar register: everything derived from it (the
  // activity bits, the skip branches) is then wave-uniform for the compiler too
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wk = wave / WN, wn = wave % WN;
  const int64_t k0 = (int64_t)tile_x * KT, n0 = (int64_t)tile_y * NT;
  const int64_t total_stages = ceil_div(nbr, G::R);
  const int64_t s_begin = (int64_t)split * stages_per_split;
  int64_t s_end = s_begin + stages_per_split;
  if (s_end > total_stages) s_end = total_stages;
  const int nstages = (int)(s_end - s_begin);
  const int64_t i_begin = s_begin * G::R;
  const int nrows = nstages * G::R;                       // block-rows of this split (may run past nbr)
  const int64_t jfirst = k0 / BC;
  int64_t jlast = (k0 + KT - 1) / BC;
  if (jlast > nbc - 1) jlast = nbc - 1;
  const int jt = (int)(jlast - jfirst + 1);

  // ---- tile index: per block-row, which block-columns of the tile are kept ----
  // sBase[rr] first holds row_ptr of block-row i_begin + rr (clamped at nbr).
  for (int rr = t; rr <= nrows; rr += kThreads) {
    const int64_t i = i_begin + rr;
    sBase[rr] = row_ptr[i < nbr ? i : nbr];
  }
  if (t < 24) (&sAct[0][0])[t] = 0u;
  __syncthreads();
  const int32_t pos0 = sBase[0];
  const int ncols = sBase[nrows] - pos0;                   // column indices of the whole split
  const bool cols_in_lds = ncols <= 2 * G::STAGE_WORDS;
  if (cols_in_lds)
    for (int e = t; e < ncols; e += kThreads) sStage[e] = (uint32_t)col_idx[pos0 + e];
  __syncthreads();
  constexpr int kRowsPerThread = (kMaxRowsPerSplit + kThreads - 1) / kThreads;
  uint32_t my_mask[kRowsPerThread];
  int32_t my_base[kRowsPerThread];
#pragma unroll
  for (int q = 0; q < kRowsPerThread; ++q) {
    const int rr = t + q * kThreads;
    uint32_t mask = 0;
    int32_t base = 0;
    if (rr < nrows) {
      const int32_t p0 = sBase[rr], p1 = sBase[rr + 1];
      bool first = true;
      for (int32_t p = p0; p < p1; ++p) {
        const int64_t j = cols_in_lds ? (int64_t)sStage[p - pos0] : (int64_t)col_idx[p];
        if (j >= jfirst && j <= jlast) {
          if (first) { base = p; first = false; }
          mask |= 1u << (int)(j - jfirst);
        }
      }
    }
    my_mask[q] = mask;
    my_base[q] = base;
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < kRowsPerThread; ++q) {
    const int rr = t + q * kThreads;
    if (rr < nrows) {
      sMask[rr] = my_mask[q];
      sBase[rr] = my_base[q];
    }
  }
  // rows / columns of the stage buffers that no stage ever writes must read as zero
  if (!G::SKIP_ONLY || G::ROWS < MS)
    for (int e = t; e < 2 * G::STAGE_WORDS; e += kThreads) sStage[e] = 0u;
  __syncthreads();

  // ---- per-thread constants of the two loaders ----
  const int wave_s = wave;
  int a_row[G::NA];            // block-row of the stage (0..R-1), or -1: vector not used
  int a_jl[G::NA];             // block-column inside the tile
  uint32_t a_src[G::NA];       // byte offset inside the block
  int a_dst[G::NA];            // element offset inside the A tile
#pragma unroll
  for (int it = 0; it < G::NA; ++it) {
    const int v = t + it * kThreads;
    const int slot = v / G::VPB, off = v % G::VPB;
    const int rbk = slot / G::JT, jl = slot % G::JT;
    const int r = (off * G::VA) / BC, c = (off * G::VA) % BC;
    const int col = (int)((jfirst + jl) * BC - k0) + c;
    const bool used = slot < G::R * G::JT && jl < jt && col >= 0 && col + G::VA <= KT;
    a_row[it] = used ? rbk : -1;
    a_jl[it] = jl;
    a_src[it] = (uint32_t)(off * G::VA * 2);
    a_dst[it] = used ? swizzled(rbk * BR + r, col) : -1;
  }
  int b_row[G::NB];            // row of the stage, or MS: vector not used
  uint32_t b_src[G::NB];       // byte offset relative to the first row of the stage (out of range if unused)
  int b_dst[G::NB];
#pragma unroll
  for (int it = 0; it < G::NB; ++it) {
    const int v = t + it * kThreads;
    const int r = v / (NT / VB), c = (v % (NT / VB)) * VB;
    const bool used = r < G::ROWS && n0 + c < N;
    b_row[it] = used ? r : MS;
    b_src[it] = used ? (uint32_t)(((int64_t)r * lddy + c) * 2) : kOutOfRange;
    b_dst[it] = used ? swizzled(r, c) : -1;
  }
  // element offsets of the LDS stores relative to stage buffer 0 (>= kDump: the dump slot)
  constexpr int kDump = 2 * G::STAGE_WORDS * 2;
  int a_lds[2][G::NA], b_lds[2][G::NB];
#pragma unroll
  for (int buf = 0; buf < 2; ++buf) {
#pragma unroll
    for (int it = 0; it < G::NA; ++it)
      a_lds[buf][it] = a_dst[it] >= 0 ? buf * G::STAGE_WORDS * 2 + a_dst[it] : kDump + t * 8;
#pragma unroll
    for (int it = 0; it < G::NB; ++it)
      b_lds[buf][it] = b_dst[it] >= 0 ? buf * G::STAGE_WORDS * 2 + MS * G::LDA + b_dst[it] : kDump + t * 8;
  }
  // dY seen from the first row / column of this workgroup; every stage gets its
  // own buffer descriptor (scalar registers), so rows past the end of the
  // matrix fall out of range by themselves
  const int64_t dy_total = M > 0 ? ((M - 1) * lddy + N) * 2 : 0;           // bytes
  const int64_t dy_first = (i_begin * BR * lddy + n0) * 2;
  const int64_t dy_stage = (int64_t)G::ROWS * lddy * 2;
  const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(values, values_bytes);
  const uint32_t lane16 = (uint32_t)(lane * G::VA * 2);

  AVec ra[D][G::NA];
  BVec rb[D][G::NB];

  // Global loads of stage index q (0-based inside the split) into ring slot d.
  // Branch-free: a vector that is pruned, outside the matrix or beyond the last
  // stage reads as zero through an out-of-range buffer offset.
  auto prefetch = [&](int d, int q) {
    const bool live = q < nstages;
    const int rr0 = live ? q * G::R : 0;
    if (G::UNIFORM_A) {
      uint32_t mask[G::R];
      uint32_t base[G::R];
#pragma unroll
      for (int rbk = 0; rbk < G::R; ++rbk) {
        mask[rbk] = (uint32_t)__builtin_amdgcn_readfirstlane((int)sMask[rr0 + rbk]);
        base[rbk] = (uint32_t)__builtin_amdgcn_readfirstlane(sBase[rr0 + rbk]);
      }
#pragma unroll
      for (int it = 0; it < G::NA; ++it) {
        const int v0 = wave_s * 64 + it * kThreads;                  // first vector of this wave's load
        const int slot = v0 / G::VPB, off0 = v0 % G::VPB;
        const int rbk = slot / G::JT, jl = slot % G::JT;
        uint32_t m = 0, b = 0;
#pragma unroll
        for (int x = 0; x < G::R; ++x)
          if (rbk == x) { m = mask[x]; b = base[x]; }
        const bool kept = live && slot < G::R * G::JT && jl < jt && ((m >> jl) & 1u);
        const uint32_t pos = b + __builtin_popcount(m & ((1u << jl) - 1u));
        const uint32_t soff = kept ? pos * (uint32_t)(BR * BC * 2) + (uint32_t)(off0 * G::VA * 2) : 0u;
        ra[d][it] = buffer_load<G::VA * 2>(rsrc_a, kept ? lane16 : kOutOfRange, soff);
      }
    } else {
      uint32_t mask[G::R];
      uint32_t base[G::R];
#pragma unroll
      for (int rbk = 0; rbk < G::R; ++rbk) {
        mask[rbk] = sMask[rr0 + rbk];
        base[rbk] = (uint32_t)sBase[rr0 + rbk];
      }
#pragma unroll
      for (int it = 0; it < G::NA; ++it) {
        uint32_t m = 0, b = 0;
#pragma unroll
        for (int rbk = 0; rbk < G::R; ++rbk)
          if (a_row[it] == rbk) { m = mask[rbk]; b = base[rbk]; }
        const bool kept = live && a_row[it] >= 0 && ((m >> a_jl[it]) & 1u);
        const uint32_t pos = b + __popc(m & ((1u << a_jl[it]) - 1u));
        ra[d][it] = buffer_load<G::VA * 2>(rsrc_a, kept ? pos * (uint32_t)(BR * BC * 2) + a_src[it] : kOutOfRange);
      }
    }
    const int64_t first = dy_first + (int64_t)q * dy_stage;
    int64_t left = live ? dy_total - first : 0;
    if (left < 0) left = 0;
    if (left > 0xFFFFFFFFll) left = 0xFFFFFFFFll;
    const __amdgpu_buffer_rsrc_t rsrc_b =
        make_rsrc(reinterpret_cast<const char *>(dY) + first, (uint32_t)left);
#pragma unroll
    for (int it = 0; it < G::NB; ++it) rb[d][it] = buffer_load<VB * 2>(rsrc_b, b_src[it]);
  };

  // Ring slot d (stage index q) -> LDS stage buffer `buf`.
  auto stage_to_lds = [&](int d, int q, int buf) {
    // unused vectors go to this thread's dump slot: no store needs a predicate
    uint16_t *s0 = reinterpret_cast<uint16_t *>(sStage);
#pragma unroll
    for (int it = 0; it < G::NA; ++it)
      *reinterpret_cast<AVec *>(&s0[a_lds[buf][it]]) = ra[d][it];   // data, zeros if pruned
#pragma unroll
    for (int it = 0; it < G::NB; ++it) *reinterpret_cast<BVec *>(&s0[b_lds[buf][it]]) = rb[d][it];
    if (!G::SKIP_ONLY) {
      // which 16-row x 32-column pieces of the activation tile hold a kept block
      const int rr0 = q * G::R;
      if (t < G::R * G::JT && q < nstages) {
        const int rbk = t / G::JT, jl = t % G::JT;
        if (jl < jt && ((sMask[rr0 + rbk] >> jl) & 1u)) {
          int c0 = (int)((jfirst + jl) * BC - k0), c1 = c0 + BC - 1;
          if (c0 < 0) c0 = 0;
          if (c1 > KT - 1) c1 = KT - 1;
          if (c0 <= c1) {
            const uint32_t bits = ((2u << (c1 >> 5)) - 1u) & ~((1u << (c0 >> 5)) - 1u);
            for (int ms = (rbk * BR) >> 4; ms <= (rbk * BR + BR - 1) >> 4; ++ms) atomicOr(&sAct[q % 3][ms], bits);
          }
        }
      }
      if (t < 8) sAct[(q + 1) % 3][t] = 0u;
    }
  };

  v16f acc[2][G::NTW];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int w = 0; w < G::NTW; ++w)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[u][w][r] = 0.f;

  const int frag_a0 = lane_fragment_offset((2 * wk) * 32), frag_a1 = lane_fragment_offset((2 * wk + 1) * 32);
  int frag_b[G::NTW];
#pragma unroll
  for (int w = 0; w < G::NTW; ++w) frag_b[w] = lane_fragment_offset((G::NTW * wn + w) * 32);

  // Multiply stage q out of LDS buffer `buf`.
#ifdef BSR_DW_PROFILE
  unsigned long long pam_dbg = 0;
#endif
  auto compute = [&](int q, int buf) {
    const uint16_t *sA = reinterpret_cast<const uint16_t *>(sStage + buf * G::STAGE_WORDS);
    const uint16_t *sB = sA + MS * G::LDA;
    // two activity bits (this wave's two 32-column pieces) per 16-row step
    uint32_t pam = 0;
    if (G::SKIP_ONLY) {
#pragma unroll
      for (int rbk = 0; rbk < G::R; ++rbk) {
        const uint32_t m = (uint32_t)__builtin_amdgcn_readfirstlane((int)sMask[q * G::R + rbk]);
        const uint32_t two = ((m >> ((2 * wk * 32) / BC)) & 1u) | (((m >> (((2 * wk + 1) * 32) / BC)) & 1u) << 1);
#pragma unroll
        for (int ms = rbk * (BR / 16); ms < (rbk + 1) * (BR / 16); ++ms) pam |= two << (2 * ms);
      }
    } else {
#pragma unroll
      for (int ms = 0; ms < G::MSUB; ++ms) {
        const uint32_t act = (uint32_t)__builtin_amdgcn_readfirstlane((int)sAct[q % 3][ms]);
        pam |= ((act >> (2 * wk)) & 3u) << (2 * ms);
      }
    }
    // Static, fully unrolled walk over the 16-row steps of the stage.  The
    // four fragments of step ms+1 are requested from LDS before the multiplies
    // of step ms are issued (their latency hides behind the matrix core); only
    // the multiplies sit under the wave-uniform skip branches.
#ifdef BSR_DW_PROFILE
    pam_dbg = pam;
#endif
    if (pam == 0) return;
    v8bf fb[G::NTW], fa0, fa1;
#pragma unroll
    for (int w = 0; w < G::NTW; ++w) fb[w] = read_fragment(sB + frag_b[w], G::LDB);
    fa0 = read_fragment(sA + frag_a0, G::LDA);
    fa1 = read_fragment(sA + frag_a1, G::LDA);
#pragma unroll
    for (int ms = 0; ms < G::MSUB; ++ms) {
      v8bf nb[G::NTW], na0 = fa0, na1 = fa1;
#pragma unroll
      for (int w = 0; w < G::NTW; ++w) nb[w] = fb[w];
      if (ms + 1 < G::MSUB) {
#pragma unroll
        for (int w = 0; w < G::NTW; ++w) nb[w] = read_fragment(sB + frag_b[w] + (ms + 1) * 16 * G::LDB, G::LDB);
        na0 = read_fragment(sA + frag_a0 + (ms + 1) * 16 * G::LDA, G::LDA);
        na1 = read_fragment(sA + frag_a1 + (ms + 1) * 16 * G::LDA, G::LDA);
      }
      const uint32_t mine = (pam >> (2 * ms)) & 3u;
      if (mine & 1u) {
#pragma unroll
        for (int w = 0; w < G::NTW; ++w)
          acc[0][w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb[w], acc[0][w], 0, 0, 0);
      }
      if (mine & 2u) {
#pragma unroll
        for (int w = 0; w < G::NTW; ++w)
          acc[1][w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb[w], acc[1][w], 0, 0, 0);
      }
#pragma unroll
      for (int w = 0; w < G::NTW; ++w) fb[w] = nb[w];
      fa0 = na0; fa1 = na1;
    }
  };

  // ---- main loop: stage q is multiplied out of LDS buffer q&1 while stage
  // q+1 moves from registers to the other buffer and stage q+1+D leaves HBM ----
#ifdef BSR_DW_PROFILE
  unsigned long long p_store = 0, p_pref = 0, p_comp = 0, p_bar = 0;
  const unsigned long long p_t0 = __builtin_readcyclecounter();
#endif
#pragma unroll
  for (int d = 0; d < D; ++d) prefetch(d, d);
  stage_to_lds(0, 0, 0);
  prefetch(0, D);
  __syncthreads();
#ifdef BSR_DW_PROFILE
  const unsigned long long p_t1 = __builtin_readcyclecounter();
#endif
  for (int q0 = 0; q0 < nstages; q0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const int q = q0 + d;
      if (q >= nstages) break;
      PROF_T(ta);
      stage_to_lds((d + 1) % D, q + 1, (d + 1) & 1);
      PROF_T(tb);
      prefetch((d + 1) % D, q + 1 + D);
      PROF_T(tc);
      compute(q, d & 1);
      PROF_T(td);
      __syncthreads();
      PROF_T(te);
#ifdef BSR_DW_PROFILE
      p_store += tb - ta; p_pref += tc - tb; p_comp += td - tc; p_bar += te - td;
      if (lane == 0 && wave == 0 && q < 64 && (blockIdx.x == 0 || blockIdx.x == 100 || blockIdx.x == 256 || blockIdx.x == 300)) {
        const int wsel = blockIdx.x == 0 ? 0 : blockIdx.x == 100 ? 1 : blockIdx.x == 256 ? 2 : 3;
        unsigned long long *g = g_trace[wsel][q];
        g[0] = ta - p_t0; g[1] = tb - p_t0; g[2] = tc - p_t0; g[3] = td - p_t0; g[4] = te - p_t0; g[5] = pam_dbg;
      }
#endif
    }
  }
#ifdef BSR_DW_PROFILE
  const unsigned long long p_t2 = __builtin_readcyclecounter();
#endif

  float *o = out + (int64_t)split * split_stride;
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int w = 0; w < G::NTW; ++w)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t k = k0 + (2 * wk + u) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int64_t n = n0 + (G::NTW * wn + w) * 32 + (lane & 31);
        if (k < K && n < N) {
          float *dst = o + k * ldo + n;
          *dst = accumulate ? *dst + acc[u][w][r] : acc[u][w][r];
        }
      }
#ifdef BSR_DW_PROFILE
  if (lane == 0 && blockIdx.x < 1024) {
    const unsigned long long p_t3 = __builtin_readcyclecounter();
    unsigned long long *g = g_prof[blockIdx.x * 4 + wave];
    g[0] = p_t1 - p_t0; g[1] = p_t2 - p_t1; g[2] = p_t3 - p_t2; g[3] = p_store; g[4] = p_pref; g[5] = p_comp;
    g[6] = p_bar; g[7] = nstages;
  }
#endif
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
  static const int target = getenv("BSR_DW_TARGET_WGS") ? atoi(getenv("BSR_DW_TARGET_WGS")) : 512;
  int64_t s = (target + tiles / 2) / (tiles > 0 ? tiles : 1);
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

template <int BR, int BC, int MS, int D, int WN>
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
  const int tiles_k = (int)ceil_div(K, 128), tiles_n = (int)ceil_div(N, 128);
  static const int xcd_map = getenv("BSR_DW_XCD_MAP") ? atoi(getenv("BSR_DW_XCD_MAP")) : 1;
  const int64_t n_items = (int64_t)p.splits * tiles_k * tiles_n;
  dim3 grid((unsigned)(xcd_map ? 8 * ceil_div(n_items, 8) : n_items));
  const uint16_t *v = static_cast<const uint16_t *>(values);
  const uint16_t *y = static_cast<const uint16_t *>(dY);
  // 32-bit buffer offsets: both operands must stay below 4 GiB (checked by dw_mfma_supported)
  const uint32_t values_bytes = (uint32_t)(nbr * nbc * BR * BC * 2);
  const uint32_t dy_bytes = M > 0 ? (uint32_t)(((M - 1) * lddy + N) * 2) : 0u;
  int vb = 8;
  while (vb > 1 && (N % vb != 0 || lddy % vb != 0 || (uintptr_t)dY % (2 * vb) != 0)) vb >>= 1;
#define BSR_DW_LAUNCH(VB)                                                                         \
  hipLaunchKernelGGL((dw_mfma_kernel<BR, BC, MS, VB, D, WN>), grid, dim3(128 * WN), 0, s,          \
                     row_ptr, col_idx, v, y, out, M, K, N, lddy, ldo, stride, nbr, nbc,            \
                     p.stages_per_split, acc_direct, tiles_k, tiles_n, p.splits, xcd_map,           \
                     values_bytes, dy_bytes)
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

bool dw_mfma_supported(int dtype, int br, int bc, const void *values, int64_t M, int64_t K, int64_t N,
                       int64_t lddy) {
  if (dtype != BSR_BF16) return false;
  if ((uintptr_t)values % 16 != 0) return false;
  const bool shape = (br == 32 && bc == 32) || (br == 64 && bc == 64) || (br == 16 && bc == 16) ||
                     (br == 14 && bc == 14);
  if (!shape) return false;
  // the kernel addresses both operands with 32-bit byte offsets
  const int64_t limit = (int64_t(1) << 32) - 64;
  if (ceil_div(M, br) * br * ceil_div(K, bc) * bc * 2 >= limit) return false;
  if (M * lddy * 2 >= limit || N > lddy) return false;
  return true;
}

// Tuning knobs (development only): stage rows and prefetch depth of the 32 x 32 kernel.
static int knob_ms32() {
  static const int v = getenv("BSR_DW_MS") ? atoi(getenv("BSR_DW_MS")) : 64;
  return v == 32 ? 32 : 64;
}
static int knob_depth() {
  static const int v = getenv("BSR_DW_DEPTH") ? atoi(getenv("BSR_DW_DEPTH")) : 2;
  return v;
}

size_t dw_mfma_ws_bytes(int64_t M, int64_t K, int64_t N, int br, int bc) {
  (void)bc;
  switch (br) {
    case 32: return knob_ms32() == 32 ? ws_for<32, 32>(M, K, N) : ws_for<32, 64>(M, K, N);
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
#define BSR_ARGS row_ptr, col_idx, values, M, K, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes, s
  static const int wn = getenv("BSR_DW_WN") ? atoi(getenv("BSR_DW_WN")) : 4;
  if (br == 32 && bc == 32) {
    if (wn == 4) return knob_ms32() == 32 ? run<32, 32, 32, 2, 4>(BSR_ARGS) : run<32, 32, 64, 2, 4>(BSR_ARGS);
    return knob_ms32() == 32 ? run<32, 32, 32, 2, 2>(BSR_ARGS) : run<32, 32, 64, 2, 2>(BSR_ARGS);
  }
  if (br == 64 && bc == 64) return wn == 4 ? run<64, 64, 64, 2, 4>(BSR_ARGS) : run<64, 64, 64, 2, 2>(BSR_ARGS);
  if (br == 16 && bc == 16) return run<16, 16, 32, 4, 2>(BSR_ARGS);
  if (br == 14 && bc == 14) return wn == 4 ? run<14, 14, 32, 2, 4>(BSR_ARGS) : run<14, 14, 32, 2, 2>(BSR_ARGS);
#undef BSR_ARGS
  return BSR_ERR_SHAPE;
}

#ifdef BSR_DW_PROFILE
extern "C" int bsr_debug_read_trace(unsigned long long *host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), sizeof(unsigned long long) * n, 0, hipMemcpyDeviceToHost);
}
extern "C" int bsr_debug_read_prof(unsigned long long *host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_prof), sizeof(unsigned long long) * n, 0, hipMemcpyDeviceToHost);
}
#endif

}  // namespace bsr
