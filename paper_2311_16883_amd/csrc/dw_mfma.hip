// Weight gradient from a BSR activation on the matrix cores (paper Sec. III,
// Fig. 2: dW = Xhat^T * dY, "BSpMM"), bfloat16 or binary32 inputs, binary32
// accumulation.  The description below is for bfloat16; binary32 differs only in
// the fragment reads (see multiply_f32).
//
// Both operands are stored with the contraction index m (activation rows) as
// the slow axis -- a kept block is [r][c] with c = output row of dW, dY is
// [m][n] -- while v_mfma_f32_32x32x16_bf16 wants every lane to hold 8
// consecutive contraction elements.  Tiles therefore go to LDS in their natural
// row-major order and the fragments come back through ds_read_b64_tr_b16, which
// transposes 4 x 16 sub-tiles across 16 lanes.
//
// Work decomposition.  A workgroup owns a KT x NT tile of dW and a contiguous
// range of block-rows (one split of the contraction).  At start it turns the BSR
// row segments that cross its tile into a table of block offsets and per-stage
// activity bits in LDS; after that the main loop reads no index from global
// memory.  The loop walks stages of MS activation rows: the kept blocks of the
// stage are copied into a dense LDS tile (zeros where a pruned block shares a
// 32-wide matrix-core tile with a kept one), dY rows next to it, and every
// 16-row x 32-column piece of the activation tile that holds no kept block is
// skipped by a wave-uniform branch -- the sparsity is exploited at matrix-core
// granularity.
//
// The waves of a workgroup have two roles.  Half of them (the loaders) only move
// data: global memory -> a ring of registers several stages deep -> LDS.  The
// other half (the multipliers) only read fragments from LDS and feed the matrix
// cores.  A wave issues in order, so a wave that does both stalls its multiplies
// whenever the texture path's queue is full and leaves the texture path idle
// while it multiplies; with the roles split the loaders keep that path (64 bytes
// per clock and compute unit, the busiest resource of this kernel) occupied all
// the time.  One barrier per stage hands LDS buffer q&1 from the loaders to the
// multipliers.  With more than one split the partial tiles go to the workspace
// and a second kernel adds them in a fixed order.
#include <utility>

#include "buffer_access.h"
#include "common.h"

namespace bsr {

namespace {

typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(16))) float v16f;

constexpr int kMaxRowsPerSplit = 512;   // block-rows of one split: its block table must fit in LDS

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose
// index is a compile-time constant in every trip, whatever its length (register
// arrays indexed with it never end up in scratch memory).
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F &&>(f));
}

// Table entry of a pruned block: still out of range after a byte offset inside a
// block is added (the activation values must stay below 2 GiB).
constexpr uint32_t kDead = 0x80000000u;

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

// LDS tiles are 128 elements wide and unpadded.  Two-byte elements (256-byte
// rows, all 64 banks): the transposing read fetches four consecutive rows per
// 16-lane group, which would all hit the same banks; so the 32-byte chunk index
// of every element is XOR-ed with twice the row's low two bits: four consecutive
// rows of one chunk, and of the neighbouring chunk read by the next lane group,
// then land on eight different bank groups.  Four-byte elements (512-byte rows):
// a fragment read takes 32 consecutive columns of two consecutive rows, which
// would share their banks; odd rows swap their 32-column halves.
constexpr int kLd = 128;
template <int E>
__device__ __forceinline__ int swizzled(int row, int col) {
  if (E == 2) return row * kLd + ((((col >> 4) ^ ((row & 3) << 1)) << 4) | (col & 15));
  return row * kLd + (col ^ ((row & 1) << 5));
}

// Element offset of this lane's part of the 16-row x 32-column fragment whose
// top-left corner is (0, col0): lanes 0-15 / 16-31 take columns 0-15 / 16-31 of
// rows 0-7, lanes 32-63 the same columns of rows 8-15.  Adding a multiple of
// 4 rows keeps the swizzle valid.
__device__ __forceinline__ int lane_fragment_offset(int col0) {
  const int l = threadIdx.x & 63, g = l >> 4, L = l & 15;
  return swizzled<2>(8 * (g >> 1) + (L >> 2), col0 + 16 * (g & 1) + 4 * (L & 3));
}


constexpr int KT = 128, NT = 128;   // dW tile of one workgroup: 2 x WN waves, 64 x (128 / WN) each

// E = bytes per element of the inputs (2: bfloat16, 4: binary32).
template <int E, int BR, int BC, int MS, int VB, int WN>
struct Geo {
  static constexpr int THREADS = 128 * WN;                // threads per role: 2 x WN waves
  static constexpr int NTW = NT / (32 * WN);               // 32-column pieces of dW per wave along N
  static constexpr int R = MS / BR;                       // block-rows per stage
  static constexpr int ROWS = R * BR;                     // rows of a stage that carry data
  static constexpr bool KALIGNED = (KT % BC == 0);
  static constexpr int JT = KALIGNED ? KT / BC : KT / BC + 2;   // block-columns that can cross a tile
  // every 16 x 32 piece of the activation tile lies inside one block: pruned
  // blocks are skipped outright and their LDS content is never read
  static constexpr bool SKIP_ONLY = (BC % 32 == 0) && (BR % 16 == 0) && KALIGNED;
  // elements per activation vector: at most 16 bytes, inside one block row
  static constexpr int VA = (E == 2 && BC % 8 == 0) ? 8 : ((BC % 4 == 0) ? 4 : ((BC % 2 == 0) ? 2 : 1));
  static constexpr int VPB = BR * BC / VA;                // vectors per block
  static constexpr int NA = (R * JT * VPB + THREADS - 1) / THREADS;
  static constexpr int NB = (ROWS * (NT / VB) + THREADS - 1) / THREADS;
  static constexpr int LDA = kLd, LDB = kLd;             // LDS rows (elements), swizzled not padded
  static constexpr int MSUB = MS / 16;
  // a wave-wide activation load (64 vectors) never straddles two blocks: the keep
  // decision and the block address are wave-uniform and live in scalar registers
  static constexpr bool UNIFORM_A = (VPB % 64 == 0);
  static constexpr int STAGE_WORDS = (MS * LDA + MS * LDB) * E / 4;   // 32-bit words of one stage (A tile, B tile)
  static_assert(MS % 16 == 0 && R >= 1 && MSUB <= 8, "stage shape");
  static_assert(JT <= 32, "tile index is a 32-bit mask");
};

// D = stages whose global loads are in flight (register ring of the loaders).
// WN = multiplier waves along N (2: 64 x 64 per wave, 4: 64 x 32 per wave); the
// workgroup has 2 x WN multiplier waves and as many loader waves.
// T = uint16_t (bfloat16 bits) or float.
// What one tensor's launch needs (kernel arguments; an array of these for a batch).
struct DwParams {
  const int32_t *row_ptr, *col_idx;
  const void *values, *dY;
  float *out;
  int64_t M, K, N, lddy, ldo, split_stride, nbr, nbc, stages_per_split;
  int accumulate, tiles_k, tiles_n, splits;
  uint32_t values_bytes;
  uint32_t wg_begin;       // first work item of this tensor in a batched launch's list
};

// wg = number of the workgroup among those of this tensor.
template <typename T, int BR, int BC, int MS, int VB, int D, int WN>
__device__ __forceinline__ void dw_mfma_body(const DwParams &prm, const uint32_t wg, const int xcd_map) {
  const int32_t *__restrict__ row_ptr = prm.row_ptr;
  const int32_t *__restrict__ col_idx = prm.col_idx;
  const T *__restrict__ values = static_cast<const T *>(prm.values);
  const T *__restrict__ dY = static_cast<const T *>(prm.dY);
  float *__restrict__ out = prm.out;
  const int64_t M = prm.M, K = prm.K, N = prm.N, lddy = prm.lddy, ldo = prm.ldo, split_stride = prm.split_stride;
  const int64_t nbr = prm.nbr, nbc = prm.nbc, stages_per_split = prm.stages_per_split;
  const int accumulate = prm.accumulate, tiles_k = prm.tiles_k, tiles_n = prm.tiles_n, splits = prm.splits;
  const uint32_t values_bytes = prm.values_bytes;
  constexpr int E = (int)sizeof(T);
  typedef Geo<E, BR, BC, MS, VB, WN> G;
  constexpr int kRole = G::THREADS;              // threads per role
  constexpr int kThreads = 2 * kRole;            // workgroup
  typedef typename Chunk<G::VA * E>::type AVec;
  typedef typename Chunk<VB * E>::type BVec;

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
    item = (wg & 7) * per_xcd + (wg >> 3);
    if ((int)(wg >> 3) >= per_xcd) return;
  } else {
    item = wg;
  }
  if (item >= items) return;
  const int split = item / tiles, tile = item % tiles;
  // Tiles are numbered fastest along the dimension with fewer tiles: when a split's tiles are
  // shared out to two XCDs (fewer splits than XCDs), each of them then needs all of the smaller
  // operand but only its part of the larger one.
  const bool n_fastest = tiles_n < tiles_k;
  const int tile_x = n_fastest ? tile / tiles_n : tile % tiles_k;
  const int tile_y = n_fastest ? tile % tiles_n : tile / tiles_k;

  // LDS: two stage buffers (A tile then B tile each) that also stage the column
  // indices of the split before the main loop, a 1 KB dump slot (16 bytes per
  // lane) for stores of unused vectors, the block table and the activity bits.
  constexpr int kTail = (D + 2) * G::R;           // block-rows the loaders may run past the split
  __shared__ __attribute__((aligned(16))) uint32_t sStage[2 * G::STAGE_WORDS + 256];
  // sTab[rr * JT + jl]: byte offset in `values` of the block in block-row rr of the
  // split and block-column jl of the tile, kDead if pruned / outside
  __shared__ uint32_t sTab[(kMaxRowsPerSplit + kTail) * G::JT];
  // first the raw column masks per block-row, then per stage the activity bits of
  // its 16-row steps (two per step, for the waves with wk = 0 in the low half-word)
  __shared__ uint32_t sPam[kMaxRowsPerSplit + 64];
  int32_t *const sPtr = reinterpret_cast<int32_t *>(sTab);   // row_ptr of the split while the table is built
  static_assert((kMaxRowsPerSplit + kTail) * G::JT > kMaxRowsPerSplit, "row_ptr fits in the table's memory");
  static_assert(kMaxRowsPerSplit <= kThreads, "one block-row per thread in the prologue");

  // the wave index lives in a scalar register: everything derived from it (the
  // role, the activity bits, the skip branches) is then wave-uniform for the
  // compiler too
  const int t = threadIdx.x, lane = t & 63;
  const int wave_wg = __builtin_amdgcn_readfirstlane(t >> 6);
  const bool loader = wave_wg >= 2 * WN;
  const int wave = loader ? wave_wg - 2 * WN : wave_wg;      // wave inside its role
  const int tg = loader ? t - kRole : t;                       // thread inside its role
  const int64_t k0 = (int64_t)tile_x * KT, n0 = (int64_t)tile_y * NT;
  const int64_t total_stages = ceil_div(nbr, G::R);
  const int64_t s_begin = (int64_t)split * stages_per_split;
  int64_t s_end = s_begin + stages_per_split;
  if (s_end > total_stages) s_end = total_stages;
  const int nstages = s_end > s_begin ? (int)(s_end - s_begin) : 0;
  const int64_t i_begin = s_begin * G::R;
  const int nrows = nstages * G::R;                       // block-rows of this split (may run past nbr)
  const int64_t jfirst = k0 / BC;
  int64_t jlast = (k0 + KT - 1) / BC;
  if (jlast > nbc - 1) jlast = nbc - 1;
  const int jt = (int)(jlast - jfirst + 1);

  // ---- block table: which blocks of the tile's block-columns each block-row keeps ----
  for (int rr = t; rr <= nrows; rr += kThreads) {
    const int64_t i = i_begin + rr;
    sPtr[rr] = row_ptr[i < nbr ? i : nbr];
  }
  __syncthreads();
  const int32_t pos0 = sPtr[0];
  const int ncols = sPtr[nrows] - pos0;                    // column indices of the whole split
  const bool cols_in_lds = ncols <= 2 * G::STAGE_WORDS;
  if (cols_in_lds)
    for (int e = t; e < ncols; e += kThreads) sStage[e] = (uint32_t)col_idx[pos0 + e];
  __syncthreads();
  uint32_t my_mask = 0;                                     // block-row t: kept block-columns of the tile
  int32_t my_base = 0;                                      // position of the first of them in col_idx / values
  if (t < nrows) {
    const int32_t p0 = sPtr[t], p1 = sPtr[t + 1];
    bool first = true;
    for (int32_t p = p0; p < p1; ++p) {
      const int64_t j = cols_in_lds ? (int64_t)sStage[p - pos0] : (int64_t)col_idx[p];
      if (j >= jfirst && j <= jlast) {
        if (first) { my_base = p; first = false; }
        my_mask |= 1u << (int)(j - jfirst);
      }
    }
  }
  __syncthreads();
  if (t < nrows) {
#pragma unroll
    for (int jl = 0; jl < G::JT; ++jl)
      sTab[t * G::JT + jl] = ((my_mask >> jl) & 1u)
                                 ? (uint32_t)(my_base + __popc(my_mask & ((1u << jl) - 1u))) * (uint32_t)(BR * BC * E)
                                 : kDead;
  }
  for (int e = t; e < kTail * G::JT; e += kThreads) sTab[nrows * G::JT + e] = kDead;
  for (int e = t; e < kMaxRowsPerSplit + 64; e += kThreads) sPam[e] = e == t ? my_mask : 0u;
  // rows / columns of the stage buffers that no stage ever writes must read as zero
  if (!G::SKIP_ONLY || G::ROWS < MS)
    for (int e = t; e < 2 * G::STAGE_WORDS; e += kThreads) sStage[e] = 0u;
  __syncthreads();
  {
    // Block-columns of the tile that overlap the two 32-column pieces of the
    // activation tile owned by the waves with wk = 0 / 1: a 16-row step of a piece
    // carries data iff a block-row it overlaps keeps one of these columns.
    uint32_t colmask[2][2] = {{0u, 0u}, {0u, 0u}};
#pragma unroll
    for (int jl = 0; jl < G::JT; ++jl) {
      const int c0 = (int)((jfirst + jl) * BC - k0), c1 = c0 + BC - 1;
#pragma unroll
      for (int x = 0; x < 4; ++x)
        if (jl < jt && c0 <= x * 32 + 31 && c1 >= x * 32) colmask[x >> 1][x & 1] |= 1u << jl;
    }
    uint32_t pam = 0;
    if (t < nstages) {
#pragma unroll
      for (int rbk = 0; rbk < G::R; ++rbk) {
        const uint32_t m = sPam[t * G::R + rbk];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          if (m & colmask[x >> 1][x & 1]) {
#pragma unroll
            for (int ms = (rbk * BR) / 16; ms <= (rbk * BR + BR - 1) / 16; ++ms)
              pam |= 1u << (16 * (x >> 1) + 2 * ms + (x & 1));
          }
        }
      }
    }
    __syncthreads();
    if (t < kMaxRowsPerSplit) sPam[t] = pam;
    __syncthreads();
  }

  if (loader) {
    // ================= loader waves =================
    // Activation vector `it` of a stage belongs to block (block-row a_row of the
    // stage, block-column a_jl of the tile); its global offset is the block's table
    // entry plus a_src.  The table entry of the next stage to fetch is read one
    // stage ahead (a_val); a_tab walks down the table by a_inc entries per stage.
    uint32_t a_src[G::NA];       // byte offset inside the block
    uint32_t a_tab[G::NA];       // index into sTab of the entry behind a_val
    uint32_t a_inc[G::NA];       // R * JT, or 0 for a vector that is never used (it stays on a dead entry)
    uint32_t a_val[G::NA];
    int a_dst[G::NA];            // element offset inside the A tile, -1: not used
#pragma unroll
    for (int it = 0; it < G::NA; ++it) {
      const int v = tg + it * kRole;
      const int slot = v / G::VPB, off = v % G::VPB;
      const int rbk = slot / G::JT, jl = slot % G::JT;
      const int r = (off * G::VA) / BC, c = (off * G::VA) % BC;
      const int col = (int)((jfirst + jl) * BC - k0) + c;
      const bool used = slot < G::R * G::JT && jl < jt && col >= 0 && col + G::VA <= KT;
      a_src[it] = (uint32_t)(off * G::VA * E);
      a_tab[it] = used ? (uint32_t)(rbk * G::JT + jl) : (uint32_t)(nrows * G::JT);
      a_inc[it] = used ? (uint32_t)(G::R * G::JT) : 0u;
      a_val[it] = sTab[a_tab[it]];
      a_dst[it] = used ? swizzled<E>(rbk * BR + r, col) : -1;
    }
    // dY is addressed through one descriptor that covers exactly the rows of this
    // split (from the tile's first column on): rows past the split or the matrix
    // end read as zero by themselves; b_cur walks down by one stage per fetch.
    uint32_t b_cur[G::NB], b_inc[G::NB];
    int b_dst[G::NB];
#pragma unroll
    for (int it = 0; it < G::NB; ++it) {
      const int v = tg + it * kRole;
      const int r = v / (NT / VB), c = (v % (NT / VB)) * VB;
      const bool used = r < G::ROWS && n0 + c < N;
      b_cur[it] = used ? (uint32_t)(((int64_t)r * lddy + c) * E) : kOutOfRange;
      b_inc[it] = used ? (uint32_t)((int64_t)G::ROWS * lddy * E) : 0u;
      b_dst[it] = used ? swizzled<E>(r, c) : -1;
    }
    // element offsets of the LDS stores relative to stage buffer 0 (>= kDump: the dump slot)
    constexpr int kStageElems = G::STAGE_WORDS * 4 / E;       // elements of one stage buffer
    constexpr int kDump = 2 * kStageElems;
    int a_lds[2][G::NA], b_lds[2][G::NB];
#pragma unroll
    for (int buf = 0; buf < 2; ++buf) {
#pragma unroll
      for (int it = 0; it < G::NA; ++it)
        a_lds[buf][it] = a_dst[it] >= 0 ? buf * kStageElems + a_dst[it] : kDump + lane * (16 / E);
#pragma unroll
      for (int it = 0; it < G::NB; ++it)
        b_lds[buf][it] = b_dst[it] >= 0 ? buf * kStageElems + MS * G::LDA + b_dst[it] : kDump + lane * (16 / E);
    }
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(values, values_bytes);
    int64_t split_rows = (i_begin + nrows) * BR;
    if (split_rows > M) split_rows = M;
    split_rows -= i_begin * BR;                                                // dY rows of this split
    const int64_t dy_split = split_rows > 0 ? ((split_rows - 1) * lddy + (N - n0)) * E : 0;
    const __amdgpu_buffer_rsrc_t rsrc_b =
        make_rsrc(reinterpret_cast<const char *>(dY) + (i_begin * BR * lddy + n0) * E, (uint32_t)dy_split);

    AVec ra[D][G::NA];
    BVec rb[D][G::NB];
    // Global load of the next stage's activation vector `it` / dY vector `it` into
    // ring slot d.  Branch-free: a vector that is pruned, outside the matrix or
    // beyond the split reads as zero through an out-of-range offset, so the number
    // of loads in flight is known at compile time.  Each call moves the vector's
    // state on by one stage.
    auto load_a = [&](int d, int it) {
      ra[d][it] = buffer_load<G::VA * E>(rsrc_a, a_val[it] + a_src[it]);
      a_tab[it] += a_inc[it];
      a_val[it] = sTab[a_tab[it]];
    };
    auto load_b = [&](int d, int it) {
      rb[d][it] = buffer_load<VB * E>(rsrc_b, b_cur[it]);
      b_cur[it] += b_inc[it];
    };
    // Ring slot d -> LDS stage buffer `buf`; unused vectors go to the dump slot,
    // so no store needs a predicate.
    T *const s0 = reinterpret_cast<T *>(sStage);
    auto store_a = [&](int d, int it, int buf) { *reinterpret_cast<AVec *>(&s0[a_lds[buf][it]]) = ra[d][it]; };
    auto store_b = [&](int d, int it, int buf) { *reinterpret_cast<BVec *>(&s0[b_lds[buf][it]]) = rb[d][it]; };

    // stages 0 .. D-1 into the ring, stage 0 on into LDS buffer 0, stage D after it
#pragma unroll
    for (int d = 0; d < D; ++d) {
#pragma unroll
      for (int it = 0; it < G::NA; ++it) load_a(d, it);
#pragma unroll
      for (int it = 0; it < G::NB; ++it) load_b(d, it);
    }
#pragma unroll
    for (int it = 0; it < G::NA; ++it) { store_a(0, it, 0); load_a(0, it); }
#pragma unroll
    for (int it = 0; it < G::NB; ++it) { store_b(0, it, 0); load_b(0, it); }
    __syncthreads();
    // While the multipliers work on stage q (buffer q&1), stage q+1 moves from its
    // ring slot to the other buffer and the slot is refilled with stage q+1+D.
    // Many trips round the ring per loop iteration: at the loop header the
    // compiler's count of loads in flight falls back to a conservative value, so
    // the first stage of an iteration waits for nearly all of them.
    constexpr int U = (D % 2 == 0 ? D : 2 * D) * 4;
    for (int q0 = 0; q0 < nstages; q0 += U) {
      static_for<U>([&](auto uc) {
        constexpr int u = decltype(uc)::value;
        if (q0 + u < nstages) {
          constexpr int d = (u + 1) % D, buf = (u + 1) & 1;
#pragma unroll
          for (int it = 0; it < G::NA; ++it) { store_a(d, it, buf); load_a(d, it); }
#pragma unroll
          for (int it = 0; it < G::NB; ++it) { store_b(d, it, buf); load_b(d, it); }
          __syncthreads();
        }
      });
    }
    return;
  }

  // ================= multiplier waves =================
  const int wk = wave / WN, wn = wave % WN;
  v16f acc[2][G::NTW];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int w = 0; w < G::NTW; ++w)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[u][w][r] = 0.f;

  // Stage q out of LDS buffer `buf` in MSUB steps of 16 activation rows; only the
  // multiplies (and for binary32 their fragment reads) sit under the wave-uniform
  // skip branches.  The activity bits of 64 stages sit in one register (lane =
  // stage) and reach a scalar register through one v_readlane.
  uint32_t pam_reg = 0;
  auto stage_pam = [&](int q) {
    if ((q & 63) == 0) pam_reg = sPam[q + lane];
    uint32_t pam = (uint32_t)__builtin_amdgcn_readlane((int)pam_reg, q & 63) >> (16 * wk);
    asm volatile("" : "+s"(pam));           // one scalar register, tested bit by bit below
    return pam;
  };

  // ---- bfloat16: v_mfma_f32_32x32x16_bf16, fragments through transposing LDS reads ----
  int frag_a0 = 0, frag_a1 = 0, frag_b[G::NTW];
  if constexpr (E == 2) {
    frag_a0 = lane_fragment_offset((2 * wk) * 32);
    frag_a1 = lane_fragment_offset((2 * wk + 1) * 32);
#pragma unroll
    for (int w = 0; w < G::NTW; ++w) frag_b[w] = lane_fragment_offset((G::NTW * wn + w) * 32);
  }
  // The fragments of step ms+1 are requested before the multiplies of step ms
  // are issued.
  auto multiply_bf16 = [&](int q, int buf) {
    const uint16_t *sA = reinterpret_cast<const uint16_t *>(sStage + buf * G::STAGE_WORDS);
    const uint16_t *sB = sA + MS * G::LDA;
    const uint32_t pam = stage_pam(q);
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
      if (pam & (1u << (2 * ms))) {
#pragma unroll
        for (int w = 0; w < G::NTW; ++w)
          acc[0][w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb[w], acc[0][w], 0, 0, 0);
      }
      if (pam & (2u << (2 * ms))) {
#pragma unroll
        for (int w = 0; w < G::NTW; ++w)
          acc[1][w] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb[w], acc[1][w], 0, 0, 0);
      }
#pragma unroll
      for (int w = 0; w < G::NTW; ++w) fb[w] = nb[w];
      fa0 = na0; fa1 = na1;
    }
  };

  // ---- binary32: v_mfma_f32_32x32x2_f32.  One instruction contracts two
  // activation rows: lane l supplies column l % 32 of row l / 32 of the pair for
  // both operands, which is how the row-major LDS tiles are laid out already (no
  // transposition); a 16-row step is 8 instructions per 32 x 32 piece.  The
  // kernel is bound by the matrix core here (16 passes per 4096 multiply-adds).
  // this lane's element of a row pair: row lane / 32, column lane % 32 of a 32-column piece; odd rows
  // have their 32-column halves swapped (see swizzled), so lanes 32-63 read the other half
  const int pair_row = (lane >> 5) * kLd, pair_col = lane & 31, pair_swap = (lane >> 5) << 5;
  auto multiply_f32 = [&](int q, int buf) {
    const float *sA = reinterpret_cast<const float *>(sStage + buf * G::STAGE_WORDS);
    const float *sB = sA + MS * G::LDA;
    const uint32_t pam = stage_pam(q);
    const int offA0 = pair_row + ((((2 * wk) * 32) ^ pair_swap) + pair_col);
    const int offA1 = pair_row + ((((2 * wk + 1) * 32) ^ pair_swap) + pair_col);
#pragma unroll
    for (int ms = 0; ms < G::MSUB; ++ms) {
      if ((pam >> (2 * ms)) & 3u) {
        float fb[G::NTW][8];
#pragma unroll
        for (int w = 0; w < G::NTW; ++w) {
          const int offB = pair_row + ((((G::NTW * wn + w) * 32) ^ pair_swap) + pair_col);
#pragma unroll
          for (int p = 0; p < 8; ++p) fb[w][p] = sB[(16 * ms + 2 * p) * kLd + offB];
        }
        if (pam & (1u << (2 * ms))) {
#pragma unroll
          for (int p = 0; p < 8; ++p) {
            const float a = sA[(16 * ms + 2 * p) * kLd + offA0];
#pragma unroll
            for (int w = 0; w < G::NTW; ++w)
              acc[0][w] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, fb[w][p], acc[0][w], 0, 0, 0);
          }
        }
        if (pam & (2u << (2 * ms))) {
#pragma unroll
          for (int p = 0; p < 8; ++p) {
            const float a = sA[(16 * ms + 2 * p) * kLd + offA1];
#pragma unroll
            for (int w = 0; w < G::NTW; ++w)
              acc[1][w] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, fb[w][p], acc[1][w], 0, 0, 0);
          }
        }
      }
    }
  };
  auto multiply = [&](int q, int buf) {
    if constexpr (E == 2) multiply_bf16(q, buf);
    else multiply_f32(q, buf);
  };

  __syncthreads();                           // stage 0 is in LDS buffer 0
  for (int q0 = 0; q0 < nstages; q0 += 2) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (q0 + u >= nstages) break;
      multiply(q0 + u, u);
      __syncthreads();
    }
  }

  // (the branch on `accumulate` is taken once, outside the store loops: inside
  // them the compiler would read the destination speculatively in both cases)
  float *o = out + (int64_t)split * split_stride;
  auto write_tile = [&](auto acc_flag) {
    constexpr bool kAcc = decltype(acc_flag)::value;
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
            if (kAcc) *dst += acc[u][w][r];
            else *dst = acc[u][w][r];
          }
        }
  };
  if (accumulate) write_tile(std::true_type{});
  else write_tile(std::false_type{});
}

template <typename T, int BR, int BC, int MS, int VB, int D, int WN>
__global__ __launch_bounds__(256 * WN) void dw_mfma_kernel(DwParams prm, int xcd_map) {
  dw_mfma_body<T, BR, BC, MS, VB, D, WN>(prm, blockIdx.x, xcd_map);
}

// Several tensors per launch.  The work items (split, tile) of all products form one list,
// product after product (wg_begin = a product's first item), and XCD x (workgroup id % 8)
// takes the contiguous part [xcd_begin[x], xcd_begin[x + 1]) of it, cut by the host so that
// every XCD gets about the same number of stages.  An XCD then works on whole splits, one
// after the other, and fetches the operands of a split into its L2 once; dealing every
// product to all eight XCDs separately puts the halves of a split on two XCDs when a
// product has fewer splits than there are XCDs (a fifth more L2 fetches at the ResMLP-S12
// shapes, at the same run time).
// With many more workgroups than compute units the table build and the write-out of one
// workgroup overlap the main loop of its neighbour on the same compute unit.
constexpr int kDwBatchMax = 24;
struct DwBatch {
  DwParams it[kDwBatchMax];
  uint32_t xcd_begin[9];
};

template <typename T, int BR, int BC, int MS, int VB, int D, int WN>
__global__ __launch_bounds__(256 * WN) void dw_mfma_batched_kernel(DwBatch b, int n) {
  const uint32_t x = blockIdx.x & 7u, slot = blockIdx.x >> 3;
  if (slot >= b.xcd_begin[x + 1] - b.xcd_begin[x]) return;
  const uint32_t g = b.xcd_begin[x] + slot;
  int i = 0;
  while (i + 1 < n && g >= b.it[i + 1].wg_begin) ++i;
  dw_mfma_body<T, BR, BC, MS, VB, D, WN>(b.it[i], g - b.it[i].wg_begin, 0);
}

struct Plan {
  int splits;
  int64_t stages_per_split;
};

// Number of splits of the contraction.  The tiles x splits work items are processed in rounds
// of one workgroup per compute unit (binary32: 128 KB of LDS each) or two (2-byte elements); a
// round costs its stages plus a fixed part (table build, partial tile write-out), and every
// split adds one pass over the K x N partial tiles (written once, read once by the
// reduction).  The constants are measured orders of magnitude on MI355X, in microseconds
// (a stage of a workgroup that shares its compute unit takes 0.7 us); only the choice of s
// depends on them.
template <int E, int BR, int MS>
Plan make_plan(int64_t M, int64_t K, int64_t N) {
  constexpr int R = MS / BR;
  constexpr int kSlots = E == 2 ? 512 : 256;
  const int64_t nbr = ceil_div(M, BR);
  const int64_t stages = ceil_div(nbr, R);
  const int64_t tiles = ceil_div(K, 128) * ceil_div(N, 128);
  Plan p;
  p.splits = 1;
  p.stages_per_split = stages > 0 ? stages : 1;
  if (stages <= 0 || tiles <= 0) return p;
  // (binary32 stages are bound by the matrix core: 16 times the passes per multiply-add)
  const double us_stage = (E == 4 ? 1.3 : 0.70) * MS / 64.0, us_round = 8.0;
  const double us_split = 2.0 * (double)K * (double)N * 4.0 / 3.0e6;
  // (at least one split per 256 block-rows, although the table would hold 512: for 16-row blocks at
  // 50176 rows 14 splits of 112 stages take 106 us where 7 of 224 take 156 us)
  const int64_t s_min = ceil_div(stages * R, (int64_t)256);
  int64_t s_max = stages < 64 ? stages : 64;
  if (s_max < s_min) s_max = s_min;
  double best = 0;
  int64_t best_s = 0;
  for (int64_t s = s_min; s <= s_max; ++s) {
    const int64_t sps = ceil_div(stages, s);
    const int64_t s_eff = ceil_div(stages, sps);
    const int64_t rounds = ceil_div(tiles * s_eff, (int64_t)kSlots);
    const double cost = (double)rounds * ((double)sps * us_stage + us_round) + (s_eff > 1 ? (double)s_eff * us_split : 0.0);
    if (best_s == 0 || cost < best) { best = cost; best_s = s_eff; }
  }
  const int64_t sps = ceil_div(stages, best_s);
  p.splits = (int)ceil_div(stages, sps);
  p.stages_per_split = sps;
  return p;
}

// elements per dY vector: 16 bytes at most
template <int E>
int dy_vector(const void *dY, int64_t N, int64_t lddy) {
  int vb = 16 / E;
  while (vb > 1 && (N % vb != 0 || lddy % vb != 0 || (uintptr_t)dY % (E * vb) != 0)) vb >>= 1;
  return vb;
}

// The plan of a product that shares its launch with `companions` - 1 others.  A product on
// its own needs enough splits to occupy every compute unit; in a batch the other products
// do that, so fewer splits will do (fewer partial tiles to write and to add up, fewer table
// builds).  The launch runs its work items about two per compute unit at a time, so its
// duration is roughly (rounds of 512 items) x (stages of an item + a fixed part); the number
// of splits is the one that makes this smallest, the partial tiles counted at what their
// traffic costs, as if the companions were products of the same shape.  Never more splits
// than on its own: the workspace is sized for that.
template <int E, int BR, int MS>
Plan make_plan_batched(int64_t M, int64_t K, int64_t N, int companions) {
  const Plan alone = make_plan<E, BR, MS>(M, K, N);
  if (companions <= 1 || alone.splits <= 1) return alone;
  constexpr int R = MS / BR;
  constexpr int64_t kSlots = 512, kFixed = 16;                 // fixed part of an item, in stages
  constexpr double kBytesPerStage = 2.0e6;                     // partial-tile bytes that cost the time of one stage (measured)
  const int64_t stages = ceil_div(ceil_div(M, BR), R);
  const int64_t tiles = ceil_div(K, 128) * ceil_div(N, 128);
  const int64_t s_min = ceil_div(stages * R, (int64_t)kMaxRowsPerSplit);
  if (s_min >= alone.splits) return alone;
  const double split_cost = (double)companions * (double)K * (double)N * 8.0 / kBytesPerStage;
  double best = 0;
  Plan p = alone;
  for (int64_t s = s_min; s <= alone.splits; ++s) {
    const int64_t sps = ceil_div(stages, s);
    const int64_t s_eff = ceil_div(stages, sps);
    const int64_t rounds = ceil_div((int64_t)companions * tiles * s_eff, kSlots);
    const double cost = (double)(rounds * (sps + kFixed)) + (double)s_eff * split_cost;
    if (s == s_min || cost < best) {
      best = cost;
      p.splits = (int)s_eff;
      p.stages_per_split = sps;
    }
  }
  return p;
}

// Kernel parameters of one product; *wgs = workgroups of its launch, *splits as planned.
template <int E, int BR, int BC, int MS>
int fill_params(const DwJob &j, DwParams *prm, uint32_t *wgs, int companions = 1) {
  const Plan p = make_plan_batched<E, BR, MS>(j.M, j.K, j.N, companions);
  const size_t need = p.splits > 1 ? (size_t)p.splits * j.K * j.N * sizeof(float) : 0;
  if (need > 0 && (j.ws == nullptr || j.ws_bytes < need)) return BSR_ERR_WORKSPACE;
  const int64_t nbr = ceil_div(j.M, BR), nbc = ceil_div(j.K, BC);
  prm->row_ptr = j.row_ptr; prm->col_idx = j.col_idx; prm->values = j.values; prm->dY = j.dY;
  prm->out = p.splits > 1 ? static_cast<float *>(j.ws) : j.dW;
  prm->M = j.M; prm->K = j.K; prm->N = j.N; prm->lddy = j.lddy;
  prm->ldo = p.splits > 1 ? j.N : j.lddw;
  prm->split_stride = p.splits > 1 ? j.K * j.N : 0;
  prm->nbr = nbr; prm->nbc = nbc; prm->stages_per_split = p.stages_per_split;
  prm->accumulate = p.splits > 1 ? 0 : j.accumulate;
  prm->tiles_k = (int)ceil_div(j.K, 128); prm->tiles_n = (int)ceil_div(j.N, 128); prm->splits = p.splits;
  // 32-bit buffer offsets: both operands must stay below 4 GiB (checked by dw_mfma_supported)
  prm->values_bytes = (uint32_t)(nbr * nbc * BR * BC * E);
  prm->wg_begin = 0;
  const int64_t n_items = (int64_t)p.splits * prm->tiles_k * prm->tiles_n;
  *wgs = (uint32_t)(8 * ceil_div(n_items, 8));        // XCD-aware work item order: whole groups of 8
  return BSR_OK;
}

template <typename T, int BR, int BC, int MS, int D, int WN>
int run(const int32_t *row_ptr, const int32_t *col_idx, const void *values, int64_t M, int64_t K,
        const void *dY, int64_t N, int64_t lddy, float *dW, int64_t lddw, int accumulate, void *ws,
        size_t ws_bytes, hipStream_t s) {
  constexpr int E = (int)sizeof(T);
  const DwJob job{row_ptr, col_idx, values, M, K, BR, BC, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes};
  DwParams prm;
  uint32_t wgs;
  int rc = fill_params<E, BR, BC, MS>(job, &prm, &wgs);
  if (rc != BSR_OK) return rc;
  const dim3 grid(wgs);
  const int xcd_map = 1;      // XCD-aware work item order (0 = plain order, kept for measurements)
  int vb = dy_vector<E>(dY, N, lddy);
#define BSR_DW_LAUNCH(VB)                                                                         \
  hipLaunchKernelGGL((dw_mfma_kernel<T, BR, BC, MS, VB, D, WN>), grid, dim3(256 * WN), 0, s, prm, xcd_map)
  if constexpr (E == 2) {
    if (vb == 8) { BSR_DW_LAUNCH(8); vb = 0; }
  }
  if (vb == 0) {}
  else if (vb == 4) BSR_DW_LAUNCH(4);
  else if (vb == 2) BSR_DW_LAUNCH(2);
  else BSR_DW_LAUNCH(1);
#undef BSR_DW_LAUNCH
  rc = check_launch();
  if (rc != BSR_OK || prm.splits == 1) return rc;
  return launch_splitk_reduce(prm.out, prm.splits, K, N, dW, lddw, accumulate, s);
}

// The jobs of one kernel instance (block shape and dY vector width `want_vb`), kDwBatchMax per launch.
template <typename T, int BR, int BC, int MS, int D, int WN>
int run_batched(const DwJob *jobs, int n, int want_vb, hipStream_t s) {
  constexpr int E = (int)sizeof(T);
  DwBatch b;
  ReduceJob red[kDwBatchMax];
  int m = 0, nred = 0;
  uint32_t total = 0;
  auto flush = [&]() -> int {
    if (m == 0) return BSR_OK;
    // cut the item list into eight parts of about equal cost: an item costs its stages plus
    // a fixed part (table build, write-out) of about sixteen stages
    int64_t cost[kDwBatchMax], all = 0;
    for (int i = 0; i < m; ++i) {
      cost[i] = b.it[i].stages_per_split + 16;
      all += cost[i] * (int64_t)b.it[i].splits * b.it[i].tiles_k * b.it[i].tiles_n;
    }
    int x = 1;
    int64_t cum = 0;
    b.xcd_begin[0] = 0;
    for (int i = 0; i < m; ++i) {
      const int64_t items = (int64_t)b.it[i].splits * b.it[i].tiles_k * b.it[i].tiles_n;
      while (x < 8 && x * all <= 8 * (cum + items * cost[i])) {
        int64_t k = ceil_div(x * all - 8 * cum, 8 * cost[i]);     // items of product i before the cut
        if (k < 0) k = 0;
        if (k > items) k = items;
        b.xcd_begin[x++] = b.it[i].wg_begin + (uint32_t)k;
      }
      cum += items * cost[i];
    }
    while (x <= 8) b.xcd_begin[x++] = total;
    uint32_t longest = 0;
    for (int q = 0; q < 8; ++q)
      if (b.xcd_begin[q + 1] - b.xcd_begin[q] > longest) longest = b.xcd_begin[q + 1] - b.xcd_begin[q];
    const dim3 grid(8 * longest), block(256 * WN);
    switch (want_vb) {
      case 8:
        if constexpr (E == 2) hipLaunchKernelGGL((dw_mfma_batched_kernel<T, BR, BC, MS, 8, D, WN>), grid, block, 0, s, b, m);
        break;
      case 4: hipLaunchKernelGGL((dw_mfma_batched_kernel<T, BR, BC, MS, 4, D, WN>), grid, block, 0, s, b, m); break;
      case 2: hipLaunchKernelGGL((dw_mfma_batched_kernel<T, BR, BC, MS, 2, D, WN>), grid, block, 0, s, b, m); break;
      default: hipLaunchKernelGGL((dw_mfma_batched_kernel<T, BR, BC, MS, 1, D, WN>), grid, block, 0, s, b, m); break;
    }
    int rc = check_launch();
    if (rc == BSR_OK && nred > 0) rc = launch_splitk_reduce_batched(red, nred, s);
    m = 0;
    nred = 0;
    total = 0;
    return rc;
  };
  int mine = 0;                                              // products of this kernel instance
  for (int i = 0; i < n; ++i)
    if (jobs[i].br == BR && jobs[i].bc == BC && dy_vector<E>(jobs[i].dY, jobs[i].N, jobs[i].lddy) == want_vb) ++mine;
  int left = mine;
  for (int i = 0; i < n; ++i) {
    const DwJob &j = jobs[i];
    if (j.br != BR || j.bc != BC || dy_vector<E>(j.dY, j.N, j.lddy) != want_vb) continue;
    uint32_t wgs;
    // products that share this launch: the rest of the list, up to the launch's capacity
    const int companions = m + (left < kDwBatchMax - m ? left : kDwBatchMax - m);
    --left;
    int rc = fill_params<E, BR, BC, MS>(j, &b.it[m], &wgs, companions);
    if (rc != BSR_OK) return rc;
    b.it[m].wg_begin = total;                                // first item of this product in the launch's list
    total += (uint32_t)(b.it[m].splits * b.it[m].tiles_k * b.it[m].tiles_n);
    (void)wgs;
    if (b.it[m].splits > 1)
      red[nred++] = ReduceJob{b.it[m].out, j.dW, j.K, j.N, j.lddw, b.it[m].splits, j.accumulate};
    if (++m == kDwBatchMax) {
      rc = flush();
      if (rc != BSR_OK) return rc;
    }
  }
  return flush();
}

template <int E, int BR, int MS>
size_t ws_for(int64_t M, int64_t K, int64_t N) {
  const Plan p = make_plan<E, BR, MS>(M, K, N);
  return p.splits > 1 ? (size_t)p.splits * K * N * sizeof(float) : 0;
}

}  // namespace

bool dw_mfma_supported(int dtype, int br, int bc, const void *values, int64_t M, int64_t K, int64_t N,
                       int64_t lddy) {
  if (dtype != BSR_BF16 && dtype != BSR_F32) return false;
  if ((uintptr_t)values % 16 != 0) return false;
  const bool shape = (br == 32 && bc == 32) || (br == 64 && bc == 64) || (br == 16 && bc == 16) ||
                     (br == 14 && bc == 14);
  if (!shape) return false;
  // the kernel addresses both operands with 32-bit byte offsets; offsets of
  // activation values at or above 2 GiB mean "pruned", and the dY offsets of the
  // stages fetched ahead past the end of a split must not wrap
  const int64_t e = elem_bytes(dtype);
  if (ceil_div(M, br) * br * ceil_div(K, bc) * bc * e >= (int64_t(1) << 31)) return false;
  if ((M + 8 * 64) * lddy * e >= (int64_t(1) << 32) - 64 || N > lddy) return false;
  return true;
}

size_t dw_mfma_ws_bytes(int dtype, int64_t M, int64_t K, int64_t N, int br, int bc) {
  (void)bc;
  const bool f32 = dtype == BSR_F32;
  switch (br) {
    case 32: return f32 ? ws_for<4, 32, 64>(M, K, N) : ws_for<2, 32, 64>(M, K, N);
    case 64: return f32 ? ws_for<4, 64, 64>(M, K, N) : ws_for<2, 64, 64>(M, K, N);
    case 16: return f32 ? ws_for<4, 16, 32>(M, K, N) : ws_for<2, 16, 32>(M, K, N);
    case 14: return f32 ? ws_for<4, 14, 32>(M, K, N) : ws_for<2, 14, 32>(M, K, N);
    default: return 0;
  }
}

int launch_dw_mfma(int dtype, const int32_t *row_ptr, const int32_t *col_idx, const void *values, int64_t M,
                   int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy, float *dW,
                   int64_t lddw, int accumulate, void *ws, size_t ws_bytes, hipStream_t s) {
  if (K == 0 || N == 0) return BSR_OK;
#define BSR_ARGS row_ptr, col_idx, values, M, K, dY, N, lddy, dW, lddw, accumulate, ws, ws_bytes, s
  if (dtype == BSR_F32) {
    if (br == 32 && bc == 32) return run<float, 32, 32, 64, 2, 4>(BSR_ARGS);
    if (br == 64 && bc == 64) return run<float, 64, 64, 64, 2, 4>(BSR_ARGS);
    if (br == 16 && bc == 16) return run<float, 16, 16, 32, 2, 4>(BSR_ARGS);
    if (br == 14 && bc == 14) return run<float, 14, 14, 32, 2, 4>(BSR_ARGS);
    return BSR_ERR_SHAPE;
  }
  if (br == 32 && bc == 32) return run<uint16_t, 32, 32, 64, 2, 4>(BSR_ARGS);
  if (br == 64 && bc == 64) return run<uint16_t, 64, 64, 64, 2, 4>(BSR_ARGS);
  if (br == 16 && bc == 16) return run<uint16_t, 16, 16, 32, 2, 4>(BSR_ARGS);
  if (br == 14 && bc == 14) return run<uint16_t, 14, 14, 32, 2, 4>(BSR_ARGS);
#undef BSR_ARGS
  return BSR_ERR_SHAPE;
}

int launch_dw_mfma_batched(int dtype, const DwJob *jobs, int n, hipStream_t s) {
  static const int kVbs[4] = {8, 4, 2, 1};
  for (int vi = 0; vi < 4; ++vi) {
    const int vb = kVbs[vi];
    int rc;
    if (dtype == BSR_F32) {
      if (vb == 8) continue;
      if ((rc = run_batched<float, 32, 32, 64, 2, 4>(jobs, n, vb, s)) != BSR_OK) return rc;
      if ((rc = run_batched<float, 64, 64, 64, 2, 4>(jobs, n, vb, s)) != BSR_OK) return rc;
      if ((rc = run_batched<float, 16, 16, 32, 2, 4>(jobs, n, vb, s)) != BSR_OK) return rc;
      if ((rc = run_batched<float, 14, 14, 32, 2, 4>(jobs, n, vb, s)) != BSR_OK) return rc;
    } else {
      if ((rc = run_batched<uint16_t, 32, 32, 64, 2, 2>(jobs, n, vb, s)) != BSR_OK) return rc;
      if ((rc = run_batched<uint16_t, 64, 64, 64, 2, 2>(jobs, n, vb, s)) != BSR_OK) return rc;
      if ((rc = run_batched<uint16_t, 16, 16, 32, 2, 2>(jobs, n, vb, s)) != BSR_OK) return rc;
      if ((rc = run_batched<uint16_t, 14, 14, 32, 2, 2>(jobs, n, vb, s)) != BSR_OK) return rc;
    }
  }
  return BSR_OK;
}

}  // namespace bsr
