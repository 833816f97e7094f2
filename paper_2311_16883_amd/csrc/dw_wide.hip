// Weight gradient from a BSR activation (paper Sec. III, Fig. 2: dW = Xhat^T * dY)
// for bfloat16 inputs and 32x32 or 64x64 blocks, with workgroup tiles that span
// 384 rows of dW, so that every row of dY is read once per 384 columns of the
// activation (once in all for the 384-wide ResMLP inputs) and every kept block
// once per 128 output columns.
//
// What bounds this operator on gfx950 is not the matrix pipeline but what feeds it.
// Both operands have the contraction index as their slow axis, so every fragment of
// v_mfma_f32_32x32x16_bf16 comes out of LDS through two transposing reads
// (ds_read_b64_tr_b16); a compute unit delivers about 360 bytes of those per
// nanosecond, 1.4 fragments per matrix instruction and SIMD, and a wave issues one
// instruction every four cycles, eight per matrix instruction.  The kernel is built
// to keep all three -- copies, fragment reads, multiplies -- busy at the same time:
//
//  * Global -> LDS copies are done by the texture path itself (buffer_load ... lds,
//    16 bytes per lane): no staging registers, no LDS store instructions, and pruned
//    blocks are simply not requested (their LDS slot keeps stale bits that no
//    instruction reads).  Every wave issues one pair of copies per stage and waits
//    for its own with an explicit vmcnt.
//  * LDS holds a ring of four stages of 32 contraction rows; a stage is a set of
//    slabs of 32 rows x 32 columns with 64-byte rows -- for 32x32 blocks a slab is
//    2 KB of `values` exactly as stored -- and the four rows that a 16-lane group of
//    a transposing read touches are 256 consecutive bytes: no bank conflicts, no
//    swizzle.  One barrier per stage.
//  * Sixteen waves, four per SIMD: what a wave can issue (an instruction every six or
//    seven cycles once scalar dependencies and branches are counted) is the scarcest
//    resource, so the per-stage work is spread over many short instruction streams.
//    Wave (wk, wn) owns 3 pieces of 32 rows x 1 strip of 32 columns of dW.  The four
//    waves of a SIMD are (0..3, wn): together they see all twelve pieces of a stage,
//    so every SIMD multiplies the same number of kept blocks however the pruned
//    blocks fall.  A fragment of the activation is read only for a kept block.
//  * The loop is software-pipelined across the barrier: after barrier q a wave first
//    requests the fragments of stage q (into one of two register sets), then issues
//    the multiplies of stage q - 1 out of the other set.  Without this, the barrier
//    puts all waves in phase -- everybody reads, then everybody multiplies -- and the
//    LDS and the matrix pipeline take turns idling.
#include <utility>

#include "buffer_access.h"
#include "common.h"

namespace bsr {

namespace {

typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(16))) float v16f;

constexpr int kTileK = 384;            // rows of dW per workgroup: 12 pieces of 32
constexpr int kPieces = kTileK / 32;
constexpr int kTileN = 128;            // columns of dW per workgroup: 4 strips of 32
constexpr int kStrips = kTileN / 32;
constexpr int kSlabBytes = 2048;       // 32 contraction rows x 32 columns of bfloat16
constexpr int kStageBytes = (kPieces + kStrips) * kSlabBytes;   // 32 KB
constexpr int kRing = 4;               // stages in LDS: 128 KB
constexpr int kWideMaxRows = 2048;     // block-rows of one split: one table word per block-row in LDS
constexpr int kWaves = 16;             // 4 (rows of dW) x 4 (columns): four waves per SIMD
constexpr int kWideThreads = 64 * kWaves;
constexpr int kPW = kPieces / 4;       // pieces per wave
constexpr int kWideMaxSplits = 16;     // splits of the contraction the planner may pick (the workspace is sized for them)
constexpr uint32_t kTableIndexLimit = 1u << 20;   // kept blocks of one split's block-rows (20 bits of a table word)

struct WideParams {
  const int32_t *row_ptr, *col_idx;
  const void *values, *dY;
  float *out;
  int64_t K, N, lddy, ldo, split_stride;
  int32_t nbr, nbc, rows_per_split, splits, tiles_k, tiles_n, accumulate;
  uint32_t values_bytes, dy_bytes;
  uint32_t wg_begin;       // first work item of this product in a batched launch's list
};

// Two global -> LDS copies of 64 lanes x 16 bytes each: lane l's bytes land at lds_addr +
// 16 * l and at lds_addr + 1024 + 16 * l; the global side is voff_lo + soff and voff_hi + soff
// + 1024 (the instruction's immediate offset moves both sides).  Inline assembly, so that the
// compiler keeps no account of these copies: it would otherwise wait for all of them (vmcnt(0))
// in front of the first LDS read that follows.  The waits are explicit (wait_copies).  (A scalar
// write of M0 needs one wait state before an instruction that reads it.)
__device__ __forceinline__ void copy_pair_to_lds(__amdgpu_buffer_rsrc_t rsrc, uint32_t lds_addr, uint32_t voff_lo,
                                                 uint32_t voff_hi, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
               "buffer_load_dwordx4 %1, %3, %4 offen lds\n\t"
               "buffer_load_dwordx4 %2, %3, %4 offen offset:1024 lds"
               :: "s"(lds_addr), "v"(voff_lo), "v"(voff_hi), "s"(rsrc), "s"(soff) : "memory", "m0");
}

// The compiler moves arithmetic on values it knows to be the same in all lanes to the scalar unit;
// this hides where a value came from, so that what is computed from it stays on the vector units.
__device__ __forceinline__ uint32_t vector_value(uint32_t x) {
  asm volatile("" : "+v"(x));
  return x;
}

// The reads of LDS that precede it in program order have completed, then the workgroup barrier.
__device__ __forceinline__ void stage_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// 16 contraction rows x 32 columns out of a slab, as the operand of one matrix
// instruction: two transposing reads of 4 rows x 16 columns per 16-lane group.
__device__ __forceinline__ v8bf read_fragment(const uint8_t *p) {
  typedef v4s __attribute__((address_space(3))) * lds_v4s;
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 256));
  v8s r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return __builtin_bit_cast(v8bf, r);
}

// Activation fragments of part of a stage in registers: the kept pieces among NP of the wave's
// three, two contraction steps of 16 rows each.
template <int NP>
struct PartFrags {
  v8bf a0[NP], a1[NP];
  uint32_t mine;      // kept pieces (bit i = piece i of the part), wave-uniform
};
constexpr int kFirst = 2;              // pieces of a wave whose fragments are requested first
struct StripFrags {
  v8bf b0, b1;        // the wave's dY strip, two contraction steps
};

// BS = block size (32 or 64).  item = (split, tile) of this product, tile = (tk, tn), tn fastest:
// workgroups that run side by side share the activation rows of their split.
template <int BS>
struct WideBody {
  static __device__ __forceinline__ void run(const WideParams &prm, const uint32_t item) {
    constexpr int JT = kTileK / BS;                  // block-columns of a tile: 12 or 6
    constexpr int SPB = BS / 32;                     // stages per block-row = pieces per block-column
    constexpr uint32_t kBlockBytes = BS * BS * 2;
    constexpr uint32_t kRowBytes = BS * 2;           // bytes of one row of a block

    __shared__ __attribute__((aligned(1024))) uint8_t sRing[kRing * kStageBytes];
    // per block-row of the split: kept block-columns of the tile (low 12 bits) and the position
    // of the first of them in col_idx / values, relative to the split's first block
    __shared__ uint32_t sTab[kWideMaxRows + 16];      // (zero words behind the split's last block-row)

    const int32_t *__restrict__ row_ptr = prm.row_ptr;
    const int32_t *__restrict__ col_idx = prm.col_idx;
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);

    const int tiles = prm.tiles_k * prm.tiles_n;
    const int split = (int)(item / (uint32_t)tiles), tile = (int)(item % (uint32_t)tiles);
    const int tk = tile / prm.tiles_n, tn = tile % prm.tiles_n;
    const int64_t k0 = (int64_t)tk * kTileK, n0 = (int64_t)tn * kTileN;
    const int i_begin = split * prm.rows_per_split;
    int nrows = prm.nbr - i_begin;
    if (nrows > prm.rows_per_split) nrows = prm.rows_per_split;
    if (nrows < 0) nrows = 0;
    const int nstages = __builtin_amdgcn_readfirstlane(nrows * SPB);
    const int jfirst = tk * JT;
    int jt = prm.nbc - jfirst;
    if (jt > JT) jt = JT;

    // ---- table: which block-columns of the tile every block-row of the split keeps ----
    int32_t pos0;
    {
      int32_t *const sPtr = reinterpret_cast<int32_t *>(sRing);                 // nrows + 1 row pointers
      uint32_t *const sCols = reinterpret_cast<uint32_t *>(sRing + 16384);      // the split's column indices
      constexpr int kColsCap = (kRing * kStageBytes - 16384) / 4;
      for (int rr = t; rr <= nrows; rr += kWideThreads) sPtr[rr] = row_ptr[i_begin + rr];
      __syncthreads();
      pos0 = sPtr[0];
      const int32_t ncols = sPtr[nrows] - pos0;
      const bool cols_in_lds = ncols >= 0 && ncols <= kColsCap;
      if (cols_in_lds)
        for (int e = t; e < ncols; e += kWideThreads) sCols[e] = (uint32_t)col_idx[pos0 + e];
      __syncthreads();
      for (int rr = t; rr < nrows; rr += kWideThreads) {
        const int32_t p0 = sPtr[rr];
        int32_t p1 = sPtr[rr + 1];
        if (p1 - p0 > prm.nbc) p1 = p0 + prm.nbc;       // a valid row never holds more
        uint32_t mask = 0;
        int32_t base = p0;
        bool first = true;
        for (int32_t p = p0; p < p1; ++p) {
          const int j = cols_in_lds ? (int)sCols[p - pos0] : (int)col_idx[p];
          if (j >= jfirst && j < jfirst + jt) {
            if (first) { base = p; first = false; }
            mask |= 1u << (j - jfirst);
          }
        }
        sTab[rr] = ((uint32_t)(base - pos0) << 12) | mask;
      }
      if (t < 16) sTab[nrows + t] = 0u;
      __syncthreads();          // the table is complete and the ring's memory is free again
    }
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)sRing;

    // What follows keeps scalar instructions out of the loop wherever it can: a compute unit issues
    // about one of them per cycle for all its waves together, and sixteen waves that each spend forty
    // on bookkeeping would need more time for that than the matrix pipeline needs for the stage.  So
    // everything that is the same for all lanes but differs from stage to stage (table words, block
    // offsets) stays in vector registers, ring slots are compile-time constants of a loop unrolled four
    // times, and a scalar value is made only where an instruction needs one: M0, and the three bits
    // that say which of the wave's pieces are kept.

    // ---- this wave's share of the copies: one pair per stage, always, into slab `wave` of the stage:
    // activation piece `wave` (waves 0-11) or dY strip `wave - 12` (waves 12-15).  A copy moves 16 rows
    // x 64 bytes, lane -> (row lane / 4, 16-byte chunk lane % 4), 1 KB in LDS in lane order; the second
    // copy of the pair takes rows 16 .. 31.  A pruned piece is "copied" from an offset beyond the
    // buffer: the hardware then writes zeros into a slab nobody reads and touches no memory, and every
    // wave has the same number of copies in flight whatever the sparsity pattern, so the wait for a
    // stage is a constant vmcnt.
    const bool is_piece = wave < kPieces;
    const __amdgpu_buffer_rsrc_t rsrc = is_piece ? make_rsrc(prm.values, prm.values_bytes) : make_rsrc(prm.dY, prm.dy_bytes);
    constexpr uint32_t kBeyond = 0xFFFF0000u;          // an offset no buffer reaches
    uint32_t v_run;             // per-lane offset of the pair's first copy for the next stage to fetch (without the block's)
    {
      const uint32_t a_lo = (uint32_t)(lane >> 2) * kRowBytes + (uint32_t)(lane & 3) * 16u + (uint32_t)pos0 * kBlockBytes +
                            (SPB == 2 ? (uint32_t)(wave & 1) * 64u : 0u);
      const int64_t row = (int64_t)i_begin * BS + (lane >> 2);
      const uint32_t b_lo = (uint32_t)((row * prm.lddy + n0 + 32 * (wave - kPieces)) * 2 + (lane & 3) * 16);
      v_run = is_piece ? a_lo : b_lo;
    }
    const uint32_t v_hi_delta = is_piece ? 16u * kRowBytes - 1024u : (uint32_t)(16 * prm.lddy * 2) - 1024u;
    const uint32_t v_step = is_piece ? 0u : (uint32_t)(32 * prm.lddy * 2);
    const uint32_t my_jl = vector_value(is_piece ? (uint32_t)(wave / SPB) : 0u);   // block-column (of the tile) of this wave's piece
    const uint32_t below = vector_value((1u << (is_piece ? wave / SPB : 0)) - 1u);
    const uint32_t always = vector_value(is_piece ? 0u : 1u);            // a dY strip is never pruned
    const uint32_t scale = vector_value(is_piece ? kBlockBytes : 0u);
    const uint32_t half_bytes = vector_value(is_piece ? 32u * kRowBytes : 0u);
    uint32_t m0_slot[kRing];
#pragma unroll
    for (int k = 0; k < kRing; ++k) m0_slot[k] = ring_lds + (uint32_t)(wave * kSlabBytes + k * kStageBytes);
    // Copies of a stage into ring slot `slot`; w = table word of the stage's block-row (in every lane),
    // second_half = the stage is the lower half of a 64-row block-row.
    auto issue = [&](uint32_t m0, uint32_t w, uint32_t second_half) {
      const uint32_t bm = w & 0xfffu;
      const uint32_t kept = ((bm >> my_jl) & 1u) | always;
      const uint32_t idx = (w >> 12) + (uint32_t)__builtin_popcount(bm & below);     // block, from the split's first
      uint32_t off = v_run + __umul24(idx, scale);
      if (SPB == 2 && second_half) off += half_bytes;
      const uint32_t lo = kept ? off : kBeyond;
      const uint32_t hi = kept ? off + v_hi_delta : kBeyond;
      copy_pair_to_lds(rsrc, m0, lo, hi, 0u);
      v_run += v_step;
    };

    const int wk = wave >> 2, wn = wave & 3;
    const int g4 = lane >> 4, L = lane & 15;
    const uint32_t frag_off = (uint32_t)((8 * (g4 >> 1) + (L >> 2)) * 64 + (16 * (g4 & 1) + 4 * (L & 3)) * 2);
    const uint8_t *const myA = sRing + (kPW * wk) * kSlabBytes + frag_off;
    const uint8_t *const myB = sRing + (kPieces + wn) * kSlabBytes + frag_off;
    v16f acc[kPW];
#pragma unroll
    for (int i = 0; i < kPW; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    // requests the activation fragments of pieces [first, first + NP) of the wave in ring slot `slot`
    auto load_part = [&](auto &f, int slot, auto first_c, uint32_t mine) {
      constexpr int first = decltype(first_c)::value;
      constexpr int NP = sizeof(f.a0) / sizeof(f.a0[0]);
      f.mine = mine;
      const uint8_t *bufA = myA + slot * kStageBytes + first * kSlabBytes;
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        if (mine & (1u << i)) {
          f.a0[i] = read_fragment(bufA + i * kSlabBytes);
          f.a1[i] = read_fragment(bufA + i * kSlabBytes + 1024);
        }
      }
    };
    auto load_strip = [&](StripFrags &f, int slot) {
      const uint8_t *bufB = myB + slot * kStageBytes;
      f.b0 = read_fragment(bufB);
      f.b1 = read_fragment(bufB + 1024);
    };
    // the multiplies of the part of a stage whose fragments are in registers
    auto multiply = [&](const auto &f, const StripFrags &b, auto first_c) {
      constexpr int first = decltype(first_c)::value;
      constexpr int NP = sizeof(f.a0) / sizeof(f.a0[0]);
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        if (f.mine & (1u << i)) {
          acc[first + i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a0[i], b.b0, acc[first + i], 0, 0, 0);
          acc[first + i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a1[i], b.b1, acc[first + i], 0, 0, 0);
        }
      }
    };
    typedef std::integral_constant<int, 0> At0;
    typedef std::integral_constant<int, kFirst> AtRest;
    const uint32_t my_shift = vector_value((uint32_t)(kPW * wk));
    // kept pieces of this wave in a stage, from the table word of the stage's block-row (vector arithmetic)
    auto my_pieces = [&](uint32_t w) -> uint32_t {
      if (SPB == 1) return (w >> my_shift) & ((1u << kPW) - 1u);
      uint32_t m = 0;
#pragma unroll
      for (int i = 0; i < kPW; ++i) m |= ((w >> ((my_shift + (uint32_t)i) >> 1)) & 1u) << i;
      return m;
    };

    // ---- main loop, four stages per trip (ring slot = stage % 4 is then a constant) ----
    const uint32_t *tab = sTab;                   // table word of stage 4 * trip (advances once per trip)
#pragma unroll
    for (int d = 0; d < kRing - 1; ++d) issue(m0_slot[d], vector_value(tab[d / SPB]), (uint32_t)(d & 1));
    PartFrags<kFirst> head;                       // pieces 0-1 of the wave
    PartFrags<kPW - kFirst> rest;                 // piece 2
    StripFrags strip[2];                          // by stage parity
    head.mine = 0u;
    rest.mine = 0u;
    uint32_t w_issue = tab[(kRing - 1) / SPB];    // table words are read one stage ahead of their use
    uint32_t w_cur = tab[0];
    // One stage, software-pipelined across the barrier by part of a stage: after barrier q the
    // fragments of the first pieces of stage q are requested, then the last piece of stage q - 1
    // is multiplied (its fragments were requested before the barrier), then the last piece of
    // stage q is requested and the first ones multiplied.  Requests and multiplies of different
    // parts overlap in every wave, whatever phase the barrier forces on the waves.
    auto stage = [&](auto slot_c) {
      constexpr int slot = decltype(slot_c)::value;                  // stage q = 4 * trip + slot
      constexpr int slot_new = (slot + kRing - 1) % kRing;           // stage q + 3 goes where stage q - 1 was
      const uint32_t mine = (uint32_t)__builtin_amdgcn_readfirstlane((int)my_pieces(vector_value(w_cur)));
      // of this wave's copies, those of stage q have landed when only the four of the two
      // stages after it are still on their way
      asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
      stage_barrier();               // ... everybody's have, and everybody has the fragments of stage q - 1
      issue(m0_slot[slot_new], vector_value(w_issue), (uint32_t)((slot + kRing - 1) & 1));
      w_issue = tab[(slot + kRing) / SPB];
      w_cur = tab[(slot + 1) / SPB];
      StripFrags &bq = strip[slot & 1];
      const StripFrags &bprev = strip[(slot + 1) & 1];
      if (mine != 0u) load_strip(bq, slot);
      load_part(head, slot, At0{}, mine & ((1u << kFirst) - 1u));
      multiply(rest, bprev, AtRest{});
      load_part(rest, slot, AtRest{}, mine >> kFirst);
      multiply(head, bq, At0{});
    };
    const int trips = (nstages + kRing - 1) / kRing;     // stages beyond the last have zero table words
    for (int trip = 0; trip < trips; ++trip) {
      stage(std::integral_constant<int, 0>{});
      stage(std::integral_constant<int, 1>{});
      stage(std::integral_constant<int, 2>{});
      stage(std::integral_constant<int, 3>{});
      tab += kRing / SPB;
    }
    // the last piece of the last stage
    multiply(rest, strip[1], AtRest{});
    // no copy may still be on its way when the workgroup gives its LDS back
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- write-out (the branch on `accumulate` is taken once, outside the store loops) ----
    float *o = prm.out + (int64_t)split * prm.split_stride;
    const int64_t K = prm.K, N = prm.N, ldo = prm.ldo;
    auto write_tile = [&](auto acc_flag) {
      constexpr bool kAcc = decltype(acc_flag)::value;
#pragma unroll
      for (int i = 0; i < kPW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t k = k0 + (kPW * wk + i) * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          const int64_t n = n0 + wn * 32 + (lane & 31);
          if (k < K && n < N) {
            float *dst = o + k * ldo + n;
            if (kAcc) *dst += acc[i][r];
            else *dst = acc[i][r];
          }
        }
    };
    if (prm.accumulate) write_tile(std::true_type{});
    else write_tile(std::false_type{});
  }
};

template <int BS>
__global__ __launch_bounds__(kWideThreads) void dw_wide_kernel(WideParams prm, int xcd_map) {
  // Workgroup ids are dealt to the 8 XCDs round-robin; XCD x takes the x-th contiguous
  // eighth of the (split, tile) list, so the tiles of one split meet in one L2.
  const int items = prm.tiles_k * prm.tiles_n * prm.splits;
  uint32_t item = blockIdx.x;
  if (xcd_map) {
    const uint32_t per_xcd = (uint32_t)(items + 7) / 8u;
    if ((blockIdx.x >> 3) >= per_xcd) return;
    item = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  }
  if (item >= (uint32_t)items) return;
  WideBody<BS>::run(prm, item);
}

constexpr int kWideBatchMax = 24;
struct WideBatch {
  WideParams it[kWideBatchMax];
  uint32_t xcd_begin[9];
};

// Several products per launch: their work items form one list, product after product, and
// XCD x takes the part [xcd_begin[x], xcd_begin[x + 1]) of it (cut by the host into eight
// parts of equal cost).
template <int BS>
__global__ __launch_bounds__(kWideThreads) void dw_wide_batched_kernel(WideBatch b, int n) {
  const uint32_t x = blockIdx.x & 7u, slot = blockIdx.x >> 3;
  if (slot >= b.xcd_begin[x + 1] - b.xcd_begin[x]) return;
  const uint32_t g = b.xcd_begin[x] + slot;
  int i = 0;
  while (i + 1 < n && g >= b.it[i + 1].wg_begin) ++i;
  const WideParams &prm = b.it[i];
  const uint32_t item = g - prm.wg_begin;
  WideBody<BS>::run(prm, item);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------

int g_wide_config = 0;        // 0: 2 x 2 waves (6 pieces x 2 strips each); 1: 1 x 4 waves (12 pieces x 1 strip each)
int g_wide_splits = 0;        // > 0: forced number of splits (measurements)
int g_wide_debug = 0;

int64_t wide_tiles(int64_t K, int64_t N) { return ceil_div(K, kTileK) * ceil_div(N, kTileN); }

// Number of splits of the contraction for a launch whose products have `tiles_all` tiles in
// all, `bytes_out` bytes of dW in all and `stages` stages each: rounds of 256 workgroups,
// each as long as its stages plus a fixed part (table, first copies, write-out), plus what
// the partial tiles cost (written once, read once by the reduction).  Measured orders of
// magnitude on MI355X; only the choice depends on them.
int wide_splits(int64_t tiles_all, int64_t stages, int64_t rows, double bytes_out) {
  if (g_wide_splits > 0) {
    int64_t s = g_wide_splits;
    const int64_t s_min = ceil_div(rows, (int64_t)kWideMaxRows);
    if (s < s_min) s = s_min;
    if (s > kWideMaxSplits && s > s_min) s = kWideMaxSplits > s_min ? kWideMaxSplits : s_min;
    if (s > rows) s = rows > 0 ? rows : 1;
    return (int)s;
  }
  const double us_stage = 0.45, fixed_stages = 14.0, bytes_per_us = 2.5e6;
  const int64_t s_min = rows > 0 ? ceil_div(rows, (int64_t)kWideMaxRows) : 1;
  int64_t s_max = rows < kWideMaxSplits ? rows : kWideMaxSplits;
  if (s_max < s_min) s_max = s_min;
  double best = 0;
  int64_t best_s = s_min;
  for (int64_t s = s_min; s <= s_max; ++s) {
    const int64_t rounds = ceil_div(tiles_all * s, (int64_t)256);
    const double sps = (double)ceil_div(stages, s);
    const double cost = (double)rounds * (sps + fixed_stages) * us_stage + (s > 1 ? 2.0 * (double)s * bytes_out / bytes_per_us : 0.0);
    if (s == s_min || cost < best) { best = cost; best_s = s; }
  }
  return (int)best_s;
}

template <int BS>
void wide_fill(const DwJob &j, int splits, WideParams *p) {
  const int64_t nbr = ceil_div(j.M, BS), nbc = ceil_div(j.K, BS);
  const int64_t rps = nbr > 0 ? ceil_div(nbr, (int64_t)splits) : 1;
  const int eff = nbr > 0 ? (int)ceil_div(nbr, rps) : 1;
  p->row_ptr = j.row_ptr; p->col_idx = j.col_idx; p->values = j.values; p->dY = j.dY;
  p->out = eff > 1 ? static_cast<float *>(j.ws) : j.dW;
  p->K = j.K; p->N = j.N; p->lddy = j.lddy;
  p->ldo = eff > 1 ? j.N : j.lddw;
  p->split_stride = eff > 1 ? j.K * j.N : 0;
  p->nbr = (int32_t)nbr; p->nbc = (int32_t)nbc; p->rows_per_split = (int32_t)rps; p->splits = eff;
  p->tiles_k = (int32_t)ceil_div(j.K, kTileK); p->tiles_n = (int32_t)ceil_div(j.N, kTileN);
  p->accumulate = eff > 1 ? 0 : j.accumulate;
  p->values_bytes = (uint32_t)(nbr * nbc * BS * BS * 2);
  p->dy_bytes = j.M > 0 ? (uint32_t)(((j.M - 1) * j.lddy + j.N) * 2) : 0u;
  p->wg_begin = 0;
}

template <int BS>
int wide_run_batched(const DwJob *jobs, int n, hipStream_t s) {
  if (n <= 0) return BSR_OK;
  // one plan for the whole list: the number of splits that suits the products together
  int64_t tiles_all = 0, stages = 0, rows = 0;
  double bytes_out = 0;
  int mine = 0;
  for (int i = 0; i < n; ++i) {
    if (jobs[i].br != BS) continue;
    ++mine;
    tiles_all += wide_tiles(jobs[i].K, jobs[i].N);
    const int64_t r = ceil_div(jobs[i].M, BS);
    if (r > rows) rows = r;
    bytes_out += 4.0 * (double)jobs[i].K * (double)jobs[i].N;
  }
  if (mine == 0) return BSR_OK;
  stages = rows * (BS / 32);
  WideBatch b;
  ReduceJob red[kWideBatchMax];
  int m = 0, nred = 0;
  uint32_t total = 0;
  // (the plan is made for up to kWideBatchMax products at a time: what one launch holds)
  const int64_t per_launch_tiles = mine > kWideBatchMax ? tiles_all * kWideBatchMax / mine : tiles_all;
  const double per_launch_bytes = mine > kWideBatchMax ? bytes_out * kWideBatchMax / mine : bytes_out;
  const int splits = wide_splits(per_launch_tiles, stages, rows, per_launch_bytes);
  auto flush = [&]() -> int {
    if (m == 0) return BSR_OK;
    int64_t cost[kWideBatchMax], all = 0;
    for (int i = 0; i < m; ++i) {
      cost[i] = (int64_t)b.it[i].rows_per_split * (BS / 32) + 14;
      all += cost[i] * (int64_t)b.it[i].splits * b.it[i].tiles_k * b.it[i].tiles_n;
    }
    int x = 1;
    int64_t cum = 0;
    b.xcd_begin[0] = 0;
    for (int i = 0; i < m; ++i) {
      const int64_t items = (int64_t)b.it[i].splits * b.it[i].tiles_k * b.it[i].tiles_n;
      while (x < 8 && x * all <= 8 * (cum + items * cost[i])) {
        int64_t k = ceil_div(x * all - 8 * cum, 8 * cost[i]);
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
    hipLaunchKernelGGL((dw_wide_batched_kernel<BS>), dim3(8 * longest), dim3(kWideThreads), 0, s, b, m);
    int rc = check_launch();
    if (rc == BSR_OK && nred > 0) rc = launch_splitk_reduce_batched(red, nred, s);
    m = 0; nred = 0; total = 0;
    return rc;
  };
  for (int i = 0; i < n; ++i) {
    const DwJob &j = jobs[i];
    if (j.br != BS) continue;
    wide_fill<BS>(j, splits, &b.it[m]);
    const size_t need = b.it[m].splits > 1 ? (size_t)b.it[m].splits * j.K * j.N * sizeof(float) : 0;
    if (need > 0 && (j.ws == nullptr || j.ws_bytes < need)) return BSR_ERR_WORKSPACE;
    b.it[m].wg_begin = total;
    total += (uint32_t)(b.it[m].splits * b.it[m].tiles_k * b.it[m].tiles_n);
    if (b.it[m].splits > 1)
      red[nred++] = ReduceJob{b.it[m].out, j.dW, j.K, j.N, j.lddw, b.it[m].splits, j.accumulate};
    if (++m == kWideBatchMax) {
      const int rc = flush();
      if (rc != BSR_OK) return rc;
    }
  }
  return flush();
}

template <int BS>
int wide_run(const DwJob &j, hipStream_t s) {
  const int64_t rows = ceil_div(j.M, BS);
  const int splits = wide_splits(wide_tiles(j.K, j.N), rows * (BS / 32), rows, 4.0 * (double)j.K * (double)j.N);
  WideParams p;
  wide_fill<BS>(j, splits, &p);
  const size_t need = p.splits > 1 ? (size_t)p.splits * j.K * j.N * sizeof(float) : 0;
  if (need > 0 && (j.ws == nullptr || j.ws_bytes < need)) return BSR_ERR_WORKSPACE;
  const int64_t items = (int64_t)p.splits * p.tiles_k * p.tiles_n;
  hipLaunchKernelGGL((dw_wide_kernel<BS>), dim3((unsigned)(8 * ceil_div(items, 8))), dim3(kWideThreads), 0, s, p, 1);
  int rc = check_launch();
  if (rc != BSR_OK || p.splits == 1) return rc;
  return launch_splitk_reduce(p.out, p.splits, j.K, j.N, j.dW, j.lddw, j.accumulate, s);
}

}  // namespace

void dw_wide_set_config(int config, int splits, int debug) {
  g_wide_config = config;
  g_wide_splits = splits;
  g_wide_debug = debug;
}

// Shapes the wide kernel takes: bfloat16, 32x32 or 64x64 blocks, dY rows that are whole
// 16-byte chunks, operands addressable with 32-bit byte offsets.
bool dw_wide_supported(int dtype, int br, int bc, const void *values, const void *dY, int64_t M, int64_t K,
                       int64_t N, int64_t lddy) {
  if (dtype != BSR_BF16 || br != bc || (br != 32 && br != 64)) return false;
  if ((uintptr_t)values % 16 != 0 || (uintptr_t)dY % 16 != 0 || N % 8 != 0 || lddy % 8 != 0 || N > lddy) return false;
  if (M <= 0 || K <= 0 || N <= 0) return false;
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  if (nbr * nbc * br * bc * 2 >= (int64_t(1) << 32) - 2 * 65536) return false;
  if ((nbr * br + 64 + 4 * 32) * lddy * 2 + 2 * N + 1024 >= (int64_t(1) << 32) - 65536) return false;
  if (nbr >= (int64_t(1) << 30) || nbc * (int64_t)kWideMaxRows >= (int64_t)kTableIndexLimit) return false;
  return true;
}

// Workspace of the wide kernel: partial tiles of the largest number of splits it may pick.
size_t dw_wide_ws_bytes(int64_t M, int64_t K, int64_t N, int br) {
  const int64_t rows = ceil_div(M, br);
  int64_t s = rows < kWideMaxSplits ? rows : kWideMaxSplits;
  const int64_t s_min = ceil_div(rows, (int64_t)kWideMaxRows);
  if (s < s_min) s = s_min;
  return s > 1 ? (size_t)s * (size_t)K * (size_t)N * sizeof(float) : 0;
}

int launch_dw_wide(const DwJob &j, hipStream_t s) {
  return j.br == 32 ? wide_run<32>(j, s) : wide_run<64>(j, s);
}

int launch_dw_wide_batched(const DwJob *jobs, int n, hipStream_t s) {
  const int rc = wide_run_batched<32>(jobs, n, s);
  if (rc != BSR_OK) return rc;
  return wide_run_batched<64>(jobs, n, s);
}

}  // namespace bsr
