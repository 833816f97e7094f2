// Weight gradient from a BSR activation (paper Sec. III, Fig. 2: dW = Xhat^T * dY)
// for bfloat16 inputs and 32x32 or 64x64 blocks, with workgroup tiles that span
// 384 rows of dW, so that every row of dY is read once per 384 columns of the
// activation (once in all for the 384-wide ResMLP inputs) and every kept block
// once per 128 output columns.
//
// What bounds this operator on gfx950 is not the matrix pipeline but everything
// around it.  Both operands have the contraction index as their slow axis, so every
// fragment of v_mfma_f32_32x32x16_bf16 comes out of LDS through two transposing
// reads (ds_read_b64_tr_b16, about 360 bytes per nanosecond and compute unit); a
// wave issues an instruction every six or seven cycles once scalar dependencies
// and taken branches are counted.  At 50 % kept blocks a stage of 32 contraction
// rows is 12 matrix instructions per SIMD, 384 cycles: a wave has a budget of a
// few dozen instructions per stage.  So:
//
//  * Sixteen waves in two roles.  Four copy waves (one per SIMD) move the stages
//    from global memory into LDS and nothing else; twelve multiplying waves, 3
//    (rows of dW) x 4 (columns), own 4 pieces of 32 rows x 1 strip of 32 columns
//    each, read fragments and issue matrix instructions and nothing else.
//  * Global -> LDS copies are done by the texture path itself (buffer_load ... lds,
//    16 bytes per lane): no staging registers, no LDS store instructions.  A copy
//    wave issues a pair of copies per stage for dY and one for each kept piece among
//    its three; a pruned piece is not copied (the texture path would spend as long on
//    a copy from beyond the buffer as on a real one).  The wave keeps count of what it
//    issued for the stages on their way, and waits for a stage with the vmcnt that
//    those counts add up to.
//  * LDS holds a ring of four stages of 32 contraction rows.  An activation piece
//    is a slab of 32 rows x 32 columns with 64-byte rows -- for 32x32 blocks 2 KB
//    of `values` exactly as stored -- where the four rows that a 16-lane group of a
//    transposing read touches are 256 consecutive bytes: no bank conflicts.  dY is
//    fetched in whole 128-byte lines, two strips side by side with 128-byte rows,
//    its 16-byte chunks permuted on the way in (by choosing which chunk a lane
//    fetches) so that its reads are conflict-free too.  One barrier per stage.
//  * Everything about the sparsity pattern is worked out before the loop: a table
//    in LDS holds, per block-row and block-column of the tile, the byte offset of
//    the kept block or an offset beyond the buffer, and per block-row the bits of
//    its kept pieces.  In the loop a copy costs a table read and two additions, a
//    multiplying wave's decision is a bit test and a branch, and a fragment of the
//    activation is read only for a kept block.  The table covers 480 block-rows;
//    longer contractions run in chunks, the accumulators carried across.
//  * The multiplying waves are software-pipelined across the barrier by half a
//    stage: the fragments of a wave's last two pieces are multiplied after the
//    next barrier, while the first reads of the next stage are on their way.
//  * Work is planned in rounds of 256 workgroups (one per compute unit: the ring
//    takes most of LDS).  With more tiles than compute units, as many products as
//    fill whole rounds are run tile by tile with no split of the contraction, and
//    the tiles left over are split just far enough to fill one more round; only
//    those go through partial tiles and the reduction kernel.
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
constexpr int kWideMaxRows = 480;      // block-rows of one split: 12 table words per block-row in LDS
constexpr int kRowPad = 12;            // table rows behind the split's last that read as "nothing kept"
constexpr int kWK = 3, kWN = 4;        // multiplying waves along the rows / columns of dW
constexpr int kMathWaves = kWK * kWN;  // 12: three per SIMD
constexpr int kCopyWaves = 4;          // one per SIMD
constexpr int kWideThreads = 64 * (kMathWaves + kCopyWaves);
constexpr int kPW = kPieces / kWK;     // pieces per multiplying wave: 4
constexpr int kFirst = 2;              // of which the fragments of the first two are requested first
constexpr int kAhead = kRing - 1;      // stages whose copies are on their way while one is multiplied
constexpr int kWideMaxSplits = 16;     // splits of the contraction the planner may pick (the workspace is sized for them)
constexpr uint32_t kBeyond = 0xFFFF0000u;          // a byte offset no buffer reaches (plus a per-lane part < 64 KB)

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
// 16 * l and at lds_addr + 1024 + 16 * l; the global side is voff_lo and voff_hi + 1024 (the
// instruction's immediate offset moves both sides).  Inline assembly, so that the compiler
// keeps no account of these copies: it would otherwise wait for all of them (vmcnt(0)) in
// front of the first LDS read that follows.  The waits are explicit.  (A scalar write of M0
// needs one wait state before an instruction that reads it.)
__device__ __forceinline__ void copy_pair_to_lds(__amdgpu_buffer_rsrc_t rsrc, uint32_t lds_addr, uint32_t voff_lo,
                                                 uint32_t voff_hi) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
               "buffer_load_dwordx4 %1, %3, 0 offen lds\n\t"
               "buffer_load_dwordx4 %2, %3, 0 offen offset:1024 lds"
               :: "s"(lds_addr), "v"(voff_lo), "v"(voff_hi), "s"(rsrc) : "memory", "m0");
}

// The compiler moves arithmetic on values it knows to be the same in all lanes to the scalar unit;
// this hides where a value came from, so that what is computed from it stays on the vector units.
__device__ __forceinline__ uint32_t vector_value(uint32_t x) {
  asm volatile("" : "+v"(x));
  return x;
}
// ... and this keeps a wave-uniform value in a scalar register as it is, so that every test of one
// of its bits is a bit test and a branch, not a mask made once and carried around.
__device__ __forceinline__ uint32_t scalar_value(uint32_t x) {
  asm volatile("" : "+s"(x));
  return x;
}

// The reads of LDS that precede it in program order have completed, then the workgroup barrier.
__device__ __forceinline__ void stage_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// 16 contraction rows x 32 columns out of a slab, as the operand of one matrix
// instruction: two transposing reads of 4 rows x 16 columns per 16-lane group.
template <int kRowPitch>
__device__ __forceinline__ v8bf read_fragment(const uint8_t *p) {
  typedef v4s __attribute__((address_space(3))) * lds_v4s;
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * kRowPitch));
  v8s r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return __builtin_bit_cast(v8bf, r);
}

// Activation fragments of part of a stage in registers: the kept pieces among NP of the wave's
// four, two contraction steps of 16 rows each.
template <int NP>
struct PartFrags {
  v8bf a0[NP], a1[NP];
  uint32_t mine;      // kept pieces (bit i = piece i of the part), wave-uniform
};
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
    // per block-row of the split and block-column of the tile: byte offset of the kept block in
    // `values`, or kBeyond; per block-row: the bits of its kept pieces
    __shared__ uint32_t sOff[(kWideMaxRows + kRowPad) * JT];
    __shared__ uint32_t sKept[kWideMaxRows + kRowPad];

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
    nrows = __builtin_amdgcn_readfirstlane(nrows);
    const int jfirst = tk * JT;
    int jt = prm.nbc - jfirst;
    if (jt > JT) jt = JT;
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)sRing;
    const bool copy_wave = wave >= kMathWaves;

    // ---- what a copy wave keeps across the chunks of the split ----
    // Copy wave c fills slabs c, c + 4, c + 8 (activation pieces) of every stage, 16 rows x 64 bytes
    // per copy (lane -> row lane / 4, 16-byte chunk lane % 4; 1 KB in LDS in lane order; the second
    // copy of a pair takes rows 16 .. 31 of the slab), and 16 rows of two strips of dY: four pairs
    // of copies per stage, always.
    const int c = wave - kMathWaves;
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(prm.values, prm.values_bytes);
    const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(prm.dY, prm.dy_bytes);
    const uint32_t a_hi_delta = 16u * kRowBytes - 1024u;
    const uint32_t b_hi_delta = (uint32_t)(8 * prm.lddy * 2) - 1024u;
    const uint32_t b_step = (uint32_t)(32 * prm.lddy * 2);
    // per-lane part of the offsets inside a block (pieces c, c + 4, c + 8 lie in the same half of
    // their 64-wide blocks)
    const uint32_t va = (uint32_t)(lane >> 2) * kRowBytes + (uint32_t)(lane & 3) * 16u + (SPB == 2 ? (uint32_t)(c & 1) * 64u : 0u);
    uint32_t m0_slot[kRing];
#pragma unroll
    for (int k = 0; k < kRing; ++k) m0_slot[k] = ring_lds + (uint32_t)(c * kSlabBytes + k * kStageBytes);
    // from the wave's first activation slab to its rows of the dY area (32 rows x 128 bytes per pair of strips)
    const uint32_t b_lds_delta = (uint32_t)((kPieces - c) * kSlabBytes + (c & 1) * 4096 + (c >> 1) * 2048);

    // ---- what a multiplying wave keeps ----
    const int wk = wave >> 2, wn = wave & 3;
    const int g4 = lane >> 4, L = lane & 15;
    const uint32_t frag_off = (uint32_t)((8 * (g4 >> 1) + (L >> 2)) * 64 + (16 * (g4 & 1) + 4 * (L & 3)) * 2);
    const uint8_t *const myA = sRing + (kPW * wk) * kSlabBytes + frag_off;
    const uint8_t *const myB = sRing + kPieces * kSlabBytes + (wn >> 1) * 4096 + (8 * (g4 >> 1) + (L >> 2)) * 128 +
                               (((wn & 1) * 4 + 2 * (g4 & 1) + ((L & 3) >> 1)) ^ (4 * ((L >> 3) & 1))) * 16 + 8 * (L & 1);
    v16f acc[kPW];
#pragma unroll
    for (int i = 0; i < kPW; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    // ---- tables: which block-columns of the tile every block-row of a chunk keeps, and where ----
    auto build_tables = [&](const int cbegin, const int crows) {
        // (built by the copy waves alone: the multiplying waves carry their accumulators through
        // here and have no registers to spare; they wait at the three barriers)
        constexpr int kTableThreads = 64 * kCopyWaves;
        const int t = c * 64 + lane;
        int32_t *const sPtr = reinterpret_cast<int32_t *>(sRing);                 // crows + 1 row pointers
        uint32_t *const sCols = reinterpret_cast<uint32_t *>(sRing + 16384);      // the chunk's column indices
        constexpr int kColsCap = (kRing * kStageBytes - 16384) / 4;
        for (int rr = t; rr <= crows; rr += kTableThreads) sPtr[rr] = row_ptr[cbegin + rr];
        __syncthreads();
        const int32_t pos0 = sPtr[0];
        const int32_t ncols = sPtr[crows] - pos0;
        const bool cols_in_lds = ncols >= 0 && ncols <= kColsCap;
        if (cols_in_lds)
          for (int e = t; e < ncols; e += kTableThreads) sCols[e] = (uint32_t)col_idx[pos0 + e];
        __syncthreads();
        for (int rr = t; rr < crows + kRowPad; rr += kTableThreads) {
          uint32_t off[JT];
#pragma unroll
          for (int jl = 0; jl < JT; ++jl) off[jl] = kBeyond;
          uint32_t mask = 0;
          if (rr < crows) {
            const int32_t p0 = sPtr[rr];
            int32_t p1 = sPtr[rr + 1];
            if (p1 - p0 > prm.nbc) p1 = p0 + prm.nbc;       // a valid row never holds more
            // eight entries at a time, so that their reads are on their way together
            for (int32_t p = p0; p < p1; p += 8) {
              int j[8];
#pragma unroll
              for (int u = 0; u < 8; ++u) {
                const int32_t q = p + u < p1 ? p + u : p1 - 1;
                j[u] = cols_in_lds ? (int)sCols[q - pos0] : (int)col_idx[q];
              }
#pragma unroll
              for (int u = 0; u < 8; ++u) {
                const uint32_t jl_kept = (uint32_t)(j[u] - jfirst);
                if (p + u < p1 && jl_kept < (uint32_t)jt) {
                  mask |= 1u << jl_kept;
#pragma unroll
                  for (int jl = 0; jl < JT; ++jl)
                    if ((uint32_t)jl == jl_kept) off[jl] = (uint32_t)(p + u) * kBlockBytes;
                }
              }
            }
          }
#pragma unroll
          for (int jl = 0; jl < JT; ++jl) sOff[rr * JT + jl] = off[jl];
          uint32_t pm = mask;                               // kept pieces from kept block-columns
          if (SPB == 2) {
            pm = 0;
#pragma unroll
            for (int jl = 0; jl < JT; ++jl) pm |= ((mask >> jl) & 1u) * (3u << (2 * jl));
          }
          sKept[rr] = pm;
        }
        __syncthreads();          // the tables are complete and the ring's memory is free again
    };
    // The block-rows of the split go in chunks whose tables fit LDS.  The two kinds of waves run
    // the same chunks and meet at the same barriers, each in code of its own.
    auto chunk_rows = [&](int r0) { return __builtin_amdgcn_readfirstlane(nrows - r0 < kWideMaxRows ? nrows - r0 : kWideMaxRows); };
    if (copy_wave) {
      for (int r0 = 0; r0 < nrows; r0 += kWideMaxRows) {
        const int crows = chunk_rows(r0), cbegin = i_begin + r0, nstages = crows * SPB;
        build_tables(cbegin, crows);
        // ================= copy waves =================
        // dY goes in whole 128-byte lines: a copy takes 8 rows x 64 columns (two strips side by
        // side); the 16-byte chunks of rows 2, 3, 6, 7 of a group are stored with bit 2 of their
        // position flipped, which keeps the transposing reads free of bank conflicts
        uint32_t vb;
        {
          const int64_t row = (int64_t)cbegin * BS + 16 * (c >> 1) + (lane >> 3);
          vb = (uint32_t)((row * prm.lddy + n0 + 64 * (c & 1)) * 2 + (((lane & 7) ^ (4 * ((lane >> 4) & 1))) * 16));
        }
        // table columns of the three pieces
        const uint32_t *offp[3] = {sOff + c / SPB, sOff + (c + 4) / SPB, sOff + (c + 8) / SPB};
        // Issues the copies of one stage and returns how many instructions that were: a pair for each
        // kept piece of the wave's three (a pruned piece is not copied at all: the texture path spends
        // as long on a copy from beyond the buffer as on a real one) and a pair for dY.
        auto issue = [&](uint32_t m0, uint32_t o0, uint32_t o1, uint32_t o2, bool lower_half) -> uint32_t {
          const uint32_t vh = va + ((SPB == 2 && lower_half) ? 32u * kRowBytes : 0u);
          uint32_t n = 2;
          if ((uint32_t)__builtin_amdgcn_readfirstlane((int)o0) != kBeyond) {
            const uint32_t l0 = o0 + vh;
            copy_pair_to_lds(rsrc_a, m0, l0, l0 + a_hi_delta);
            n += 2;
          }
          if ((uint32_t)__builtin_amdgcn_readfirstlane((int)o1) != kBeyond) {
            const uint32_t l1 = o1 + vh;
            copy_pair_to_lds(rsrc_a, m0 + 4u * kSlabBytes, l1, l1 + a_hi_delta);
            n += 2;
          }
          if ((uint32_t)__builtin_amdgcn_readfirstlane((int)o2) != kBeyond) {
            const uint32_t l2 = o2 + vh;
            copy_pair_to_lds(rsrc_a, m0 + 8u * kSlabBytes, l2, l2 + a_hi_delta);
            n += 2;
          }
          copy_pair_to_lds(rsrc_b, m0 + b_lds_delta, vb, vb + b_hi_delta);
          vb += b_step;
          return n;
        };
        // Waits until at most `allowed` of this wave's copies are on their way (allowed = 4, 6, .. 16: the
        // copies of the two stages behind the one that must have landed).
        auto wait_copies = [&](uint32_t allowed) {
          if (allowed >= 12u) {
            if (allowed >= 16u) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
            else if (allowed >= 14u) asm volatile("s_waitcnt vmcnt(14)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
          } else if (allowed >= 8u) {
            if (allowed >= 10u) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
          } else {
            if (allowed >= 6u) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
          }
        };
        uint32_t cnt[kAhead];                               // copies issued for the stages q .. q + 2
#pragma unroll
        for (int d = 0; d < kAhead; ++d)
          cnt[d] = issue(m0_slot[d], vector_value(offp[0][(d / SPB) * JT]), vector_value(offp[1][(d / SPB) * JT]),
                         vector_value(offp[2][(d / SPB) * JT]), (d & 1) != 0);
        uint32_t c1 = cnt[1], c2 = cnt[2];                  // of the stages q + 1 and q + 2
        // table entries are read one stage ahead of their use
        uint32_t n0_ = offp[0][(kAhead / SPB) * JT], n1_ = offp[1][(kAhead / SPB) * JT], n2_ = offp[2][(kAhead / SPB) * JT];
        auto stage = [&](auto slot_c) {
          constexpr int slot = decltype(slot_c)::value;                  // stage q = 4 * trip + slot
          constexpr int slot_new = (slot + kAhead) % kRing;              // stage q + 3 goes where stage q - 1 was
          // the copies of stage q have landed when only those of the two stages after it are on their way
          wait_copies(c1 + c2);
          stage_barrier();
          const uint32_t c3 = issue(m0_slot[slot_new], vector_value(n0_), vector_value(n1_), vector_value(n2_),
                                    ((slot + kAhead) & 1) != 0);
          c1 = c2;
          c2 = c3;
          n0_ = offp[0][((slot + kAhead + 1) / SPB) * JT];
          n1_ = offp[1][((slot + kAhead + 1) / SPB) * JT];
          n2_ = offp[2][((slot + kAhead + 1) / SPB) * JT];
        };
        const int trips = (nstages + kRing - 1) / kRing;
        for (int trip = 0; trip < trips; ++trip) {
          stage(std::integral_constant<int, 0>{});
          stage(std::integral_constant<int, 1>{});
          stage(std::integral_constant<int, 2>{});
          stage(std::integral_constant<int, 3>{});
#pragma unroll
          for (int u = 0; u < 3; ++u) offp[u] += (kRing / SPB) * JT;
        }
        // no copy may still be on its way when the ring is reused or the workgroup gives its LDS back
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();        // the ring and the tables are free for the next chunk
      }
      return;
    }
    for (int r0 = 0; r0 < nrows; r0 += kWideMaxRows) {
      const int crows = chunk_rows(r0), nstages = crows * SPB;
      __syncthreads();          // (the three barriers of the table build)
      __syncthreads();
      __syncthreads();
        // ================= multiplying waves =================
        // requests the activation fragments of pieces [first, first + NP) of the wave in ring slot `slot`
        auto load_part = [&](auto &f, int slot, auto first_c, uint32_t mine) {
          constexpr int first = decltype(first_c)::value;
          constexpr int NP = sizeof(f.a0) / sizeof(f.a0[0]);
          f.mine = mine;
          const uint8_t *bufA = myA + slot * kStageBytes + first * kSlabBytes;
          const uint32_t m = scalar_value(mine);
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            if (m & (1u << i)) {
              f.a0[i] = read_fragment<64>(bufA + i * kSlabBytes);
              f.a1[i] = read_fragment<64>(bufA + i * kSlabBytes + 1024);
            }
          }
        };
        auto load_strip = [&](StripFrags &f, int slot) {
          const uint8_t *bufB = myB + slot * kStageBytes;
          f.b0 = read_fragment<128>(bufB);
          f.b1 = read_fragment<128>(bufB + 2048);
        };
        // the multiplies of the part of a stage whose fragments are in registers
        auto multiply = [&](const auto &f, const StripFrags &b, auto first_c) {
          constexpr int first = decltype(first_c)::value;
          constexpr int NP = sizeof(f.a0) / sizeof(f.a0[0]);
          const uint32_t m = scalar_value(f.mine);
#pragma unroll
          for (int i = 0; i < NP; ++i) {
            if (m & (1u << i)) {
              acc[first + i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a0[i], b.b0, acc[first + i], 0, 0, 0);
              acc[first + i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a1[i], b.b1, acc[first + i], 0, 0, 0);
            }
          }
        };
        typedef std::integral_constant<int, 0> At0;
        typedef std::integral_constant<int, kFirst> AtRest;

        // ---- main loop, four stages per trip (ring slot = stage % 4 is then a constant).  Stages
        // beyond the chunk's last find "nothing kept" in the padded table rows.
        const uint32_t *kept = sKept;                 // of stage 4 * trip; advances once per trip
        PartFrags<kFirst> head;                       // pieces 0-1 of the wave
        PartFrags<kPW - kFirst> rest;                 // pieces 2-3
        StripFrags strip[2];                          // by stage parity
        head.mine = 0u;
        rest.mine = 0u;
        uint32_t kept_next = kept[0];                 // read one stage ahead of its use
        const uint32_t my_shift = (uint32_t)(kPW * wk);
        // One stage, software-pipelined across the barrier by part of a stage: after barrier q the
        // fragments of the first pieces of stage q are requested, then the last pieces of stage q - 1
        // are multiplied (their fragments were requested before the barrier), then the last pieces of
        // stage q are requested and the first ones multiplied.
        auto stage = [&](auto slot_c) {
          constexpr int slot = decltype(slot_c)::value;                  // stage q = 4 * trip + slot
          const uint32_t mine =
              (uint32_t)__builtin_amdgcn_readfirstlane((int)((vector_value(kept_next) >> my_shift) & ((1u << kPW) - 1u)));
          stage_barrier();               // everybody's copies of stage q have landed, and everybody has the fragments of stage q - 1
          kept_next = kept[(slot + 1) / SPB];
          StripFrags &bq = strip[slot & 1];
          const StripFrags &bprev = strip[(slot + 1) & 1];
          if (mine != 0u) load_strip(bq, slot);
          load_part(head, slot, At0{}, mine & ((1u << kFirst) - 1u));
          multiply(rest, bprev, AtRest{});
          load_part(rest, slot, AtRest{}, mine >> kFirst);
          multiply(head, bq, At0{});
        };
        const int trips = (nstages + kRing - 1) / kRing;
        for (int trip = 0; trip < trips; ++trip) {
          stage(std::integral_constant<int, 0>{});
          stage(std::integral_constant<int, 1>{});
          stage(std::integral_constant<int, 2>{});
          stage(std::integral_constant<int, 3>{});
          kept += kRing / SPB;
        }
        multiply(rest, strip[1], AtRest{});              // the last pieces of the last stage
      __syncthreads();        // the ring and the tables are free for the next chunk
    }

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

constexpr int kWideBatchMax = 24;
struct WideBatch {
  WideParams it[kWideBatchMax];
  // Two lists of work items: list 0 = the products [0, n0) of `it`, list 1 = the rest.  XCD x takes
  // the part [xcd_begin[l][x], xcd_begin[l][x + 1]) of list l, first its part of list 0.
  uint32_t xcd_begin[2][9];
  int32_t n0;
};

// Several products per launch: their work items form two lists (the products that are not
// split, then those that are), product after product, and every XCD takes a part of equal
// cost of each list (cut by the host).
template <int BS>
__global__ __launch_bounds__(kWideThreads) void dw_wide_batched_kernel(WideBatch b, int n) {
  const uint32_t x = blockIdx.x & 7u;
  uint32_t slot = blockIdx.x >> 3;
  const uint32_t mine0 = b.xcd_begin[0][x + 1] - b.xcd_begin[0][x];
  int i, last;
  uint32_t g;
  if (slot < mine0) {
    g = b.xcd_begin[0][x] + slot;
    i = 0;
    last = b.n0;
  } else {
    slot -= mine0;
    if (slot >= b.xcd_begin[1][x + 1] - b.xcd_begin[1][x]) return;
    g = b.xcd_begin[1][x] + slot;
    i = b.n0;
    last = n;
  }
  while (i + 1 < last && g >= b.it[i + 1].wg_begin) ++i;
  const WideParams &prm = b.it[i];
  const uint32_t item = g - prm.wg_begin;
  WideBody<BS>::run(prm, item);
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------

int64_t wide_tiles(int64_t K, int64_t N) { return ceil_div(K, kTileK) * ceil_div(N, kTileN); }

// The plan of one launch.  The products [0, whole) are not split: one workgroup runs all the
// block-rows of a tile and writes dW itself.  The others are split `splits` ways along the
// contraction, into partial tiles that a second kernel adds up.  With many tiles the first
// group fills the chip in whole rounds of 256 workgroups, and the second group's tiles are
// split just far enough that what is left over fills one more round.
struct WidePlan {
  int whole, splits;
};

// Cost model, in units of one stage: a workgroup costs its stages plus a fixed part (tables,
// first copies, write-out); work is done in rounds of 256 workgroups; a partial tile is
// written once and read once by the reduction.  Measured orders of magnitude on MI355X;
// only the choice depends on them.
WidePlan wide_plan(const int64_t *tiles, const int64_t *stages, const int64_t *rows, const double *bytes_out, int m) {
  const double us_stage = 0.5, fixed_stages = 30.0, bytes_per_us = 3.0e6;
  int64_t min_rows = rows[0];
  for (int i = 1; i < m; ++i) min_rows = rows[i] < min_rows ? rows[i] : min_rows;
  int64_t s_max = min_rows < kWideMaxSplits ? min_rows : kWideMaxSplits;
  if (s_max < 1) s_max = 1;
  WidePlan best{0, 1};
  double best_cost = 0;
  bool first = true;
  for (int w = 0; w <= m; ++w) {
    int64_t tiles_a = 0, tiles_b = 0, stages_a = 0, stages_b = 0;
    double bytes_b = 0;
    for (int i = 0; i < m; ++i) {
      if (i < w) { tiles_a += tiles[i]; stages_a = stages[i] > stages_a ? stages[i] : stages_a; }
      else { tiles_b += tiles[i]; stages_b = stages[i] > stages_b ? stages[i] : stages_b; bytes_b += bytes_out[i]; }
    }
    const double cost_a = (double)ceil_div(tiles_a, (int64_t)256) * ((double)stages_a + fixed_stages) * us_stage;
    for (int64_t s = 1; s <= (w == m ? 1 : s_max); ++s) {
      double cost = cost_a;
      if (w < m) {
        cost += (double)ceil_div(tiles_b * s, (int64_t)256) * ((double)ceil_div(stages_b, s) + fixed_stages) * us_stage;
        if (s > 1) cost += 2.0 * (double)s * bytes_b / bytes_per_us;
      }
      if (first || cost < best_cost) { best_cost = cost; best = WidePlan{w, (int)s}; first = false; }
    }
  }
  return best;
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

// Cuts the work items of the products [lo, hi) of a launch, in their order, into eight parts of
// equal cost, one per XCD; returns the most items any XCD got.
template <int BS>
uint32_t wide_cut(const WideBatch &b, int lo, int hi, uint32_t *begin) {
  int64_t cost[kWideBatchMax], all = 0;
  uint32_t first = 0, total = 0;
  for (int i = lo; i < hi; ++i) {
    cost[i] = (int64_t)b.it[i].rows_per_split * (BS / 32) + 30;
    const int64_t items = (int64_t)b.it[i].splits * b.it[i].tiles_k * b.it[i].tiles_n;
    all += cost[i] * items;
    if (i == lo) first = b.it[i].wg_begin;
    total = b.it[i].wg_begin + (uint32_t)items;
  }
  int x = 1;
  int64_t cum = 0;
  begin[0] = first;
  for (int i = lo; i < hi; ++i) {
    const int64_t items = (int64_t)b.it[i].splits * b.it[i].tiles_k * b.it[i].tiles_n;
    while (x < 8 && x * all <= 8 * (cum + items * cost[i])) {
      int64_t k = ceil_div(x * all - 8 * cum, 8 * cost[i]);
      if (k < 0) k = 0;
      if (k > items) k = items;
      begin[x++] = b.it[i].wg_begin + (uint32_t)k;
    }
    cum += items * cost[i];
  }
  while (x <= 8) begin[x++] = hi > lo ? total : first;
  uint32_t longest = 0;
  for (int q = 0; q < 8; ++q)
    if (begin[q + 1] - begin[q] > longest) longest = begin[q + 1] - begin[q];
  return longest;
}

// One launch of up to kWideBatchMax products of block size BS, and the reduction of those it splits.
template <int BS>
int wide_launch(const DwJob *const *jobs, int m, hipStream_t s, std::vector<ReduceJob> *later) {
  if (m <= 0) return BSR_OK;
  int64_t tiles[kWideBatchMax], stages[kWideBatchMax], rows[kWideBatchMax];
  double bytes_out[kWideBatchMax];
  for (int i = 0; i < m; ++i) {
    tiles[i] = wide_tiles(jobs[i]->K, jobs[i]->N);
    rows[i] = ceil_div(jobs[i]->M, (int64_t)BS);
    stages[i] = rows[i] * (BS / 32);
    bytes_out[i] = 4.0 * (double)jobs[i]->K * (double)jobs[i]->N;
  }
  const WidePlan plan = wide_plan(tiles, stages, rows, bytes_out, m);
  WideBatch b;
  ReduceJob red[kWideBatchMax];
  int nred = 0;
  uint32_t total = 0;
  for (int i = 0; i < m; ++i) {
    const DwJob &j = *jobs[i];
    if (i == plan.whole) total = 0;           // the second list counts its items from 0 again
    wide_fill<BS>(j, i < plan.whole ? 1 : plan.splits, &b.it[i]);
    const size_t need = b.it[i].splits > 1 ? (size_t)b.it[i].splits * j.K * j.N * sizeof(float) : 0;
    if (need > 0 && (j.ws == nullptr || j.ws_bytes < need)) return BSR_ERR_WORKSPACE;
    b.it[i].wg_begin = total;
    total += (uint32_t)(b.it[i].splits * b.it[i].tiles_k * b.it[i].tiles_n);
    if (b.it[i].splits > 1)
      red[nred++] = ReduceJob{b.it[i].out, j.dW, j.K, j.N, j.lddw, b.it[i].splits, j.accumulate};
  }
  b.n0 = plan.whole;
  const uint32_t longest = wide_cut<BS>(b, 0, plan.whole, b.xcd_begin[0]) + wide_cut<BS>(b, plan.whole, m, b.xcd_begin[1]);
  if (longest == 0) return BSR_OK;
  hipLaunchKernelGGL((dw_wide_batched_kernel<BS>), dim3(8 * longest), dim3(kWideThreads), 0, s, b, m);
  int rc = check_launch();
  if (rc == BSR_OK && nred > 0) {
    if (later != nullptr) later->insert(later->end(), red, red + nred);
    else rc = launch_splitk_reduce_batched(red, nred, s);
  }
  return rc;
}

template <int BS>
int wide_run_batched(const DwJob *jobs, int n, hipStream_t s, std::vector<ReduceJob> *later) {
  const DwJob *mine[kWideBatchMax];
  int m = 0;
  for (int i = 0; i < n; ++i) {
    if (jobs[i].br != BS) continue;
    mine[m++] = &jobs[i];
    if (m == kWideBatchMax) {
      const int rc = wide_launch<BS>(mine, m, s, later);
      if (rc != BSR_OK) return rc;
      m = 0;
    }
  }
  return wide_launch<BS>(mine, m, s, later);
}

}  // namespace

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
  if (nbr >= (int64_t(1) << 30) || nbc >= (int64_t(1) << 30)) return false;
  return true;
}

// Workspace of the wide kernel: partial tiles of the largest number of splits it may pick.
size_t dw_wide_ws_bytes(int64_t M, int64_t K, int64_t N, int br) {
  const int64_t rows = ceil_div(M, br);
  const int64_t s = rows < kWideMaxSplits ? rows : kWideMaxSplits;
  return s > 1 ? (size_t)s * (size_t)K * (size_t)N * sizeof(float) : 0;
}

int launch_dw_wide(const DwJob &j, hipStream_t s) {
  const DwJob *one = &j;
  return j.br == 32 ? wide_launch<32>(&one, 1, s, nullptr) : wide_launch<64>(&one, 1, s, nullptr);
}

int launch_dw_wide_batched(const DwJob *jobs, int n, hipStream_t s, std::vector<ReduceJob> *later) {
  const int rc = wide_run_batched<32>(jobs, n, s, later);
  if (rc != BSR_OK) return rc;
  return wide_run_batched<64>(jobs, n, s, later);
}

}  // namespace bsr
