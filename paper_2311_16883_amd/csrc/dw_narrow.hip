// Weight gradient from a BSR activation (paper Sec. III, Fig. 2: dW = Xhat^T * dY)
// for bfloat16 inputs with small square blocks and a small weight matrix: blocks
// of b x b, b even and at most 16, at most 14 block-columns, N <= 224 -- the
// cross-patch linear layers of ResMLP (196 x 196 weights, 14 x 14 blocks over the
// patch axis).
//
// dW is small (at most 7 x 7 matrix-core tiles of 32 x 32) and the contraction
// is long, so one workgroup owns ALL of dW for a range of block-rows: every byte
// of the kept blocks and of dY is read exactly once, and the operator is bound
// by HBM.  With blocks narrower than a matrix-core tile nothing can be skipped
// at tile granularity; the kept blocks are laid out as a dense tile of the
// masked activation, zeros where a block was pruned, and multiplied as such.
//
//  * A stage is two block-rows.  In LDS a block-row is a group of 16 rows (b data
//    rows, the rest zero) = one contraction step of v_mfma_f32_32x32x16_bf16.  In
//    the activation group every block-column has a slot of 16 columns (32 bytes: a
//    matrix-core tile is two slots; the columns of a slot beyond b belong to no row
//    of dW and hold whatever follows the block's row in memory); rows are 576 bytes
//    apart: 448 of slots and padding that puts the four rows a transposing read
//    touches into different banks.  The dY group has its rows padded to the next of
//    64, 192, 320, 448 bytes for the same reason (with the 392-byte rows of memory,
//    45 % of the LDS cycles were bank conflicts).
//  * Both operands go from global memory to LDS through the texture path
//    (buffer_load ... lds), a ring of four stages deep, by four copy waves that do
//    nothing else, 16 bytes per lane.  LDS fills in lane order, and a lane fetches
//    the 16 bytes that belong where it writes: of dY, a piece of the block-row (one
//    contiguous piece of memory), or nothing in the padding of a row; of the
//    activation, half a slot = 16 bytes of one row of the kept block of that
//    block-column -- or nothing (an offset beyond the buffer, which makes the copy
//    write zeros) when the block was pruned or the row or column lies outside the
//    block or the matrix.  The range check is per dword, so a copy that reaches over
//    the end of the buffer delivers what is inside.  Every wave issues the same
//    number of copies per stage (9 or 8), so waiting for a stage is a constant vmcnt.
//  * A table in LDS, built once per workgroup, holds for every block-row of its
//    range the position of its first kept block and, per block-column, the rank of
//    that column among the kept ones of the row (or "pruned"): col_idx may be in any
//    order inside a block-row.
//  * Seven multiplying waves: wave p owns the tile columns 32 p .. 32 p + 31 of the
//    activation (the rows of dW of block-columns 2 p and 2 p + 1) and all columns of
//    dW (7 accumulator tiles), so a fragment of the activation is read once and a
//    fragment of dY once per wave.
//  * The block-rows are split over workgroups; partial matrices go to the workspace
//    and the split-K reduction kernel adds them in a fixed order.
#include "buffer_access.h"
#include "common.h"

namespace bsr {

namespace {

typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(16))) float v16f;

constexpr int kNT = 7;                     // tiles of 32 along K and along N: 224
constexpr int kMathWaves = 7;
constexpr int kCopyWaves = 4;
constexpr int kNarrowThreads = 64 * (kMathWaves + kCopyWaves);
constexpr int kSlots = 14;                 // block-columns of the activation tile: a slot of 16 columns (32 bytes) each
constexpr int kPitchA = 576;               // bytes per row of the activation tile: 448 of slots, and padding that puts rows 16 banks apart
constexpr int kGroupA = 16 * kPitchA;      // 9 KB: one block-row of the activation tile
constexpr int kGroupB = 8192;              // one block-row of dY: at most 16 rows x 448 bytes, copied 8 x 1 KB
constexpr int kStage = 2 * kGroupA + 2 * kGroupB;      // 34 KB
constexpr int kRing = 4;
constexpr int kAhead = kRing - 1;
constexpr int kNarrowMaxRows = 768;        // block-rows of one workgroup's range (its table lives in LDS)
constexpr int kRowPad = 8;                 // table rows behind the range's last that read as "all pruned"
constexpr int kNarrowMaxSplits = 128;
constexpr uint32_t kBeyond = 0xFFFF0000u;  // a byte offset no buffer reaches

struct NarrowParams {
  const int32_t *row_ptr, *col_idx;
  const void *values, *dY;
  float *out;              // dW, or the partial matrices [splits][K][N]
  int64_t K, N, ldo, split_stride;
  int32_t nbr, nbc, b, rows_per_split, splits, accumulate;
  uint32_t values_bytes, dy_bytes;
  uint32_t wg_begin;       // first workgroup of this product in a launch of several
};

// Global -> LDS copies.  LDS address = M0 + IMM + 16 * lane, global address = resource base + voff + IMM.
__device__ __forceinline__ void set_m0(uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" :: "s"(lds_addr) : "memory", "m0");
}
template <int IMM>
__device__ __forceinline__ void dma_dwordx4(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff) {
  asm volatile("buffer_load_dwordx4 %0, %1, 0 offen offset:%2 lds" :: "v"(voff), "s"(rsrc), "n"(IMM) : "memory", "m0");
}
__device__ __forceinline__ void stage_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// 16 contraction rows x 32 columns as the operand of one matrix instruction: two transposing
// reads of 4 rows x 16 columns per 16-lane group; `pitch` = bytes per row.
__device__ __forceinline__ v8bf read_fragment(const uint8_t *p, int pitch) {
  typedef v4s __attribute__((address_space(3))) * lds_v4s;
  const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p));
  const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(p + 4 * pitch));
  v8s r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return __builtin_bit_cast(v8bf, r);
}

// NS = strips of 32 columns of dW (ceil(N / 32)): a compile-time constant, so that the loop over a stage's
// matrix instructions has no branches and fragments are requested two instructions ahead of their use.
template <int NS>
__device__ __forceinline__ void narrow_body(const NarrowParams &prm, const uint32_t split) {
  __shared__ __attribute__((aligned(1024))) uint8_t sRing[kRing * kStage];
  __shared__ uint32_t sStart[kNarrowMaxRows + kRowPad];           // position of the block-row's first kept block
  __shared__ __attribute__((aligned(16))) uint8_t sRank[(kNarrowMaxRows + kRowPad) * 16];   // per block-column: rank among the kept, or 0xFF

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int b = prm.b, nbc = prm.nbc;
  const int i_begin = (int)split * prm.rows_per_split;
  int nrows = prm.nbr - i_begin;
  if (nrows > prm.rows_per_split) nrows = prm.rows_per_split;
  if (nrows < 0) nrows = 0;
  nrows = __builtin_amdgcn_readfirstlane(nrows);
  const int nstages = (nrows + 1) / 2;

  // ---- table (the ring's memory holds the range's column indices meanwhile) ----
  {
    const int32_t *__restrict__ row_ptr = prm.row_ptr;
    const int32_t *__restrict__ col_idx = prm.col_idx;
    int32_t *const sCols = reinterpret_cast<int32_t *>(sRing);
    const int32_t pos0 = nrows > 0 ? row_ptr[i_begin] : 0;
    const int32_t pos1 = nrows > 0 ? row_ptr[i_begin + nrows] : 0;
    int32_t ncols = pos1 - pos0;
    const bool in_lds = ncols >= 0 && ncols <= (int)(sizeof(sRing) / 4);
    if (in_lds)
      for (int e = t; e < ncols; e += kNarrowThreads) sCols[e] = col_idx[pos0 + e];
    __syncthreads();
    for (int rr = t; rr < nrows + kRowPad; rr += kNarrowThreads) {
      uint32_t rank[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
      uint32_t start = 0;
      if (rr < nrows) {
        const int32_t p0 = row_ptr[i_begin + rr];
        int32_t cnt = row_ptr[i_begin + rr + 1] - p0;
        if (cnt > nbc) cnt = nbc;                           // a valid row never holds more
        start = (uint32_t)p0;
        for (int e = 0; e < cnt; ++e) {
          const int j = in_lds ? sCols[p0 - pos0 + e] : col_idx[p0 + e];
          if (j >= 0 && j < 16) {
            const uint32_t sh = 8u * (uint32_t)(j & 3);
            rank[j >> 2] = (rank[j >> 2] & ~(0xFFu << sh)) | ((uint32_t)e << sh);
          }
        }
      }
      sStart[rr] = start;
      uint32_t *dst = reinterpret_cast<uint32_t *>(sRank + rr * 16);
      dst[0] = rank[0]; dst[1] = rank[1]; dst[2] = rank[2]; dst[3] = rank[3];
    }
    __syncthreads();            // the table is complete and the ring's memory is free again
  }
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)sRing;
  // Bytes per row of dY in memory, and in LDS: there the pitch is the next of 64, 192, 320, 448, so that the
  // four rows that a 16-lane group of a transposing read touches start 16 banks apart (as in the activation tile).
  const int pitch_mem = (int)prm.N * 2;
  const int pitch_b = 64 + 128 * ((pitch_mem + 63) / 128);

  if (wave >= kMathWaves) {
    // ================= copy waves =================
    // Copy wave c serves block-row g = c / 2 of every stage: of the nine 1 KB pieces of its activation
    // group the first five (c even) or the last four, and four of the eight 1 KB pieces of its dY group:
    // 9 or 8 copies per stage, always.
    const int c = wave - kMathWaves, g = c >> 1, rh = c & 1;
    const __amdgpu_buffer_rsrc_t rsrc_a = make_rsrc(prm.values, prm.values_bytes);
    const uint32_t block_bytes = (uint32_t)(b * b * 2), row_bytes = (uint32_t)(b * 2);
    constexpr uint32_t kDead = kBeyond + 4096u;
    // Activation tile: LDS fills in lane order, 16 bytes per lane.  The 16 bytes at byte o of the group
    // are row o / 576 of the tile and, inside the row, half h of the 32-byte slot of block-column j:
    // bytes 16 h .. 16 h + 15 of that row of block j -- fetched if the block is kept, else (and in the
    // padding of a tile row, in rows beyond the block, in block-columns beyond the matrix) nothing is
    // fetched and zeros are written.  The second half of a slot reaches beyond the 2 b bytes of the
    // block's row: what follows in memory lands in tile columns that belong to no row of dW.
    const int na = rh == 0 ? 5 : 4, ka0 = rh == 0 ? 0 : 5;
    uint32_t a_col[5], a_off[5];                            // block-column (0xFF: nothing to fetch), byte inside the block
#pragma unroll
    for (int k = 0; k < 5; ++k) {
      const uint32_t o = (uint32_t)(1024 * (ka0 + k) + 16 * lane);
      const uint32_t row = o / (uint32_t)kPitchA, cb = o - row * (uint32_t)kPitchA;
      const uint32_t j = cb >> 5, h = (cb >> 4) & 1u;
      const bool fetch = k < na && cb < 32u * kSlots && row < (uint32_t)b && j < (uint32_t)nbc && 16u * h < row_bytes;
      a_col[k] = fetch ? j : 0xFFu;
      a_off[k] = row * row_bytes + 16u * h;
    }
    const uint32_t group_bytes_b = (uint32_t)(b * pitch_mem);
    // dY: the wave's four copies of 1 KB fill LDS in lane order; the 16 bytes at byte o of the group in LDS are
    // row o / pitch_b, byte o % pitch_b of the block-row in memory -- or nothing, in the padding of a row.  (A
    // chunk may reach over the end of its row: into the padding go the first bytes of the next row, or zeros
    // at the end of the block-row, as the range check is per dword.)
    uint32_t lane_b[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t o = (uint32_t)(4096 * rh + 1024 * k + 16 * lane);
      const uint32_t row = o / (uint32_t)pitch_b, cb = o - row * (uint32_t)pitch_b;
      lane_b[k] = cb < (uint32_t)pitch_mem ? row * (uint32_t)pitch_mem + cb : kDead;
    }
    auto issue = [&](int q) {                               // the copies of stage q of the range
      const uint32_t slot = ring_lds + (uint32_t)((q & (kRing - 1)) * kStage);
      const int i = 2 * q + g;                              // block-row of the range (table rows beyond it: all pruned)
      const uint32_t start = sStart[i];
      const uint32_t group_a = slot + (uint32_t)(g * kGroupA + 1024 * ka0);
#pragma unroll
      for (int k = 0; k < 5; ++k) {
        if (k < na) {                                       // (wave-uniform)
          const uint32_t rk = a_col[k] < 16u ? (uint32_t)sRank[i * 16 + (int)a_col[k]] : 0xFFu;
          const uint32_t v = rk == 0xFFu ? kDead : (start + rk) * block_bytes + a_off[k];
          set_m0(group_a + 1024u * (uint32_t)k);
          dma_dwordx4<0>(rsrc_a, v);
        }
      }
      // this block-row of dY as a buffer of its own: what lies beyond it (or beyond the matrix) reads as zero
      const int64_t at = (int64_t)(i_begin + i) * group_bytes_b;
      int64_t left = i < nrows ? (int64_t)prm.dy_bytes - at : 0;
      if (left > group_bytes_b) left = group_bytes_b;
      if (left < 0) left = 0;
      const __amdgpu_buffer_rsrc_t rsrc_b = make_rsrc(static_cast<const char *>(prm.dY) + (left > 0 ? at : 0), (uint32_t)left);
      const uint32_t group_lds = slot + (uint32_t)(2 * kGroupA + g * kGroupB + 4 * rh * 1024);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        set_m0(group_lds + 1024u * (uint32_t)k);
        dma_dwordx4<0>(rsrc_b, lane_b[k]);
      }
    };
#pragma unroll
    for (int d = 0; d < kAhead; ++d) issue(d);
    for (int q = 0; q < nstages; ++q) {
      // the copies of stage q have landed when only those of the two stages after it are on their way
      if (rh == 0) asm volatile("s_waitcnt vmcnt(18)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
      stage_barrier();
      issue(q + kAhead);                                    // into the slot of stage q - 1, which everybody has left
    }
    // no copy may still be on its way when the workgroup gives its LDS back
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    return;
  }

  // ================= multiplying waves =================
  const int p = wave;                                       // tile columns 32 p .. 32 p + 31: the block-columns 2 p and 2 p + 1
  const int g4 = lane >> 4, L = lane & 15;
  const int frag_row = 8 * (g4 >> 1) + (L >> 2), frag_col = 16 * (g4 & 1) + 4 * (L & 3);
  const uint8_t *const myA = sRing + frag_row * kPitchA + (32 * p + frag_col) * 2;
  const uint8_t *const myB = sRing + 2 * kGroupA + frag_row * pitch_b + frag_col * 2;
  const bool active = 2 * p < nbc;
  v16f acc[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;
  for (int q = 0; q < nstages; ++q) {
    stage_barrier();              // everybody's copies of stage q have landed, and everybody is done with stage q - 1
    if (active) {
      const uint8_t *const pa = myA + (q & (kRing - 1)) * kStage;
      const uint8_t *const pb = myB + (q & (kRing - 1)) * kStage;
      // 2 NS matrix instructions: block-row g = idx / NS of the stage, strip idx % NS
      auto strip_fragment = [&](int idx) { return read_fragment(pb + (idx / NS) * kGroupB + (idx % NS) * 64, pitch_b); };
      v8bf a[2], bf[3];
      a[0] = read_fragment(pa, kPitchA);
      bf[0] = strip_fragment(0);
      if (NS > 0) bf[1] = strip_fragment(1);
      a[1] = read_fragment(pa + kGroupA, kPitchA);
#pragma unroll
      for (int idx = 0; idx < 2 * NS; ++idx) {
        if (idx + 2 < 2 * NS) bf[(idx + 2) % 3] = strip_fragment(idx + 2);
        acc[idx % NS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[idx / NS], bf[idx % 3], acc[idx % NS], 0, 0, 0);
      }
    }
  }
  if (!active) return;
  float *o = prm.out + (int64_t)split * prm.split_stride;
  const int64_t K = prm.K, N = prm.N, ldo = prm.ldo;
  const bool add = prm.accumulate != 0;
#pragma unroll
  for (int s = 0; s < NS; ++s) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      // tile column -> row of dW: column c of the slot of block-column j is row j b + c, for c < b
      const int tc = 32 * p + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      const int64_t k = (int64_t)(tc >> 4) * b + (tc & 15);
      const int64_t n = 32 * s + (lane & 31);
      if ((tc & 15) < b && k < K && n < N) {
        float *dst = o + k * ldo + n;
        *dst = add ? *dst + acc[s][r] : acc[s][r];
      }
    }
  }
}

constexpr int kNarrowBatchMax = 24;
struct NarrowBatch {
  NarrowParams it[kNarrowBatchMax];
};

// Workgroup w belongs to the product whose range of workgroups holds w, and is one split of it.  All products
// of a launch have the same number NS of 32-column strips.
template <int NS>
__global__ __launch_bounds__(kNarrowThreads) void dw_narrow_batched_kernel(NarrowBatch bt, int n) {
  int i = 0;
  while (i + 1 < n && blockIdx.x >= bt.it[i + 1].wg_begin) ++i;
  narrow_body<NS>(bt.it[i], blockIdx.x - bt.it[i].wg_begin);
}

void narrow_fill(const DwJob &j, int splits, NarrowParams *p) {
  const int64_t nbr = ceil_div(j.M, (int64_t)j.br), nbc = ceil_div(j.K, (int64_t)j.bc);
  const int64_t rps = nbr > 0 ? ceil_div(nbr, (int64_t)splits) : 1;
  const int eff = nbr > 0 ? (int)ceil_div(nbr, rps) : 1;
  p->row_ptr = j.row_ptr; p->col_idx = j.col_idx; p->values = j.values; p->dY = j.dY;
  p->out = eff > 1 ? static_cast<float *>(j.ws) : j.dW;
  p->K = j.K; p->N = j.N;
  p->ldo = eff > 1 ? j.N : j.lddw;
  p->split_stride = eff > 1 ? j.K * j.N : 0;
  p->nbr = (int32_t)nbr; p->nbc = (int32_t)nbc; p->b = j.br; p->rows_per_split = (int32_t)rps; p->splits = eff;
  p->accumulate = eff > 1 ? 0 : j.accumulate;
  p->values_bytes = (uint32_t)(nbr * nbc * j.br * j.bc * 2);
  p->dy_bytes = (uint32_t)(j.M * j.N * 2);
  p->wg_begin = 0;
}

}  // namespace

// Shapes the narrow-block kernel takes: bfloat16, square blocks of an even size up to 16, at most 14
// block-columns and 224 columns of dW, dY rows contiguous in memory with every block-row of dY
// starting on a 16-byte boundary, operands addressable with 32-bit byte offsets.
bool dw_narrow_supported(int dtype, int br, int bc, const void *values, const void *dY, int64_t M, int64_t K,
                         int64_t N, int64_t lddy) {
  if (dtype != BSR_BF16 || br != bc || br < 2 || br > 16 || (br & 1)) return false;
  if (M <= 0 || K <= 0 || N <= 0 || K > 32 * kNT || N > 32 * kNT || N % 4 != 0 || lddy != N) return false;
  if ((uintptr_t)values % 4 != 0 || (uintptr_t)dY % 16 != 0 || ((int64_t)br * N * 2) % 16 != 0) return false;
  const int64_t nbr = ceil_div(M, (int64_t)br), nbc = ceil_div(K, (int64_t)bc);
  if (nbc > kSlots) return false;
  if (nbr * nbc * br * bc * 2 >= (int64_t(1) << 32) - 2 * 65536) return false;
  if ((nbr + 2 * kRing) * br * N * 2 >= (int64_t(1) << 32) - 2 * 65536) return false;
  return nbr < (int64_t(1) << 30);
}

// Splits of the contraction: one round of workgroups on the 256 compute units for the whole
// launch (a workgroup takes most of a compute unit's LDS), at least two stages per workgroup.
static int narrow_splits(int64_t nbr, int products) {
  int64_t s = 256 / (products > 0 ? products : 1);
  if (s > kNarrowMaxSplits) s = kNarrowMaxSplits;
  if (s > nbr / 4) s = nbr / 4;
  const int64_t s_min = ceil_div(nbr, (int64_t)kNarrowMaxRows);
  if (s < s_min) s = s_min;
  return (int)(s < 1 ? 1 : s);
}

size_t dw_narrow_ws_bytes(int64_t M, int64_t K, int64_t N, int br) {
  const int64_t nbr = ceil_div(M, (int64_t)br);
  int64_t s = nbr / 4 < kNarrowMaxSplits ? nbr / 4 : kNarrowMaxSplits;
  const int64_t s_min = ceil_div(nbr, (int64_t)kNarrowMaxRows);
  if (s < s_min) s = s_min;
  return s > 1 ? (size_t)s * (size_t)K * (size_t)N * sizeof(float) : 0;
}

int launch_dw_narrow_batched(const DwJob *jobs, int n, hipStream_t s, std::vector<ReduceJob> *later) {
  // the products with the same number of 32-column strips share launches, kNarrowBatchMax per launch
  for (int ns = 1; ns <= kNT; ++ns) {
    int mine = 0;
    for (int i = 0; i < n; ++i)
      if (ceil_div(jobs[i].N, (int64_t)32) == ns) ++mine;
    int left = mine, at = 0;
    while (left > 0) {
      const int m = left < kNarrowBatchMax ? left : kNarrowBatchMax;
      NarrowBatch bt;
      ReduceJob red[kNarrowBatchMax];
      int nred = 0, k = 0;
      uint32_t total = 0;
      for (; at < n && k < m; ++at) {
        const DwJob &j = jobs[at];
        if (ceil_div(j.N, (int64_t)32) != ns) continue;
        const int64_t nbr = ceil_div(j.M, (int64_t)j.br);
        narrow_fill(j, narrow_splits(nbr, m), &bt.it[k]);
        const size_t need = bt.it[k].splits > 1 ? (size_t)bt.it[k].splits * j.K * j.N * sizeof(float) : 0;
        if (need > 0 && (j.ws == nullptr || j.ws_bytes < need)) return BSR_ERR_WORKSPACE;
        bt.it[k].wg_begin = total;
        total += (uint32_t)bt.it[k].splits;
        if (bt.it[k].splits > 1)
          red[nred++] = ReduceJob{bt.it[k].out, j.dW, j.K, j.N, j.lddw, bt.it[k].splits, j.accumulate};
        ++k;
      }
      const dim3 grid(total), block(kNarrowThreads);
      switch (ns) {
        case 1: hipLaunchKernelGGL(dw_narrow_batched_kernel<1>, grid, block, 0, s, bt, m); break;
        case 2: hipLaunchKernelGGL(dw_narrow_batched_kernel<2>, grid, block, 0, s, bt, m); break;
        case 3: hipLaunchKernelGGL(dw_narrow_batched_kernel<3>, grid, block, 0, s, bt, m); break;
        case 4: hipLaunchKernelGGL(dw_narrow_batched_kernel<4>, grid, block, 0, s, bt, m); break;
        case 5: hipLaunchKernelGGL(dw_narrow_batched_kernel<5>, grid, block, 0, s, bt, m); break;
        case 6: hipLaunchKernelGGL(dw_narrow_batched_kernel<6>, grid, block, 0, s, bt, m); break;
        default: hipLaunchKernelGGL(dw_narrow_batched_kernel<7>, grid, block, 0, s, bt, m); break;
      }
      int rc = check_launch();
      if (rc == BSR_OK && nred > 0) {
        if (later != nullptr) later->insert(later->end(), red, red + nred);
        else rc = launch_splitk_reduce_batched(red, nred, s);
      }
      if (rc != BSR_OK) return rc;
      left -= m;
    }
  }
  return BSR_OK;
}

}  // namespace bsr
