// dW for block shapes the matrix-core kernel has no variant of (1 x b row segments
// -- the shape the paper's Table II overheads imply --, b = K whole-row pruning,
// rectangular or odd blocks): the BSR operand is re-tiled into 32x32 blocks in the
// workspace and the 32x32 kernel runs on that.
//
// A matrix-core instruction contracts 16 rows of a 32-column strip at once, so it
// can only skip work where all of those 16 x 32 positions are pruned; with row
// segments that practically never happens, and the arithmetic of the re-tiled
// operand (every 32x32 block present, pruned positions +0.0) is what any
// matrix-core formulation does.  What the BSR form still saves is the memory the
// activation occupies between forward and backward pass (paper Sec. III).
//
// reblock_kernel: a workgroup owns 32 matrix rows x a chunk of columns.  It zeroes
// an LDS tile, copies every stored block that intersects the tile into it (the
// entries of consecutive block-rows are consecutive in col_idx / values, so they
// are one index range), and writes the tile out as 32x32 blocks with their
// row_ptr / col_idx (all blocks present, columns ascending).
#include <climits>

#include "common.h"

namespace bsr {

namespace {

constexpr int kRbEntries = 2048;          // entries listed in LDS per round
constexpr int kRbTileBytes = 32768;       // LDS tile: 32 rows x chunk

// WORDS: blocks of at most 32 rows whose rows are whole 32-bit words.  The stored blocks
// of the tile's block-rows are one contiguous run of words in `values`; it is read
// linearly, eight loads in flight per thread, and every word finds its place in the
// tile from (entry, row, word) = decode(position).  Otherwise `group` lanes walk the
// part of each block that lies inside the tile, element by element.
template <typename T, bool WORDS>
__global__ __launch_bounds__(256) void reblock_kernel(
    const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx, const T *__restrict__ values,
    int64_t K, int br, int bc, int64_t nbr, int64_t nbr2, int64_t nbc2, int kc, int group, int ebatch,
    uint32_t magic_blk, uint32_t magic_seg, int32_t *__restrict__ rp2, int32_t *__restrict__ ci2,
    T *__restrict__ values2) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  T *tile = reinterpret_cast<T *>(smem);                                        // [32][kc]
  int32_t *erow = reinterpret_cast<int32_t *>(smem + (size_t)32 * kc * sizeof(T));   // tile row of an entry's first row
  int32_t *ecol = erow + kRbEntries;                                            // tile column of its first column
  __shared__ int32_t rp[34];
  const int t = threadIdx.x;
  const int64_t k0 = (int64_t)blockIdx.x * kc;
  const int gl = t & (group - 1), grp = t / group, ngrp = 256 / group;
  constexpr int kVec = 16 / (int)sizeof(T);                                     // elements per 16-byte vector
  for (int64_t I = blockIdx.y; I < nbr2; I += gridDim.y) {
    const int64_t m0 = I * 32;
    const int64_t i_first = m0 / br;
    int64_t i_last = (m0 + 31) / br;
    if (i_last > nbr - 1) i_last = nbr - 1;
    const int ni = (int)(i_last - i_first + 1);                                 // source block-rows: 1 .. 32
    if (t <= ni) rp[t] = row_ptr[i_first + t];
    uint4 *t4 = reinterpret_cast<uint4 *>(tile);
    for (int v = t; v < 32 * kc / kVec; v += 256) t4[v] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    const int64_t P0 = rp[0], P1 = rp[ni];
    for (int64_t pb = P0; pb < P1; pb += ebatch) {
      const int nb = (int)((P1 - pb) < ebatch ? (P1 - pb) : ebatch);
      for (int q = t; q < nb; q += 256) {
        const int64_t p = pb + q;
        int lo = 0, hi = ni - 1;                                                // last source block-row with rp <= p
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (p >= rp[mid]) lo = mid; else hi = mid - 1;
        }
        const int64_t j = col_idx[p];
        const int64_t c0 = j * bc - k0;
        erow[q] = (int32_t)((i_first + lo) * br - m0);                          // -br < . < 32
        ecol[q] = (j < 0 || c0 >= kc || c0 + bc <= 0) ? INT_MIN : (int32_t)c0;
      }
      __syncthreads();
      if (WORDS) {
        constexpr int kPerWord = 4 / (int)sizeof(T);
        const uint32_t seg_words = (uint32_t)bc / kPerWord, blk_words = (uint32_t)br * seg_words;
        const int kcw = kc / kPerWord;
        const uint32_t total = (uint32_t)nb * blk_words;                       // < 2^16 (ebatch)
        const uint32_t *vw = reinterpret_cast<const uint32_t *>(values) + pb * blk_words;
        uint32_t *tw = reinterpret_cast<uint32_t *>(tile);
        for (uint32_t w0 = 0; w0 < total; w0 += 8 * 256) {
          uint32_t reg[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const uint32_t w = w0 + t + 256 * k;
            reg[k] = w < total ? vw[w] : 0u;
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) {
            const uint32_t w = w0 + t + 256 * k;
            if (w < total) {
              const uint32_t q = span_div(w, blk_words, magic_blk), rem = w - q * blk_words;
              const uint32_t r = span_div(rem, seg_words, magic_seg), c = rem - r * seg_words;
              const int32_t ec = ecol[q];
              const int row = erow[q] + (int)r;
              const int col = ec / kPerWord + (int)c;                           // ec is a multiple of the word size
              if (ec != INT_MIN && row >= 0 && row < 32 && col >= 0 && col < kcw) tw[row * kcw + col] = reg[k];
            }
          }
        }
      } else
      // `group` lanes per entry: they walk the part of the block that lies inside the tile
      for (int q = grp; q < nb; q += ngrp) {
        const int32_t er = erow[q], ec = ecol[q];
        if (ec == INT_MIN) continue;
        const int rs0 = er < 0 ? -er : 0;
        const int rs1 = br < 32 - er ? br : 32 - er;
        const int cs0 = ec < 0 ? -ec : 0;
        const int cs1 = bc < kc - ec ? bc : kc - ec;
        const int nr = rs1 - rs0, ncol = cs1 - cs0;
        if (nr <= 0 || ncol <= 0) continue;
        const T *src = values + ((pb + q) * br + rs0) * (int64_t)bc + cs0;
        T *dst = tile + (er + rs0) * kc + ec + cs0;
        int r = gl / ncol, c = gl - r * ncol;
        while (r < nr) {
          dst[r * kc + c] = src[(int64_t)r * bc + c];
          c += group;
          while (c >= ncol) { c -= ncol; ++r; }
        }
      }
      __syncthreads();
    }
    // ---- the tile as 32x32 blocks ----
    const int jb = kc / 32;                                                     // blocks in the chunk
    const int64_t J0 = k0 / 32;
    constexpr int kVpb = 32 / kVec;                                             // vectors per block row
    for (int v = t; v < 32 * jb * kVpb; v += 256) {
      const int vv = v % kVpb, r = (v / kVpb) % 32, jl = v / (kVpb * 32);
      if (J0 + jl < nbc2) {
        const uint4 val = *reinterpret_cast<const uint4 *>(tile + r * kc + jl * 32 + vv * kVec);
        *reinterpret_cast<uint4 *>(values2 + (((I * nbc2 + J0 + jl) * 32 + r) * 32 + vv * kVec)) = val;
      }
    }
    if (blockIdx.x == 0) {
      for (int64_t J = t; J < nbc2; J += 256) ci2[I * nbc2 + J] = (int32_t)J;
      if (t == 0) {
        rp2[I] = (int32_t)(I * nbc2);
        if (I == nbr2 - 1) rp2[nbr2] = (int32_t)(nbr2 * nbc2);
      }
    }
    __syncthreads();
  }
  (void)K;
}

struct ReblockPlan {
  int64_t nbr2, nbc2;
  size_t values_off, rp_off, ci_off, inner_off, total;
};

ReblockPlan reblock_plan(int dtype, int64_t M, int64_t K, int64_t N) {
  ReblockPlan p;
  p.nbr2 = ceil_div(M, 32);
  p.nbc2 = ceil_div(K, 32);
  p.values_off = 0;
  p.rp_off = align_up((size_t)p.nbr2 * p.nbc2 * 1024 * elem_bytes(dtype), 256);
  p.ci_off = p.rp_off + align_up((size_t)(p.nbr2 + 1) * 4, 256);
  p.inner_off = p.ci_off + align_up((size_t)p.nbr2 * p.nbc2 * 4, 256);
  p.total = p.inner_off + align_up(dw_mfma_ws_bytes(dtype, M, K, N, 32, 32), 256);
  return p;
}

}  // namespace

bool dw_reblock_supported(int dtype, int br, int bc, int64_t M, int64_t K, int64_t N, int64_t lddy) {
  if (M <= 0 || K <= 0 || N <= 0) return false;
  if (ceil_div(M, 32) * ceil_div(K, 32) >= (int64_t(1) << 31)) return false;
  (void)br;
  (void)bc;
  return dw_mfma_supported(dtype, 32, 32, nullptr, M, K, N, lddy);
}

size_t dw_reblock_ws_bytes(int dtype, int64_t M, int64_t K, int64_t N) { return reblock_plan(dtype, M, K, N).total; }

int launch_dw_reblocked(int dtype, const int32_t *row_ptr, const int32_t *col_idx, const void *values, int64_t M,
                        int64_t K, int br, int bc, const void *dY, int64_t N, int64_t lddy, float *dW,
                        int64_t lddw, int accumulate, void *ws, size_t ws_bytes, hipStream_t s) {
  const ReblockPlan p = reblock_plan(dtype, M, K, N);
  if (ws_bytes < p.total) return BSR_ERR_WORKSPACE;
  char *w = static_cast<char *>(ws);
  int32_t *rp2 = reinterpret_cast<int32_t *>(w + p.rp_off);
  int32_t *ci2 = reinterpret_cast<int32_t *>(w + p.ci_off);
  const int e = elem_bytes(dtype);
  const int64_t k2 = p.nbc2 * 32;
  const int kc_max = kRbTileBytes / (32 * e);
  const int kc = (int)(k2 < kc_max ? k2 : kc_max);
  // lanes per stored block: about its area inside a tile, a power of two
  const int64_t area = (int64_t)(br < 32 ? br : 32) * (bc < kc ? bc : kc);
  int group = 1;
  while (group < 64 && group < area) group <<= 1;
  const int64_t nbr = ceil_div(M, br);
  const dim3 grid((unsigned)ceil_div(k2, kc), (unsigned)(p.nbr2 < 65535 ? p.nbr2 : 65535));
  const size_t lds = (size_t)32 * kc * e + 2 * (size_t)kRbEntries * 4;
  // word mode: rows of whole words, at most 32 rows, few column chunks (every chunk reads the whole run)
  const int64_t blk_words = (int64_t)br * bc * e / 4;
  const bool words = ((int64_t)bc * e) % 4 == 0 && br <= 32 && blk_words <= 4096 && grid.x <= 4 &&
                     (uintptr_t)values % 4 == 0;
  int ebatch = kRbEntries;
  uint32_t magic_blk = 0, magic_seg = 0;
  if (words) {
    if (ebatch > 65536 / blk_words) ebatch = (int)(65536 / blk_words);
    auto magic = [](uint32_t d) { return (uint32_t)(((uint64_t(1) << 32) + d - 1) / d); };
    magic_blk = magic((uint32_t)blk_words);
    magic_seg = magic((uint32_t)(bc * e / 4));
  }
#define BSR_REBLOCK(T, W)                                                                                   \
  hipLaunchKernelGGL((reblock_kernel<T, W>), grid, dim3(256), lds, s, row_ptr, col_idx,                     \
                     static_cast<const T *>(values), K, br, bc, nbr, p.nbr2, p.nbc2, kc, group, ebatch,     \
                     magic_blk, magic_seg, rp2, ci2, reinterpret_cast<T *>(w + p.values_off))
  if (dtype == BSR_F32) {
    if (words) BSR_REBLOCK(float, true); else BSR_REBLOCK(float, false);
  } else {
    if (words) BSR_REBLOCK(uint16_t, true); else BSR_REBLOCK(uint16_t, false);
  }
#undef BSR_REBLOCK
  const int rc = check_launch();
  if (rc != BSR_OK) return rc;
  return launch_dw_mfma(dtype, rp2, ci2, w + p.values_off, M, K, 32, 32, dY, N, lddy, dW, lddw, accumulate,
                        w + p.inner_off, ws_bytes - p.inner_off, s);
}

}  // namespace bsr
