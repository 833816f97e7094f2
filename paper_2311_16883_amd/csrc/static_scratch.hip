// bsr_score_select_static: bsr_score_select for callers that cannot allocate
// (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  The workspace of the selection -- the block scores when the caller
// wants none, the bucket counts, the control block and the candidate list of the
// grid-wide passes -- lives in a device array of fixed size that is part of the
// library's code object, one copy per GPU, instead of a buffer of the caller.
#include <mutex>

#include "common.h"

namespace bsr {
namespace {

// Capacity: matrices of up to kStaticMaxBlocks blocks.  What the selection needs
// per block (8 B score, 8 B candidate key, 4 B candidate index) plus its fixed
// part (256 x 256 bucket counts, control block) and alignment slack.
constexpr int64_t kStaticMaxBlocks = int64_t(1) << 19;
constexpr size_t kScratchBytes = (size_t)kStaticMaxBlocks * 20 + 256 * 256 * 4 + 16 * 256;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of `scratch` on every GPU this process has used it on.  In host
// code the array's name is only a handle for hipGetSymbolAddress, never an address.
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of the array (resolved once per device).
int scratch_address(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { set_hip_error((int)e); return BSR_ERR_HIP; }
  if (dev < 0 || dev >= kMaxDevices) return BSR_ERR_SHAPE;
  std::lock_guard<std::mutex> guard(g_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      set_hip_error((int)e);
      return BSR_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return BSR_OK;
}

}  // namespace
}  // namespace bsr

using namespace bsr;

extern "C" {

int64_t bsr_score_select_static_max_blocks(void) { return kStaticMaxBlocks; }

int bsr_static_scratch_init(void) {
  void *p = nullptr;
  return scratch_address(&p);
}

int bsr_score_select_static(const void *X, int dtype, int64_t M, int64_t K, int64_t ldx, int br, int bc,
                            double keep, double *scores, uint8_t *keep_mask, void *stream) {
  // sizes first: an oversized problem is refused before anything touches the GPU
  if (dtype != BSR_F32 && dtype != BSR_BF16) return BSR_ERR_DTYPE;
  if (M < 0 || K < 0 || br < 1 || bc < 1) return BSR_ERR_SHAPE;
  const int64_t nbr = ceil_div(M, br), nbc = ceil_div(K, bc);
  if (nbr > kStaticMaxBlocks || nbc > kStaticMaxBlocks || nbr * nbc > kStaticMaxBlocks) return BSR_ERR_LIMIT;
  const size_t need = bsr_workspace_bytes(BSR_OP_SCORE_SELECT, M, K, 0, br, bc, dtype);
  if (need > kScratchBytes) return BSR_ERR_LIMIT;
  void *ws = nullptr;
  const int rc = scratch_address(&ws);
  if (rc != BSR_OK) return rc;
  return bsr_score_select(X, dtype, M, K, ldx, br, bc, keep, scores, keep_mask, ws, kScratchBytes, stream);
}

}  // extern "C"
