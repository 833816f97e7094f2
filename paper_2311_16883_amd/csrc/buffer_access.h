// Raw buffer loads / stores (device code only): accesses through a buffer
// resource are range-checked by the hardware, which predicates them without a
// branch, and take a wave-uniform offset from a scalar register next to the
// per-lane one.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bsr {

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

// Byte store at base + off + soff; out-of-range lanes store nothing.
__device__ __forceinline__ void buffer_store_u8(__amdgpu_buffer_rsrc_t r, uint32_t off, uint32_t soff, uint8_t v) {
  __builtin_amdgcn_raw_buffer_store_b8(v, r, off, soff, 0);
}

}  // namespace bsr
