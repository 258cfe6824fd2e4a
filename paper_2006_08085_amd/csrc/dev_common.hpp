// Device-side helpers shared by the kernels: state storage types and checks.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace detag {

// bfloat16 storage, handled as raw 16-bit patterns; arithmetic is always fp32.
struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float(uint32_t(v.bits) << 16); }

// Round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ uint16_t bf16_bits_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

template <typename ST>
__device__ __forceinline__ ST from_f32(float f);
template <>
__device__ __forceinline__ float from_f32<float>(float f) {
  return f;
}
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) {
  bf16_t r;
  r.bits = bf16_bits_rne(f);
  return r;
}

// Row-tile access through buffer resources.  A resource describes `bytes` valid
// bytes starting at a wavefront-uniform base (tile base + row * pitch); lanes
// address it with a 32-bit byte offset.  The base lives in scalar registers, so
// no per-row 64-bit vector addresses are built, and the hardware range check
// makes out-of-range lanes read zero and drop their stores: ragged tails need
// no branches.
using rsrc_t = __amdgpu_buffer_rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, int(bytes), 0x00020000);
}

// Row i of a tile: `valid` columns starting at column `tile` of row i.
template <typename E>
__device__ __forceinline__ rsrc_t row_of(const E *base, int64_t tile, int64_t ld, int i, uint32_t valid) {
  return make_rsrc(base + tile + int64_t(i) * ld, valid * uint32_t(sizeof(E)));
}

// Cache-policy bits of the buffer instructions on gfx950 (the `aux` operand):
// bit 0 = sc0, bit 1 = nt, bit 4 = sc1.  State tiles are touched exactly once
// per kernel, so they are streamed with nt (non-temporal).
constexpr int kAuxLoad = 2, kAuxStore = 2;

template <typename ST>
__device__ __forceinline__ float buf_load(rsrc_t r, uint32_t byte_off);
template <>
__device__ __forceinline__ float buf_load<float>(rsrc_t r, uint32_t byte_off) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, int(byte_off), 0, kAuxLoad));
}
template <>
__device__ __forceinline__ float buf_load<bf16_t>(rsrc_t r, uint32_t byte_off) {
  const uint16_t h = uint16_t(__builtin_amdgcn_raw_buffer_load_b16(r, int(byte_off), 0, kAuxLoad));
  return __uint_as_float(uint32_t(h) << 16);
}

template <typename ST>
__device__ __forceinline__ void buf_store(rsrc_t r, uint32_t byte_off, float v);
template <>
__device__ __forceinline__ void buf_store<float>(rsrc_t r, uint32_t byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), r, int(byte_off), 0, kAuxStore);
}
template <>
__device__ __forceinline__ void buf_store<bf16_t>(rsrc_t r, uint32_t byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b16(short(bf16_bits_rne(v)), r, int(byte_off), 0, kAuxStore);
}

// Hides a uniform pointer's value from the optimiser (it stays in scalar
// registers).  Used between the load and the store phase of a tile so the row
// bases are recomputed with a few scalar adds instead of being kept alive, one
// register pair per row, across the whole kernel.
template <typename P>
__device__ __forceinline__ P *launder_uniform(P *p) {
  asm volatile("" : "+s"(p));
  return p;
}

// Forces a value to exist in a vector register at this point of the program.
// Without it the compiler sinks "v = y + gn - go" below the code that does not
// use v yet and carries the three operands instead of the one result.
__device__ __forceinline__ void pin_vgpr(float &v) { asm volatile("" : "+v"(v)); }

inline int hip_rc(hipError_t e) { return static_cast<int>(e); }

inline int ceil_div_i64(int64_t a, int64_t b) { return static_cast<int>((a + b - 1) / b); }

}  // namespace detag
