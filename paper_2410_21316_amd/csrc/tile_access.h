// Device-side helpers for kernels that address one tile of a flat array through
// a buffer descriptor (gfx950).  The cache policy of every access is an operand
// of the compiler's buffer builtins (bit 0 sc0, bit 1 nt, bit 4 sc1 on gfx950),
// so the compiler, not hand-written instructions, keeps the wait states and
// counters right; and the descriptor's size makes the hardware drop accesses
// past the end of what is left of the array, so a ragged last tile needs no
// branch (loads return 0, stores are discarded).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dos {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool NTL>
constexpr int load_aux() { return NTL ? 2 : 0; }
// Store policies: 0 plain, 1 non-temporal, 2 non-temporal at system scope without
// the wave-level bit (sc1 nt), 3 non-temporal at system scope (sc0 sc1 nt).
template <int SP>
constexpr int store_aux() { return SP == 0 ? 0 : SP == 1 ? 2 : SP == 2 ? 18 : 19; }

// Descriptor over `bytes` bytes starting at `base` (wave-uniform): raw buffer, no
// stride, 32-bit data format.  A tile is a few KiB, so clamping the size of what
// is left of an array to 32 bits never cuts into the tile.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const void* base, uint64_t bytes) {
  const uint32_t rec = bytes > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)bytes;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)rec, 0x00020000);
}
template <bool NTL>
__device__ __forceinline__ f32x4 buf_ld4(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, load_aux<NTL>()));
}
template <bool NTL>
__device__ __forceinline__ u32x2 buf_ld2(__amdgpu_buffer_rsrc_t r, uint32_t off) {
  return __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, load_aux<NTL>());
}
template <int SP>
__device__ __forceinline__ void buf_st4(__amdgpu_buffer_rsrc_t r, uint32_t off, f32x4 val) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, val), r, (int)off, 0, store_aux<SP>());
}
template <int SP>
__device__ __forceinline__ void buf_st2(__amdgpu_buffer_rsrc_t r, uint32_t off, u32x2 val) {
  __builtin_amdgcn_raw_buffer_store_b64(val, r, (int)off, 0, store_aux<SP>());
}

}  // namespace dos
