// Fused mixed-precision AdamW over one subgroup for gfx950 (MI355X).
//
// One pass over five arrays: FP32 p, m, v are read and rewritten in place, bf16
// gradients are read and the bf16 copy of the new parameters is written --
// 28 bytes of HBM traffic per element and nothing else (Section 4.1 of the
// paper stages p, m, v and the gradient on the device, Algorithm 1 updates them
// there and emits the 16-bit parameters; here the update and the downscale are
// one kernel).  The kernel is bound by HBM bandwidth: ~0.5 flop per byte, no
// reuse, so there is no LDS staging and no MFMA.  Every lane moves 16 bytes per
// FP32 access; a wave's accesses are contiguous; a block owns a contiguous tile
// so DRAM pages are opened once.  The same launch exists for Adagrad and RMSProp
// (Section 4.1 names them next to Adam): p and one accumulator, 20 bytes per
// element.  The default launch is the untiled one (adam_kernel_tile /
// accum_kernel_tile); the tiled layouts stay for launch-shape sweeps.
//
// Arithmetic: each operation is one IEEE binary32 operation (the file is built
// with -ffp-contract=off, correctly rounded divide and square root, denormals
// kept), in the order documented in dos.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>

#include "dos_internal.h"
#include "tile_access.h"

namespace dos {
namespace {

// Dynamic LDS requested per 64-thread block of the default launch, on a compute
// unit with 160 KiB of LDS (gfx950).  The kernel never touches it: 160 KiB /
// 14.5 KiB = 11 blocks per CU, i.e. about three waves per SIMD instead of the
// eight the register count would allow.  Measured on MI355X over 100M-parameter
// subgroups: 6.7 TB/s with 10-11 waves per CU, 6.05 with 32, 6.45 with 9, 4.1
// with 5 -- fewer waves keep fewer DRAM pages open at once, too few no longer
// cover the latency.  On a device that reports another LDS size per compute unit
// the request is scaled with it, so that the cap stays at the same number of waves.
constexpr int64_t kLdsPerCuAssumed = 160 * 1024;
constexpr int64_t kDefaultLdsThrottle = 14848;
// The two-array rules (Adagrad, RMSProp) move 20 instead of 28 bytes per element, so a
// wave holds less traffic and the best cap is higher: 15 waves per CU (6.7 TB/s; 6.6 with
// 11 or 17 waves).
constexpr int64_t kDefaultLdsThrottleTwoArrays = 10923;

// LDS per compute unit of the current device (queried once per device; the value gfx950
// has if the query fails).
int64_t lds_per_cu() {
  static std::atomic<int64_t> cache[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
    (void)hipGetLastError();
    return kLdsPerCuAssumed;
  }
  int64_t v = cache[dev].load(std::memory_order_relaxed);
  if (v == 0) {
    int bytes = 0;
    if (hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess ||
        bytes < 64 * 1024) {
      (void)hipGetLastError();
      bytes = (int)kLdsPerCuAssumed;
    }
    v = bytes;
    cache[dev].store(v, std::memory_order_relaxed);
  }
  return v;
}

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* ptr) {
  if constexpr (NT) return __builtin_nontemporal_load(ptr);
  else return *ptr;
}
// Stores of the layouts that address memory through plain pointers: plain or
// non-temporal.
template <int SP, typename T>
__device__ __forceinline__ void st(T* ptr, T val) {
  static_assert(SP == 0 || SP == 1, "system-scope store policies exist in the untiled layout only");
  if constexpr (SP == 1) __builtin_nontemporal_store(val, ptr);
  else *ptr = val;
}

// binary32 -> bf16 bit pattern, round to nearest even; NaN kept as quiet NaN.
__device__ __forceinline__ uint32_t bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
  return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? ((u >> 16) | 0x0040u) : r;
}

// One element; returns the bf16 bits of the new parameter.
__device__ __forceinline__ uint32_t adam_element(const AdamScalars& s, float& p, float& m, float& v,
                                                 uint32_t g_bits_hi) {
  const float g = __uint_as_float(g_bits_hi);  // bf16 in the upper half: exact widening
  const float mt = s.beta1 * m + s.omb1 * g;
  const float vt = s.beta2 * v + (s.omb2 * g) * g;
  const float d = __builtin_sqrtf(vt) * s.inv_sqrt_bc2 + s.eps;
  const float pt = p * s.decay - s.step_size * (mt / d);
  m = mt;
  v = vt;
  p = pt;
  return bf16_rne(pt);
}

// Adagrad (RMS = false: v += g*g) and RMSProp (RMS = true: v = a*v + (1-a)*g*g): one
// element of p and its accumulator v, no first moment; returns the bf16 bits of the
// new parameter.
template <bool RMS>
__device__ __forceinline__ uint32_t accum_element(const AdamScalars& s, float& p, float& v, uint32_t g_bits_hi) {
  const float g = __uint_as_float(g_bits_hi);
  const float vt = RMS ? s.beta2 * v + (s.omb2 * g) * g : v + g * g;
  const float d = __builtin_sqrtf(vt) + s.eps;
  const float pt = p * s.decay - s.step_size * (g / d);
  v = vt;
  p = pt;
  return bf16_rne(pt);
}

template <bool RMS>
__device__ __forceinline__ u32x2 accum_quad(const AdamScalars& s, f32x4& p, f32x4& v, u32x2 g) {
  float p0 = p.x, p1 = p.y, p2 = p.z, p3 = p.w;
  float v0 = v.x, v1 = v.y, v2 = v.z, v3 = v.w;
  const uint32_t b0 = accum_element<RMS>(s, p0, v0, g.x << 16);
  const uint32_t b1 = accum_element<RMS>(s, p1, v1, g.x & 0xFFFF0000u);
  const uint32_t b2 = accum_element<RMS>(s, p2, v2, g.y << 16);
  const uint32_t b3 = accum_element<RMS>(s, p3, v3, g.y & 0xFFFF0000u);
  p.x = p0; p.y = p1; p.z = p2; p.w = p3;
  v.x = v0; v.y = v1; v.z = v2; v.w = v3;
  u32x2 out;
  out.x = b0 | (b1 << 16);
  out.y = b2 | (b3 << 16);
  return out;
}

// Four consecutive elements held by one lane.
__device__ __forceinline__ u32x2 adam_quad(const AdamScalars& s, f32x4& p, f32x4& m, f32x4& v, u32x2 g) {
  float p0 = p.x, p1 = p.y, p2 = p.z, p3 = p.w;
  float m0 = m.x, m1 = m.y, m2 = m.z, m3 = m.w;
  float v0 = v.x, v1 = v.y, v2 = v.z, v3 = v.w;
  const uint32_t b0 = adam_element(s, p0, m0, v0, g.x << 16);
  const uint32_t b1 = adam_element(s, p1, m1, v1, g.x & 0xFFFF0000u);
  const uint32_t b2 = adam_element(s, p2, m2, v2, g.y << 16);
  const uint32_t b3 = adam_element(s, p3, m3, v3, g.y & 0xFFFF0000u);
  p.x = p0; p.y = p1; p.z = p2; p.w = p3;
  m.x = m0; m.y = m1; m.z = m2; m.w = m3;
  v.x = v0; v.y = v1; v.z = v2; v.w = v3;
  u32x2 out;
  out.x = b0 | (b1 << 16);
  out.y = b2 | (b3 << 16);
  return out;
}

// Elements [4*n_quads, n): at most three, handled by the first lanes of block 0.
__device__ __forceinline__ void adam_tail(float* p, float* m, float* v, const uint16_t* g,
                                          uint16_t* p_lp, uint64_t n_quads, uint64_t n,
                                          const AdamScalars& s) {
  const uint64_t i = n_quads * 4 + threadIdx.x;
  if (blockIdx.x == 0 && i < n) {
    float pi = p[i], mi = m[i], vi = v[i];
    const uint32_t b = adam_element(s, pi, mi, vi, (uint32_t)g[i] << 16);
    p[i] = pi; m[i] = mi; v[i] = vi;
    p_lp[i] = (uint16_t)b;
  }
}

// Layout A: a lane handles 4 consecutive elements per trip, TRIPS trips per tile,
// trips of one tile are blockDim.x*4 elements apart (every wave access is 1 KiB
// contiguous for FP32, 512 B for bf16).
template <int TRIPS, bool NTL, int NTS>
__global__ __launch_bounds__(512) void adam_kernel_quads(float* __restrict__ p, float* __restrict__ m,
                                                         float* __restrict__ v,
                                                         const uint16_t* __restrict__ g,
                                                         uint16_t* __restrict__ p_lp, uint64_t n,
                                                         AdamScalars s) {
  const uint64_t n_quads = n >> 2;
  const uint64_t tile = (uint64_t)blockDim.x * TRIPS;
  const uint64_t n_tiles = (n_quads + tile - 1) / tile;
  f32x4* __restrict__ p4 = reinterpret_cast<f32x4*>(p);
  f32x4* __restrict__ m4 = reinterpret_cast<f32x4*>(m);
  f32x4* __restrict__ v4 = reinterpret_cast<f32x4*>(v);
  const u32x2* __restrict__ g4 = reinterpret_cast<const u32x2*>(g);
  u32x2* __restrict__ o4 = reinterpret_cast<u32x2*>(p_lp);

  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const uint64_t base = t * tile + threadIdx.x;
    f32x4 P[TRIPS], M[TRIPS], V[TRIPS];
    u32x2 G[TRIPS];
#pragma unroll
    for (int k = 0; k < TRIPS; ++k) {
      const uint64_t q = base + (uint64_t)k * blockDim.x;
      if (q < n_quads) {
        G[k] = ld<NTL>(g4 + q);
        P[k] = ld<NTL>(p4 + q);
        M[k] = ld<NTL>(m4 + q);
        V[k] = ld<NTL>(v4 + q);
      }
    }
#pragma unroll
    for (int k = 0; k < TRIPS; ++k) {
      const uint64_t q = base + (uint64_t)k * blockDim.x;
      if (q < n_quads) {
        const u32x2 o = adam_quad(s, P[k], M[k], V[k], G[k]);
        st<NTS>(m4 + q, M[k]);
        st<NTS>(v4 + q, V[k]);
        st<NTS>(p4 + q, P[k]);
        st<NTS>(o4 + q, o);
      }
    }
  }
  adam_tail(p, m, v, g, p_lp, n_quads, n, s);
}

// Layout A without the tile loop: block b owns Q * blockDim quads, nothing else:
// lane l handles quads l, l + blockDim, ... of the tile, so every load or store
// instruction of a wave covers 1 KiB of whole lines (512 B for the 16-bit arrays)
// and the Q instructions for one array follow each other.  Q = 1 is the shortest
// possible wave: five descriptors, four loads, the update, four stores.
template <bool NTL, int NTS, int Q>
__global__ __launch_bounds__(512) void adam_kernel_tile(float* __restrict__ p, float* __restrict__ m,
                                                        float* __restrict__ v, const uint16_t* __restrict__ g,
                                                        uint16_t* __restrict__ p_lp, uint64_t n, AdamScalars s,
                                                        uint32_t xcd_shift) {
  const uint64_t whole = (n >> 2) << 2;                                // elements in whole quads
  // Blocks are handed to the 8 XCDs round-robin.  Natural mapping (xcd_shift = 32 or more): block b
  // owns tile b, so the XCDs interleave tile by tile.  Otherwise each XCD takes 2^xcd_shift
  // consecutive tiles at a time: dispatch slot seq of XCD x owns tile ((seq >> k) * 8 + x) << k | low
  // bits of seq (the grid is a multiple of 8 << k, tiles past the end are dropped by the range check).
  uint64_t t = blockIdx.x;
  if (xcd_shift < 32) {
    const uint64_t x = t & 7, seq = t >> 3;
    t = ((((seq >> xcd_shift) << 3) + x) << xcd_shift) | (seq & ((1ull << xcd_shift) - 1));
  }
  const uint64_t e0 = t * blockDim.x * (4 * Q);                        // first element of this tile
  const uint64_t left = whole > e0 ? whole - e0 : 0;                   // whole-quad elements from e0 on
  const __amdgpu_buffer_rsrc_t rp = tile_rsrc(p + e0, left * 4), rm = tile_rsrc(m + e0, left * 4),
                               rv = tile_rsrc(v + e0, left * 4), rg = tile_rsrc(g + e0, left * 2),
                               ro = tile_rsrc(p_lp + e0, left * 2);
  u32x2 G[Q], O[Q];
  f32x4 P[Q], M[Q], V[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) G[q] = buf_ld2<NTL>(rg, (q * blockDim.x + threadIdx.x) * 8);
#pragma unroll
  for (int q = 0; q < Q; ++q) P[q] = buf_ld4<NTL>(rp, (q * blockDim.x + threadIdx.x) * 16);
#pragma unroll
  for (int q = 0; q < Q; ++q) M[q] = buf_ld4<NTL>(rm, (q * blockDim.x + threadIdx.x) * 16);
#pragma unroll
  for (int q = 0; q < Q; ++q) V[q] = buf_ld4<NTL>(rv, (q * blockDim.x + threadIdx.x) * 16);
#pragma unroll
  for (int q = 0; q < Q; ++q) O[q] = adam_quad(s, P[q], M[q], V[q], G[q]);
#pragma unroll
  for (int q = 0; q < Q; ++q) buf_st4<NTS>(rm, (q * blockDim.x + threadIdx.x) * 16, M[q]);
#pragma unroll
  for (int q = 0; q < Q; ++q) buf_st4<NTS>(rv, (q * blockDim.x + threadIdx.x) * 16, V[q]);
#pragma unroll
  for (int q = 0; q < Q; ++q) buf_st4<NTS>(rp, (q * blockDim.x + threadIdx.x) * 16, P[q]);
#pragma unroll
  for (int q = 0; q < Q; ++q) buf_st2<NTS>(ro, (q * blockDim.x + threadIdx.x) * 8, O[q]);
  adam_tail(p, m, v, g, p_lp, n >> 2, n, s);
}

// The same launch for the rules that keep p and one accumulator (Adagrad, RMSProp):
// 20 bytes per element (reads 4+4+2, writes 4+4+2), the m array is never touched.
template <bool RMS, bool NTL, int NTS>
__global__ __launch_bounds__(512) void accum_kernel_tile(float* __restrict__ p, float* __restrict__ v,
                                                         const uint16_t* __restrict__ g,
                                                         uint16_t* __restrict__ p_lp, uint64_t n, AdamScalars s) {
  const uint64_t whole = (n >> 2) << 2;
  const uint64_t e0 = (uint64_t)blockIdx.x * blockDim.x * 4;
  const uint64_t left = whole > e0 ? whole - e0 : 0;
  const __amdgpu_buffer_rsrc_t rp = tile_rsrc(p + e0, left * 4), rv = tile_rsrc(v + e0, left * 4),
                               rg = tile_rsrc(g + e0, left * 2), ro = tile_rsrc(p_lp + e0, left * 2);
  const uint32_t off4 = threadIdx.x * 16, off2 = threadIdx.x * 8;
  const u32x2 G = buf_ld2<NTL>(rg, off2);
  f32x4 P = buf_ld4<NTL>(rp, off4);
  f32x4 V = buf_ld4<NTL>(rv, off4);
  const u32x2 o = accum_quad<RMS>(s, P, V, G);
  buf_st4<NTS>(rv, off4, V);
  buf_st4<NTS>(rp, off4, P);
  buf_st2<NTS>(ro, off2, o);
  // elements [whole, n): at most three, handled by the first lanes of block 0
  const uint64_t i = whole + threadIdx.x;
  if (blockIdx.x == 0 && i < n) {
    float pi = p[i], vi = v[i];
    const uint32_t b = accum_element<RMS>(s, pi, vi, (uint32_t)g[i] << 16);
    p[i] = pi; v[i] = vi;
    p_lp[i] = (uint16_t)b;
  }
}

// Layout B: a lane handles 8 consecutive elements per trip (two adjacent 16-byte
// FP32 accesses, one 16-byte bf16 access).
template <bool NTL, int NTS>
__global__ __launch_bounds__(512) void adam_kernel_octets(float* __restrict__ p, float* __restrict__ m,
                                                          float* __restrict__ v,
                                                          const uint16_t* __restrict__ g,
                                                          uint16_t* __restrict__ p_lp, uint64_t n,
                                                          AdamScalars s) {
  const uint64_t n_oct = n >> 3;
  f32x4* __restrict__ p4 = reinterpret_cast<f32x4*>(p);
  f32x4* __restrict__ m4 = reinterpret_cast<f32x4*>(m);
  f32x4* __restrict__ v4 = reinterpret_cast<f32x4*>(v);
  const u32x4* __restrict__ g8 = reinterpret_cast<const u32x4*>(g);
  u32x4* __restrict__ o8 = reinterpret_cast<u32x4*>(p_lp);
  const uint64_t n_tiles = (n_oct + blockDim.x - 1) / blockDim.x;
  for (uint64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
    const uint64_t q = t * blockDim.x + threadIdx.x;
    if (q < n_oct) {
      const u32x4 G = ld<NTL>(g8 + q);
      f32x4 P0 = ld<NTL>(p4 + 2 * q), P1 = ld<NTL>(p4 + 2 * q + 1);
      f32x4 M0 = ld<NTL>(m4 + 2 * q), M1 = ld<NTL>(m4 + 2 * q + 1);
      f32x4 V0 = ld<NTL>(v4 + 2 * q), V1 = ld<NTL>(v4 + 2 * q + 1);
      u32x2 ga, gb;
      ga.x = G.x; ga.y = G.y; gb.x = G.z; gb.y = G.w;
      const u32x2 oa = adam_quad(s, P0, M0, V0, ga);
      const u32x2 ob = adam_quad(s, P1, M1, V1, gb);
      u32x4 O;
      O.x = oa.x; O.y = oa.y; O.z = ob.x; O.w = ob.y;
      st<NTS>(m4 + 2 * q, M0); st<NTS>(m4 + 2 * q + 1, M1);
      st<NTS>(v4 + 2 * q, V0); st<NTS>(v4 + 2 * q + 1, V1);
      st<NTS>(p4 + 2 * q, P0); st<NTS>(p4 + 2 * q + 1, P1);
      st<NTS>(o8 + q, O);
    }
  }
  // elements [8*n_oct, n): at most seven, scalar, first lanes of block 0
  const uint64_t i = n_oct * 8 + threadIdx.x;
  if (blockIdx.x == 0 && i < n) {
    float pi = p[i], mi = m[i], vi = v[i];
    const uint32_t b = adam_element(s, pi, mi, vi, (uint32_t)g[i] << 16);
    p[i] = pi; m[i] = mi; v[i] = vi;
    p_lp[i] = (uint16_t)b;
  }
}

// Pull copy: lanes read 16 bytes each from (pinned, device-mapped) host memory
// and write them to device memory.  Used for the 16-bit parameter uploads of the
// host lane, which would otherwise queue behind the bulk prefetches on the DMA
// engine that serves the host-to-device direction.
__global__ __launch_bounds__(256) void pull_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                        uint64_t n_vec, uint16_t* __restrict__ dst16,
                                                        const uint16_t* __restrict__ src16, uint64_t n16) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride)
    dst[i] = __builtin_nontemporal_load(src + i);
  // trailing 16-bit words (fewer than 8)
  const uint64_t t = n_vec * 8 + threadIdx.x;
  if (blockIdx.x == 0 && t < n16) dst16[t] = src16[t];
}

template <bool NTL, int NTS>
dos_status launch_layout(int layout, dim3 grid, dim3 block, size_t lds, hipStream_t st_, float* p, float* m, float* v,
                         const uint16_t* g, uint16_t* lp, uint64_t n, const AdamScalars& s, uint32_t xcd_shift) {
  if (s.opt != DOS_OPT_ADAMW) {  // the accumulator rules exist in the one-quad untiled layout only
    if (layout != 4) return DOS_EINVAL;
    if (s.opt == DOS_OPT_RMSPROP)
      hipLaunchKernelGGL((accum_kernel_tile<true, NTL, NTS>), grid, block, lds, st_, p, v, g, lp, n, s);
    else
      hipLaunchKernelGGL((accum_kernel_tile<false, NTL, NTS>), grid, block, lds, st_, p, v, g, lp, n, s);
    return DOS_OK;
  }
  if (layout == 5) {
    hipLaunchKernelGGL((adam_kernel_tile<NTL, NTS, 2>), grid, block, lds, st_, p, m, v, g, lp, n, s, xcd_shift);
    return DOS_OK;
  }
  if (layout == 6) {
    hipLaunchKernelGGL((adam_kernel_tile<NTL, NTS, 4>), grid, block, lds, st_, p, m, v, g, lp, n, s, xcd_shift);
    return DOS_OK;
  }
  if constexpr (NTS >= 2) {  // system-scope stores exist in the untiled layouts only
    if (layout != 4) return DOS_EINVAL;
    hipLaunchKernelGGL((adam_kernel_tile<NTL, NTS, 1>), grid, block, lds, st_, p, m, v, g, lp, n, s, xcd_shift);
    return DOS_OK;
  } else {
  switch (layout) {
    case 0: hipLaunchKernelGGL((adam_kernel_quads<2, NTL, NTS>), grid, block, lds, st_, p, m, v, g, lp, n, s); break;
    case 1: hipLaunchKernelGGL((adam_kernel_quads<1, NTL, NTS>), grid, block, lds, st_, p, m, v, g, lp, n, s); break;
    case 2: hipLaunchKernelGGL((adam_kernel_quads<4, NTL, NTS>), grid, block, lds, st_, p, m, v, g, lp, n, s); break;
    case 3: hipLaunchKernelGGL((adam_kernel_octets<NTL, NTS>), grid, block, lds, st_, p, m, v, g, lp, n, s); break;
    case 4: hipLaunchKernelGGL((adam_kernel_tile<NTL, NTS, 1>), grid, block, lds, st_, p, m, v, g, lp, n, s, xcd_shift); break;
    default: return DOS_EINVAL;
  }
  return DOS_OK;
  }
}

}  // namespace

dos_status launch_adam(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n,
                       const AdamScalars& s, void* stream, const dos_launch_cfg* cfg) {
  if (n == 0) return DOS_OK;
  // Default shape (measured best on MI355X): one tile of 256 elements per one-wave
  // block, no tile loop, non-temporal loads, non-temporal system-scope stores (each
  // store instruction of a wave covers 1 KiB of whole cache lines, so writing through
  // loses nothing and measures 2.5 % faster), waves per CU capped through the LDS
  // request.
  int variant = cfg ? cfg->variant : 0x74;
  int threads = (cfg && cfg->block_threads) ? cfg->block_threads : 64;
  int64_t blocks = cfg ? cfg->grid_blocks : 0;
  // The kernel uses no LDS; a dynamic allocation only caps how many waves a CU holds.
  int64_t lds;
  if (cfg && cfg->lds_bytes) {
    lds = cfg->lds_bytes;
  } else {
    lds = s.opt == DOS_OPT_ADAMW ? kDefaultLdsThrottle : kDefaultLdsThrottleTwoArrays;
    const int64_t have = lds_per_cu();
    if (have != kLdsPerCuAssumed) lds = std::min<int64_t>(65536, lds * have / kLdsPerCuAssumed);
  }
  if (lds < 0) lds = 0;
  if (lds > 65536) return DOS_EINVAL;
  if (variant < 0 || threads < 64 || threads > 512 || (threads % 64) != 0 || blocks < 0) return DOS_EINVAL;
  const int layout = variant & 0xF;
  const bool ntl = (variant & 0x10) != 0;
  const int sp = (variant >> 5) & 3;  // 0 plain, 1 nt, 2 sc1 nt, 3 sc0 sc1 nt
  if (layout > 6 || (variant & ~0x7F)) return DOS_EINVAL;
  if (layout >= 4 && blocks != 0) return DOS_EINVAL;  // these layouts have no tile loop
  static const int trips_of[7] = {2, 1, 4, 1, 1, 2, 4};
  const uint64_t units = (layout == 3) ? (n >> 3) : (n >> 2);
  const uint64_t tile = (uint64_t)threads * trips_of[layout];
  uint64_t n_tiles = (units + tile - 1) / tile;
  if (n_tiles == 0) n_tiles = 1;  // tail only
  if (blocks == 0 || (uint64_t)blocks > n_tiles) blocks = (int64_t)n_tiles;
  if (blocks > 0x7FFFFFFF) {
    if (layout >= 4) return DOS_EINVAL;  // one block per tile: more tiles than a grid can hold
    blocks = 0x7FFFFFFF;                 // grid-stride covers the rest
  }
  // XCD-grouped tile order (untiled AdamW layout only): the grid becomes a multiple of 8 << k
  uint32_t xcd_shift = 32;
  if (cfg && cfg->xcd_group) {
    const int64_t grp = cfg->xcd_group;
    if (layout < 4 || s.opt != DOS_OPT_ADAMW || grp < 1 || grp > (1 << 20) || (grp & (grp - 1))) return DOS_EINVAL;
    xcd_shift = (uint32_t)__builtin_ctzll((unsigned long long)grp);
    const int64_t unit = 8 * grp;
    blocks = (blocks + unit - 1) / unit * unit;
    if (blocks > 0x7FFFFFFF) return DOS_EINVAL;
  }
  dim3 grid((unsigned)blocks), block((unsigned)threads);
  hipStream_t st_ = reinterpret_cast<hipStream_t>(stream);
  dos_status rc;
#define DOS_LAUNCH(L, S) \
  rc = launch_layout<L, S>(layout, grid, block, (size_t)lds, st_, p, m, v, g, p_lp, n, s, xcd_shift)
  switch ((ntl ? 4 : 0) | sp) {
    case 0: DOS_LAUNCH(false, 0); break;
    case 1: DOS_LAUNCH(false, 1); break;
    case 2: DOS_LAUNCH(false, 2); break;
    case 3: DOS_LAUNCH(false, 3); break;
    case 4: DOS_LAUNCH(true, 0); break;
    case 5: DOS_LAUNCH(true, 1); break;
    case 6: DOS_LAUNCH(true, 2); break;
    default: DOS_LAUNCH(true, 3); break;
  }
#undef DOS_LAUNCH
  if (rc != DOS_OK) return rc;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error((int)e, "launch of the fused AdamW kernel");
    return DOS_EHIP;
  }
  return DOS_OK;
}

dos_status launch_pull_copy_u16(uint16_t* dst_dev, const uint16_t* src_host, uint64_t n, void* stream) {
  if (n == 0) return DOS_OK;
  const uint64_t n_vec = n >> 3;
  uint64_t blocks = (n_vec + 255) / 256;
  if (blocks > 64) blocks = 64;  // a few CUs keep enough reads in flight for the host link
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(pull_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                     reinterpret_cast<u32x4*>(dst_dev), reinterpret_cast<const u32x4*>(src_host), n_vec, dst_dev,
                     src_host, n);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error((int)e, "launch of the upload copy kernel");
    return DOS_EHIP;
  }
  return DOS_OK;
}

}  // namespace dos
