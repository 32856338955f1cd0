// Host side of the AdamW update: per-step scalars, argument checks, and the
// host-core update used for CPU-planned subgroups (Algorithm 1, cpu_update, with
// the FP32->16-bit downscale of Section 4.1 fused into the same pass).
//
// The host loop performs the same binary32 operations in the same order as the
// device kernel; the file is built with -ffp-contract=off and without fast-math,
// so the auto-vectorised code (IEEE divide and square root in every x86 vector
// width) is bit-identical to the device result.
#include <math.h>
#include <string.h>
#if defined(__x86_64__)
#include <immintrin.h>
#endif

#include <thread>
#include <vector>

#include "dos_internal.h"

namespace dos {

dos_status make_scalars(const dos_hparams* hp, AdamScalars* out) {
  if (!hp || !out) return DOS_EINVAL;
  const float lr = hp->lr, b1 = hp->beta1, b2 = hp->beta2, eps = hp->eps, wd = hp->weight_decay;
  const int opt = hp->optimizer;
  if (opt != DOS_OPT_ADAMW && opt != DOS_OPT_ADAGRAD && opt != DOS_OPT_RMSPROP) return DOS_EINVAL;
  if (hp->step < 1) return DOS_EINVAL;
  if (!isfinite(lr) || !isfinite(wd) || !isfinite(eps) || !(eps >= 0.0f)) return DOS_EINVAL;
  if (opt == DOS_OPT_ADAMW && !(b1 >= 0.0f && b1 < 1.0f)) return DOS_EINVAL;
  if (opt != DOS_OPT_ADAGRAD && !(b2 >= 0.0f && b2 < 1.0f)) return DOS_EINVAL;
  memset(out, 0, sizeof *out);
  out->opt = opt;
  out->eps = eps;
  out->decay = (float)(1.0 - (double)lr * (double)wd);
  if (opt == DOS_OPT_ADAMW) {
    const double t = (double)hp->step;
    const double bc1 = 1.0 - pow((double)b1, t);
    const double bc2 = 1.0 - pow((double)b2, t);
    out->beta1 = b1;
    out->beta2 = b2;
    out->omb1 = 1.0f - b1;
    out->omb2 = 1.0f - b2;
    out->step_size = (float)((double)lr / bc1);
    out->inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));
  } else {
    out->step_size = lr;  // no bias correction: the step index does not enter
    if (opt == DOS_OPT_RMSPROP) {
      out->beta2 = b2;
      out->omb2 = 1.0f - b2;
    }
  }
  return DOS_OK;
}

dos_status check_subgroup_pointers(const dos_subgroup* sg, bool needs_m) {
  if (!sg) return DOS_EINVAL;
  if (sg->n == 0) return DOS_OK;
  if (!sg->p || (needs_m && !sg->m) || !sg->v || !sg->g || !sg->p_lp) return DOS_EINVAL;
  const uintptr_t bits = (uintptr_t)sg->p | (needs_m ? (uintptr_t)sg->m : 0) | (uintptr_t)sg->v |
                         (uintptr_t)sg->g | (uintptr_t)sg->p_lp;
  if (bits & 15u) return DOS_EALIGN;
  return DOS_OK;
}

namespace {

inline uint16_t bf16_rne_host(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  const uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
  const uint32_t q = (u >> 16) | 0x0040u;
  return (uint16_t)(((u & 0x7FFFFFFFu) > 0x7F800000u) ? q : r);
}

// The loop the compiler vectorises.  Clones for wider vector units are picked at
// load time; all of them perform the same IEEE operations.  (Sanitizer builds
// define DOS_NO_TARGET_CLONES: the load-time resolver runs before their runtime
// is up.)
#ifndef DOS_NO_TARGET_CLONES
__attribute__((target_clones("avx512f", "avx2", "default")))
#endif
void adam_block(float* __restrict__ p, float* __restrict__ m, float* __restrict__ v,
                const uint16_t* __restrict__ g, uint16_t* __restrict__ p_lp, uint64_t n,
                const AdamScalars s) {
  for (uint64_t i = 0; i < n; ++i) {
    const uint32_t gb = (uint32_t)g[i] << 16;
    float gi;
    memcpy(&gi, &gb, 4);
    const float mt = s.beta1 * m[i] + s.omb1 * gi;
    const float vt = s.beta2 * v[i] + (s.omb2 * gi) * gi;
    const float d = sqrtf(vt) * s.inv_sqrt_bc2 + s.eps;
    const float pt = p[i] * s.decay - s.step_size * (mt / d);
    m[i] = mt;
    v[i] = vt;
    p[i] = pt;
    p_lp[i] = bf16_rne_host(pt);
  }
}

// Adagrad (RMS = false: v += g*g) and RMSProp (RMS = true: v = a*v + (1-a)*g*g) over
// p and v; same operation order as the device kernel.
template <bool RMS>
inline void accum_body(float* __restrict__ p, float* __restrict__ v, const uint16_t* __restrict__ g,
                       uint16_t* __restrict__ p_lp, uint64_t n, const AdamScalars s) {
  for (uint64_t i = 0; i < n; ++i) {
    const uint32_t gb = (uint32_t)g[i] << 16;
    float gi;
    memcpy(&gi, &gb, 4);
    const float vt = RMS ? s.beta2 * v[i] + (s.omb2 * gi) * gi : v[i] + gi * gi;
    const float d = sqrtf(vt) + s.eps;
    const float pt = p[i] * s.decay - s.step_size * (gi / d);
    v[i] = vt;
    p[i] = pt;
    p_lp[i] = bf16_rne_host(pt);
  }
}
#ifndef DOS_NO_TARGET_CLONES
__attribute__((target_clones("avx512f", "avx2", "default")))
#endif
void adagrad_block(float* __restrict__ p, float* __restrict__ v, const uint16_t* __restrict__ g,
                   uint16_t* __restrict__ p_lp, uint64_t n, const AdamScalars s) {
  accum_body<false>(p, v, g, p_lp, n, s);
}
#ifndef DOS_NO_TARGET_CLONES
__attribute__((target_clones("avx512f", "avx2", "default")))
#endif
void rmsprop_block(float* __restrict__ p, float* __restrict__ v, const uint16_t* __restrict__ g,
                   uint16_t* __restrict__ p_lp, uint64_t n, const AdamScalars s) {
  accum_body<true>(p, v, g, p_lp, n, s);
}

}  // namespace

namespace {

// Copies n 16-bit words from a small cache-resident buffer to memory that is written through the
// PCIe BAR, with non-temporal 32-byte stores where the destination allows: each is one full posted
// write instead of a cached store the core has to push out.
#if defined(__x86_64__)
__attribute__((target("avx2"))) void stream_copy_u16_avx2(uint16_t* dst, const uint16_t* src, uint64_t n) {
  uint64_t i = 0;
  while (i < n && ((uintptr_t)(dst + i) & 31u)) {  // head up to a 32-byte boundary
    dst[i] = src[i];
    ++i;
  }
  for (; i + 16 <= n; i += 16)
    _mm256_stream_si256(reinterpret_cast<__m256i*>(dst + i),
                        _mm256_loadu_si256(reinterpret_cast<const __m256i*>(src + i)));
  for (; i < n; ++i) dst[i] = src[i];
}
#endif

void stream_copy_u16(uint16_t* dst, const uint16_t* src, uint64_t n) {
#if defined(__x86_64__)
  static const bool avx2 = __builtin_cpu_supports("avx2");
  if (avx2) {
    stream_copy_u16_avx2(dst, src, n);
    return;
  }
#endif
  memcpy(dst, src, n * 2);
}

}  // namespace

void host_adam_range_streamed(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp_dev, uint64_t n,
                              const AdamScalars& s) {
  constexpr uint64_t kBlock = 2048;  // 4 KiB of 16-bit output: stays in the first-level cache
  alignas(64) uint16_t tmp[kBlock];
  for (uint64_t off = 0; off < n; off += kBlock) {
    const uint64_t cnt = n - off < kBlock ? n - off : kBlock;
    host_adam_range(p + off, m ? m + off : nullptr, v + off, g + off, tmp, cnt, s);
    stream_copy_u16(p_lp_dev + off, tmp, cnt);
  }
}

void store_fence() {
#if defined(__x86_64__) || defined(__i386__)
  __builtin_ia32_sfence();
#else
  __atomic_thread_fence(__ATOMIC_SEQ_CST);
#endif
}

void host_adam_range(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n,
                     const AdamScalars& s) {
  if (s.opt == DOS_OPT_ADAGRAD) adagrad_block(p, v, g, p_lp, n, s);
  else if (s.opt == DOS_OPT_RMSPROP) rmsprop_block(p, v, g, p_lp, n, s);
  else adam_block(p, m, v, g, p_lp, n, s);
}

}  // namespace dos

extern "C" dos_status dos_adam_step_host(const dos_subgroup* sg, const dos_hparams* hp, int32_t threads) {
  dos::AdamScalars s;
  dos_status rc = dos::make_scalars(hp, &s);
  if (rc != DOS_OK) return rc;
  rc = dos::check_subgroup_pointers(sg, s.opt == DOS_OPT_ADAMW);
  if (rc != DOS_OK) return rc;
  if (sg->n == 0) return DOS_OK;
  if (sg->state_loc == DOS_DEVICE || sg->grad_loc == DOS_DEVICE) return DOS_ESTATE;
  if (sg->state_loc < DOS_HOST_PINNED || sg->state_loc > DOS_HOST_PAGEABLE || sg->grad_loc < DOS_HOST_PINNED ||
      sg->grad_loc > DOS_HOST_PAGEABLE)
    return DOS_EINVAL;
  const uint64_t n = sg->n;
  int T = threads < 1 ? 1 : threads;
  const uint64_t min_per_thread = 1u << 16;
  if ((uint64_t)T > (n + min_per_thread - 1) / min_per_thread) T = (int)((n + min_per_thread - 1) / min_per_thread);
  if (T <= 1) {
    dos::host_adam_range(sg->p, sg->m, sg->v, sg->g, sg->p_lp, n, s);
    return DOS_OK;
  }
  float* const m = sg->m;  // NULL for the rules without a first moment: never offset
  // static split on 64-element boundaries
  const uint64_t per = (((n + T - 1) / T) + 63) & ~(uint64_t)63;
  // Slices that found no thread (the system refused one) are updated by the calling thread, so
  // the call always completes the whole subgroup and nothing leaves it as an exception.
  std::vector<std::thread> pool;
  int started = 0;
  try {
    pool.reserve(T);
    for (; started < T; ++started) {
      const uint64_t lo = (uint64_t)started * per;
      if (lo >= n) break;
      const uint64_t cnt = (lo + per <= n) ? per : n - lo;
      pool.emplace_back([=]() {
        dos::host_adam_range(sg->p + lo, m ? m + lo : nullptr, sg->v + lo, sg->g + lo, sg->p_lp + lo, cnt, s);
      });
    }
  } catch (...) {
  }
  for (int t = started; t < T; ++t) {
    const uint64_t lo = (uint64_t)t * per;
    if (lo >= n) break;
    const uint64_t cnt = (lo + per <= n) ? per : n - lo;
    dos::host_adam_range(sg->p + lo, m ? m + lo : nullptr, sg->v + lo, sg->g + lo, sg->p_lp + lo, cnt, s);
  }
  for (auto& th : pool) th.join();
  return DOS_OK;
}
