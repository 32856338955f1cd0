// Host-side measurement aid of the benchmark (see dos_probe.h): a host-memory
// stream with the host update's access pattern.  Built into libdos_probe.so,
// never into libdos.so.
#include <string.h>
#if defined(__x86_64__)
#include <immintrin.h>
#endif

#include <atomic>
#include <chrono>
#include <thread>
#include <vector>

#include "dos_probe.h"

namespace {

// One block of the host stream: reads p, m, v, g, rewrites p, m, v, emits 16 bits
// per element.  The additions keep the compiler from dropping the store-back.
#if defined(__x86_64__)
__attribute__((target_clones("avx512f", "avx2", "default")))
#endif
void stream_block(float* __restrict__ p, float* __restrict__ m, float* __restrict__ v,
                  const uint16_t* __restrict__ g, uint16_t* __restrict__ out, uint64_t n) {
  for (uint64_t i = 0; i < n; ++i) {
    const uint32_t gb = (uint32_t)g[i] << 16;
    float gf;
    memcpy(&gf, &gb, 4);
    const float pt = p[i] + gf, mt = m[i] + gf, vt = v[i] + gf;
    p[i] = pt;
    m[i] = mt;
    v[i] = vt;
    uint32_t u;
    memcpy(&u, &pt, 4);
    out[i] = (uint16_t)(u >> 16);
  }
}

#if defined(__x86_64__)
__attribute__((target("avx2"))) void nt_copy_u16(uint16_t* dst, const uint16_t* src, uint64_t n) {
  uint64_t i = 0;
  while (i < n && ((uintptr_t)(dst + i) & 31u)) {
    dst[i] = src[i];
    ++i;
  }
  for (; i + 16 <= n; i += 16)
    _mm256_stream_si256(reinterpret_cast<__m256i*>(dst + i),
                        _mm256_loadu_si256(reinterpret_cast<const __m256i*>(src + i)));
  for (; i < n; ++i) dst[i] = src[i];
}
#endif

void copy_out(uint16_t* dst, const uint16_t* src, uint64_t n) {
#if defined(__x86_64__)
  static const bool avx2 = __builtin_cpu_supports("avx2");
  if (avx2) {
    nt_copy_u16(dst, src, n);
    return;
  }
#endif
  memcpy(dst, src, n * 2);
}

}  // namespace

extern "C" dos_status dos_probe_host_stream(float* p, float* m, float* v, const uint16_t* g, uint16_t* out16, uint64_t n,
                                 uint64_t out_n, int32_t threads, int32_t reps, int32_t streamed, double* seconds) {
  if (!p || !m || !v || !g || !out16 || !seconds || n == 0 || threads < 1 || threads > 1024 || reps < 1)
    return DOS_EINVAL;
  if (!streamed && out_n < n) return DOS_EINVAL;
  const int T = threads;
  constexpr uint64_t kChunk = (uint64_t)1 << 20;  // the threads take chunks from a shared counter, as the phase's workers do
  constexpr uint64_t kBlock = 2048;               // 4 KiB of output: stays in the first-level cache
  const uint64_t n_chunks = (n + kChunk - 1) / kChunk, total = n_chunks * (uint64_t)reps;
  const uint64_t window = (out_n / (uint64_t)T) & ~(uint64_t)(kBlock - 1);  // per thread, streamed output only
  if (streamed && window < 2 * kBlock) return DOS_EBUDGET;
  try {
    std::atomic<uint64_t> next{0};
    std::vector<std::thread> pool;
    pool.reserve(T);
    const auto t0 = std::chrono::steady_clock::now();
    for (int t = 0; t < T; ++t) {
      pool.emplace_back([&, t] {
        alignas(64) uint16_t tmp[kBlock];
        uint16_t* const win = out16 + (uint64_t)t * window;
        uint64_t wpos = 0;
        for (;;) {
          const uint64_t k = next.fetch_add(1, std::memory_order_relaxed);
          if (k >= total) break;
          const uint64_t lo = (k % n_chunks) * kChunk, cnt = kChunk < n - lo ? kChunk : n - lo;
          if (!streamed) {
            stream_block(p + lo, m + lo, v + lo, g + lo, out16 + lo, cnt);
            continue;
          }
          for (uint64_t off = 0; off < cnt; off += kBlock) {
            const uint64_t c = cnt - off < kBlock ? cnt - off : kBlock;
            stream_block(p + lo + off, m + lo + off, v + lo + off, g + lo + off, tmp, c);
            if (streamed == 1) {
              copy_out(win + wpos, tmp, c);
              wpos = wpos + 2 * kBlock <= window ? wpos + kBlock : 0;
            }
          }
        }
      });
    }
    for (auto& th : pool) th.join();
    *seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  } catch (...) {
    return DOS_EINVAL;
  }
  return DOS_OK;
}
