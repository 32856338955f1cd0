// Runs dos_run_update_phase on the CPU against the stand-in HIP runtime (see
// hip_stub/): the "device" kernels below are the library's own host update, so
// the result must equal dos_adam_step_host bit for bit.  Built by
// tests/test_sanitizers.py with phase.cpp, plan.cpp and adam_host.cpp under
// ASan/UBSan and under TSan (worker pool, upload ring, lane timers), and once more
// with -DDOS_COUNT_ALLOCS, where every heap allocation of the process is counted
// (operator new replaced here, malloc and friends wrapped by the linker) and the
// count must not move across dos_run_update_phase: the phase allocates nothing.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <random>
#include <vector>

#include "dos_internal.h"

#ifdef DOS_COUNT_ALLOCS
#include <atomic>
#include <new>
static std::atomic<long> g_allocs{0};
extern "C" {
void* __real_malloc(size_t);
void* __real_calloc(size_t, size_t);
void* __real_realloc(void*, size_t);
void* __real_aligned_alloc(size_t, size_t);
int __real_posix_memalign(void**, size_t, size_t);
void* __wrap_malloc(size_t n) { ++g_allocs; return __real_malloc(n); }
void* __wrap_calloc(size_t a, size_t b) { ++g_allocs; return __real_calloc(a, b); }
void* __wrap_realloc(void* q, size_t n) { ++g_allocs; return __real_realloc(q, n); }
void* __wrap_aligned_alloc(size_t a, size_t n) { ++g_allocs; return __real_aligned_alloc(a, n); }
int __wrap_posix_memalign(void** q, size_t a, size_t n) { ++g_allocs; return __real_posix_memalign(q, a, n); }
}
void* operator new(size_t n) {
  ++g_allocs;
  void* q = __real_malloc(n ? n : 1);
  if (!q) throw std::bad_alloc();
  return q;
}
void* operator new[](size_t n) { return operator new(n); }
void* operator new(size_t n, std::align_val_t a) {
  ++g_allocs;
  void* q = nullptr;
  if (__real_posix_memalign(&q, (size_t)a < sizeof(void*) ? sizeof(void*) : (size_t)a, n ? n : 1)) throw std::bad_alloc();
  return q;
}
void* operator new[](size_t n, std::align_val_t a) { return operator new(n, a); }
void operator delete(void* q) noexcept { free(q); }
void operator delete[](void* q) noexcept { free(q); }
void operator delete(void* q, size_t) noexcept { free(q); }
void operator delete[](void* q, size_t) noexcept { free(q); }
void operator delete(void* q, std::align_val_t) noexcept { free(q); }
void operator delete[](void* q, std::align_val_t) noexcept { free(q); }
void operator delete(void* q, size_t, std::align_val_t) noexcept { free(q); }
void operator delete[](void* q, size_t, std::align_val_t) noexcept { free(q); }
static long allocs_now() { return g_allocs.load(); }
#else
static long allocs_now() { return 0; }
#endif

namespace dos {
void note_hip_error(int, const char*) {}
dos_status launch_adam(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n,
                       const AdamScalars& s, void*, const dos_launch_cfg*) {
  host_adam_range(p, m, v, g, p_lp, n, s);
  return DOS_OK;
}
dos_status launch_pull_copy_u16(uint16_t* dst, const uint16_t* src, uint64_t n, void*) {
  memcpy(dst, src, n * 2);
  return DOS_OK;
}
}  // namespace dos

// (api.cpp, where the real one lives, is not part of this build)
extern "C" dos_status dos_host_advise_hugepages(void*, uint64_t) { return DOS_OK; }

static int fail(const char* what) {
  fprintf(stderr, "phase_driver: %s\n", what);
  return 1;
}

struct Arrays {
  std::vector<float*> p, m, v;
  std::vector<uint16_t*> g, lp;
};

static void* aligned(size_t bytes) {
  void* q = nullptr;
  if (posix_memalign(&q, 256, bytes ? bytes : 256)) abort();
  return q;
}

int main() {
  std::mt19937_64 rng(77);
  for (int it = 0; it < 40; ++it) {
    const int n_sg = 1 + (int)(rng() % 9);
    std::vector<uint64_t> sizes(n_sg);
    for (auto& s : sizes) s = (rng() % 5 == 0) ? rng() % 70 : rng() % 300000;
    const int n_slots = (int)(rng() % 4);                       // 0 = no staging at all
    const uint64_t slot_params = 64 * (1 + rng() % 2000);
    const bool slots_hold_grads = rng() % 2;
    const uint64_t chunk = 64 * (1 + rng() % 500);
    const int ring = 2 + (int)(rng() % 6);
    const int threads = 1 + (int)(rng() % 6);

    Arrays a, b;  // a: through the phase, b: straight through dos_adam_step_host
    std::vector<dos_subgroup> sgs(n_sg), ref(n_sg);
    std::vector<uint8_t> target(n_sg), resident(n_sg, 0);
    std::vector<int32_t> order(n_sg);
    for (int i = 0; i < n_sg; ++i) order[i] = i;
    std::shuffle(order.begin(), order.end(), rng);
    for (int i = 0; i < n_sg; ++i) {
      const uint64_t n = sizes[i];
      target[i] = (n_slots > 0) ? (uint8_t)(rng() % 2) : DOS_ON_CPU;
      const bool is_resident = target[i] == DOS_ON_GPU && rng() % 4 == 0;
      const bool grads_on_device = target[i] == DOS_ON_GPU && (is_resident || !slots_hold_grads || rng() % 2);
      for (Arrays* x : {&a, &b}) {
        x->p.push_back((float*)aligned(n * 4));
        x->m.push_back((float*)aligned(n * 4));
        x->v.push_back((float*)aligned(n * 4));
        x->g.push_back((uint16_t*)aligned(n * 2));
        x->lp.push_back((uint16_t*)aligned(n * 2));
      }
      for (uint64_t k = 0; k < n; ++k) {
        a.p[i][k] = b.p[i][k] = 0.01f * (float)((int)(rng() % 200) - 100);
        a.m[i][k] = b.m[i][k] = 0.0f;
        a.v[i][k] = b.v[i][k] = 0.0f;
        a.g[i][k] = b.g[i][k] = (uint16_t)(((rng() % 2) ? 0x3A00 : 0xBA00) + rng() % 256);
        a.lp[i][k] = b.lp[i][k] = 0;
      }
      sgs[i] = dos_subgroup{a.p[i], a.m[i], a.v[i], a.g[i], a.lp[i], n,
                            is_resident ? DOS_DEVICE : DOS_HOST_PINNED,
                            grads_on_device ? DOS_DEVICE : DOS_HOST_PINNED};
      ref[i] = dos_subgroup{b.p[i], b.m[i], b.v[i], b.g[i], b.lp[i], n, DOS_HOST_PINNED, DOS_HOST_PINNED};
    }
    const uint64_t bpp = slots_hold_grads ? 14 : 12;
    void* slot_mem = aligned((uint64_t)(n_slots ? n_slots : 1) * bpp * slot_params);
    void* stage = aligned((uint64_t)ring * chunk * 2);
    dos_ctx_config cfg{};
    cfg.slot_mem = n_slots ? slot_mem : nullptr;
    cfg.slot_bytes = (uint64_t)n_slots * bpp * slot_params;
    cfg.slot_params = slot_params;
    cfg.n_slots = n_slots;
    cfg.host_threads = threads;
    cfg.pinned_stage = stage;
    cfg.pinned_stage_bytes = (uint64_t)ring * chunk * 2;
    cfg.upload_chunk_params = chunk;
    cfg.flags = (it % 2) ? DOS_CTX_PROFILE : 0;
    if (it % 4 >= 2) {                       // direct uploads: no ring at all
      cfg.flags |= DOS_CTX_UPLOAD_DIRECT;
      if (it % 8 >= 4) {
        cfg.pinned_stage = nullptr;
        cfg.pinned_stage_bytes = 0;
      }
    }
    dos_ctx* ctx = nullptr;
    if (dos_ctx_create(&ctx, &cfg) != DOS_OK) return fail("dos_ctx_create failed");
    dos_plan plan{};
    plan.n_sg = n_sg;
    plan.n_slots = n_slots;
    plan.slot_params = slot_params;
    plan.target = target.data();
    plan.order = order.data();
    plan.resident = resident.data();
    for (int64_t step = 1; step <= 3; ++step) {
      // the rule rotates with the iteration: AdamW, Adagrad, RMSProp
      dos_hparams hp{1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, step, (int32_t)(it % 3)};
      dos_phase_stats st{};
      const long allocs_before = allocs_now();
      const dos_status rc = dos_run_update_phase(ctx, sgs.data(), n_sg, &plan, &hp, &st);
      if (allocs_now() != allocs_before) {
        fprintf(stderr, "%ld heap allocations inside dos_run_update_phase\n", allocs_now() - allocs_before);
        return fail("the update phase allocated host memory");
      }
      if (rc != DOS_OK) {
        fprintf(stderr, "status %d\n", (int)rc);
        return fail("dos_run_update_phase failed");
      }
      uint64_t total = 0;
      for (auto s : sizes) total += s;
      if (st.params_gpu + st.params_cpu + st.params_resident != total) return fail("stats do not add up");
      if (st.d2h_bytes != (it % 3 ? 8.0 : 12.0) * (double)st.params_gpu) return fail("flush bytes do not fit the rule");
      for (int i = 0; i < n_sg; ++i) {
        if (dos_adam_step_host(&ref[i], &hp, 1) != DOS_OK) return fail("dos_adam_step_host failed");
        const uint64_t n = sizes[i];
        if (memcmp(a.p[i], b.p[i], n * 4) || memcmp(a.m[i], b.m[i], n * 4) || memcmp(a.v[i], b.v[i], n * 4) ||
            memcmp(a.lp[i], b.lp[i], n * 2))
          return fail("phase result differs from the direct host update");
      }
    }
    // a plan the context cannot serve must be refused before anything is touched
    if (n_slots == 0 && n_sg > 0 && sizes[0] > 0) {
      std::vector<uint8_t> all_gpu(n_sg, DOS_ON_GPU);
      dos_plan bad = plan;
      bad.target = all_gpu.data();
      dos_hparams hp{1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 4};
      std::vector<float> before(a.p[0], a.p[0] + sizes[0]);
      if (dos_run_update_phase(ctx, sgs.data(), n_sg, &bad, &hp, nullptr) != DOS_EBUDGET)
        return fail("GPU plan without slots accepted");
      if (memcmp(before.data(), a.p[0], sizes[0] * 4)) return fail("state touched by a refused call");
    }
    dos_ctx_destroy(ctx);
    for (Arrays* x : {&a, &b})
      for (int i = 0; i < n_sg; ++i) {
        free(x->p[i]); free(x->m[i]); free(x->v[i]); free(x->g[i]); free(x->lp[i]);
      }
    free(slot_mem);
    free(stage);
  }
  // A phase with more pieces or chunks than the context reserved at creation (16384 and 65536) is
  // refused before anything is touched, instead of growing the work lists.
  {
    const uint64_t n = 64ull * 65537;  // 65537 chunks of 64; 16385 pieces of 256 would need n >= 4194560
    std::vector<float> p(n, 0.5f), m(n, 0.0f), v(n, 0.0f);
    std::vector<uint16_t> g(n, 0x3A00), lp(n, 0);
    void* slot_mem = aligned(2 * 14 * 64);
    void* stage = aligned(4 * 64 * 2);
    dos_ctx_config cfg{};
    cfg.slot_mem = slot_mem;
    cfg.slot_bytes = 2 * 14 * 64;
    cfg.slot_params = 64;
    cfg.n_slots = 2;
    cfg.host_threads = 2;
    cfg.pinned_stage = stage;
    cfg.pinned_stage_bytes = 4 * 64 * 2;
    cfg.upload_chunk_params = 64;
    dos_ctx* ctx = nullptr;
    if (dos_ctx_create(&ctx, &cfg) != DOS_OK) return fail("dos_ctx_create (small slots) failed");
    dos_subgroup sg{p.data(), m.data(), v.data(), g.data(), lp.data(), n, DOS_HOST_PINNED, DOS_HOST_PINNED};
    if (((uintptr_t)p.data() | (uintptr_t)m.data() | (uintptr_t)v.data() | (uintptr_t)g.data() | (uintptr_t)lp.data()) & 15)
      return fail("test arrays are not 16-byte aligned");
    uint8_t target = DOS_ON_CPU;
    int32_t order = 0;
    dos_plan plan{};
    plan.n_sg = 1;
    plan.n_slots = 2;
    plan.slot_params = 64;
    plan.target = &target;
    plan.order = &order;
    dos_hparams hp{1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 1, 0};
    if (dos_run_update_phase(ctx, &sg, 1, &plan, &hp, nullptr) != DOS_EBUDGET) return fail("65537 chunks accepted");
    target = DOS_ON_GPU;
    if (dos_run_update_phase(ctx, &sg, 1, &plan, &hp, nullptr) != DOS_EBUDGET) return fail("65537 pieces accepted");
    for (uint64_t k = 0; k < n; k += 4097)
      if (p[k] != 0.5f || m[k] != 0.0f || lp[k] != 0) return fail("state touched by a refused phase");
    // one element fewer per list limit is fine: 16384 pieces exactly
    sg.n = 64ull * 16384;
    if (dos_run_update_phase(ctx, &sg, 1, &plan, &hp, nullptr) != DOS_OK) return fail("16384 pieces refused");
    if (p[0] == 0.5f) return fail("accepted phase did nothing");
    dos_ctx_destroy(ctx);
    free(slot_mem);
    free(stage);
  }
  printf("phase_driver ok\n");
  return 0;
}
