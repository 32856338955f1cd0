// C-ABI entry points that need no context: the device-resident update, pinned
// host memory, and error text.
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <string.h>
#if defined(__linux__)
#include <sys/mman.h>
#endif

#include <atomic>
#include <thread>
#include <vector>

#include "dos_internal.h"

namespace dos {

static thread_local char g_hip_error[256] = "";

void note_hip_error(int code, const char* what) {
  snprintf(g_hip_error, sizeof g_hip_error, "%s: %s (%d)", what, hipGetErrorString((hipError_t)code), code);
}

}  // namespace dos

extern "C" {

dos_status dos_adam_step_cfg(const dos_subgroup* sg, const dos_hparams* hp, void* hip_stream,
                             const dos_launch_cfg* cfg) {
  dos::AdamScalars s;
  dos_status rc = dos::make_scalars(hp, &s);
  if (rc != DOS_OK) return rc;
  rc = dos::check_subgroup_pointers(sg, s.opt == DOS_OPT_ADAMW);
  if (rc != DOS_OK) return rc;
  if (sg->n == 0) return DOS_OK;
  if (sg->state_loc != DOS_DEVICE || sg->grad_loc != DOS_DEVICE) return DOS_ESTATE;
  return dos::launch_adam(sg->p, sg->m, sg->v, sg->g, sg->p_lp, sg->n, s, hip_stream, cfg);
}

dos_status dos_adam_step(const dos_subgroup* sg, const dos_hparams* hp, void* hip_stream) {
  return dos_adam_step_cfg(sg, hp, hip_stream, nullptr);
}

dos_status dos_device_large_bar(int32_t device, int32_t* yes) {
  if (!yes) return DOS_EINVAL;
  int v = 0;
  hipError_t e = hipDeviceGetAttribute(&v, hipDeviceAttributeIsLargeBar, device);
  if (e != hipSuccess) {
    dos::note_hip_error((int)e, "hipDeviceGetAttribute");
    (void)hipGetLastError();
    return DOS_EHIP;
  }
  *yes = v ? 1 : 0;
  return DOS_OK;
}

dos_status dos_pinned_alloc(void** out, uint64_t bytes) {
  if (!out || bytes == 0) return DOS_EINVAL;
  *out = nullptr;
  void* ptr = nullptr;
  hipError_t e = hipHostMalloc(&ptr, (size_t)bytes, hipHostMallocDefault);
  if (e != hipSuccess) {
    dos::note_hip_error((int)e, "hipHostMalloc");
    (void)hipGetLastError();
    return DOS_EHIP;
  }
  *out = ptr;
  return DOS_OK;
}

dos_status dos_pinned_free(void* ptr) {
  if (!ptr) return DOS_OK;
  hipError_t e = hipHostFree(ptr);
  if (e != hipSuccess) {
    dos::note_hip_error((int)e, "hipHostFree");
    (void)hipGetLastError();
    return DOS_EHIP;
  }
  return DOS_OK;
}

dos_status dos_host_advise_hugepages(void* ptr, uint64_t bytes) {
  if (!ptr && bytes) return DOS_EINVAL;
#if defined(__linux__) && defined(MADV_HUGEPAGE)
  const uintptr_t page = 4096;
  const uintptr_t lo = ((uintptr_t)ptr + page - 1) & ~(page - 1);
  const uintptr_t hi = ((uintptr_t)ptr + bytes) & ~(page - 1);
  if (hi > lo && madvise(reinterpret_cast<void*>(lo), hi - lo, MADV_HUGEPAGE) != 0) return DOS_ESTATE;
#endif
  return DOS_OK;
}

dos_status dos_host_prefault(void* ptr, uint64_t bytes, int32_t threads) {
  if (!ptr && bytes) return DOS_EINVAL;
  if (bytes == 0) return DOS_OK;
  int T = threads < 1 ? 1 : (threads > 256 ? 256 : threads);
  const uint64_t page = 4096;
  const uint64_t pages = (bytes + page - 1) / page;
  if ((uint64_t)T > pages) T = (int)pages;
  std::atomic<uint64_t> sink{0};
  volatile unsigned char* base = static_cast<volatile unsigned char*>(ptr);
  auto touch = [=, &sink](int t) {
    const uint64_t lo = pages * t / T, hi = pages * (t + 1) / T;
    uint64_t acc = 0;
    for (uint64_t pg = lo; pg < hi; ++pg) {
      const unsigned char b = base[pg * page];
      base[pg * page] = b;  // a write fault gives the page real memory, not the shared zero page
      acc += b;
    }
    sink.fetch_add(acc, std::memory_order_relaxed);
  };
  // shares that found no thread are touched by the calling thread: nothing leaves as an exception
  std::vector<std::thread> pool;
  int started = 0;
  try {
    pool.reserve(T);
    for (; started < T; ++started) pool.emplace_back(touch, started);
  } catch (...) {
  }
  for (int t = started; t < T; ++t) touch(t);
  for (auto& th : pool) th.join();
  return DOS_OK;
}

const char* dos_strerror(dos_status s) {
  switch (s) {
    case DOS_OK: return "ok";
    case DOS_EINVAL: return "invalid argument";
    case DOS_EALIGN: return "array not 16-byte aligned";
    case DOS_EBUDGET: return "GPU budget or staging memory too small";
    case DOS_EHIP: return "HIP call failed";
    case DOS_ESTATE: return "memory location does not fit the requested target";
    case DOS_ENOMEM: return "host memory or a thread could not be obtained";
  }
  return "unknown status";
}

const char* dos_last_hip_error(void) { return dos::g_hip_error; }

int32_t dos_version(void) { return 120; }

}  // extern "C"
