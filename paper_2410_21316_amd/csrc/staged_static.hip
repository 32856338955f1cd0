// dos_gpu_update_staged: the GPU lane of the update phase for one host-resident
// subgroup -- prefetch, fused update, flush (Algorithm 1: prefetch_in, gpu_update,
// flush_out) -- through a staging buffer that is part of the library's own code
// object instead of memory the caller hands in.  For callers that cannot
// allocate: nothing here calls hipMalloc, hipFree or any allocating routine.
//
// The staging buffer is a file-scope device array.  In host code its name is a
// stand-in, not a device address: the address is asked for once per device with
// hipGetSymbolAddress and kept, and only that pointer is ever given to copies and
// kernels.  Every GPU holds its own copy of the array from the moment the code
// object is loaded there until the process ends.
#include <hip/hip_runtime.h>

#include <mutex>

#include "dos_internal.h"

namespace {

constexpr uint64_t kMaxParams = DOS_STAGED_MAX_PARAMS;
// p | m | v (FP32) | g (16-bit), each kMaxParams elements
constexpr uint64_t kScratchBytes = 14 * kMaxParams;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once known

// Device address of the calling thread's current device's copy of the array.
dos_status scratch_address(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    dos::note_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidDevice), "hipGetDevice");
    (void)hipGetLastError();
    return DOS_EHIP;
  }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      dos::note_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidSymbol), "hipGetSymbolAddress of the staging array");
      (void)hipGetLastError();
      return DOS_EHIP;
    }
    g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return DOS_OK;
}

#define STAGED_TRY(call, what)              \
  do {                                      \
    hipError_t e_ = (call);                 \
    if (e_ != hipSuccess) {                 \
      dos::note_hip_error((int)e_, what);   \
      (void)hipGetLastError();              \
      return DOS_EHIP;                      \
    }                                       \
  } while (0)

}  // namespace

extern "C" dos_status dos_gpu_update_staged(const dos_subgroup* sg, const dos_hparams* hp, void* hip_stream) {
  dos::AdamScalars sc;
  dos_status rc = dos::make_scalars(hp, &sc);
  if (rc != DOS_OK) return rc;
  const bool needs_m = sc.opt == DOS_OPT_ADAMW;
  rc = dos::check_subgroup_pointers(sg, needs_m);
  if (rc != DOS_OK) return rc;
  if (sg->n == 0) return DOS_OK;
  if (sg->state_loc != DOS_HOST_PINNED) return DOS_ESTATE;
  if (sg->grad_loc != DOS_HOST_PINNED && sg->grad_loc != DOS_DEVICE) return DOS_ESTATE;
  if (sg->n > kMaxParams) return DOS_EBUDGET;  // larger than the library's staging array

  unsigned char* base = nullptr;
  if ((rc = scratch_address(&base)) != DOS_OK) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  float* const sp = reinterpret_cast<float*>(base);
  float* const sm = reinterpret_cast<float*>(base + 4 * kMaxParams);
  float* const sv = reinterpret_cast<float*>(base + 8 * kMaxParams);
  uint16_t* const sgr = reinterpret_cast<uint16_t*>(base + 12 * kMaxParams);
  const size_t fb = (size_t)sg->n * 4;

  // Everything is ordered by the one stream: prefetch, update, flush.  The copies fill exactly
  // the elements the kernel reads, so nothing of an earlier call's contents is ever looked at.
  STAGED_TRY(hipMemcpyAsync(sp, sg->p, fb, hipMemcpyHostToDevice, st), "prefetch of p");
  if (needs_m) STAGED_TRY(hipMemcpyAsync(sm, sg->m, fb, hipMemcpyHostToDevice, st), "prefetch of m");
  STAGED_TRY(hipMemcpyAsync(sv, sg->v, fb, hipMemcpyHostToDevice, st), "prefetch of v");
  const uint16_t* gdev = sg->g;
  if (sg->grad_loc == DOS_HOST_PINNED) {
    STAGED_TRY(hipMemcpyAsync(sgr, sg->g, (size_t)sg->n * 2, hipMemcpyHostToDevice, st), "prefetch of g");
    gdev = sgr;
  }
  rc = dos::launch_adam(sp, sm, sv, gdev, sg->p_lp, sg->n, sc, st, nullptr);
  if (rc != DOS_OK) return rc;
  STAGED_TRY(hipMemcpyAsync(sg->p, sp, fb, hipMemcpyDeviceToHost, st), "flush of p");
  if (needs_m) STAGED_TRY(hipMemcpyAsync(sg->m, sm, fb, hipMemcpyDeviceToHost, st), "flush of m");
  STAGED_TRY(hipMemcpyAsync(sg->v, sv, fb, hipMemcpyDeviceToHost, st), "flush of v");
  return DOS_OK;
}
