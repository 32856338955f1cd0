// Internal declarations shared by the translation units of libdos.
#pragma once

#include <stdint.h>

#include "dos.h"

namespace dos {

// The binary32 scalars of one step, derived once on the host (formed in double,
// each rounded to binary32 once), and the update rule they belong to.  Adagrad
// and RMSProp use beta2 / omb2 (RMSProp's smoothing constant), step_size (the
// learning rate itself: no bias correction), eps and decay.
struct AdamScalars {
  float beta1, beta2, omb1, omb2, step_size, inv_sqrt_bc2, eps, decay;
  int32_t opt;  // dos_optimizer
};

// FP32 state arrays the rule keeps per subgroup: p, m, v or p, v.
inline int fp32_arrays_of(int opt) { return opt == DOS_OPT_ADAMW ? 3 : 2; }

// Validates the hyper-parameters and derives the scalars.
dos_status make_scalars(const dos_hparams* hp, AdamScalars* out);

// DOS_OK when every pointer of the subgroup the rule uses is non-NULL (or n == 0)
// and 16-byte aligned; m is only looked at when needs_m.
dos_status check_subgroup_pointers(const dos_subgroup* sg, bool needs_m = true);

// Enqueues the fused kernel over n elements on `stream`.  Pointers are device
// memory, 16-byte aligned (checked by the callers).  Returns DOS_EHIP when the
// launch fails, DOS_EINVAL for an unknown launch shape.
dos_status launch_adam(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n,
                       const AdamScalars& s, void* stream, const dos_launch_cfg* cfg);

// Enqueues a copy kernel that reads n 16-bit words from pinned (device-mapped)
// host memory and writes them to device memory; both pointers 16-byte aligned.
dos_status launch_pull_copy_u16(uint16_t* dst_dev, const uint16_t* src_host, uint64_t n, void* stream);

// Host update of elements [0, n) on the calling thread (vectorised, bit-identical
// to the device kernel).
void host_adam_range(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp, uint64_t n,
                     const AdamScalars& s);

// The same update with the 16-bit output going to memory the host writes through the PCIe BAR
// (device memory): the output of each small block is formed in a cache-resident buffer and sent
// with non-temporal stores.
void host_adam_range_streamed(float* p, float* m, float* v, const uint16_t* g, uint16_t* p_lp_dev, uint64_t n,
                              const AdamScalars& s);

// Drains the calling core's write-combining buffers (x86 sfence).
void store_fence();

// Records the text of a failed HIP call for dos_last_hip_error().
void note_hip_error(int code, const char* what);

}  // namespace dos
