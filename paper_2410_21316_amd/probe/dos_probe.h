/*
 * libdos_probe -- measurement aids for the benchmark of libdos.  Not part of the
 * product library and not declared in include/dos.h: the benchmark loads this
 * library only for its ceiling measurements and for the known-size copy kernel
 * that scales hardware traffic counters.  Several of these calls overwrite the
 * arrays they are given; never point them at optimizer state that is still
 * needed.
 */
#ifndef DOS_PROBE_H
#define DOS_PROBE_H

#include <stdint.h>

#include "dos.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The dynamic LDS request with which dos_adam_step caps the resident waves per
 * compute unit for AdamW (see dos_launch_cfg.lds_bytes in dos.h). */
#define DOS_PROBE_DEFAULT_LDS_CAP 14848

/* A plain device-to-device copy kernel (reads `bytes`, writes `bytes`; multiple
 * of 16; both pointers device memory, 16-byte aligned), asynchronous on
 * hip_stream.  Hardware traffic counters read for this kernel give the scale of
 * the same counters read for the update kernels. */
dos_status dos_probe_copy(void* dst_dev, const void* src_dev, uint64_t bytes, void* hip_stream);

/* The default launch of dos_adam_step over a device-resident subgroup with parts
 * taken out -- mode 0 performs only its loads (14 B/param), mode 1 only its
 * stores (14 B/param; p, m, v and p_lp become 0), mode 2 loads and stores
 * without the arithmetic (it flips the sign of p, m, v).  Modes 1 and 2 destroy
 * the state they run on.  The rates of modes 0 and 1 are what the memory system
 * reaches in each direction alone; the AdamW kernel's mixed rate is judged
 * against them.  lds_bytes: dynamic LDS requested per block (caps the resident
 * waves per CU), 0 = none, at most 65536.  Elements past the last multiple of
 * four are not touched. */
dos_status dos_probe_adam_traffic(const dos_subgroup* sg, int32_t mode, int32_t lds_bytes, void* hip_stream);

/* Host-memory stream with the access pattern of the host update and no
 * arithmetic to speak of: `threads` threads share out `reps` passes over
 * p, m, v (FP32, read and rewritten in place) and g (16-bit, read) in chunks of
 * 1 Mi elements taken from a common counter (as the workers of the update phase
 * take theirs) and write one 16-bit word per element to out16 -- ordinary host
 * memory of out_n >= n elements (streamed = 0), a window of out_n elements of
 * device memory that the host writes through the PCIe BAR with non-temporal
 * stores (streamed = 1; each thread rewrites its own part of the window), or
 * nowhere (streamed = 2: the 16-bit words are formed and dropped, which shows
 * what the output path costs).  *seconds is the wall time of all passes: 26
 * bytes of host memory traffic per element and pass (28 when out16 is host
 * memory, more where its lines are read before they are written).  Use a
 * buffer far beyond the host's caches (hundreds of MB per thread) and enough
 * passes for a few tenths of a second.  The ceiling against which the host lane
 * of the update phase is judged.  Synchronous; allocates only its threads. */
dos_status dos_probe_host_stream(float* p, float* m, float* v, const uint16_t* g, uint16_t* out16, uint64_t n,
                                 uint64_t out_n, int32_t threads, int32_t reps, int32_t streamed, double* seconds);

#ifdef __cplusplus
}
#endif
#endif /* DOS_PROBE_H */
