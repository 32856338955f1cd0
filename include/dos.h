/*
 * libdos -- the optimizer-update hot path of "Deep Optimizer States"
 * (arXiv 2410.21316) for one AMD MI355X (gfx950) GPU and its host cores.
 *
 * Plain C ABI: raw pointers (each documented as host or device), sizes and
 * status codes.  No function prints or aborts, and none lets a C++ exception
 * cross the boundary: where host memory or a thread cannot be had the call
 * returns DOS_ENOMEM.  Unless stated otherwise, validation precedes work: when a
 * call returns an error no element of any caller array has been modified.  The
 * library never allocates or pins memory inside dos_adam_step or
 * dos_run_update_phase, host memory included (Section 4.1: interleaving must not
 * incur allocation costs; all host buffers are pre-allocated and pre-pinned) --
 * staging memory and streams are handed in at context creation, and the work
 * lists and statistics buffers of a phase are sized then.  dos_adam_step_host
 * allocates nothing but its threads.
 *
 * The update (Sections 1, 2 "mixed precision", 4.1: FP32 parameters, momentum
 * and variance; 16-bit gradients in, 16-bit parameter copy out; Adam).  The
 * paper prints no equations; this library implements bias-corrected Adam with
 * decoupled weight decay, every per-element operation one IEEE binary32
 * operation rounded to nearest-even, unfused, gradual underflow:
 *
 *   scalars, once per call, formed in double and rounded to binary32 once:
 *     step_size    = lr / (1 - beta1^step)
 *     inv_sqrt_bc2 = 1 / sqrt(1 - beta2^step)
 *     decay        = 1 - lr * weight_decay
 *     omb1 = 1.0f - beta1,  omb2 = 1.0f - beta2        (binary32 subtraction)
 *   per element i:
 *     g = widen(g16[i])
 *     m = beta1*m[i] + omb1*g
 *     v = beta2*v[i] + (omb2*g)*g
 *     d = sqrt(v)*inv_sqrt_bc2 + eps
 *     p = p[i]*decay - step_size*(m/d)
 *     m[i]=m, v[i]=v, p[i]=p, p_lp[i]=bf16_round_nearest_even(p)
 */
#ifndef DOS_H
#define DOS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dos_status {
  DOS_OK = 0,
  DOS_EINVAL = -1,  /* NULL pointer, bad hyper-parameter, bad size or count          */
  DOS_EALIGN = -2,  /* an array is not 16-byte aligned                               */
  DOS_EBUDGET = -3, /* GPU budget / staging memory too small for one slot            */
  DOS_EHIP = -4,    /* a HIP call failed (sticky in a context)                       */
  DOS_ESTATE = -5,  /* memory location and requested target do not fit together      */
  DOS_ENOMEM = -6   /* host memory or a thread could not be obtained                 */
} dos_status;

typedef enum dos_loc {
  DOS_HOST_PINNED = 0,   /* page-locked host memory: the DMA engines can reach it           */
  DOS_DEVICE = 1,        /* device memory                                                   */
  DOS_HOST_PAGEABLE = 2  /* ordinary host memory: only the host cores touch it, so only a
                            CPU-planned subgroup may live there                             */
} dos_loc;
typedef enum dos_target { DOS_ON_CPU = 0, DOS_ON_GPU = 1 } dos_target;

/* One subgroup of the flat optimizer partition (Section 2 "ZeRO": a rank's
 * parameters are cut into subgroups; p16, g16, p32, m32, v32 are cut alike).
 * All five arrays have n elements and are owned by the caller.  p, m, v live
 * where state_loc says (pinned host memory or device memory), g where grad_loc
 * says.  p_lp is device memory in dos_adam_step and dos_run_update_phase (it is
 * a slice of the 16-bit model on the GPU) and host memory in
 * dos_adam_step_host.  Every pointer must be 16-byte aligned. */
typedef struct dos_subgroup {
  float* p;          /* FP32 master parameters, in/out, updated in place  */
  float* m;          /* FP32 first moment (momentum), in/out              */
  float* v;          /* FP32 second moment (variance), in/out             */
  const uint16_t* g; /* bf16 gradient bit patterns, in                    */
  uint16_t* p_lp;    /* bf16 bit patterns of the updated parameters, out  */
  uint64_t n;        /* elements; 0 is allowed and is a no-op             */
  int32_t state_loc; /* dos_loc of p, m, v                                */
  int32_t grad_loc;  /* dos_loc of g                                      */
} dos_subgroup;

/* Update rules.  Section 4.1 names Adam, Adagrad and RMSProp as the adaptive
 * optimizers whose per-element independence the interleaving relies on.
 *   DOS_OPT_ADAMW    bias-corrected Adam with decoupled weight decay; state p, m, v
 *   DOS_OPT_ADAGRAD  v += g*g;                   p = p*(1-lr*wd) - lr*g/(sqrt(v)+eps)
 *   DOS_OPT_RMSPROP  v = a*v + (1-a)*g*g (a = beta2, uncentred, no momentum);
 *                                                p = p*(1-lr*wd) - lr*g/(sqrt(v)+eps)
 * Adagrad and RMSProp keep p and v only: the m pointer of a subgroup is not
 * read and may be NULL, the interleaved phase stages two FP32 arrays instead of
 * three (8 bytes per parameter each way), and the resident update moves 20 bytes
 * per parameter (reads 4+4+2, writes 4+4+2). */
typedef enum dos_optimizer { DOS_OPT_ADAMW = 0, DOS_OPT_ADAGRAD = 1, DOS_OPT_RMSPROP = 2 } dos_optimizer;

/* Hyper-parameters as binary32 values; step is 1-based and names the step
 * being taken (it is not modified).  Valid: step >= 1, eps >= 0, all values
 * finite, optimizer one of dos_optimizer; 0 <= beta < 1 for the betas the rule
 * uses (AdamW both, RMSProp beta2 as its smoothing constant, Adagrad none).  A
 * zero-initialised optimizer field means AdamW. */
typedef struct dos_hparams {
  float lr, beta1, beta2, eps, weight_decay;
  int64_t step;
  int32_t optimizer; /* dos_optimizer; last, so that initialisers written for the
                        first six members keep meaning AdamW */
} dos_hparams;

/* Launch shape of the fused kernel, for tuning sweeps. */
typedef struct dos_launch_cfg {
  int32_t variant;       /* kernel layout variant, see dos_adam_step_cfg          */
  int32_t block_threads; /* 0 = default (64); multiple of 64, <= 512              */
  int32_t grid_blocks;   /* 0 = one tile per block; else grid-stride over tiles   */
  int32_t lds_bytes;     /* dynamic LDS per block, used only to cap the number of
                            resident waves per CU (160 KiB / lds_bytes blocks);
                            0 = default, negative = none                           */
  int32_t xcd_group;     /* 0 = block b owns tile b (blocks, and so tiles, go round
                            the 8 XCDs one by one); a power of two k = each XCD takes k
                            consecutive tiles at a time (layouts 4-6, AdamW only)    */
} dos_launch_cfg;

/* ---- device-resident update (Algorithm 1, gpu_update) ---------------------
 * Fused update (hp->optimizer; AdamW unless said otherwise) over one subgroup
 * whose arrays are all device memory.
 * Asynchronous on hip_stream (a hipStream_t, NULL = the default stream); no
 * allocation, no synchronisation, so a stream under HIP graph capture records
 * just the kernel launch (the per-step scalars are kernel arguments: a replay
 * repeats the captured step number).  HBM traffic is 28 bytes per element (reads
 * 4+4+4+2, writes 4+4+4+2; 20 bytes for the rules without a first moment).
 * n may exceed 2^32 (arrays are addressed with 64-bit offsets); the limit is
 * 2^31 - 1 tiles of 256 elements, far beyond what device memory holds.
 * Errors: DOS_EINVAL (NULL, bad hyper-parameters, n beyond that limit),
 * DOS_ESTATE (state_loc or grad_loc not DOS_DEVICE), DOS_EALIGN, DOS_EHIP. */
dos_status dos_adam_step(const dos_subgroup* sg, const dos_hparams* hp, void* hip_stream);

/* Same, with an explicit launch shape.  The low four bits of `variant` pick the
 * layout -- 0: each lane handles 4 consecutive elements per trip (16-byte FP32
 * accesses, 8-byte bf16), two trips unrolled; 1: one trip; 2: four trips; 3: each
 * lane handles 8 consecutive elements (two 16-byte FP32 accesses, 16-byte bf16);
 * 4: one trip and no tile loop (block b owns tile b and nothing else; grid_blocks
 * must be 0); 5, 6: as 4 with two and four trips per lane (a block owns 2 or 4
 * consecutive bursts of 16 bytes per lane in each array, loaded and stored array by
 * array; AdamW only); bit 4 (0x10) makes the loads non-temporal; bits 5-6 pick the
 * store policy: 0x20 non-temporal, 0x40 non-temporal at system scope without the
 * wave-level bit (sc1 nt), 0x60 non-temporal at system scope (sc0 sc1 nt); the two
 * system-scope policies exist in layouts 4 to 6 only.
 * dos_adam_step uses variant 0x74 with 64-thread blocks and an LDS request of
 * 14848 bytes per block (11 one-wave blocks per compute unit).  A NULL cfg means
 * those defaults; unknown values, lds_bytes above 65536: DOS_EINVAL.  Adagrad and
 * RMSProp exist in layout 4 only (other layouts: DOS_EINVAL). */
dos_status dos_adam_step_cfg(const dos_subgroup* sg, const dos_hparams* hp, void* hip_stream,
                             const dos_launch_cfg* cfg);

/* ---- host update (Algorithm 1, cpu_update + the FP32->16-bit downscale, fused)
 * The same arithmetic on host cores over host memory, bit-identical to the
 * device kernel.  All five arrays are host pointers (p_lp too).  threads <= 0
 * means one thread.  Synchronous. */
dos_status dos_adam_step_host(const dos_subgroup* sg, const dos_hparams* hp, int32_t threads);

/* ---- planner (Section 4.2 performance model, Section 4.3 Algorithm 1) ------ */

/* Measured or assumed rates.  h2d/d2h in bytes per second (per direction, under
 * duplex load), update rates in parameters per second.  downscale_params_per_s
 * is the paper's D_c; 0 means the downscale is fused into the host update
 * (1/D_c = 0). */
typedef struct dos_cost_model {
  double h2d_Bps, d2h_Bps;
  double gpu_params_per_s, cpu_params_per_s;
  double downscale_params_per_s;
  double launch_overhead_s;
  int32_t fp32_arrays; /* FP32 state arrays staged per subgroup: 3 (p, m, v; also
                          meant by 0) or 2 (p, v: Adagrad, RMSProp)               */
  double cpu_cost_per_dma_byte; /* host-update work, in parameters, that one byte staged
                          through the GPU lane (either direction) takes away from the
                          host lane: both lanes share the host's memory system (the
                          paper's CPU-cores-per-GPU study, Section 5.4, observes the
                          same contention).  The host lane is priced as
                          (N_C + cost * staged bytes) / cpu_params_per_s; 0 = the lanes
                          do not disturb each other.  Above 1 / (2 * 4 * fp32_arrays)
                          staging a subgroup costs the host lane more than it saves.    */
  double fit[5];       /* running sums of dos_cost_model_observe; zero-initialise      */
} dos_cost_model;

enum { DOS_PLAN_STRIDE = 0, DOS_PLAN_BALANCED = 1 };

/* Output of the planner.  target, order and resident are caller-provided arrays
 * of n_sg entries (resident may be NULL). */
typedef struct dos_plan {
  int32_t n_sg;
  int32_t n_slots;       /* staging slots that fit the budget (capped)                 */
  uint64_t slot_params;  /* capacity of one slot in parameters (<= largest subgroup)   */
  uint8_t* target;       /* dos_target per subgroup                                    */
  int32_t* order;        /* processing order: a permutation of 0..n_sg-1               */
  uint8_t* resident;     /* 1 = keep p,m,v on the GPU across steps (static resident)   */
  int32_t stride_k;      /* Eq. 1 rounded (stride mode), 0 = no dynamic GPU subgroup   */
  double stride_k_real;  /* Eq. 1 before rounding                                      */
  double predicted_s;    /* cost-model makespan of the plan                            */
  double lower_bound_s;  /* max(H2D bytes / h2d_Bps, D2H bytes / d2h_Bps) of the plan  */
} dos_plan;

/* Pure, deterministic, host-only.
 *   mode DOS_PLAN_STRIDE:   k = (3/B + 1/U_g) / (1/U_c + 1/D_c - 1/(2B)) with B in
 *     parameters/s (h2d_Bps/4), rounded to nearest, at least 1; subgroup i goes
 *     to the GPU when (i+1) % k == 0 (Eq. 1 and Algorithm 1).  The 3 is the
 *     number of FP32 arrays that cross the link each way (cm->fp32_arrays: 2
 *     for Adagrad and RMSProp).
 *   mode DOS_PLAN_BALANCED: minimises this library's own makespan estimate
 *     (dos_plan_cost) over the number and choice of GPU subgroups: exhaustively
 *     for up to 16 non-resident subgroups, otherwise an even spread of the best
 *     count (Algorithm 1's stride pattern for n/k) improved by single moves and
 *     pair swaps.
 * gpu_budget_bytes is the device memory the phase may use for FP32 staging and
 * static residents; bytes_per_param_slot is 12 (p, m, v) or 14 (gradients
 * staged too).  Subgroups stream through the slots in pieces: a slot holds
 * min(largest subgroup, 16 Mi) parameters when at least two such slots fit the
 * budget, otherwise a third of the budget; at most 3 slots are used; fewer than
 * 64 Ki parameters per slot is DOS_EBUDGET.  With n_resident_max > 0
 * the planner may mark up to that many trailing subgroups as static residents
 * if they fit the budget next to the staging slots (Section 4.1: residents are
 * placed last).
 * cpu_only (n_sg entries, or NULL for none) marks subgroups that cannot be staged
 * through the GPU -- those whose state is in pageable host memory because the
 * machine cannot pin all of it.  They are never dynamically GPU-planned (they may
 * still be chosen as static residents: a resident's state lives on the device);
 * the stride of mode DOS_PLAN_STRIDE counts over the stageable subgroups only. */
dos_status dos_plan_subgroups(const dos_cost_model* cm, const uint64_t* sizes, const uint8_t* cpu_only,
                              int32_t n_sg, uint64_t gpu_budget_bytes, int32_t bytes_per_param_slot,
                              int32_t mode, int32_t n_resident_max, dos_plan* out);

/* The makespan estimate the balanced mode minimises, for any assignment:
 * predicted = max(host lane, GPU lane), lower = max(link time per direction).
 * slot_params = 0 means whole subgroups are staged. */
dos_status dos_plan_cost(const dos_cost_model* cm, const uint64_t* sizes, const uint8_t* target,
                         const uint8_t* resident, int32_t n_sg, int32_t n_slots, uint64_t slot_params,
                         double* predicted_s, double* lower_bound_s);

/* ---- interleaved update phase (Sections 4.1, 4.3) ------------------------- */

typedef struct dos_ctx dos_ctx;

enum {
  DOS_CTX_PROFILE = 1,    /* time every copy and kernel with events                            */
  DOS_CTX_UPLOAD_DMA = 2, /* send 16-bit uploads with hipMemcpyAsync instead of the default
                             pull-copy kernel (DMA uploads queue behind the bulk prefetches)  */
  DOS_CTX_UPLOAD_DIRECT = 8, /* the host workers write the 16-bit parameters of CPU-planned
                             subgroups straight into p_lp -- device memory, written by the host
                             cores through the PCIe BAR -- instead of into the pinned ring: no
                             ring, no upload kernels, and 4 bytes per parameter less host-memory
                             traffic.  Needs a device whose whole memory is mapped into the host's
                             address space (dos_device_large_bar); creation fails with DOS_ESTATE
                             otherwise.  pinned_stage may then be NULL                         */
  DOS_CTX_SPIN_WAIT = 4   /* the two threads that drive the GPU lane spin while they wait for
                             a slot or a piece instead of sleeping (takes cores from the host
                             workers)                                                         */
};

typedef struct dos_ctx_config {
  void* slot_mem;          /* device memory for the staging ring (caller allocates)   */
  uint64_t slot_bytes;     /* its size                                                */
  uint64_t slot_params;    /* capacity of one slot in parameters                      */
  int32_t n_slots;         /* slots to use (<= 16); each takes 12*slot_params bytes of
                              slot_mem, or 14*slot_params if that fits (then host-
                              resident gradients of GPU-planned subgroups are staged) */
  int32_t host_threads;    /* worker threads for CPU-planned subgroups (>= 1)         */
  void* h2d_stream;        /* hipStream_t for prefetches; NULL (for any of the four) =
                              the library's own stream for that role, created once per
                              device and kept until the process ends                  */
  void* compute_stream;    /* hipStream_t for kernels                                 */
  void* d2h_stream;        /* hipStream_t for flushes                                 */
  void* upload_stream;     /* hipStream_t for 16-bit parameter uploads                */
  void* pinned_stage;      /* pinned host memory for the 16-bit upload ring           */
  uint64_t pinned_stage_bytes;
  uint64_t upload_chunk_params; /* 0 = default (4 Mi)                                 */
  int32_t flags;
  int32_t device;          /* HIP device ordinal                                      */
} dos_ctx_config;

typedef struct dos_phase_stats {
  double wall_s;                  /* call entry to join                               */
  double h2d_bytes, d2h_bytes;    /* bytes moved over the host link per direction     */
  double h2d_busy_s, d2h_busy_s;  /* summed copy durations (DOS_CTX_PROFILE), else -1 */
  double gpu_busy_s;              /* summed kernel durations (DOS_CTX_PROFILE)        */
  double duplex_overlap_s;        /* time both directions were busy at once           */
  double cpu_lane_s;              /* first host update start to last upload enqueued  */
  double gpu_lane_s;              /* phase start to last flush landed                 */
  double cpu_compute_s;           /* host update time, summed over worker threads     */
  double cpu_wait_s;              /* waiting for a free upload-ring entry, summed     */
  double cpu_enqueue_s;           /* enqueueing uploads, summed over worker threads   */
  uint64_t params_gpu, params_cpu, params_resident;
  int32_t n_gpu, n_cpu, n_resident, n_slots;
  int32_t n_pieces, host_threads;
  double h2d_span_s, d2h_span_s;  /* first copy start to last copy end per direction
                                     (DOS_CTX_PROFILE), else -1: span - busy is the
                                     time a direction sat idle between its copies    */
} dos_phase_stats;

/* Creates a context: everything a phase needs besides the caller's memory is
 * made here, once, so that the phases themselves allocate nothing (Section 4.1:
 * the buffers of the interleaved update are pre-allocated and pre-pinned, because
 * allocation inside the update would cost more than the overlap gains) -- events,
 * worker threads, the prefetch thread of the GPU lane, the lists of pieces and
 * chunks (a phase may have up to 16384 staged pieces and 65536 host chunks; one
 * that needs more is refused with DOS_EBUDGET), the statistics buffers and
 * (unless given) streams.  slot_mem
 * and pinned_stage stay owned by the caller and must outlive the context.  A
 * context runs one phase at a time; contexts that use the library's own streams
 * on the same device share them, so their phases should not overlap either.
 * Errors: DOS_EINVAL (NULL, host_threads < 1, slot_params not a multiple of 64,
 * chunk not a multiple of 64), DOS_EALIGN (slot_mem / pinned_stage not 256-byte
 * aligned), DOS_EBUDGET (slot_bytes < n_slots * 12 * slot_params, ring smaller
 * than two chunks), DOS_EHIP, DOS_ENOMEM. */
dos_status dos_ctx_create(dos_ctx** out, const dos_ctx_config* cfg);
/* Joins the context's threads and releases the events; NULL is allowed. */
void dos_ctx_destroy(dos_ctx* ctx);

/* One update phase over all subgroups (Algorithm 1 run_update, re-designed as
 * two concurrent lanes).  GPU-planned subgroups in pinned host memory are
 * prefetched into a staging slot (H2D stream, enqueued by the context's prefetch
 * thread), updated there (compute stream) and flushed back (D2H stream, both
 * enqueued by the calling thread), slot by slot, piece by piece; static residents
 * (state_loc == DOS_DEVICE) are updated in place, last; CPU-planned subgroups
 * (state and gradients in pinned or pageable host memory) are updated in place
 * by the host worker threads, which write the 16-bit parameters into the pinned
 * upload ring and send them to p_lp on the upload stream (or store them straight
 * into p_lp, DOS_CTX_UPLOAD_DIRECT).  n_sg may be at most 65536.  hp->optimizer selects
 * the rule for all of them; Adagrad and RMSProp stage and flush p and v only.
 * Synchronous at the boundary: on return every p, m, v is back where state_loc
 * says and every p_lp has landed on the device.  plan->target decides the lane
 * of each subgroup, plan->order the order in which each lane takes its subgroups
 * (plan->n_slots, slot_params and resident are informative: the context's slots
 * and each subgroup's state_loc are what the phase uses).  Errors leave all state
 * untouched when they are detected by validation (DOS_EINVAL, DOS_EALIGN,
 * DOS_ESTATE, DOS_EBUDGET -- the last also for a phase with more pieces or chunks
 * than the context was created for); DOS_EHIP is sticky and state is then
 * undefined.  Allocates nothing, on the device or on the host. */
dos_status dos_run_update_phase(dos_ctx* ctx, dos_subgroup* sgs, int32_t n_sg, const dos_plan* plan,
                                const dos_hparams* hp, dos_phase_stats* stats);

/* Measures the inputs of the performance model (Section 4.2: the link rate B,
 * the GPU and CPU update rates U_g and U_c; the downscale rate D_c is reported as
 * 0 = fused) on this machine, with the context's own slots, streams and worker
 * threads and through the paths its phases use:
 *   h2d_Bps, d2h_Bps   pinned copies in both directions at once (the paper gives
 *                      one B; the directions differ under duplex load), between
 *                      slot 0 and the upload ring -- or, for a context without a
 *                      ring, pinned memory obtained for the duration of the call;
 *   gpu_params_per_s, launch_overhead_s   the fused kernel over one slot;
 *   cpu_params_per_s   the host update with all worker threads, taking chunks
 *                      from a shared counter as the phases' workers do, over a
 *                      temporary host buffer of 16 Mi parameters per thread
 *                      (470 MB each, 7.5 GB for 16 threads: far beyond the
 *                      caches -- a buffer of 1.9 GB still reads 13 % too fast
 *                      on a many-chiplet host), its 16-bit output going where
 *                      the phases send it: with DOS_CTX_UPLOAD_DIRECT into
 *                      device memory through the PCIe BAR (the staging slots
 *                      serve as the target), otherwise into host memory as into
 *                      the upload ring.
 * The rates are stand-alone peaks: what staged traffic takes away from the host
 * cores when both lanes run (Section 5.4, CPU cores per GPU) is left to
 * dos_cost_model_observe.  Not part of the update phase: the call allocates and
 * frees its temporary buffers and overwrites the staging slots and the ring.
 * Errors: DOS_EBUDGET (no slot, or slot / ring below 1 MiB), DOS_ENOMEM, DOS_EHIP. */
dos_status dos_calibrate(dos_ctx* ctx, dos_cost_model* out);

/* Timeline of the GPU lane of the context's last phase (contexts created with
 * DOS_CTX_PROFILE, phases run with a non-NULL stats argument): for each staged
 * piece, in the order they were processed, six times in milliseconds since the
 * phase's first command -- prefetch start and end, kernel start and end, flush
 * start and end.  Writes at most max_pieces
 * rows of six floats into ms6 (a host buffer) and the number of pieces the phase
 * had into *n_pieces (0 when nothing was timed). */
dos_status dos_ctx_last_timeline(const dos_ctx* ctx, float* ms6, int32_t max_pieces, int32_t* n_pieces);

/* Feeds what the phase that produced `st` actually reached back into `cm`
 * (Section 4.2 takes B, U_g, U_c as constants measured once; Section 5.4, "CPU
 * cores per GPU", shows that host update and transfers slow each other down
 * when they share the host's memory system -- this call measures by how much).
 * Host lane: its time is fitted as (N_C + cost * staged bytes) / cpu_params_per_s
 * over the phases seen so far (older ones fade), which separates the host cores'
 * own rate from what the GPU lane's traffic takes away from them as soon as two
 * phases with different splits have been seen; until then cpu_cost_per_dma_byte
 * keeps its value and only the rate moves.  Link, when the context profiles:
 * bytes / summed copy time per direction, where the host-to-device direction also
 * counts the 16-bit upload bytes that moved while prefetches were busy (the model
 * charges them to that direction), and both rates are then lowered by a common
 * factor until the model reproduces the measured GPU-lane time; without
 * profiling: bytes / lane time as an upper bound on the time (rates only drop).
 * Call it after every phase and re-plan: the plan then tracks contention between
 * the two lanes, and falls back to the host cores alone where staging does not pay. */
dos_status dos_cost_model_observe(dos_cost_model* cm, const dos_phase_stats* st);

/* ---- for callers that cannot allocate -------------------------------------- */

/* Largest subgroup dos_gpu_update_staged accepts, in parameters.  Its staging
 * array holds 14 bytes per parameter (p, m, v and the gradient): 28 MiB on every
 * GPU the library runs on, from the first use of the library there until the
 * process ends. */
#define DOS_STAGED_MAX_PARAMS 2097152

/* The GPU lane of dos_run_update_phase for ONE subgroup whose p, m, v live in
 * pinned host memory, with no context and no memory handed in: prefetch into the
 * library's own staging array, fused update (hp->optimizer), flush back -- all
 * enqueued on hip_stream (a hipStream_t, NULL = the default stream) and ordered by
 * it alone; the call returns without waiting, and the result is the same, bit for
 * bit, as that of dos_run_update_phase with this subgroup GPU-planned.
 * For callers that cannot call hipMalloc -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation: this function calls no
 * hipMalloc, hipFree or other allocating routine.  (Its first call on a device
 * looks up the device address of the staging array; make that call outside any
 * capture.)  sg->g is device memory (grad_loc DOS_DEVICE) or pinned host memory
 * (staged with the state); sg->p_lp is device memory; sg->m may be NULL for
 * Adagrad and RMSProp.  All calls on one GPU share that GPU's staging array, which
 * keeps the last call's contents (every call overwrites what it reads): calls
 * whose work overlaps in time on one GPU -- on different streams, or from
 * different threads -- race; order them on one stream or with events.
 * Errors: DOS_EINVAL, DOS_EALIGN, DOS_ESTATE (state not in pinned host memory),
 * DOS_EBUDGET (sg->n > DOS_STAGED_MAX_PARAMS: the subgroup does not fit the
 * staging array; nothing has been touched), DOS_EHIP. */
dos_status dos_gpu_update_staged(const dos_subgroup* sg, const dos_hparams* hp, void* hip_stream);

/* ---- utilities ------------------------------------------------------------ */

/* *yes = 1 when the whole memory of HIP device `device` is mapped into the host's
 * address space (resizable / large PCIe BAR), so that host cores can write device
 * memory directly: what DOS_CTX_UPLOAD_DIRECT needs. */
dos_status dos_device_large_bar(int32_t device, int32_t* yes);

/* Pinned (page-locked) host memory of exactly `bytes` bytes, 4 KiB aligned. */
dos_status dos_pinned_alloc(void** out, uint64_t bytes);
dos_status dos_pinned_free(void* ptr);

/* Asks the kernel to back a range of ordinary (pageable) host memory with huge
 * pages where it can (Linux madvise MADV_HUGEPAGE on the whole pages inside the
 * range; a no-op elsewhere).  Call it before the memory is first touched: the host
 * update streams through four arrays, and with 2 MiB pages the hardware
 * prefetchers are not stopped every 4 KiB.  DOS_ESTATE if the kernel refuses. */
dos_status dos_host_advise_hugepages(void* ptr, uint64_t bytes);

/* Reads one byte of every 4 KiB page of a buffer and writes it back, with
 * `threads` threads, so that the first host update of a host buffer that so far
 * was only written by DMA, or never touched, does not pay for the page faults
 * inside the update phase.  Also for device memory on a large-BAR machine (the
 * 16-bit model that DOS_CTX_UPLOAD_DIRECT lets the host cores write): the first
 * host access to a device page maps it, which costs about as much.  Nobody else
 * may write the buffer during the call. */
dos_status dos_host_prefault(void* ptr, uint64_t bytes, int32_t threads);

const char* dos_strerror(dos_status s);
/* Text of the last HIP error seen by the calling thread ("" if none). */
const char* dos_last_hip_error(void);
int32_t dos_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DOS_H */
