// The interleaved update phase (Sections 4.1 and 4.3 of the paper), re-designed
// for one MI355X and its host cores as two concurrent lanes:
//
//   GPU lane   -- every GPU-planned subgroup that lives in pinned host memory is
//                 cut into pieces of at most one staging slot; piece j uses slot
//                 j mod n_slots:  H2D stream: wait(slot free), copy p, m, v (and
//                 g when it is host-resident) in, record(ready);  compute stream:
//                 wait(ready), fused AdamW kernel, record(done);  D2H stream:
//                 wait(done), copy p, m, v back, record(free).  Two threads
//                 drive this as a software pipeline with a bounded look-ahead:
//                 the context's prefetch thread enqueues a prefetch as soon as
//                 its slot is free, the calling thread kernel + flush of piece j
//                 once j has landed (enqueueing a copy can block the caller
//                 while earlier copies of that direction are in flight, so each
//                 direction has its own thread); prefetch and flush run full
//                 duplex.  Static residents (state already in device memory)
//                 are updated in place, last.
//   host lane  -- persistent worker threads take chunks of the CPU-planned
//                 subgroups and run the host update, which emits the 16-bit
//                 parameters in the same pass (the paper's separate downscale
//                 pass is fused away): straight into the device model through
//                 the PCIe BAR where the device memory is host-mapped
//                 (DOS_CTX_UPLOAD_DIRECT), else into a pinned ring from which
//                 each chunk is sent to the device model on a fourth stream.
//
// The call joins both lanes before it returns.  Nothing is allocated here: slots,
// ring, streams, events and threads belong to the context.
#include <hip/hip_runtime_api.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "dos_internal.h"

namespace {

using clk = std::chrono::steady_clock;
inline double secs(clk::time_point a, clk::time_point b) {
  return std::chrono::duration<double>(b - a).count();
}

constexpr int kMaxSlots = 16;
constexpr int kProfPieces = 4096;  // pieces per phase that can be timed individually
// Capacity of the per-phase work lists, reserved when the context is created so that a
// phase never grows them: a phase that would need more is refused (DOS_EBUDGET).
constexpr size_t kMaxChunks = (size_t)1 << 16;
constexpr size_t kMaxPieces = (size_t)1 << 14;

struct Chunk {  // a piece of a CPU-planned subgroup
  int sg;
  uint64_t off, cnt;
};

struct Piece {  // a piece of a GPU-planned, host-resident subgroup
  int sg;
  uint64_t off, cnt;
};

}  // namespace

struct dos_ctx {
  int device = 0;
  int flags = 0;
  hipStream_t h2d = nullptr, comp = nullptr, d2h = nullptr, upl = nullptr;
  // staging ring on the device
  char* slot_mem = nullptr;
  uint64_t slot_params = 0, slot_stride = 0;
  int n_slots = 0;
  bool slots_hold_grads = false;
  hipEvent_t ready[kMaxSlots] = {}, done[kMaxSlots] = {}, freed[kMaxSlots] = {};
  // 16-bit upload ring in pinned host memory
  char* stage = nullptr;
  uint64_t chunk_params = 0;
  int ring_n = 0;
  std::vector<hipEvent_t> ring_ev;
  std::vector<std::atomic<int64_t>> ring_seq;  // last chunk index recorded on each ring entry
  // profiling events
  std::vector<hipEvent_t> prof;  // 6 per piece
  std::vector<float> timeline;   // the last phase's event times, 6 per piece (ms since t0)
  std::vector<std::pair<double, double>> iv_up, iv_down;  // copy intervals of the last phase (statistics)
  hipEvent_t cal_ev[4] = {nullptr, nullptr, nullptr, nullptr};  // timing events of dos_calibrate
  hipEvent_t t0 = nullptr;  // start of the phase on the H2D stream (origin of the profile timeline)
  // end of the GPU lane: tail[0], tail[1] close the H2D and compute streams, lane_end follows both
  // and the last flush on the D2H stream; the driver thread sleeps on it
  hipEvent_t tail[2] = {nullptr, nullptr}, lane_end = nullptr;
  // host workers
  int T = 1;
  std::vector<std::thread> workers;
  std::mutex mu;
  std::condition_variable cv_start, cv_done;
  uint64_t generation = 0;
  int running = 0;
  bool quit = false;
  // the job the workers see
  const dos_subgroup* job_sgs = nullptr;
  const std::vector<Chunk>* job_chunks = nullptr;
  dos::AdamScalars job_scalars{};
  std::atomic<int64_t> next_chunk{0};
  std::atomic<int> job_error{0};
  std::mutex upl_mu;
  clk::time_point cpu_first, cpu_last;
  struct alignas(64) LaneTimes { double compute = 0, wait = 0, enqueue = 0; };
  std::vector<LaneTimes> lane_times;  // one per worker, reset every phase
  std::atomic<bool> cpu_started{false};
  std::atomic<uint32_t> direct_sink{0};  // keeps the read-backs of the direct uploads alive
  // prefetch thread of the GPU lane: it enqueues the host-to-device copies, the
  // calling thread the kernels and the flushes (an enqueue of a copy can block its
  // caller while earlier copies of the same direction are in flight; with one thread
  // per direction a blocked prefetch enqueue no longer delays the flushes)
  std::thread prefetcher;
  std::mutex pipe_mu;
  std::condition_variable pipe_cv;
  uint64_t pf_generation = 0;       // bumped to start a prefetch job
  bool pf_busy = false;             // a prefetch job is running
  bool pf_prof = false;             // the job records profile events
  bool pf_needs_m = true;           // the rule keeps a first moment: m is staged too
  const dos_subgroup* pf_sgs = nullptr;
  int64_t pf_enqueued = -1;         // last piece whose prefetch and ready event are enqueued
  int64_t fl_enqueued = -1;         // last piece whose flush and freed event are enqueued
  bool pipe_abort = false;          // the calling thread gave up: the prefetcher stops
  bool pf_quit = false;             // the context is being destroyed
  hipError_t pf_error = hipSuccess; // first failure of the prefetcher
  const char* pf_error_what = "";
  // scratch lists reused across phases (reserved at creation)
  std::vector<Chunk> chunks;
  std::vector<Piece> pieces;
  dos_status sticky = DOS_OK;
};

namespace {

// Streams the library creates are created once per device and kept until the
// process ends.  Measured on MI355X / ROCm 7: after the copy streams of a context
// had been destroyed and new ones created, prefetches and flushes of every later
// context ran strictly one after the other (no duplex overlap) for the rest of
// the process; streams that are never destroyed keep both directions concurrent.
struct DeviceStreams {
  hipStream_t s[4] = {nullptr, nullptr, nullptr, nullptr};
  bool made = false;
};
std::mutex g_streams_mu;
DeviceStreams g_streams[64];

hipError_t library_streams(int device, hipStream_t out[4]) {
  if (device < 0 || device >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_streams_mu);
  DeviceStreams& d = g_streams[device];
  if (!d.made) {
    for (int i = 0; i < 4; ++i) {
      if (d.s[i]) continue;  // made by an earlier call that failed further on
      hipError_t e = hipStreamCreateWithFlags(&d.s[i], hipStreamNonBlocking);
      if (e != hipSuccess) {
        d.s[i] = nullptr;
        return e;
      }
    }
    d.made = true;
  }
  for (int i = 0; i < 4; ++i) out[i] = d.s[i];
  return hipSuccess;
}

#define HIP_TRY(ctx, call, what)                \
  do {                                          \
    hipError_t e_ = (call);                     \
    if (e_ != hipSuccess) {                     \
      dos::note_hip_error((int)e_, what);       \
      (void)hipGetLastError();                  \
      (ctx)->sticky = DOS_EHIP;                 \
      return DOS_EHIP;                          \
    }                                           \
  } while (0)

void worker_main(dos_ctx* c, int tid) {
  (void)hipSetDevice(c->device);
  uint64_t seen = 0;
  for (;;) {
    {
      std::unique_lock<std::mutex> lk(c->mu);
      c->cv_start.wait(lk, [&] { return c->quit || c->generation != seen; });
      if (c->quit) return;
      seen = c->generation;
    }
    const std::vector<Chunk>& chunks = *c->job_chunks;
    const int64_t total = (int64_t)chunks.size();
    dos_ctx::LaneTimes& lt = c->lane_times[tid];
    lt = dos_ctx::LaneTimes();
    const volatile uint16_t* last_direct = nullptr;  // last word this worker wrote into device memory
    for (;;) {
      const int64_t ci = c->next_chunk.fetch_add(1);
      if (ci >= total || c->job_error.load()) break;
      if (!c->cpu_started.exchange(true)) c->cpu_first = clk::now();
      const Chunk& ch = chunks[ci];
      const dos_subgroup& sg = c->job_sgs[ch.sg];
      if (c->flags & DOS_CTX_UPLOAD_DIRECT) {
        // the 16-bit parameters go straight into the device model: p_lp is device memory that this
        // core writes through the PCIe BAR (posted writes, combined into whole lines on the way)
        const auto td0 = clk::now();
        uint16_t* dst = sg.p_lp + ch.off;
        dos::host_adam_range_streamed(sg.p + ch.off, sg.m ? sg.m + ch.off : nullptr, sg.v + ch.off, sg.g + ch.off,
                                      dst, ch.cnt, c->job_scalars);
        last_direct = dst + (ch.cnt - 1);
        lt.compute += secs(td0, clk::now());
        continue;
      }
      const int r = (int)(ci % c->ring_n);
      // the ring entry is free once the upload of chunk ci - ring_n has landed
      const auto tw0 = clk::now();
      if (ci >= c->ring_n) {
        while (c->ring_seq[r].load(std::memory_order_acquire) != ci - c->ring_n) {
          if (c->job_error.load()) break;
          std::this_thread::yield();
        }
        if (c->job_error.load()) break;
        if (hipEventSynchronize(c->ring_ev[r]) != hipSuccess) {
          c->job_error.store(1);
          break;
        }
      }
      uint16_t* out = reinterpret_cast<uint16_t*>(c->stage + (uint64_t)r * c->chunk_params * 2);
      const auto tw1 = clk::now();
      dos::host_adam_range(sg.p + ch.off, sg.m ? sg.m + ch.off : nullptr, sg.v + ch.off, sg.g + ch.off, out,
                           ch.cnt, c->job_scalars);
      const auto tw2 = clk::now();
      {
        std::lock_guard<std::mutex> lk(c->upl_mu);
        hipError_t e = hipSuccess;
        if (c->flags & DOS_CTX_UPLOAD_DMA) {
          e = hipMemcpyAsync(sg.p_lp + ch.off, out, ch.cnt * 2, hipMemcpyHostToDevice, c->upl);
        } else if (dos::launch_pull_copy_u16(sg.p_lp + ch.off, out, ch.cnt, c->upl) != DOS_OK) {
          e = hipErrorLaunchFailure;
        }
        if (e == hipSuccess) e = hipEventRecord(c->ring_ev[r], c->upl);
        if (e != hipSuccess) {
          dos::note_hip_error((int)e, "upload of 16-bit parameters");
          c->job_error.store(1);
        }
      }
      c->ring_seq[r].store(ci, std::memory_order_release);
      const auto tw3 = clk::now();
      lt.wait += secs(tw0, tw1);
      lt.compute += secs(tw1, tw2);
      lt.enqueue += secs(tw2, tw3);
    }
    if (last_direct) {
      // The writes through the BAR are posted.  A store fence drains this core's write-combining
      // buffers, and reading one of the written words back cannot complete before the writes ahead
      // of it have reached the device: after this, work launched on the GPU sees them.
      std::atomic_thread_fence(std::memory_order_seq_cst);
      dos::store_fence();
      c->direct_sink.fetch_add(*last_direct, std::memory_order_relaxed);
    }
    {
      std::lock_guard<std::mutex> lk(c->mu);
      c->cpu_last = clk::now();
      if (--c->running == 0) c->cv_done.notify_all();
    }
  }
}

struct SlotPtrs {
  float *p, *m, *v;
  uint16_t* g;
};
inline SlotPtrs slot_of(const dos_ctx* c, size_t j) {
  char* base = c->slot_mem + (uint64_t)(j % (size_t)c->n_slots) * c->slot_stride;
  return SlotPtrs{(float*)base, (float*)(base + 4 * c->slot_params), (float*)(base + 8 * c->slot_params),
                  (uint16_t*)(base + 12 * c->slot_params)};
}

// Prefetch of piece j into its slot (H2D stream).  The slot is free once the flush
// of piece j - n_slots has landed: a host wait, so that no stream ever holds a long
// chain of blocked commands.  The caller has made sure that flush is enqueued.
hipError_t prefetch_piece(dos_ctx* c, const dos_subgroup* sgs, const Piece& pc, size_t j, bool prof,
                          bool needs_m, const char** what) {
  const dos_subgroup& sg = sgs[pc.sg];
  const int s = (int)(j % (size_t)c->n_slots);
  const SlotPtrs sl = slot_of(c, j);
  const size_t fb = pc.cnt * 4;
  hipEvent_t* pe = prof ? &c->prof[j * 6] : nullptr;
  hipError_t e = hipSuccess;
  *what = "hipEventSynchronize";
  if (j >= (size_t)c->n_slots && (e = hipEventSynchronize(c->freed[s])) != hipSuccess) return e;
  *what = "hipEventRecord";
  if (pe && (e = hipEventRecord(pe[0], c->h2d)) != hipSuccess) return e;
  *what = "prefetch of p";
  if ((e = hipMemcpyAsync(sl.p, sg.p + pc.off, fb, hipMemcpyHostToDevice, c->h2d)) != hipSuccess) return e;
  *what = "prefetch of m";
  if (needs_m && (e = hipMemcpyAsync(sl.m, sg.m + pc.off, fb, hipMemcpyHostToDevice, c->h2d)) != hipSuccess)
    return e;
  *what = "prefetch of v";
  if ((e = hipMemcpyAsync(sl.v, sg.v + pc.off, fb, hipMemcpyHostToDevice, c->h2d)) != hipSuccess) return e;
  *what = "prefetch of g";
  if (sg.grad_loc == DOS_HOST_PINNED &&
      (e = hipMemcpyAsync(sl.g, sg.g + pc.off, pc.cnt * 2, hipMemcpyHostToDevice, c->h2d)) != hipSuccess)
    return e;
  *what = "hipEventRecord";
  if (pe && (e = hipEventRecord(pe[1], c->h2d)) != hipSuccess) return e;
  return hipEventRecord(c->ready[s], c->h2d);
}

void prefetcher_main(dos_ctx* c) {
  (void)hipSetDevice(c->device);
  uint64_t seen = 0;
  for (;;) {
    {
      std::unique_lock<std::mutex> lk(c->pipe_mu);
      c->pipe_cv.wait(lk, [&] { return c->pf_quit || c->pf_generation != seen; });
      if (c->pf_quit) return;
      seen = c->pf_generation;
    }
    const std::vector<Piece>& pieces = c->pieces;
    const dos_subgroup* sgs = c->pf_sgs;
    const bool prof = c->pf_prof, needs_m = c->pf_needs_m;
    for (size_t j = 0; j < pieces.size(); ++j) {
      if (j >= (size_t)c->n_slots) {
        // the flush that frees this slot must have been enqueued before its event means anything
        std::unique_lock<std::mutex> lk(c->pipe_mu);
        c->pipe_cv.wait(lk, [&] { return c->pipe_abort || c->fl_enqueued >= (int64_t)(j - (size_t)c->n_slots); });
        if (c->pipe_abort) break;
      }
      const char* what = "";
      const hipError_t e = prefetch_piece(c, sgs, pieces[j], j, prof, needs_m, &what);
      std::lock_guard<std::mutex> lk(c->pipe_mu);
      if (e != hipSuccess) {
        c->pf_error = e;
        c->pf_error_what = what;
        c->pipe_cv.notify_all();
        break;
      }
      c->pf_enqueued = (int64_t)j;
      c->pipe_cv.notify_all();
    }
    {
      std::lock_guard<std::mutex> lk(c->pipe_mu);
      c->pf_busy = false;
      c->pipe_cv.notify_all();
    }
  }
}

void destroy(dos_ctx* c) {
  {
    std::lock_guard<std::mutex> lk(c->mu);
    c->quit = true;
  }
  c->cv_start.notify_all();
  {
    std::lock_guard<std::mutex> lk(c->pipe_mu);
    c->pf_quit = true;
    c->pipe_cv.notify_all();
  }
  if (c->prefetcher.joinable()) c->prefetcher.join();
  for (auto& t : c->workers) t.join();
  (void)hipSetDevice(c->device);
  for (int s = 0; s < kMaxSlots; ++s) {
    if (c->ready[s]) (void)hipEventDestroy(c->ready[s]);
    if (c->done[s]) (void)hipEventDestroy(c->done[s]);
    if (c->freed[s]) (void)hipEventDestroy(c->freed[s]);
  }
  for (auto e : c->ring_ev)
    if (e) (void)hipEventDestroy(e);
  for (auto e : c->prof)
    if (e) (void)hipEventDestroy(e);
  if (c->t0) (void)hipEventDestroy(c->t0);
  for (hipEvent_t e : c->cal_ev)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : {c->tail[0], c->tail[1], c->lane_end})
    if (e) (void)hipEventDestroy(e);
  delete c;
}

// Length of the union of [a,b) intervals intersected with the union of another set.
// Works in place on the two lists (sorted and merged where they stand): no allocation.
double overlap_of_unions(std::vector<std::pair<double, double>>& a, std::vector<std::pair<double, double>>& b) {
  auto merge = [](std::vector<std::pair<double, double>>& v) {
    if (v.empty()) return;
    std::sort(v.begin(), v.end());
    size_t w = 0;
    for (size_t r = 1; r < v.size(); ++r) {
      if (v[r].first <= v[w].second) v[w].second = std::max(v[w].second, v[r].second);
      else v[++w] = v[r];
    }
    v.resize(w + 1);
  };
  merge(a);
  merge(b);
  double tot = 0;
  size_t i = 0, j = 0;
  while (i < a.size() && j < b.size()) {
    const double lo = std::max(a[i].first, b[j].first), hi = std::min(a[i].second, b[j].second);
    if (hi > lo) tot += hi - lo;
    if (a[i].second < b[j].second) ++i; else ++j;
  }
  return tot;
}

}  // namespace

namespace {

dos_status ctx_create(dos_ctx** out, const dos_ctx_config* cfg, dos_ctx*& c) {
  if (!cfg || cfg->host_threads < 1 || cfg->host_threads > 1024 || cfg->n_slots < 0 || cfg->n_slots > kMaxSlots)
    return DOS_EINVAL;
  if (cfg->n_slots > 0) {
    if (!cfg->slot_mem || cfg->slot_params == 0 || (cfg->slot_params & 63)) return DOS_EINVAL;
    if ((uintptr_t)cfg->slot_mem & 255) return DOS_EALIGN;
    if (cfg->slot_bytes / (uint64_t)cfg->n_slots / 12 < cfg->slot_params) return DOS_EBUDGET;
  }
  const uint64_t chunk = cfg->upload_chunk_params ? cfg->upload_chunk_params : (4u << 20);
  if (chunk & 63) return DOS_EINVAL;
  int ring_n = 0;
  if (cfg->pinned_stage) {
    if ((uintptr_t)cfg->pinned_stage & 255) return DOS_EALIGN;
    ring_n = (int)std::min<uint64_t>(cfg->pinned_stage_bytes / (chunk * 2), 4096);
    if (ring_n < 2) return DOS_EBUDGET;
  }
  if (hipSetDevice(cfg->device) != hipSuccess) {
    (void)hipGetLastError();
    return DOS_EHIP;
  }
  if (cfg->flags & DOS_CTX_UPLOAD_DIRECT) {
    // host cores may write device memory only where all of it is mapped into the host's address space
    int large_bar = 0;
    if (hipDeviceGetAttribute(&large_bar, hipDeviceAttributeIsLargeBar, cfg->device) != hipSuccess) {
      (void)hipGetLastError();
      return DOS_EHIP;
    }
    if (!large_bar) return DOS_ESTATE;
  }
  c = new dos_ctx();
  c->device = cfg->device;
  c->flags = cfg->flags;
  c->T = cfg->host_threads;
  c->slot_mem = (char*)cfg->slot_mem;
  c->slot_params = cfg->slot_params;
  c->n_slots = cfg->n_slots;
  if (c->n_slots > 0) {
    const uint64_t per = cfg->slot_bytes / (uint64_t)c->n_slots;
    c->slots_hold_grads = per / 14 >= c->slot_params;
    c->slot_stride = (c->slots_hold_grads ? 14 : 12) * c->slot_params;
  }
  c->stage = (char*)cfg->pinned_stage;
  c->chunk_params = chunk;
  c->ring_n = ring_n;

  auto fail = [&](hipError_t e, const char* what) {
    dos::note_hip_error((int)e, what);
    (void)hipGetLastError();
    destroy(c);
    c = nullptr;
    return DOS_EHIP;
  };
  hipError_t e;
  struct { void* given; hipStream_t* dst; } st[4] = {{cfg->h2d_stream, &c->h2d}, {cfg->compute_stream, &c->comp},
                                                     {cfg->d2h_stream, &c->d2h}, {cfg->upload_stream, &c->upl}};
  hipStream_t lib_streams[4];
  if ((e = library_streams(c->device, lib_streams)) != hipSuccess) return fail(e, "hipStreamCreate");
  for (int i = 0; i < 4; ++i) *st[i].dst = st[i].given ? (hipStream_t)st[i].given : lib_streams[i];
  for (int s = 0; s < c->n_slots; ++s) {
    if ((e = hipEventCreateWithFlags(&c->ready[s], hipEventDisableTiming | ((c->flags & DOS_CTX_SPIN_WAIT) ? 0u : (unsigned)hipEventBlockingSync))) != hipSuccess)
      return fail(e, "hipEventCreate");
    if ((e = hipEventCreateWithFlags(&c->done[s], hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
    // the prefetch thread sleeps on this one, the calling thread on `ready` (neither may take a core
    // from the workers)
    if ((e = hipEventCreateWithFlags(&c->freed[s], hipEventDisableTiming | ((c->flags & DOS_CTX_SPIN_WAIT) ? 0u : (unsigned)hipEventBlockingSync))) != hipSuccess)
      return fail(e, "hipEventCreate");
  }
  c->ring_ev.assign(ring_n, nullptr);
  c->ring_seq = std::vector<std::atomic<int64_t>>(ring_n);
  for (int r = 0; r < ring_n; ++r)
    if ((e = hipEventCreateWithFlags(&c->ring_ev[r], hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
  if ((e = hipEventCreate(&c->t0)) != hipSuccess) return fail(e, "hipEventCreate");
  for (hipEvent_t* ev : {&c->tail[0], &c->tail[1]})
    if ((e = hipEventCreateWithFlags(ev, hipEventDisableTiming)) != hipSuccess) return fail(e, "hipEventCreate");
  if ((e = hipEventCreateWithFlags(&c->lane_end, hipEventDisableTiming | ((c->flags & DOS_CTX_SPIN_WAIT) ? 0u : (unsigned)hipEventBlockingSync))) != hipSuccess)
    return fail(e, "hipEventCreate");
  for (hipEvent_t& ev : c->cal_ev)
    if ((e = hipEventCreate(&ev)) != hipSuccess) return fail(e, "hipEventCreate");
  if (c->flags & DOS_CTX_PROFILE) {
    c->prof.assign((size_t)kProfPieces * 6, nullptr);
    c->timeline.reserve((size_t)kProfPieces * 6);
    c->iv_up.reserve(kProfPieces);
    c->iv_down.reserve(kProfPieces);
    for (auto& ev : c->prof)
      if ((e = hipEventCreate(&ev)) != hipSuccess) return fail(e, "hipEventCreate");
  }
  c->chunks.reserve(kMaxChunks);
  c->pieces.reserve(kMaxPieces);
  c->lane_times.resize(c->T);
  c->workers.reserve(c->T);
  for (int t = 0; t < c->T; ++t) c->workers.emplace_back(worker_main, c, t);
  if (c->n_slots > 0) c->prefetcher = std::thread(prefetcher_main, c);
  *out = c;
  return DOS_OK;
}

}  // namespace

extern "C" dos_status dos_ctx_create(dos_ctx** out, const dos_ctx_config* cfg) {
  if (!out) return DOS_EINVAL;
  *out = nullptr;
  dos_ctx* c = nullptr;
  // Containers and threads are created here; a failure of either must not leave the C boundary as
  // an exception.  destroy() joins whatever threads were started.
  try {
    return ctx_create(out, cfg, c);
  } catch (...) {
    if (c) {
      try {
        destroy(c);
      } catch (...) {
      }
    }
    *out = nullptr;
    return DOS_ENOMEM;
  }
}

extern "C" void dos_ctx_destroy(dos_ctx* ctx) {
  if (ctx) destroy(ctx);
}

namespace {

dos_status run_update_phase(dos_ctx* c, dos_subgroup* sgs, int32_t n_sg, const dos_plan* plan, const dos_hparams* hp,
                            dos_phase_stats* stats) {
  const auto t_entry = clk::now();
  if (!c || !plan || n_sg < 0 || (n_sg > 0 && (!sgs || !plan->target || !plan->order))) return DOS_EINVAL;
  if (c->sticky != DOS_OK) return c->sticky;
  if (plan->n_sg != n_sg) return DOS_EINVAL;
  dos::AdamScalars sc;
  dos_status rc = dos::make_scalars(hp, &sc);
  if (rc != DOS_OK) return rc;

  // ---- validation: nothing is touched before every subgroup has been checked
  std::vector<Chunk>& chunks = c->chunks;
  std::vector<Piece>& pieces = c->pieces;
  chunks.clear();
  pieces.clear();
  {
    // order must be a permutation
    uint64_t seen_words[(1 << 16) / 64] = {};
    if (n_sg > (1 << 16)) return DOS_EINVAL;
    for (int k = 0; k < n_sg; ++k) {
      const int i = plan->order[k];
      if (i < 0 || i >= n_sg || (seen_words[i >> 6] >> (i & 63) & 1)) return DOS_EINVAL;
      seen_words[i >> 6] |= (uint64_t)1 << (i & 63);
    }
  }
  uint64_t params_gpu = 0, params_cpu = 0, params_res = 0;
  int n_gpu = 0, n_cpu = 0, n_res = 0;
  const bool needs_m = sc.opt == DOS_OPT_ADAMW;  // Adagrad, RMSProp: p and v only
  for (int k = 0; k < n_sg; ++k) {
    const int i = plan->order[k];
    const dos_subgroup& sg = sgs[i];
    if ((rc = dos::check_subgroup_pointers(&sg, needs_m)) != DOS_OK) return rc;
    if (plan->target[i] > DOS_ON_GPU) return DOS_EINVAL;
    if (sg.state_loc < DOS_HOST_PINNED || sg.state_loc > DOS_HOST_PAGEABLE) return DOS_EINVAL;
    if (sg.grad_loc < DOS_HOST_PINNED || sg.grad_loc > DOS_HOST_PAGEABLE) return DOS_EINVAL;
    if (sg.n == 0) continue;
    if (plan->target[i] == DOS_ON_CPU) {
      // the host cores read and write it in place: pinned or pageable, but not device memory
      if (sg.state_loc == DOS_DEVICE || sg.grad_loc == DOS_DEVICE) return DOS_ESTATE;
      if (c->ring_n < 2 && !(c->flags & DOS_CTX_UPLOAD_DIRECT)) return DOS_EBUDGET;
      if ((sg.n + c->chunk_params - 1) / c->chunk_params > kMaxChunks - chunks.size()) return DOS_EBUDGET;
      for (uint64_t off = 0; off < sg.n; off += c->chunk_params)
        chunks.push_back({i, off, std::min(c->chunk_params, sg.n - off)});
      params_cpu += sg.n;
      ++n_cpu;
    } else if (sg.state_loc == DOS_DEVICE) {  // static resident
      if (sg.grad_loc != DOS_DEVICE) return DOS_ESTATE;
      params_res += sg.n;
      ++n_res;
    } else {
      // the DMA engines must reach it: pageable state or gradients cannot be staged
      if (sg.state_loc == DOS_HOST_PAGEABLE || sg.grad_loc == DOS_HOST_PAGEABLE) return DOS_ESTATE;
      if (c->n_slots < 1) return DOS_EBUDGET;
      if (sg.grad_loc == DOS_HOST_PINNED && !c->slots_hold_grads) return DOS_EBUDGET;
      if ((sg.n + c->slot_params - 1) / c->slot_params > kMaxPieces - pieces.size()) return DOS_EBUDGET;
      for (uint64_t off = 0; off < sg.n; off += c->slot_params)
        pieces.push_back({i, off, std::min(c->slot_params, sg.n - off)});
      params_gpu += sg.n;
      ++n_gpu;
    }
  }

  HIP_TRY(c, hipSetDevice(c->device), "hipSetDevice");
  const bool prof = (c->flags & DOS_CTX_PROFILE) && pieces.size() <= (size_t)kProfPieces;

  // ---- host lane: wake the workers
  if (!chunks.empty()) {
    std::lock_guard<std::mutex> lk(c->mu);
    c->job_sgs = sgs;
    c->job_chunks = &chunks;
    c->job_scalars = sc;
    c->next_chunk.store(0);
    c->job_error.store(0);
    c->cpu_started.store(false);
    for (int r = 0; r < c->ring_n; ++r) c->ring_seq[r].store(-1);
    c->running = c->T;
    ++c->generation;
  }
  if (!chunks.empty()) c->cv_start.notify_all();

  // ---- GPU lane: enqueue every piece
  dos_status gpu_rc = DOS_OK;
  auto enqueue_gpu = [&]() -> dos_status {
    HIP_TRY(c, hipEventRecord(c->t0, c->h2d), "hipEventRecord");
    // the other streams start no earlier than t0 (keeps the timeline comparable)
    // kernel over the slot (compute stream) and flush back to the host (D2H stream)
    auto enqueue_update_and_flush = [&](size_t j) -> dos_status {
      const Piece& pc = pieces[j];
      const dos_subgroup& sg = sgs[pc.sg];
      const int s = (int)(j % (size_t)c->n_slots);
      const SlotPtrs sl = slot_of(c, j);
      const size_t fb = pc.cnt * 4;
      hipEvent_t* pe = prof ? &c->prof[j * 6] : nullptr;
      const uint16_t* gdev = (sg.grad_loc == DOS_HOST_PINNED) ? sl.g : sg.g + pc.off;
      HIP_TRY(c, hipStreamWaitEvent(c->comp, c->ready[s], 0), "hipStreamWaitEvent");
      if (pe) HIP_TRY(c, hipEventRecord(pe[2], c->comp), "hipEventRecord");
      dos_status k = dos::launch_adam(sl.p, sl.m, sl.v, gdev, sg.p_lp + pc.off, pc.cnt, sc, c->comp, nullptr);
      if (k != DOS_OK) {
        c->sticky = k;
        return k;
      }
      if (pe) HIP_TRY(c, hipEventRecord(pe[3], c->comp), "hipEventRecord");
      HIP_TRY(c, hipEventRecord(c->done[s], c->comp), "hipEventRecord");
      HIP_TRY(c, hipStreamWaitEvent(c->d2h, c->done[s], 0), "hipStreamWaitEvent");
      if (pe) HIP_TRY(c, hipEventRecord(pe[4], c->d2h), "hipEventRecord");
      HIP_TRY(c, hipMemcpyAsync(sg.p + pc.off, sl.p, fb, hipMemcpyDeviceToHost, c->d2h), "flush of p");
      if (needs_m) HIP_TRY(c, hipMemcpyAsync(sg.m + pc.off, sl.m, fb, hipMemcpyDeviceToHost, c->d2h), "flush of m");
      HIP_TRY(c, hipMemcpyAsync(sg.v + pc.off, sl.v, fb, hipMemcpyDeviceToHost, c->d2h), "flush of v");
      if (pe) HIP_TRY(c, hipEventRecord(pe[5], c->d2h), "hipEventRecord");
      HIP_TRY(c, hipEventRecord(c->freed[s], c->d2h), "hipEventRecord");
      return DOS_OK;
    };
    // Software pipeline driven by two threads.  The prefetch thread enqueues the
    // prefetch of piece j as soon as its slot is free (the flush of piece
    // j - n_slots has landed); this thread enqueues kernel and flush of piece j
    // once piece j has landed.  Prefetches therefore run at most n_slots - 1
    // pieces ahead, and when the D2H stream submits a copy the DMA engine that
    // serves the prefetches is busy, so the runtime (which picks a free engine
    // per stream at submission time) never puts both directions on one engine.
    const size_t np = pieces.size();
    if (np > 0) {
      {
        std::lock_guard<std::mutex> lk(c->pipe_mu);
        c->pf_sgs = sgs;
        c->pf_prof = prof;
        c->pf_needs_m = needs_m;
        c->pf_enqueued = c->fl_enqueued = -1;
        c->pipe_abort = false;
        c->pf_error = hipSuccess;
        c->pf_busy = true;
        ++c->pf_generation;
      }
      c->pipe_cv.notify_all();
      dos_status r = DOS_OK;
      for (size_t j = 0; j < np && r == DOS_OK; ++j) {
        {
          std::unique_lock<std::mutex> lk(c->pipe_mu);
          c->pipe_cv.wait(lk, [&] { return c->pf_error != hipSuccess || c->pf_enqueued >= (int64_t)j; });
          if (c->pf_error != hipSuccess) {
            dos::note_hip_error((int)c->pf_error, c->pf_error_what);
            c->sticky = r = DOS_EHIP;
            break;
          }
        }
        r = [&]() -> dos_status {
          HIP_TRY(c, hipEventSynchronize(c->ready[j % (size_t)c->n_slots]), "hipEventSynchronize");
          return enqueue_update_and_flush(j);
        }();
        if (r == DOS_OK) {
          std::lock_guard<std::mutex> lk(c->pipe_mu);
          c->fl_enqueued = (int64_t)j;
          c->pipe_cv.notify_all();
        }
      }
      {
        // the prefetch thread is idle again before anything else touches the H2D stream
        std::unique_lock<std::mutex> lk(c->pipe_mu);
        if (r != DOS_OK) c->pipe_abort = true;
        c->pipe_cv.notify_all();
        c->pipe_cv.wait(lk, [&] { return !c->pf_busy; });
      }
      if (r != DOS_OK) return r;
    }
    // static residents, placed last: their kernels overlap the tail transfers
    for (int k = 0; k < n_sg; ++k) {
      const int i = plan->order[k];
      const dos_subgroup& sg = sgs[i];
      if (sg.n == 0 || plan->target[i] != DOS_ON_GPU || sg.state_loc != DOS_DEVICE) continue;
      dos_status kr = dos::launch_adam(sg.p, sg.m, sg.v, sg.g, sg.p_lp, sg.n, sc, c->comp, nullptr);
      if (kr != DOS_OK) {
        c->sticky = kr;
        return kr;
      }
    }
    // the lane ends when all three streams have drained: one event behind all of them
    HIP_TRY(c, hipEventRecord(c->tail[0], c->h2d), "hipEventRecord");
    HIP_TRY(c, hipEventRecord(c->tail[1], c->comp), "hipEventRecord");
    HIP_TRY(c, hipStreamWaitEvent(c->d2h, c->tail[0], 0), "hipStreamWaitEvent");
    HIP_TRY(c, hipStreamWaitEvent(c->d2h, c->tail[1], 0), "hipStreamWaitEvent");
    HIP_TRY(c, hipEventRecord(c->lane_end, c->d2h), "hipEventRecord");
    return DOS_OK;
  };
  gpu_rc = enqueue_gpu();

  // ---- join: the GPU lane (asleep on its last event, so that the lane's own end is
  // timed and no core is taken from the workers), the host lane, then the streams
  hipError_t e0 = gpu_rc == DOS_OK ? hipEventSynchronize(c->lane_end) : hipSuccess;
  const auto t_gpu_done = clk::now();
  if (!chunks.empty()) {
    std::unique_lock<std::mutex> lk(c->mu);
    c->cv_done.wait(lk, [&] { return c->running == 0; });
  }
  hipError_t e1 = hipStreamSynchronize(c->h2d);
  hipError_t e2 = hipStreamSynchronize(c->comp);
  hipError_t e3 = hipStreamSynchronize(c->d2h);
  hipError_t e4 = hipStreamSynchronize(c->upl);
  const auto t_exit = clk::now();
  if (gpu_rc != DOS_OK) return gpu_rc;
  for (hipError_t e : {e0, e1, e2, e3, e4})
    if (e != hipSuccess) {
      dos::note_hip_error((int)e, "hipStreamSynchronize at the end of the update phase");
      (void)hipGetLastError();
      c->sticky = DOS_EHIP;
      return DOS_EHIP;
    }
  if (c->job_error.load()) {
    c->sticky = DOS_EHIP;
    return DOS_EHIP;
  }

  if (stats) {
    memset(stats, 0, sizeof *stats);
    stats->wall_s = secs(t_entry, t_exit);
    const double state_bytes = 4.0 * dos::fp32_arrays_of(sc.opt);  // per parameter and direction
    stats->h2d_bytes = state_bytes * (double)params_gpu + 2.0 * (double)params_cpu;
    for (const Piece& pc : pieces)
      if (sgs[pc.sg].grad_loc == DOS_HOST_PINNED) stats->h2d_bytes += 2.0 * (double)pc.cnt;
    stats->d2h_bytes = state_bytes * (double)params_gpu;
    stats->h2d_busy_s = stats->d2h_busy_s = stats->gpu_busy_s = stats->duplex_overlap_s = -1.0;
    stats->h2d_span_s = stats->d2h_span_s = -1.0;
    stats->cpu_lane_s = chunks.empty() ? 0.0 : secs(c->cpu_first, c->cpu_last);
    stats->gpu_lane_s = secs(t_entry, t_gpu_done);
    stats->params_gpu = params_gpu;
    stats->params_cpu = params_cpu;
    stats->params_resident = params_res;
    stats->n_gpu = n_gpu;
    stats->n_cpu = n_cpu;
    stats->n_resident = n_res;
    stats->n_slots = c->n_slots;
    stats->n_pieces = (int32_t)pieces.size();
    stats->host_threads = c->T;
    if (!chunks.empty())
      for (const auto& lt : c->lane_times) {
        stats->cpu_compute_s += lt.compute;
        stats->cpu_wait_s += lt.wait;
        stats->cpu_enqueue_s += lt.enqueue;
      }
    c->timeline.clear();
    if (prof && !pieces.empty()) {
      // (pieces.size() <= kProfPieces here, which is what the two lists were reserved for)
      std::vector<std::pair<double, double>>&up = c->iv_up, &down = c->iv_down;
      up.clear();
      down.clear();
      double hb = 0, db = 0, gb = 0;
      bool ok = true;
      for (size_t j = 0; j < pieces.size() && ok; ++j) {
        hipEvent_t* pe = &c->prof[j * 6];
        float t[6];
        for (int q = 0; q < 6; ++q)
          if (hipEventElapsedTime(&t[q], c->t0, pe[q]) != hipSuccess) {
            (void)hipGetLastError();
            ok = false;
          }
        if (!ok) break;
        hb += (t[1] - t[0]) * 1e-3;
        gb += (t[3] - t[2]) * 1e-3;
        db += (t[5] - t[4]) * 1e-3;
        up.emplace_back(t[0] * 1e-3, t[1] * 1e-3);
        down.emplace_back(t[4] * 1e-3, t[5] * 1e-3);
        c->timeline.insert(c->timeline.end(), t, t + 6);
      }
      if (!ok) c->timeline.clear();
      if (ok) {
        stats->h2d_busy_s = hb;
        stats->d2h_busy_s = db;
        stats->gpu_busy_s = gb;
        // (pieces are processed in order on each stream: first and last copy bound the span)
        stats->h2d_span_s = up.back().second - up.front().first;
        stats->d2h_span_s = down.back().second - down.front().first;
        stats->duplex_overlap_s = overlap_of_unions(up, down);
      }
    }
  }
  return DOS_OK;
}

}  // namespace

extern "C" dos_status dos_run_update_phase(dos_ctx* c, dos_subgroup* sgs, int32_t n_sg, const dos_plan* plan,
                                           const dos_hparams* hp, dos_phase_stats* stats) {
  try {
    return run_update_phase(c, sgs, n_sg, plan, hp, stats);
  } catch (...) {
    // nothing in the phase allocates, so nothing is expected here; should a lock or a wait fail all
    // the same, the state of the subgroups is unknown
    if (c) c->sticky = DOS_EHIP;
    return DOS_ENOMEM;
  }
}

extern "C" dos_status dos_ctx_last_timeline(const dos_ctx* c, float* ms6, int32_t max_pieces, int32_t* n_pieces) {
  if (!c || !n_pieces || max_pieces < 0 || (max_pieces > 0 && !ms6)) return DOS_EINVAL;
  const size_t have = c->timeline.size() / 6;
  *n_pieces = (int32_t)have;
  const size_t take = std::min(have, (size_t)max_pieces);
  if (take) memcpy(ms6, c->timeline.data(), take * 6 * sizeof(float));
  return DOS_OK;
}

// Rates of the cost model measured with the context's own resources (the inputs of the
// performance model, Section 4.2: B per direction, U_g, U_c; D_c is zero because the
// downscale is fused into the host update).
namespace {

dos_status calibrate(dos_ctx* c, dos_cost_model* out) {
  if (c->sticky != DOS_OK) return c->sticky;
  if (c->n_slots < 1) return DOS_EBUDGET;
  HIP_TRY(c, hipSetDevice(c->device), "hipSetDevice");
  memset(out, 0, sizeof *out);
  const uint64_t slot_bytes = c->slot_stride;
  const uint64_t stage_bytes = (uint64_t)c->ring_n * c->chunk_params * 2;

  // ---- host link, both directions at once.  Host side: the upload ring, or (contexts without
  // one) pinned memory obtained for the duration of the measurement.  Device side: the two halves
  // of slot 0.
  uint64_t nbytes = (slot_bytes / 2) & ~(uint64_t)255;
  char* pinned_tmp = nullptr;
  char *host_a, *host_b;
  if (c->ring_n >= 2) {
    const uint64_t half = (stage_bytes / 2) & ~(uint64_t)255;
    nbytes = std::min(nbytes, half);
    host_a = c->stage;
    host_b = c->stage + half;
  } else {
    nbytes = std::min<uint64_t>(nbytes, (uint64_t)256 << 20);
    if (nbytes >= (1u << 20)) {
      void* q = nullptr;
      const hipError_t he = hipHostMalloc(&q, 2 * nbytes, hipHostMallocDefault);
      if (he != hipSuccess) {  // no pinned memory to be had: the context itself is as good as before
        dos::note_hip_error((int)he, "hipHostMalloc for the link calibration");
        (void)hipGetLastError();
        return DOS_EHIP;
      }
      pinned_tmp = (char*)q;
    }
    host_a = pinned_tmp;
    host_b = pinned_tmp + nbytes;
  }
  if (nbytes < (1u << 20)) return DOS_EBUDGET;
  auto release = [&] {
    if (pinned_tmp) (void)hipHostFree(pinned_tmp);
    pinned_tmp = nullptr;
  };
  char* dev_a = c->slot_mem;
  char* dev_b = c->slot_mem + nbytes;
  memset(host_a, 0, nbytes);
  memset(host_b, 0, nbytes);
  hipEvent_t* ev = c->cal_ev;
  hipError_t e = hipMemsetAsync(c->slot_mem, 0, slot_bytes, c->comp);
  if (e == hipSuccess) e = hipStreamSynchronize(c->comp);
  const int reps = (int)std::max<uint64_t>(2, std::min<uint64_t>(64, ((uint64_t)2 << 30) / nbytes));
  // warm-up, then both directions at once
  for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {
    e = hipEventRecord(ev[0], c->h2d);
    if (e == hipSuccess) e = hipEventRecord(ev[2], c->d2h);
    for (int r = 0; r < (pass ? reps : 1) && e == hipSuccess; ++r) {
      e = hipMemcpyAsync(dev_a, host_a, nbytes, hipMemcpyHostToDevice, c->h2d);
      if (e == hipSuccess) e = hipMemcpyAsync(host_b, dev_b, nbytes, hipMemcpyDeviceToHost, c->d2h);
    }
    if (e == hipSuccess) e = hipEventRecord(ev[1], c->h2d);
    if (e == hipSuccess) e = hipEventRecord(ev[3], c->d2h);
    if (e == hipSuccess) e = hipStreamSynchronize(c->h2d);
    if (e == hipSuccess) e = hipStreamSynchronize(c->d2h);
  }
  float ms_up = 0, ms_down = 0;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms_up, ev[0], ev[1]);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms_down, ev[2], ev[3]);
  release();
  HIP_TRY(c, e, "calibration copies");
  out->h2d_Bps = (double)nbytes * reps / (ms_up * 1e-3);
  out->d2h_Bps = (double)nbytes * reps / (ms_down * 1e-3);

  // ---- device kernel over slot 0: five arrays carved out of the slot
  {
    const uint64_t n = (slot_bytes / 28) & ~(uint64_t)63;
    float* p = (float*)c->slot_mem;
    float* m = p + n;
    float* v = m + n;
    uint16_t* g = (uint16_t*)(v + n);
    uint16_t* lp = g + n;
    dos::AdamScalars sc{0.9f, 0.999f, 0.1f, 0.001f, 1e-3f, 1.0f, 1e-8f, 1.0f, DOS_OPT_ADAMW};
    const int kreps = 5;
    dos_status k = dos::launch_adam(p, m, v, g, lp, n, sc, c->comp, nullptr);  // warm-up
    hipError_t he = hipEventRecord(ev[0], c->comp);
    for (int r = 0; r < kreps && k == DOS_OK; ++r) k = dos::launch_adam(p, m, v, g, lp, n, sc, c->comp, nullptr);
    if (he == hipSuccess) he = hipEventRecord(ev[1], c->comp);
    if (he == hipSuccess) he = hipStreamSynchronize(c->comp);
    float ms = 0;
    if (he == hipSuccess) he = hipEventElapsedTime(&ms, ev[0], ev[1]);
    if (k != DOS_OK) return k;
    HIP_TRY(c, he, "calibration kernel");
    out->gpu_params_per_s = (double)n * kreps / (ms * 1e-3);
    // launch overhead: the same kernel over 64 elements
    he = hipEventRecord(ev[0], c->comp);
    for (int r = 0; r < 20 && k == DOS_OK; ++r) k = dos::launch_adam(p, m, v, g, lp, 64, sc, c->comp, nullptr);
    if (he == hipSuccess) he = hipEventRecord(ev[1], c->comp);
    if (he == hipSuccess) he = hipStreamSynchronize(c->comp);
    if (he == hipSuccess) he = hipEventElapsedTime(&ms, ev[0], ev[1]);
    if (k != DOS_OK) return k;
    HIP_TRY(c, he, "calibration kernel");
    out->launch_overhead_s = ms * 1e-3 / 20;
  }

  // ---- host update with all worker threads, through the path the phase will use: with direct
  // uploads the 16-bit output is stored into device memory through the PCIe BAR (here: into the
  // staging slots, every thread rewriting its own window of them), otherwise it goes to host memory
  // as it does into the upload ring.  The threads take 1 Mi-parameter chunks from a shared counter, as
  // the phase's workers take theirs, sweep after sweep over a temporary buffer of 16 Mi parameters per
  // thread (470 MB; 7.5 GB for 16 threads; at least 64 Mi parameters).  The footprint matters: on this
  // machine's host every core has tens of MiB of last-level cache within reach, a 1.9 GB buffer swept
  // again and again by 16 threads reads 13 % faster than the tens of GB a phase streams through (18.2
  // against 16.1 G params/s), and a ring-sized one three to four times faster.
  {
    const bool direct = (c->flags & DOS_CTX_UPLOAD_DIRECT) != 0;
    const int T = c->T;
    uint64_t n = std::min<uint64_t>((uint64_t)512 << 20, std::max<uint64_t>((uint64_t)64 << 20, (uint64_t)T << 24));
    char* big = nullptr;
    constexpr uint64_t kHuge = (uint64_t)2 << 20;  // 2 MiB-aligned, so that the kernel can back it with huge pages
    while (!(big = static_cast<char*>(aligned_alloc(kHuge, (n * 28 + kHuge - 1) & ~(kHuge - 1)))) &&
           n > ((uint64_t)64 << 20))
      n >>= 1;
    if (big) (void)dos_host_advise_hugepages(big, n * 28);  // before the first touch; a refusal costs 2 %
    char* base = big;
    if (!big) {
      if (c->ring_n < 2) return DOS_ENOMEM;
      n = (stage_bytes / 28) & ~(uint64_t)63;
      base = c->stage;
    }
    // device window of each thread for the direct path, in 16-bit words
    uint16_t* const dev_out = reinterpret_cast<uint16_t*>(c->slot_mem);
    const uint64_t window = (((uint64_t)c->n_slots * slot_bytes / 2) / (uint64_t)T) & ~(uint64_t)63;
    if (direct && window < 4096) {
      if (big) free(big);
      return DOS_EBUDGET;
    }
    float* p = (float*)base;
    float* m = p + n;
    float* v = m + n;
    uint16_t* g = (uint16_t*)(v + n);
    uint16_t* lp = g + n;
    dos::AdamScalars sc{0.9f, 0.999f, 0.1f, 0.001f, 1e-3f, 1.0f, 1e-8f, 1.0f, DOS_OPT_ADAMW};
    const uint64_t per = (((n + T - 1) / T) + 63) & ~(uint64_t)63;
    const uint64_t chunk = (uint64_t)1 << 20, n_chunks = (n + chunk - 1) / chunk;
    std::atomic<uint64_t> next{0};
    // sweeps == 0: every thread fills its own slice (first touch by one owner per region);
    // otherwise the threads share out `sweeps` passes over all chunks
    auto run = [&](int sweeps) {
      next.store(0);
      const uint64_t total = n_chunks * (uint64_t)sweeps;
      std::vector<std::thread> th;
      th.reserve(T);
      struct Joiner {  // threads already started are joined also when starting the next one fails
        std::vector<std::thread>& v;
        ~Joiner() {
          for (auto& t : v)
            if (t.joinable()) t.join();
        }
      } joiner{th};
      for (int t = 0; t < T; ++t) {
        th.emplace_back([&, t] {
          if (sweeps == 0) {
            const uint64_t lo = (uint64_t)t * per;
            for (uint64_t i = lo; i < std::min(n, lo + per); ++i) {
              p[i] = 0.01f;
              m[i] = v[i] = 0.0f;
              g[i] = (uint16_t)(0x3A00 + (i & 127));
              lp[i] = 0;
            }
            return;
          }
          uint16_t* const win = dev_out + (uint64_t)t * window;
          for (;;) {
            const uint64_t k = next.fetch_add(1, std::memory_order_relaxed);
            if (k >= total) break;
            const uint64_t lo = (k % n_chunks) * chunk, cnt = std::min(chunk, n - lo);
            if (!direct) {
              dos::host_adam_range(p + lo, m + lo, v + lo, g + lo, lp + lo, cnt, sc);
              continue;
            }
            for (uint64_t off = 0; off < cnt; off += window)
              dos::host_adam_range_streamed(p + lo + off, m + lo + off, v + lo + off, g + lo + off, win,
                                            std::min(window, cnt - off), sc);
          }
          if (direct) {  // drain the posted writes, as the phase's workers do
            dos::store_fence();
            (void)*reinterpret_cast<volatile uint16_t*>(win);
          }
        });
      }
    };
    double rate = 0;
    try {
      run(0);
      auto a = clk::now();
      run(1);
      const double t1 = secs(a, clk::now());
      // three measurements of ~0.25 s each; the rate is a stand-alone peak, so the best one counts
      // (on a shared host single measurements scatter)
      const int sweeps = (int)std::max(1.0, std::min(400.0, 0.25 / t1));
      for (int k = 0; k < 3; ++k) {
        a = clk::now();
        run(sweeps);
        rate = std::max(rate, (double)n * sweeps / secs(a, clk::now()));
      }
    } catch (...) {
      if (big) free(big);
      return DOS_ENOMEM;
    }
    out->cpu_params_per_s = rate;
    if (big) free(big);
    else memset(c->stage, 0, stage_bytes);
  }
  out->downscale_params_per_s = 0.0;
  return DOS_OK;
}

}  // namespace

extern "C" dos_status dos_calibrate(dos_ctx* c, dos_cost_model* out) {
  if (!c || !out) return DOS_EINVAL;
  try {
    return calibrate(c, out);
  } catch (...) {
    return DOS_ENOMEM;
  }
}
