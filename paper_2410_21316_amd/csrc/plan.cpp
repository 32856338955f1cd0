// CPU/GPU subgroup planner: the performance model of Section 4.2 (Eq. 1), the
// stride placement of Algorithm 1 (Section 4.3), and a "balanced" mode that
// minimises this library's own makespan estimate for unequal subgroup sizes,
// per-direction link rates and a fused host downscale.  Pure host code.
#include <math.h>

#include <algorithm>
#include <vector>

#include "dos_internal.h"

namespace {

// Three slots are enough to keep prefetch, kernel and flush of consecutive pieces
// overlapped; on MI355X more outstanding prefetches slow the flushes down.
constexpr int kMaxSlots = 3;
constexpr uint64_t kMinSlotParams = 1u << 16;
// Pieces of 16 Mi parameters (192 MiB of FP32 state) copy at full link rate and
// keep fill/drain of the pipeline and the wait of anything queued behind it short.
constexpr uint64_t kPieceParams = 16u << 20;

struct Cost {
  double predicted, lower;
};

// Bytes of FP32 state per parameter that cross the link in each direction.
double state_bytes_of(const dos_cost_model& cm) { return cm.fp32_arrays == 2 ? 8.0 : 12.0; }

bool valid_cost_model(const dos_cost_model* cm) {
  return cm && (cm->fp32_arrays == 0 || cm->fp32_arrays == 2 || cm->fp32_arrays == 3) &&
         cm->cpu_cost_per_dma_byte >= 0 && isfinite(cm->cpu_cost_per_dma_byte) && cm->h2d_Bps > 0 && cm->d2h_Bps > 0 && cm->gpu_params_per_s > 0 &&
         cm->cpu_params_per_s > 0 && cm->downscale_params_per_s >= 0 && cm->launch_overhead_s >= 0 &&
         isfinite(cm->h2d_Bps) && isfinite(cm->d2h_Bps) && isfinite(cm->gpu_params_per_s) &&
         isfinite(cm->cpu_params_per_s) && isfinite(cm->downscale_params_per_s) &&
         isfinite(cm->launch_overhead_s);
}

// Makespan estimate of one phase.  CPU-planned subgroups: n/U_c on the host and
// 2 B/param of H2D.  Dynamic GPU subgroups: 12 B/param each way plus n/U_g and a
// launch.  Residents: GPU time only.  With >= 2 slots the lanes overlap and only
// the first prefetch + kernel lead the D2H lane; with one slot they serialise.
Cost evaluate(const dos_cost_model& cm, const uint64_t* sizes, const uint8_t* target,
              const uint8_t* resident, int n, int n_slots, uint64_t slot_params) {
  double NG = 0, NC = 0, NR = 0, first = -1;
  int cg = 0, cr = 0;
  for (int i = 0; i < n; ++i) {
    const double s = (double)sizes[i];
    if (target[i] == DOS_ON_CPU) {
      NC += s;
    } else if (resident && resident[i]) {
      NR += s;
      ++cr;
    } else {
      if (first < 0) first = s;
      NG += s;
      ++cg;
    }
  }
  const double sb = state_bytes_of(cm);
  const double h2d_bytes = sb * NG + 2.0 * NC, d2h_bytes = sb * NG;
  const double t_h2d = h2d_bytes / cm.h2d_Bps, t_d2h = d2h_bytes / cm.d2h_Bps;
  // the staged traffic (both directions) takes host memory bandwidth from the host update
  const double t_cpu = (NC + cm.cpu_cost_per_dma_byte * 2.0 * sb * NG) / cm.cpu_params_per_s;
  const double t_gpu = (NG + NR) / cm.gpu_params_per_s + cm.launch_overhead_s * (cg + cr);
  double lane;
  if (cg == 0) {
    lane = std::max(t_h2d, t_gpu);
  } else if (n_slots >= 2) {
    if (slot_params > 0 && first > (double)slot_params) first = (double)slot_params;  // pieces
    const double lead = sb * first / cm.h2d_Bps + first / cm.gpu_params_per_s + cm.launch_overhead_s;
    lane = std::max(std::max(t_h2d, lead + t_d2h), t_gpu);
  } else {
    lane = std::max(sb * NG / cm.h2d_Bps + t_gpu + t_d2h, t_h2d);
  }
  return {std::max(t_cpu, lane), std::max(t_h2d, t_d2h)};
}

}  // namespace

extern "C" dos_status dos_plan_cost(const dos_cost_model* cm, const uint64_t* sizes, const uint8_t* target,
                                    const uint8_t* resident, int32_t n_sg, int32_t n_slots,
                                    uint64_t slot_params, double* predicted_s, double* lower_bound_s) {
  if (!valid_cost_model(cm) || n_sg < 0 || n_slots < 1 || !predicted_s || !lower_bound_s) return DOS_EINVAL;
  if (n_sg > 0 && (!sizes || !target)) return DOS_EINVAL;
  for (int i = 0; i < n_sg; ++i) {
    if (target[i] > DOS_ON_GPU) return DOS_EINVAL;
    if (resident && resident[i] && target[i] != DOS_ON_GPU) return DOS_ESTATE;
  }
  const Cost c = evaluate(*cm, sizes, target, resident, n_sg, n_slots, slot_params);
  *predicted_s = c.predicted;
  *lower_bound_s = c.lower;
  return DOS_OK;
}

namespace {

dos_status plan_subgroups(const dos_cost_model* cm, const uint64_t* sizes, const uint8_t* cpu_only, int32_t n_sg,
                          uint64_t gpu_budget_bytes, int32_t bytes_per_param_slot, int32_t mode,
                          int32_t n_resident_max, dos_plan* out) {
  if (!valid_cost_model(cm) || !out || n_sg < 0 || n_resident_max < 0) return DOS_EINVAL;
  if (mode != DOS_PLAN_STRIDE && mode != DOS_PLAN_BALANCED) return DOS_EINVAL;
  if (bytes_per_param_slot != 12 && bytes_per_param_slot != 14) return DOS_EINVAL;
  if (n_sg > 0 && (!sizes || !out->target || !out->order)) return DOS_EINVAL;
  if (n_resident_max > 0 && !out->resident) return DOS_EINVAL;
  uint64_t s_max = 0;
  for (int i = 0; i < n_sg; ++i) s_max = std::max(s_max, sizes[i]);

  // ---- staging slots from the budget
  const uint64_t bpp = (uint64_t)bytes_per_param_slot;
  uint64_t slot_params;
  int n_slots;
  const uint64_t s_pad = (s_max + 63) & ~(uint64_t)63;  // keeps every slot array 16-byte aligned
  const uint64_t want = std::min<uint64_t>(s_pad, kPieceParams);  // subgroups stream through in pieces
  if (want > 0 && gpu_budget_bytes / bpp / 2 >= want) {
    slot_params = want;
    n_slots = (int)std::min<uint64_t>(kMaxSlots, gpu_budget_bytes / (bpp * want));
  } else {
    slot_params = (gpu_budget_bytes / (kMaxSlots * bpp)) & ~(uint64_t)0xFFFF;  // multiple of 64 Ki
    n_slots = kMaxSlots;
  }
  if (n_sg > 0 && slot_params < kMinSlotParams) return DOS_EBUDGET;

  std::vector<uint8_t> target(n_sg, DOS_ON_CPU), resident(n_sg, 0);

  // ---- static residents: trailing subgroups that fit next to the slots
  uint64_t left = gpu_budget_bytes - std::min<uint64_t>(gpu_budget_bytes, (uint64_t)n_slots * bpp * slot_params);
  int n_res = 0;
  // (a resident's state lives on the device, so it does not matter whether its
  // host copy could be pinned: cpu_only does not exclude residency)
  for (int i = n_sg - 1; i >= 0 && n_res < n_resident_max; --i) {
    const uint64_t need = (uint64_t)state_bytes_of(*cm) * sizes[i];
    if (need > left) break;
    left -= need;
    resident[i] = 1;
    target[i] = DOS_ON_GPU;
    ++n_res;
  }
  std::vector<int> movable;  // subgroups that may be staged through the GPU, in index order
  for (int i = 0; i < n_sg; ++i)
    if (!resident[i] && (!cpu_only || !cpu_only[i])) movable.push_back(i);
  const int n_dyn = (int)movable.size();

  // ---- Eq. 1 (reported in both modes)
  const double B = cm->h2d_Bps / 4.0;  // link rate in FP32 parameters per second
  const double inv_dc = cm->downscale_params_per_s > 0 ? 1.0 / cm->downscale_params_per_s : 0.0;
  const double den = 1.0 / cm->cpu_params_per_s + inv_dc - 1.0 / (2.0 * B);
  double k_real = 0.0;
  int k = 0;
  if (den > 0.0) {
    // (the 3 of Eq. 1 is the number of FP32 arrays that cross the link each way)
    k_real = (state_bytes_of(*cm) / 4.0 / B + 1.0 / cm->gpu_params_per_s) / den;
    k = std::max(1, (int)(k_real + 0.5));
  }

  auto cost_of = [&](const std::vector<uint8_t>& t) {
    return evaluate(*cm, sizes, t.data(), resident.data(), n_sg, n_slots, slot_params);
  };

  if (mode == DOS_PLAN_STRIDE) {
    for (int q = 0; q < n_dyn; ++q)
      if (k >= 1 && (q + 1) % k == 0) target[movable[q]] = DOS_ON_GPU;
  } else if (n_dyn <= 16) {
    // few subgroups: every assignment is tried
    std::vector<uint8_t> best = target, cand = target;
    double best_cost = cost_of(best).predicted;
    for (uint32_t bits = 1; bits < (1u << n_dyn); ++bits) {
      for (int q = 0; q < n_dyn; ++q) cand[movable[q]] = (bits >> q) & 1u;
      const double cc = cost_of(cand).predicted;
      if (cc < best_cost) {
        best_cost = cc;
        best = cand;
      }
    }
    target = best;
  } else {
    // evenly spread c GPU subgroups among the dynamic ones (for c = n/k this is
    // Algorithm 1's stride pattern), pick the best count ...
    std::vector<uint8_t> best = target, cand = target;
    double best_cost = cost_of(best).predicted;
    for (int c = 1; c <= n_dyn; ++c) {
      for (int q = 0; q < n_dyn; ++q)
        cand[movable[q]] = ((int64_t)(q + 1) * c / n_dyn > (int64_t)q * c / n_dyn) ? DOS_ON_GPU : DOS_ON_CPU;
      const double cc = cost_of(cand).predicted;
      if (cc < best_cost) {
        best_cost = cc;
        best = cand;
      }
    }
    // ... then improve by single moves and pair swaps while the estimate drops
    // (unequal sizes make the best subset differ from the even spread).
    bool improved = true;
    for (int pass = 0; improved && pass < 64; ++pass) {
      improved = false;
      for (int q = 0; q < n_dyn; ++q) {
        const int i = movable[q];
        best[i] ^= 1;
        const double cc = cost_of(best).predicted;
        if (cc < best_cost * (1.0 - 1e-12)) {
          best_cost = cc;
          improved = true;
        } else {
          best[i] ^= 1;
        }
      }
      if (n_dyn <= 96) {
        for (int qi = 0; qi < n_dyn; ++qi)
          for (int qj = qi + 1; qj < n_dyn; ++qj) {
            const int i = movable[qi], j = movable[qj];
            if (best[i] == best[j] || sizes[i] == sizes[j]) continue;
            std::swap(best[i], best[j]);
            const double cc = cost_of(best).predicted;
            if (cc < best_cost * (1.0 - 1e-12)) {
              best_cost = cc;
              improved = true;
            } else {
              std::swap(best[i], best[j]);
            }
          }
      }
    }
    target = best;
  }

  const Cost c = cost_of(target);
  out->n_sg = n_sg;
  out->n_slots = n_slots;
  out->slot_params = slot_params;
  out->stride_k = k;
  out->stride_k_real = k_real;
  out->predicted_s = c.predicted;
  out->lower_bound_s = c.lower;
  for (int i = 0; i < n_sg; ++i) {
    out->target[i] = target[i];
    out->order[i] = i;
    if (out->resident) out->resident[i] = resident[i];
  }
  return DOS_OK;
}

}  // namespace

extern "C" dos_status dos_plan_subgroups(const dos_cost_model* cm, const uint64_t* sizes, const uint8_t* cpu_only,
                                         int32_t n_sg, uint64_t gpu_budget_bytes, int32_t bytes_per_param_slot,
                                         int32_t mode, int32_t n_resident_max, dos_plan* out) {
  try {  // the work lists are heap-allocated; the caller's arrays are written last, so an error leaves them as they were
    return plan_subgroups(cm, sizes, cpu_only, n_sg, gpu_budget_bytes, bytes_per_param_slot, mode, n_resident_max,
                          out);
  } catch (...) {
    return DOS_ENOMEM;
  }
}

// Feeds one phase's measured lane rates back into the cost model, so that the
// next plan balances the lanes as they really ran (host DRAM contention between
// the host update and the DMA traffic makes both slower than when calibrated
// alone -- the paper observes the same in its CPU-cores-per-GPU study, Section 5.4).
extern "C" dos_status dos_cost_model_observe(dos_cost_model* cm, const dos_phase_stats* st) {
  if (!cm || !st) return DOS_EINVAL;
  if (st->params_cpu > 0 && st->cpu_lane_s > 0.0) {
    // Host lane: least-squares fit of  lane time = a * N_C + b * staged bytes  over the phases
    // seen so far (weights fade by a quarter per phase); rate = 1/a, cost per byte = b/a.
    const double x1 = (double)st->params_cpu * 1e-9;
    const double staged_bytes = std::max(0.0, st->h2d_bytes - 2.0 * (double)st->params_cpu) + st->d2h_bytes;
    const double x2 = staged_bytes * 1e-9, y = st->cpu_lane_s;
    double* f = cm->fit;  // sums of x1*x1, x1*x2, x2*x2, x1*y, x2*y
    for (int i = 0; i < 5; ++i) f[i] = isfinite(f[i]) ? f[i] * 0.75 : 0.0;
    f[0] += x1 * x1; f[1] += x1 * x2; f[2] += x2 * x2; f[3] += x1 * y; f[4] += x2 * y;
    const double det = f[0] * f[2] - f[1] * f[1];
    bool fitted = false;
    if (f[2] > 0.0 && det > 1e-4 * f[0] * f[2]) {  // phases with different splits have been seen
      const double a = (f[3] * f[2] - f[4] * f[1]) / det, b = (f[4] * f[0] - f[3] * f[1]) / det;
      if (a > 0.0 && b >= 0.0) {
        cm->cpu_params_per_s = 1e9 / a;
        // a byte of traffic cannot displace much more host work than the update's own bytes per
        // parameter allow (about 1/32); a larger fit is measurement noise on nearly equal splits
        cm->cpu_cost_per_dma_byte = std::min(b / a, 0.125);
        fitted = true;
      } else if (a > 0.0 && f[3] > 0.0) {  // staging did not slow the host lane down: no cost
        cm->cpu_params_per_s = 1e9 * f[0] / f[3];
        cm->cpu_cost_per_dma_byte = 0.0;
        fitted = true;
      }
    }
    // one split only (or a fit that makes no sense): the cost keeps its value, the rate explains this phase
    if (!fitted) cm->cpu_params_per_s = ((double)st->params_cpu + cm->cpu_cost_per_dma_byte * staged_bytes) / y;
  }
  if (st->params_gpu > 0 && st->h2d_busy_s > 0.0 && st->d2h_busy_s > 0.0) {
    // summed copy durations (DOS_CTX_PROFILE) give the rate each direction reached while busy.
    // The 16-bit uploads of the host lane share the host-to-device direction with the
    // prefetches and the cost model charges them to it, so the bytes they moved while
    // prefetches were running count towards its rate (uploads are spread evenly over the
    // host lane).
    const double uploads = 2.0 * (double)st->params_cpu;
    const double staged = st->h2d_bytes - uploads;  // bytes the prefetches moved
    const double share = st->cpu_lane_s > 0.0 ? std::min(1.0, st->h2d_busy_s / st->cpu_lane_s) : 0.0;
    cm->h2d_Bps = (staged + uploads * share) / st->h2d_busy_s;
    cm->d2h_Bps = st->d2h_bytes / st->d2h_busy_s;
    // The lane as a whole may have run longer than its busier direction explains
    // (a direction idles while it waits for the other one's piece): both rates are
    // lowered so that the model reproduces the lane time of the phase it was fed.
    const double lane = std::max(st->h2d_bytes / cm->h2d_Bps, st->d2h_bytes / cm->d2h_Bps);
    if (st->gpu_lane_s > lane && lane > 0.0) {
      cm->h2d_Bps *= lane / st->gpu_lane_s;
      cm->d2h_Bps *= lane / st->gpu_lane_s;
    }
  } else if (st->params_gpu > 0 && st->gpu_lane_s > 0.0 && st->d2h_bytes > 0.0) {
    // without per-copy timing: the lane as a whole bounds both directions
    const double rate = st->d2h_bytes / st->gpu_lane_s;
    if (rate < cm->d2h_Bps) cm->d2h_Bps = rate;
    if (rate < cm->h2d_Bps) cm->h2d_Bps = rate;
  }
  return DOS_OK;
}
