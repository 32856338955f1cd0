// Exercises the host-only parts of libdos (planner, host AdamW) under the
// sanitizers: built by tests/test_sanitizers.py with g++ -fsanitize=..., linked
// with plan.cpp and adam_host.cpp only (no HIP).  Exit status 0 = no finding.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <random>
#include <vector>

#include "dos.h"

namespace dos {
void note_hip_error(int, const char*) {}  // the HIP-facing units are not linked here
}

static int fail(const char* what) {
  fprintf(stderr, "host_driver: %s\n", what);
  return 1;
}

int main() {
  std::mt19937_64 rng(241021316);
  // ---- planner: both modes, with and without residents, many shapes
  for (int it = 0; it < 300; ++it) {
    const int n = (int)(rng() % 140);
    std::vector<uint64_t> sizes(n);
    for (auto& s : sizes) s = (1u << 20) + rng() % (300u << 20);
    dos_cost_model cm{(10.0 + rng() % 50) * 1e9, (10.0 + rng() % 50) * 1e9, (20.0 + rng() % 200) * 1e9,
                      (0.3 + rng() % 20) * 1e9, (rng() % 2) ? 8.7e9 : 0.0, 5e-6};
    std::vector<uint8_t> target(n + 1), resident(n + 1);
    std::vector<int32_t> order(n + 1);
    dos_plan plan{};
    plan.target = target.data();
    plan.order = order.data();
    plan.resident = resident.data();
    const uint64_t budget = (uint64_t)(1 + rng() % 64) * 1000000000ull;
    std::vector<uint8_t> cpu_only(n + 1);
    for (auto& f : cpu_only) f = (uint8_t)(rng() % 3 == 0);
    const dos_status rc = dos_plan_subgroups(&cm, sizes.data(), (rng() % 2) ? cpu_only.data() : nullptr, n, budget, (rng() % 2) ? 12 : 14, (int)(rng() % 2),
                                             (int)(rng() % (n + 1)), &plan);
    if (rc != DOS_OK) return fail("dos_plan_subgroups failed");
    double pred = 0, low = 0;
    if (dos_plan_cost(&cm, sizes.data(), target.data(), resident.data(), n, plan.n_slots, plan.slot_params, &pred,
                      &low) != DOS_OK)
      return fail("dos_plan_cost failed");
    if (n > 0 && !(pred == plan.predicted_s)) return fail("plan and cost disagree");
    dos_phase_stats st{};
    st.params_cpu = 1000;
    st.cpu_lane_s = 1e-3;
    if (dos_cost_model_observe(&cm, &st) != DOS_OK) return fail("dos_cost_model_observe failed");
  }
  // ---- host AdamW: ragged sizes, several thread counts, exact-size heap blocks so
  // that any access past the end is caught
  const uint64_t ns[] = {1, 3, 15, 16, 17, 63, 64, 65, 1000, 4097, 65536, 65537, 200003};
  for (uint64_t n : ns) {
    for (int threads : {1, 2, 5, 16}) {
      // 16-byte aligned, exactly n elements each
      float *p, *m, *v;
      uint16_t *g, *lp;
      if (posix_memalign((void**)&p, 16, n * 4) || posix_memalign((void**)&m, 16, n * 4) ||
          posix_memalign((void**)&v, 16, n * 4) || posix_memalign((void**)&g, 16, n * 2) ||
          posix_memalign((void**)&lp, 16, n * 2))
        return fail("allocation failed");
      for (uint64_t i = 0; i < n; ++i) {
        p[i] = 0.01f * (float)((int)(rng() % 200) - 100);
        m[i] = 0.0f;
        v[i] = 0.0f;
        g[i] = (uint16_t)(0x3A00 + rng() % 256);
        lp[i] = 0;
      }
      dos_subgroup sg{p, m, v, g, lp, n, DOS_HOST_PINNED, DOS_HOST_PINNED};
      for (int64_t step = 1; step <= 3; ++step) {
        dos_hparams hp{1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, step};
        if (dos_adam_step_host(&sg, &hp, threads) != DOS_OK) return fail("dos_adam_step_host failed");
      }
      double acc = 0;
      for (uint64_t i = 0; i < n; ++i) acc += v[i] + lp[i];
      if (!(acc > 0)) return fail("nothing was updated");
      free(p); free(m); free(v); free(g); free(lp);
    }
  }
  // ---- argument errors
  dos_hparams bad{1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 0};
  dos_subgroup empty{nullptr, nullptr, nullptr, nullptr, nullptr, 0, DOS_HOST_PINNED, DOS_HOST_PINNED};
  if (dos_adam_step_host(&empty, &bad, 1) != DOS_EINVAL) return fail("step 0 accepted");
  printf("host_driver ok\n");
  return 0;
}
