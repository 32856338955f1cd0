"""Pins for the planner reference (oracle/plan_ref.py): the numbers and the
placement the paper itself prints."""
import os

import pytest

from oracle import plan_ref as ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_second_machine_worked_example():
    """Section 5.4: B=3, U_g=35, U_c=2, D_c=8.7 G params/s 'results in k=2'."""
    (B, Ug, Uc, Dc, k_paper), = rows("perf_model_second_machine.txt")
    B, Ug, Uc, Dc = (float(x) * 1e9 for x in (B, Ug, Uc, Dc))
    k = ref.stride_k_real(B, Ug, Uc, Dc)
    assert k == pytest.approx(2.2945, abs=5e-4)      # (3/3 + 1/35) / (1/2 + 1/8.7 - 1/6)
    assert ref.stride_k(B, Ug, Uc, Dc) == int(k_paper)


def test_eq1_balances_host_time_against_link_plus_gpu_time():
    """Eq. 1 itself: k (S/U_c + S/D_c) = 3S/B + kS/(2B) + S/U_g at the solution,
    for any subgroup size S (Section 4.2: k does not depend on S)."""
    B, Ug, Uc, Dc = 4.6e9, 180e9, 1.5e9, 20e9
    k = ref.stride_k_real(B, Ug, Uc, Dc)
    for S in (1e6, 1e8, 4e8):
        lhs = k * (S / Uc + S / Dc)
        rhs = max(3 * S / B, 3 * S / B + k * S / (2 * B)) + S / Ug
        assert lhs == pytest.approx(rhs, rel=1e-12)
    # units: scaling every rate by the same factor leaves k unchanged
    assert ref.stride_k_real(2 * B, 2 * Ug, 2 * Uc, 2 * Dc) == pytest.approx(k, rel=1e-12)


def test_faster_host_means_larger_stride_and_faster_link_smaller():
    base = dict(B=3e9, U_g=35e9, U_c=2e9, D_c=8.7e9)
    k0 = ref.stride_k_real(**base)
    assert ref.stride_k_real(**{**base, "U_c": 4e9}) > k0
    assert ref.stride_k_real(**{**base, "D_c": 20e9}) > k0
    assert ref.stride_k_real(**{**base, "B": 6e9}) < k0
    assert ref.stride_k_real(**{**base, "U_g": 70e9}) < k0


def test_stride_two_is_every_alternate_subgroup():
    """Sections 5.3 / 5.4: k=2, i.e. every alternate subgroup, 50 % on the GPU."""
    t = ref.stride_targets(10, 2)
    assert t == [0, 1] * 5
    assert sum(t) / len(t) == 0.5
    assert ref.stride_targets(5, 1) == [1] * 5            # k=1: everything on the GPU
    assert ref.stride_targets(5, 0) == [0] * 5            # marker for 'never'


def test_update_figure_timeline():
    """Section 4.1 update-step figure: 8 subgroups, one GPU update for every two
    CPU updates, S7 and S8 resident and placed last."""
    (n, k, res, gpu), = rows("update_timeline_8_subgroups.txt")
    n, k = int(n), int(k)
    res = [int(x) for x in res.split(",")]
    gpu = [int(x) for x in gpu.split(",")]
    t = ref.stride_targets(n, k, res)
    assert [i for i, x in enumerate(t) if x == ref.ON_GPU] == gpu
    # the dynamic part is 33 %: one in three of the non-resident subgroups
    dyn = [x for i, x in enumerate(t) if i not in res]
    assert sum(dyn) / len(dyn) == pytest.approx(1 / 3)
    trace = ref.run_update_trace(n, k, res)
    # order of the update actions follows the subgroup order
    upd = [(a, i) for a, i in trace if a in ("gpu_update", "cpu_update")]
    assert upd == [("cpu_update", 0), ("cpu_update", 1), ("gpu_update", 2), ("cpu_update", 3),
                   ("cpu_update", 4), ("gpu_update", 5), ("gpu_update", 6), ("gpu_update", 7)]
    # while S3 (index 2) is on the GPU, the two CPU-updated subgroups before it
    # are handed to the downscale; after it, S3 is flushed and S6 prefetched
    # before the CPU carries on with S4
    i = trace.index(("gpu_update", 2))
    assert trace[i + 1] == ("cpu_downscale", [0, 1])
    assert trace[i + 2:i + 5] == [("flush_out", 2), ("prefetch_in", 5), ("cpu_update", 3)]
    # the very first step prefetches the first GPU subgroup while the CPU starts
    assert trace[0] == ("prefetch_in", 2) and trace[1] == ("cpu_update", 0)


def test_every_subgroup_is_updated_exactly_once():
    for n in (1, 2, 7, 16):
        for k in (0, 1, 2, 3, 5):
            for res in ((), (n - 1,), tuple(range(max(0, n - 2), n))):
                tr = ref.run_update_trace(n, k, res)
                upd = sorted(i for a, i in tr if a in ("gpu_update", "cpu_update"))
                assert upd == list(range(n))
                tgt = ref.stride_targets(n, k, res)
                for a, i in tr:
                    if a == "gpu_update":
                        assert tgt[i] == ref.ON_GPU
                    if a == "cpu_update":
                        assert tgt[i] == ref.ON_CPU


COST = dict(h2d_Bps=55e9, d2h_Bps=50e9, gpu_params_per_s=200e9, cpu_params_per_s=1.5e9,
            launch_overhead_s=10e-6, n_slots=3)


def test_cost_function_limits():
    sizes = [100_000_000] * 10
    all_cpu, lb0 = ref.phase_cost(sizes, [0] * 10, **COST)
    assert all_cpu == pytest.approx(1e9 / 1.5e9)
    assert lb0 == pytest.approx(2e9 / 55e9)
    all_gpu, lb1 = ref.phase_cost(sizes, [1] * 10, **COST)
    assert lb1 == pytest.approx(12e9 / 50e9)
    assert all_gpu >= lb1
    # one slot serialises prefetch, kernel and flush
    one, _ = ref.phase_cost(sizes, [1] * 10, **{**COST, "n_slots": 1})
    assert one == pytest.approx(12e9 / 55e9 + 12e9 / 50e9 + 1e9 / 200e9 + 10 * 10e-6)


def test_brute_force_beats_both_extremes():
    sizes = [100_000_000] * 8
    best, tgt = ref.brute_force_plan(sizes, **COST)
    assert best < ref.phase_cost(sizes, [0] * 8, **COST)[0]
    assert best <= ref.phase_cost(sizes, [1] * 8, **COST)[0]
    assert 0 < sum(tgt) <= 8
