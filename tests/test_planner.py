"""dos_plan_subgroups / dos_plan_cost (host-only part of the C ABI) against the
planner reference: Eq. 1 and Algorithm 1's stride placement, the cost function,
and the balanced mode against brute force."""
import ctypes as C
import random

import pytest

import paper_2410_21316_amd as dos
from oracle import plan_ref as ref

G = 1e9


def cm_from_paper_units(B, Ug, Uc, Dc):
    """The paper quotes all four rates in FP32 parameters per second; the C ABI
    takes the link in bytes per second (4 bytes per FP32 parameter)."""
    return dos.cost_model(4 * B, 4 * B, Ug, Uc, Dc, 0.0)


def test_stride_mode_reproduces_the_papers_worked_example():
    """Section 5.4: (B, U_g, U_c, D_c) = (3, 35, 2, 8.7) G params/s gives k = 2,
    'every alternate subgroup'."""
    cm = cm_from_paper_units(3 * G, 35 * G, 2 * G, 8.7 * G)
    sizes = [100_000_000] * 70
    plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, dos.DOS_PLAN_STRIDE)
    assert plan.c.stride_k == 2
    assert plan.c.stride_k_real == pytest.approx(ref.stride_k_real(3 * G, 35 * G, 2 * G, 8.7 * G), rel=1e-12)
    assert plan.c.stride_k_real == pytest.approx(2.2945, abs=5e-4)
    assert plan.targets == ref.stride_targets(70, 2)
    assert plan.orders == list(range(70))
    assert sum(plan.targets) == 35                     # 50 % on the GPU


@pytest.mark.parametrize("rates", [(4.6, 180, 1.5, 20), (14, 190, 7.5, 0), (3, 35, 2, 8.7), (12, 25, 8, 15.5),
                                   (1, 100, 0.3, 5), (50, 200, 100, 0)])
def test_stride_mode_matches_reference_for_any_rates(rates):
    B, Ug, Uc, Dc = (x * G for x in rates)
    cm = cm_from_paper_units(B, Ug, Uc, Dc)
    for n_sg in (1, 2, 7, 33, 130):
        plan = dos.dos_plan_subgroups(cm, [50_000_000] * n_sg, 8 * 10**9, dos.DOS_PLAN_STRIDE)
        k = ref.stride_k(B, Ug, Uc, Dc if Dc else float("inf"))
        assert plan.c.stride_k == k
        assert plan.targets == ref.stride_targets(n_sg, k)


def test_stride_does_not_depend_on_subgroup_size():
    """Section 4.2: k is independent of the subgroup size."""
    cm = cm_from_paper_units(3 * G, 35 * G, 2 * G, 8.7 * G)
    base = dos.dos_plan_subgroups(cm, [100_000_000] * 24, 64 * 10**9, dos.DOS_PLAN_STRIDE)
    for scale in (0.5, 2, 4, 10):
        other = dos.dos_plan_subgroups(cm, [int(100_000_000 * scale)] * 24, 64 * 10**9, dos.DOS_PLAN_STRIDE)
        assert other.targets == base.targets and other.c.stride_k == base.c.stride_k


def test_update_figure_placement_with_residents_last():
    """Section 4.1 figure: 8 subgroups, stride 3, two static residents placed
    last -> GPU set {S3, S6, S7, S8}.  Rates chosen so that Eq. 1 gives 3."""
    B, Ug, Uc, Dc = 3 * G, 35 * G, 2.8 * G, 8.7 * G
    assert ref.stride_k(B, Ug, Uc, Dc) == 3
    sizes = [10_000_000] * 8
    slots = 3 * 12 * 10_000_000
    plan = dos.dos_plan_subgroups(cm_from_paper_units(B, Ug, Uc, Dc), sizes, slots + 2 * 12 * 10_000_000,
                                  dos.DOS_PLAN_STRIDE, n_resident_max=2)
    assert plan.residents == [0, 0, 0, 0, 0, 0, 1, 1]
    assert [i for i, t in enumerate(plan.targets) if t] == [2, 5, 6, 7]
    assert plan.targets == ref.stride_targets(8, 3, residents=(6, 7))


COST = dict(h2d_Bps=55e9, d2h_Bps=48e9, gpu_params_per_s=190e9, cpu_params_per_s=7e9, launch_overhead_s=8e-6)


def test_cost_function_matches_reference():
    """dos_plan_cost against the reference's estimate for random assignments, slot counts, piece sizes,
    residents, both state widths (three arrays for AdamW, two for Adagrad / RMSProp) and with and without
    the charge for what staged traffic takes away from the host lane."""
    rng = random.Random(7)
    for _ in range(400):
        arrays = rng.choice([3, 3, 2])
        contention = rng.choice([0.0, 0.0, 0.01, 0.04, 0.11])
        cm = dos.cost_model(COST["h2d_Bps"], COST["d2h_Bps"], COST["gpu_params_per_s"], COST["cpu_params_per_s"], 0.0,
                            COST["launch_overhead_s"], fp32_arrays=arrays, cpu_cost_per_dma_byte=contention)
        n = rng.randint(1, 14)
        sizes = [rng.randint(1, 400) * 1_000_000 for _ in range(n)]
        tgt = [rng.randint(0, 1) for _ in range(n)]
        n_res = rng.randint(0, 2)
        res = [0] * n
        for i in range(n - 1, max(-1, n - 1 - n_res), -1):
            res[i] = 1
            tgt[i] = 1
        slots = rng.choice([1, 2, 3])
        sp = rng.choice([0, 16 << 20])
        got = dos.dos_plan_cost(cm, sizes, tgt, slots, res, sp)
        want = ref.phase_cost(sizes, tgt, n_slots=slots, resident=[i for i in range(n) if res[i]], slot_params=sp,
                              fp32_arrays=arrays, cpu_cost_per_dma_byte=contention, **COST)
        assert got[0] == pytest.approx(want[0], rel=1e-12)
        assert got[1] == pytest.approx(want[1], rel=1e-12)


@pytest.mark.parametrize("seed", range(8))
def test_balanced_mode_with_contention_and_two_arrays_finds_the_brute_force_optimum(seed):
    """The same exhaustive check with the two product terms the first one leaves at their defaults."""
    rng = random.Random(1000 + seed)
    n = rng.randint(4, 11)
    sizes = [rng.randint(40, 160) * 1_000_000 for _ in range(n)]
    cost = dict(COST)
    cost["cpu_params_per_s"] = rng.choice([1e9, 3e9, 7e9, 14e9])
    extra = dict(fp32_arrays=rng.choice([2, 3]), cpu_cost_per_dma_byte=rng.choice([0.0, 0.01, 0.03, 0.06]))
    cm = dos.cost_model(cost["h2d_Bps"], cost["d2h_Bps"], cost["gpu_params_per_s"], cost["cpu_params_per_s"], 0.0,
                        cost["launch_overhead_s"], **extra)
    plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, dos.DOS_PLAN_BALANCED)
    best, _ = ref.brute_force_plan(sizes, n_slots=plan.c.n_slots, slot_params=plan.c.slot_params, **cost, **extra)
    mine, low = ref.phase_cost(sizes, plan.targets, n_slots=plan.c.n_slots, slot_params=plan.c.slot_params, **cost,
                               **extra)
    assert plan.c.predicted_s == pytest.approx(mine, rel=1e-12)
    assert plan.c.lower_bound_s == pytest.approx(low, rel=1e-12)
    assert mine <= best * (1 + 1e-12)


@pytest.mark.parametrize("seed", range(12))
def test_balanced_mode_is_close_to_the_brute_force_optimum(seed):
    """For up to 12 subgroups of random, unequal sizes the planner finds the
    exhaustive optimum of the cost function."""
    rng = random.Random(seed)
    n = rng.randint(4, 12)
    sizes = [rng.randint(40, 160) * 1_000_000 for _ in range(n)]
    cost = dict(COST)
    cost["cpu_params_per_s"] = rng.choice([1e9, 3e9, 7e9, 20e9])
    cost["d2h_Bps"] = rng.choice([24e9, 48e9])
    cm = dos.cost_model(cost["h2d_Bps"], cost["d2h_Bps"], cost["gpu_params_per_s"], cost["cpu_params_per_s"], 0.0,
                        cost["launch_overhead_s"])
    plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, dos.DOS_PLAN_BALANCED)
    best, _ = ref.brute_force_plan(sizes, n_slots=plan.c.n_slots, slot_params=plan.c.slot_params, **cost)
    mine, low = ref.phase_cost(sizes, plan.targets, n_slots=plan.c.n_slots, slot_params=plan.c.slot_params, **cost)
    assert plan.c.predicted_s == pytest.approx(mine, rel=1e-12)
    assert plan.c.lower_bound_s == pytest.approx(low, rel=1e-12)
    assert mine <= best * (1 + 1e-12)


def test_balanced_mode_heuristic_gap_beyond_sixteen_subgroups():
    """18 unequal subgroups (heuristic search): within 5 % of brute force."""
    rng = random.Random(99)
    sizes = [rng.randint(40, 160) * 1_000_000 for _ in range(18)]
    cm = dos.cost_model(COST["h2d_Bps"], COST["d2h_Bps"], COST["gpu_params_per_s"], 3e9, 0.0, COST["launch_overhead_s"])
    plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, dos.DOS_PLAN_BALANCED)
    cost = {**COST, "cpu_params_per_s": 3e9}
    best, _ = ref.brute_force_plan(sizes, n_slots=plan.c.n_slots, slot_params=plan.c.slot_params, **cost)
    assert plan.c.predicted_s <= best * 1.05


def test_balanced_mode_on_equal_subgroups_beats_every_stride():
    sizes = [100_000_000] * 130
    cm = dos.cost_model(55e9, 48e9, 190e9, 7e9, 0.0, 8e-6)
    plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, dos.DOS_PLAN_BALANCED)
    for k in range(1, 9):
        t = ref.stride_targets(130, k)
        c, _ = ref.phase_cost(sizes, t, n_slots=plan.c.n_slots, slot_params=plan.c.slot_params,
                              **{**COST, "cpu_params_per_s": 7e9})
        assert plan.c.predicted_s <= c * (1 + 1e-12)
    # the GPU subgroups are spread through the order, not bunched at one end
    g = [i for i, t in enumerate(plan.targets) if t]
    assert 0 < len(g) < 130
    gaps = [b - a for a, b in zip(g, g[1:])]
    assert max(gaps) <= 2 * (130 // len(g) + 1)


def test_slots_follow_the_budget():
    cm = dos.cost_model(55e9, 48e9, 190e9, 7e9)
    sizes = [100_000_000] * 10
    p = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9)
    assert (p.c.n_slots, p.c.slot_params) == (3, 16 << 20)              # pieces of 16 Mi parameters
    p = dos.dos_plan_subgroups(cm, [1_000_000] * 10, 40 * 10**9)
    assert (p.c.n_slots, p.c.slot_params) == (3, 1_000_000)             # whole (small) subgroups
    p = dos.dos_plan_subgroups(cm, [1_000_001] * 10, 40 * 10**9)
    assert p.c.slot_params == 1_000_064                                  # padded to 64 elements
    p = dos.dos_plan_subgroups(cm, sizes, 2 * 12 * (16 << 20))
    assert (p.c.n_slots, p.c.slot_params) == (2, 16 << 20)
    p = dos.dos_plan_subgroups(cm, sizes, 100 * 10**6)                   # ~8.3M parameters of staging in all
    assert p.c.n_slots == 3 and p.c.slot_params == (100 * 10**6 // 36) // 65536 * 65536
    p = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, bytes_per_param_slot=14)
    assert p.c.n_slots == 3
    with pytest.raises(dos.DosError) as e:
        dos.dos_plan_subgroups(cm, sizes, 1_000_000)
    assert e.value.status == dos.DOS_EBUDGET


def test_residents_take_what_the_budget_leaves():
    cm = dos.cost_model(55e9, 48e9, 190e9, 7e9)
    sizes = [100_000_000] * 130
    p = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, n_resident_max=130)
    staging = 3 * 12 * (16 << 20)
    n_res = (40 * 10**9 - staging) // (12 * 100_000_000)
    assert sum(p.residents) == n_res == 32
    assert p.residents == [0] * (130 - n_res) + [1] * n_res              # placed last (Section 4.1)
    assert all(t == 1 for t, r in zip(p.targets, p.residents) if r)
    p0 = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, n_resident_max=0)
    assert p.c.predicted_s < p0.c.predicted_s and sum(p0.residents) == 0
    p5 = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, n_resident_max=5)
    assert sum(p5.residents) == 5


def test_planner_rejects_bad_arguments():
    lib = dos.load()
    cm = dos.cost_model(55e9, 48e9, 190e9, 7e9)
    sizes = (C.c_uint64 * 4)(*[1 << 20] * 4)
    pl = dos.Plan(4)

    def call(cm_=cm, n=4, budget=10**9, bpp=12, mode=1, nres=0, out=pl.c, sz=sizes):
        return lib.dos_plan_subgroups(C.byref(cm_) if cm_ is not None else None, sz, None, n, budget, bpp, mode, nres,
                                      C.byref(out) if out is not None else None)

    assert call() == dos.DOS_OK
    assert call(cm_=None) == dos.DOS_EINVAL
    assert call(out=None) == dos.DOS_EINVAL
    assert call(n=-1) == dos.DOS_EINVAL
    assert call(mode=2) == dos.DOS_EINVAL
    assert call(bpp=13) == dos.DOS_EINVAL
    assert call(nres=-1) == dos.DOS_EINVAL
    assert call(sz=None) == dos.DOS_EINVAL
    assert call(budget=0) == dos.DOS_EBUDGET
    for field in ("h2d_Bps", "d2h_Bps", "gpu_params_per_s", "cpu_params_per_s"):
        bad = dos.cost_model(55e9, 48e9, 190e9, 7e9)
        setattr(bad, field, 0.0)
        assert call(cm_=bad) == dos.DOS_EINVAL
        setattr(bad, field, float("nan"))
        assert call(cm_=bad) == dos.DOS_EINVAL
    assert call(n=0) == dos.DOS_OK and pl.c.n_sg == 0


def test_planner_is_deterministic():
    cm = dos.cost_model(55e9, 48e9, 190e9, 3e9)
    sizes = [random.Random(3).randint(50, 150) * 1_000_000 for _ in range(40)]
    a = dos.dos_plan_subgroups(cm, sizes, 16 * 10**9)
    b = dos.dos_plan_subgroups(cm, sizes, 16 * 10**9)
    assert a.targets == b.targets and a.c.predicted_s == b.c.predicted_s


def test_cost_model_observe_takes_the_measured_rates():
    cm = dos.cost_model(56e9, 48e9, 200e9, 8e9)
    st = dos.dos_phase_stats()
    st.params_cpu, st.cpu_lane_s = 3_600_000_000, 0.45
    st.params_gpu = 1_300_000_000
    st.h2d_bytes = 12.0 * st.params_gpu + 2.0 * st.params_cpu
    st.d2h_bytes = 12.0 * st.params_gpu
    st.h2d_busy_s, st.d2h_busy_s, st.gpu_lane_s = 0.40, 0.43, 0.43
    dos.dos_cost_model_observe(cm, st)
    assert cm.cpu_params_per_s == pytest.approx(8e9)
    # prefetch bytes plus the share of the 16-bit uploads that ran while prefetches were busy
    assert cm.h2d_Bps == pytest.approx((12.0 * 1.3e9 + 2.0 * 3.6e9 * (0.40 / 0.45)) / 0.40)
    assert cm.d2h_Bps == pytest.approx(12.0 * 1.3e9 / 0.43)
    assert cm.gpu_params_per_s == 200e9
    # the model is then consistent with the phase it was taken from: the host-to-device time it
    # predicts for the same plan is the time that direction was busy, stretched to the host lane
    assert (st.h2d_bytes / cm.h2d_Bps) == pytest.approx(0.40 * st.h2d_bytes / (12.0 * 1.3e9 + 7.2e9 * 0.40 / 0.45))
    # uploads never outlast the host lane: a prefetch stream busier than the host lane gets all of them
    cm1 = dos.cost_model(56e9, 48e9, 200e9, 8e9)
    st.h2d_busy_s = 0.50
    dos.dos_cost_model_observe(cm1, st)
    assert cm1.h2d_Bps == pytest.approx(st.h2d_bytes / 0.50)
    st.h2d_busy_s = 0.40
    # a lane that ran longer than its busier direction explains lowers both rates by the same factor,
    # so that the model gives back the lane time it was fed
    cm4 = dos.cost_model(56e9, 48e9, 200e9, 8e9)
    st.gpu_lane_s = 0.50
    dos.dos_cost_model_observe(cm4, st)
    assert max(st.h2d_bytes / cm4.h2d_Bps, st.d2h_bytes / cm4.d2h_Bps) == pytest.approx(0.50)
    assert cm4.h2d_Bps / cm4.d2h_Bps == pytest.approx(cm.h2d_Bps / cm.d2h_Bps)
    st.gpu_lane_s = 0.46
    # without per-copy timing only an upper bound on the time is known: rates may only drop
    cm2 = dos.cost_model(56e9, 48e9, 200e9, 8e9)
    st.h2d_busy_s = st.d2h_busy_s = -1.0
    dos.dos_cost_model_observe(cm2, st)
    assert cm2.d2h_Bps == pytest.approx(12.0 * 1.3e9 / 0.46) and cm2.h2d_Bps == pytest.approx(12.0 * 1.3e9 / 0.46)
    # nothing measured on a lane: that lane's rate stays
    cm3 = dos.cost_model(56e9, 48e9, 200e9, 8e9)
    dos.dos_cost_model_observe(cm3, dos.dos_phase_stats())
    assert (cm3.h2d_Bps, cm3.d2h_Bps, cm3.cpu_params_per_s) == (56e9, 48e9, 8e9)
    lib = dos.load()
    assert lib.dos_cost_model_observe(None, C.byref(st)) == dos.DOS_EINVAL


def test_two_array_rules_move_eight_bytes_per_parameter():
    """Adagrad and RMSProp keep p and v only (Section 4.1 names them next to Adam): the link terms of
    the estimate and of Eq. 1 shrink from three FP32 arrays to two, and residents need 8 B/param."""
    sizes = [100_000_000] * 20
    tg = [i % 2 for i in range(20)]
    cm3 = dos.cost_model(50e9, 40e9, 200e9, 4e9)
    cm2 = dos.cost_model(50e9, 40e9, 200e9, 4e9, fp32_arrays=2)
    assert dos.cost_model(50e9, 40e9, 200e9, 4e9, fp32_arrays=0).fp32_arrays == 0   # 0 means 3
    p3, l3 = dos.dos_plan_cost(cm3, sizes, tg, 3, None, 16 << 20)
    p2, l2 = dos.dos_plan_cost(cm2, sizes, tg, 3, None, 16 << 20)
    p0, l0 = dos.dos_plan_cost(dos.cost_model(50e9, 40e9, 200e9, 4e9, fp32_arrays=0), sizes, tg, 3, None, 16 << 20)
    assert (p0, l0) == (p3, l3)
    ng = nc = 1e9
    assert l3 == pytest.approx(max((12 * ng + 2 * nc) / 50e9, 12 * ng / 40e9))
    assert l2 == pytest.approx(max((8 * ng + 2 * nc) / 50e9, 8 * ng / 40e9))
    # Eq. 1 with two arrays: k = (2/B + 1/U_g) / (1/U_c - 1/(2B)), B in parameters per second
    B = 50e9 / 4
    plan = dos.dos_plan_subgroups(cm2, sizes, 4 * 10**9, dos.DOS_PLAN_STRIDE)
    assert plan.c.stride_k_real == pytest.approx((2 / B + 1 / 200e9) / (1 / 4e9 - 1 / (2 * B)))
    # cheaper staging moves more subgroups to the GPU
    n3 = sum(dos.dos_plan_subgroups(cm3, sizes, 4 * 10**9).targets)
    n2 = sum(dos.dos_plan_subgroups(cm2, sizes, 4 * 10**9).targets)
    assert n2 > n3 > 0
    # residents: 8 bytes per parameter of budget each
    budget = 3 * 12 * (16 << 20) + 5 * 8 * 100_000_000
    assert sum(dos.dos_plan_subgroups(cm2, sizes, budget, n_resident_max=20).residents) == 5
    assert sum(dos.dos_plan_subgroups(cm3, sizes, budget, n_resident_max=20).residents) == 3
    bad = dos.cost_model(50e9, 40e9, 200e9, 4e9, fp32_arrays=4)
    with pytest.raises(dos.DosError):
        dos.dos_plan_subgroups(bad, sizes, 4 * 10**9)


def _phase(n_c, n_g, u0, beta, t_gpu_lane=None):
    """Stats of a phase on a machine whose host lane takes (N_C + beta * staged bytes) / u0."""
    st = dos.dos_phase_stats()
    st.params_cpu, st.params_gpu = int(n_c), int(n_g)
    st.h2d_bytes = 12.0 * n_g + 2.0 * n_c
    st.d2h_bytes = 12.0 * n_g
    st.cpu_lane_s = (n_c + beta * 24.0 * n_g) / u0
    st.h2d_busy_s = st.d2h_busy_s = -1.0
    st.gpu_lane_s = t_gpu_lane if t_gpu_lane is not None else st.cpu_lane_s
    return st


def test_observe_separates_the_host_rate_from_what_staging_costs_it():
    """Both lanes share the host's memory system (Section 5.4 of the paper sees the same contention).
    From phases with different splits the feedback recovers the host cores' own rate and the host work
    that a staged byte takes away; the planner then stops staging where it costs more than it saves."""
    u0, beta = 12.0e9, 0.035
    cm = dos.cost_model(56e9, 48e9, 230e9, 15e9)                 # calibrated stand-alone: optimistic
    dos.dos_cost_model_observe(cm, _phase(9.0e9, 4.0e9, u0, beta))
    # one split: the cost keeps its value (0), the rate alone explains the phase
    assert cm.cpu_cost_per_dma_byte == 0.0
    assert cm.cpu_params_per_s == pytest.approx(9.0e9 / ((9.0e9 + beta * 96e9) / u0))
    dos.dos_cost_model_observe(cm, _phase(11.0e9, 2.0e9, u0, beta))
    assert cm.cpu_params_per_s == pytest.approx(u0, rel=1e-6)
    assert cm.cpu_cost_per_dma_byte == pytest.approx(beta, rel=1e-6)
    # more phases of the same machine keep the fit where it is, also when the split no longer changes
    for _ in range(6):
        dos.dos_cost_model_observe(cm, _phase(11.0e9, 2.0e9, u0, beta))
    assert cm.cpu_params_per_s == pytest.approx(u0, rel=1e-3) and cm.cpu_cost_per_dma_byte == pytest.approx(beta, rel=1e-3)
    # an all-CPU phase fits the same line
    dos.dos_cost_model_observe(cm, _phase(13.0e9, 0.0, u0, beta))
    assert cm.cpu_params_per_s == pytest.approx(u0, rel=1e-3)
    # the machine changes (another tenant takes memory bandwidth): the fit follows within a few phases
    for k in range(12):
        dos.dos_cost_model_observe(cm, _phase(10.0e9 + 1e9 * (k % 3), 3.0e9 - 1e9 * (k % 3), 9.0e9, 0.02))
    assert cm.cpu_params_per_s == pytest.approx(9.0e9, rel=0.02) and cm.cpu_cost_per_dma_byte == pytest.approx(0.02, rel=0.1)


def test_planner_prices_contention_and_falls_back_to_the_host_cores():
    sizes = [100_000_000] * 40
    tg = [1 if i % 4 == 0 else 0 for i in range(40)]
    ng, nc = 1.0e9, 3.0e9
    cm = dos.cost_model(56e9, 48e9, 230e9, 12e9, cpu_cost_per_dma_byte=0.03)
    pred, low = dos.dos_plan_cost(cm, sizes, tg, 3, None, 16 << 20)
    lead = 12.0 * (16 << 20) / 56e9 + (16 << 20) / 230e9
    want = max((nc + 0.03 * 24.0 * ng) / 12e9, (12 * ng + 2 * nc) / 56e9, lead + 12 * ng / 48e9)
    assert pred == pytest.approx(want) and low == pytest.approx(max((12 * ng + 2 * nc) / 56e9, 12 * ng / 48e9))
    # a staged subgroup takes 24 B/param of traffic: at more than 1/24 parameters per byte it costs the host
    # lane more work than it removes, and the balanced plan keeps everything on the host cores
    for cost, staged in ((0.0, True), (0.02, True), (0.045, False), (0.2, False)):
        cm = dos.cost_model(56e9, 48e9, 230e9, 12e9, cpu_cost_per_dma_byte=cost)
        plan = dos.dos_plan_subgroups(cm, sizes, 4 * 10**9)
        assert (sum(plan.targets) > 0) == staged, cost
        if not staged:
            assert plan.c.predicted_s == pytest.approx(4.0e9 / 12e9)
    # below that point a growing cost slows the host lane down, so the balance moves towards the GPU and
    # the predicted time grows
    plans = [dos.dos_plan_subgroups(dos.cost_model(56e9, 48e9, 230e9, 6e9, cpu_cost_per_dma_byte=c), sizes, 4 * 10**9)
             for c in (0.0, 0.01, 0.02, 0.03)]
    counts = [sum(pl.targets) for pl in plans]
    times = [pl.c.predicted_s for pl in plans]
    assert counts == sorted(counts) and counts[0] > 0 and times == sorted(times) and times[0] < times[-1]
    assert times[-1] < 4.0e9 / 6e9                     # still better than the host cores alone
    with pytest.raises(dos.DosError):
        dos.dos_plan_subgroups(dos.cost_model(56e9, 48e9, 230e9, 6e9, cpu_cost_per_dma_byte=-0.1), sizes, 4 * 10**9)


@pytest.mark.parametrize("u0,beta,h2d,d2h,stages", [
    (2.0e9, 0.004, 50e9, 45e9, True),      # slow host (the paper's regime): staging pays
    (12.0e9, 0.035, 47e9, 45e9, True),     # fast host, mild contention: a small staged share pays
    (16.0e9, 0.12, 40e9, 45e9, False),     # fast host whose stores share the link: staging costs more than it saves
])
def test_plan_observe_loop_converges_on_a_simulated_machine(u0, beta, h2d, d2h, stages):
    """Closed loop, as a training run uses the library: plan, run a phase, observe, plan again -- on a
    simulated machine with known rates, contention and 2 % timing noise.  The loop has to end within a few
    percent of the best split for that machine (found by trying every count), whether that split stages
    subgroups or keeps them all on the host cores."""
    rng = random.Random(int(u0 / 1e6) + int(beta * 1e4))
    sizes = [100_000_000] * 60
    s_gpu = 230e9

    def machine(n_gpu_sg, noise=True):
        ng, nc = 1e8 * n_gpu_sg, 1e8 * (60 - n_gpu_sg)
        jit = (lambda: 1.0 + rng.uniform(-0.02, 0.02)) if noise else (lambda: 1.0)
        t_cpu = (nc + beta * 24.0 * ng) / u0 * jit()
        t_h2d, t_d2h = (12 * ng + 2 * nc) / h2d * jit(), 12 * ng / d2h * jit()
        t_gpu = max(t_h2d, t_d2h + 0.004, ng / s_gpu) if ng else 0.0
        return ng, nc, t_cpu, t_gpu, t_h2d, t_d2h

    best = min(max(machine(k, False)[2], machine(k, False)[3]) for k in range(61))
    all_cpu = machine(0, False)[2]
    cm = dos.cost_model(56e9, 48e9, s_gpu, 1.2 * u0)               # calibrated stand-alone: optimistic
    walls = []
    for it in range(14):
        if it == 0:
            k = 0                                                  # first phase on the host cores alone
        else:
            k = sum(dos.dos_plan_subgroups(cm, sizes, 40 * 10**9).targets)
        ng, nc, t_cpu, t_gpu, t_h2d, t_d2h = machine(k)
        st = dos.dos_phase_stats()
        st.params_cpu, st.params_gpu = int(nc), int(ng)
        st.h2d_bytes, st.d2h_bytes = 12.0 * ng + 2.0 * nc, 12.0 * ng
        st.cpu_lane_s, st.gpu_lane_s = t_cpu, t_gpu
        # the prefetches are busy for their own bytes' share of the direction's time
        st.h2d_busy_s = t_h2d * (12.0 * ng) / (12.0 * ng + 2.0 * nc) if ng else -1.0
        st.d2h_busy_s = t_d2h if ng else -1.0
        dos.dos_cost_model_observe(cm, st)
        walls.append((k, max(t_cpu, t_gpu)))
    tail = walls[-4:]
    assert all(w <= 1.06 * best for _, w in tail), (walls, best)
    assert all((k > 0) == stages for k, _ in tail), walls
    if stages:
        assert max(w for _, w in tail) < all_cpu


@pytest.mark.parametrize("seed", range(20))
def test_balanced_plan_invariants_on_random_machines(seed):
    """Whatever the rates: the balanced plan is never worse (by its own estimate)
    than all-CPU, all-GPU or any stride of Algorithm 1; its order is a permutation;
    scaling every subgroup by the same factor keeps the placement (the paper's
    observation that the split does not depend on the subgroup size, Section 4.2)."""
    rng = random.Random(500 + seed)
    n = rng.choice([5, 17, 40, 130, 260])
    base = rng.choice([50, 100, 200, 400]) * 1_000_000
    sizes = [base] * n if rng.random() < 0.5 else [int(base * rng.uniform(0.5, 1.5)) for _ in range(n)]
    cost = dict(h2d_Bps=rng.uniform(10, 64) * 1e9, d2h_Bps=rng.uniform(10, 64) * 1e9,
                gpu_params_per_s=rng.uniform(20, 250) * 1e9, cpu_params_per_s=rng.uniform(0.3, 20) * 1e9,
                launch_overhead_s=0.0)
    cm = dos.cost_model(cost["h2d_Bps"], cost["d2h_Bps"], cost["gpu_params_per_s"], cost["cpu_params_per_s"], 0.0, 0.0)
    plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9)
    kw = dict(n_slots=plan.c.n_slots, slot_params=plan.c.slot_params, **cost)
    assert sorted(plan.orders) == list(range(n))
    assert set(plan.targets) <= {0, 1}
    mine = ref.phase_cost(sizes, plan.targets, **kw)[0]
    assert plan.c.predicted_s == pytest.approx(mine, rel=1e-12)
    assert plan.c.lower_bound_s <= plan.c.predicted_s * (1 + 1e-12)
    for other in ([0] * n, [1] * n, *(ref.stride_targets(n, k) for k in range(2, 7))):
        assert mine <= ref.phase_cost(sizes, other, **kw)[0] * (1 + 1e-9)
    if len(set(sizes)) == 1 and n > 16:
        # equal subgroups: the same placement for 3x larger subgroups (slots already at the 16 Mi cap)
        big = dos.dos_plan_subgroups(cm, [3 * s for s in sizes], 40 * 10**9)
        assert big.targets == plan.targets
        assert big.c.predicted_s == pytest.approx(3 * plan.c.predicted_s, rel=0.02)


def test_cpu_only_subgroups_are_never_moved_to_the_gpu():
    """Subgroups whose state sits in pageable host memory must stay on the host
    cores; the rest is planned as usual, and for few subgroups still optimally."""
    rng = random.Random(11)
    cm = dos.cost_model(COST["h2d_Bps"], COST["d2h_Bps"], COST["gpu_params_per_s"], 3e9, 0.0, COST["launch_overhead_s"])
    cost = {**COST, "cpu_params_per_s": 3e9}
    for n in (6, 12, 40, 130):
        sizes = [rng.randint(40, 160) * 1_000_000 for _ in range(n)]
        mask = [rng.random() < 0.5 for _ in range(n)]
        for mode in (dos.DOS_PLAN_BALANCED, dos.DOS_PLAN_STRIDE):
            plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, mode, n_resident_max=3, cpu_only=mask)
            for t, r, forced in zip(plan.targets, plan.residents, mask):
                assert not (forced and t and not r)          # never staged; residency is allowed
            # residents are the trailing subgroups (Section 4.1), whatever the mask says
            assert plan.residents == [0] * (n - sum(plan.residents)) + [1] * sum(plan.residents)
            assert sum(plan.residents) == 3
        if n <= 12:
            plan = dos.dos_plan_subgroups(cm, sizes, 40 * 10**9, cpu_only=mask)
            assert sum(plan.residents) == 0
            free = [i for i in range(n) if not mask[i]]
            best = None
            for bits in range(1 << len(free)):
                t = [0] * n
                for q, i in enumerate(free):
                    t[i] = (bits >> q) & 1
                c = ref.phase_cost(sizes, t, n_slots=plan.c.n_slots, slot_params=plan.c.slot_params, **cost)[0]
                best = c if best is None else min(best, c)
            assert plan.c.predicted_s <= best * (1 + 1e-12)
    # stride mode counts over the movable subgroups only
    mask = [0, 1, 0, 0, 1, 0, 0, 0]
    cmp_ = cm_from_paper_units(3 * G, 35 * G, 2 * G, 8.7 * G)          # k = 2
    plan = dos.dos_plan_subgroups(cmp_, [10_000_000] * 8, 10**9, dos.DOS_PLAN_STRIDE, cpu_only=mask)
    assert plan.targets == [0, 0, 1, 0, 0, 1, 0, 1]
    # everything forced to the host
    plan = dos.dos_plan_subgroups(cm, [10_000_000] * 5, 10**9, cpu_only=[1] * 5)
    assert plan.targets == [0] * 5 and plan.residents == [0] * 5
