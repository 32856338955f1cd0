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


def test_stride_rounding_follows_the_reading_taken():
    """The paper's only worked example (2.294 -> 2) is met by rounding down and by rounding to nearest
    alike, so the paper does not pin the rounding.  This build reads it as round-to-nearest, at least 1,
    and a non-positive denominator (host faster than its uploads) as 'no dynamic GPU subgroup'; the
    values below pin that reading, not the paper."""
    B, Ug, Dc = 3e9, 35e9, 8.7e9
    # U_c chosen so that Eq. 1 gives 2.6 and 3.4: den = (3/B + 1/U_g) / k
    for k_real, k_int in ((2.6, 3), (3.4, 3), (0.3, 1)):
        den = (3.0 / B + 1.0 / Ug) / k_real
        Uc = 1.0 / (den - 1.0 / Dc + 1.0 / (2.0 * B))
        assert ref.stride_k_real(B, Ug, Uc, Dc) == pytest.approx(k_real, rel=1e-12)
        assert ref.stride_k(B, Ug, Uc, Dc) == k_int
    assert ref.stride_k(1e9, 35e9, 50e9, float("inf")) == 0      # 1/U_c < 1/(2B): the host never lags


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


# ---- the makespan estimate, branch by branch, against numbers worked out by hand -------------------
# Ten subgroups of 1e8 parameters; H2D 60 GB/s, D2H 40 GB/s, U_g 200 G params/s, launch 10 us.
# Section 4.2's terms: a staged subgroup moves 3S (FP32 parameters) = 12 bytes/param each way, a
# CPU-updated one sends S/2 = 2 bytes/param up, a kernel takes S/U_g.
HAND = dict(h2d_Bps=60e9, d2h_Bps=40e9, gpu_params_per_s=200e9, cpu_params_per_s=20e9, launch_overhead_s=10e-6)
S8 = 100_000_000
MIXED = [0, 0, 1, 0, 0, 1, 0, 1, 0, 1]             # four staged (N_G = 4e8), six on the host (N_C = 6e8)


def test_overlapped_lane_waits_for_the_flushes_behind_the_first_piece():
    """Three slots.  H2D: (12*4e8 + 2*6e8) / 60e9 = 0.100 s.  D2H: 12*4e8 / 40e9 = 0.120 s, and it cannot
    start before the first subgroup has been prefetched and updated: 12e8/60e9 + 1e8/200e9 + 1e-5 =
    0.02051 s.  Kernels: 4e8/200e9 + 4e-5 = 0.00204 s.  Host: 6e8/20e9 = 0.030 s.
    Lane = max(0.100, 0.02051 + 0.120, 0.00204) = 0.14051 s."""
    pred, low = ref.phase_cost([S8] * 10, MIXED, n_slots=3, **HAND)
    assert pred == pytest.approx(0.14051, rel=1e-9)
    assert low == pytest.approx(0.120, rel=1e-9)
    # two slots overlap just the same
    assert ref.phase_cost([S8] * 10, MIXED, n_slots=2, **HAND)[0] == pytest.approx(0.14051, rel=1e-9)
    # the first *staged* subgroup leads, whatever its position: make it a small one
    sizes = [S8] * 10
    sizes[2] = 10_000_000                            # N_G = 3.1e8
    lead = 12 * 1e7 / 60e9 + 1e7 / 200e9 + 1e-5      # 0.00206
    assert ref.phase_cost(sizes, MIXED, n_slots=3, **HAND)[0] == pytest.approx(lead + 12 * 3.1e8 / 40e9, rel=1e-9)


def test_pieces_shorten_the_lead():
    """Slots of 16 Mi parameters: only the first piece leads the flushes.
    12*16777216/60e9 + 16777216/200e9 + 1e-5 = 0.0033554432 + 0.0000838861 + 0.00001 = 0.0034493293 s;
    lane = 0.0034493293 + 0.120 = 0.1234493293 s."""
    pred, _ = ref.phase_cost([S8] * 10, MIXED, n_slots=3, slot_params=16 << 20, **HAND)
    assert pred == pytest.approx(0.1234493293, rel=1e-9)
    # a slot larger than the subgroup changes nothing
    assert ref.phase_cost([S8] * 10, MIXED, n_slots=3, slot_params=1 << 30, **HAND)[0] == pytest.approx(0.14051, rel=1e-9)


def test_single_slot_serialises_the_staged_subgroups_next_to_the_uploads():
    """One slot: 12*4e8/60e9 + (4e8/200e9 + 4e-5) + 12*4e8/40e9 = 0.080 + 0.00204 + 0.120 = 0.20204 s
    (the uploads of the host lane, 0.020 s, ride alongside).  With a host that is slow enough for its
    uploads to outlast that (nothing staged is the limit case) the H2D direction bounds the lane."""
    pred, low = ref.phase_cost([S8] * 10, MIXED, n_slots=1, **HAND)
    assert pred == pytest.approx(0.20204, rel=1e-9)
    assert low == pytest.approx(0.120, rel=1e-9)
    # 1 staged, 99 on the host, slow D2H irrelevant: H2D = (12e8 + 2*99e8)/60e9 = 0.350 s outlasts
    # the serial chain 0.020 + 0.00051 + 0.030 = 0.05051 s
    tgt = [1] + [0] * 99
    pred, _ = ref.phase_cost([S8] * 100, tgt, n_slots=1, **{**HAND, "cpu_params_per_s": 1e12})
    assert pred == pytest.approx(0.350, rel=1e-9)


def test_residents_cost_gpu_time_only():
    """Subgroups 8 and 9 resident, 2 and 5 staged, six on the host; a slow GPU (1 G params/s) so that
    the kernels bound the lane: (2e8 + 2e8)/1e9 + 4e-5 = 0.40004 s.  Link: H2D (12*2e8 + 2*6e8)/60e9 =
    0.060 s, D2H 12*2e8/40e9 = 0.060 s -- the residents' state never crosses it."""
    tgt = [0, 0, 1, 0, 0, 1, 0, 0, 1, 1]
    kw = {**HAND, "gpu_params_per_s": 1e9}
    pred, low = ref.phase_cost([S8] * 10, tgt, n_slots=3, resident=[8, 9], **kw)
    assert pred == pytest.approx(0.40004, rel=1e-9)
    assert low == pytest.approx(0.060, rel=1e-9)
    # residents only, nothing staged: kernels 2e8/1e9 + 2e-5 against uploads 2*8e8/60e9
    tgt = [0] * 8 + [1, 1]
    pred, low = ref.phase_cost([S8] * 10, tgt, n_slots=3, resident=[8, 9], **kw)
    assert pred == pytest.approx(0.20002, rel=1e-9)
    assert low == pytest.approx(1.6e9 / 60e9, rel=1e-9)
    with pytest.raises(AssertionError):               # a resident is GPU-planned by definition
        ref.phase_cost([S8] * 10, [0] * 10, n_slots=3, resident=[9], **kw)


def test_two_array_rules_move_eight_bytes_per_parameter():
    """Adagrad / RMSProp keep p and one accumulator: 8 bytes/param each way.  H2D (8*4e8 + 2*6e8)/60e9 =
    0.07333 s, D2H 8*4e8/40e9 = 0.080 s, lead 8e8/60e9 + 0.0005 + 1e-5 = 0.0138433 s -> 0.0938433 s."""
    pred, low = ref.phase_cost([S8] * 10, MIXED, n_slots=3, fp32_arrays=2, **HAND)
    assert pred == pytest.approx(8e8 / 60e9 + 0.00051 + 0.080, rel=1e-9)
    assert pred == pytest.approx(0.09384333, rel=1e-6)
    assert low == pytest.approx(0.080, rel=1e-9)


def test_staged_traffic_is_charged_to_the_host_lane():
    """Contention (Section 5.4): with 0.05 parameters of host work lost per staged byte, the 2*12*4e8 =
    9.6e9 staged bytes cost the host 4.8e8 parameters: (6e8 + 4.8e8) / 2e9 = 0.540 s (0.300 s without)."""
    kw = {**HAND, "cpu_params_per_s": 2e9}
    assert ref.phase_cost([S8] * 10, MIXED, n_slots=3, **kw)[0] == pytest.approx(0.300, rel=1e-9)
    pred, low = ref.phase_cost([S8] * 10, MIXED, n_slots=3, cpu_cost_per_dma_byte=0.05, **kw)
    assert pred == pytest.approx(0.540, rel=1e-9)
    assert low == pytest.approx(0.120, rel=1e-9)      # the bound prices the link only
    # with two arrays 2*8*4e8 = 6.4e9 bytes -> (6e8 + 3.2e8)/2e9 = 0.460 s
    assert ref.phase_cost([S8] * 10, MIXED, n_slots=3, cpu_cost_per_dma_byte=0.05, fp32_arrays=2,
                          **kw)[0] == pytest.approx(0.460, rel=1e-9)
    # residents are not staged: no charge
    tgt = [0] * 8 + [1, 1]
    assert ref.phase_cost([S8] * 10, tgt, n_slots=3, resident=[8, 9], cpu_cost_per_dma_byte=0.05,
                          **kw)[0] == pytest.approx(8e8 / 2e9, rel=1e-9)


def test_eq1_balance_is_the_models_balance():
    """Eq. 1 (Section 4.2) equates, per GPU-updated subgroup, the host time of k subgroups with the
    link time 3S/B + k S/(2B) and the kernel S/U_g.  With a GPU and a D2H direction fast enough not to
    matter and a fused downscale (1/D_c = 0), B = 3 and U_c = 1.5 G params/s give k = 2 exactly; a
    phase of four such periods (two on the host for each staged one) must then have both lanes end
    together, and at the link bound."""
    B, Uc = 3e9, 1.5e9
    assert ref.stride_k_real(B, float("inf"), Uc, float("inf")) == pytest.approx(2.0, rel=1e-12)
    sizes = [S8] * 12
    tgt = [0, 0, 1] * 4
    kw = dict(h2d_Bps=4 * B, d2h_Bps=1e30, gpu_params_per_s=1e30, cpu_params_per_s=Uc, launch_overhead_s=0.0,
              n_slots=3)
    pred, low = ref.phase_cost(sizes, tgt, **kw)
    host = 8 * S8 / Uc
    assert pred == pytest.approx(host, rel=1e-12) and low == pytest.approx(host, rel=1e-12)
    # one more on the host makes the host lane the longer one, one more on the GPU the link
    more_cpu = ref.phase_cost(sizes, [0, 0, 1] * 3 + [0, 0, 0], **kw)
    more_gpu = ref.phase_cost(sizes, [0, 0, 1] * 3 + [0, 1, 1], **kw)
    assert more_cpu[0] == pytest.approx(9 * S8 / Uc, rel=1e-12) and more_cpu[0] > more_cpu[1]
    assert more_gpu[0] == pytest.approx(more_gpu[1], rel=1e-12) and more_gpu[0] > host


def simulate_pipeline(pieces, n_slots, h2d_Bps, d2h_Bps, gpu_params_per_s, launch_overhead_s, state_bytes=12.0):
    """Event-by-event timeline of the staged lane: piece j is prefetched into slot j mod n_slots once
    that slot's previous occupant has been flushed, updated once it has landed and the previous kernel
    is done, flushed once updated and the previous flush is done.  Returns the time the last flush ends."""
    h_end, k_end, d_end = [], [], []
    for j, n in enumerate(pieces):
        h0 = max(h_end[-1] if h_end else 0.0, d_end[j - n_slots] if j >= n_slots else 0.0)
        h_end.append(h0 + state_bytes * n / h2d_Bps)
        k0 = max(h_end[-1], k_end[-1] if k_end else 0.0)
        k_end.append(k0 + n / gpu_params_per_s + launch_overhead_s)
        d0 = max(k_end[-1], d_end[-1] if d_end else 0.0)
        d_end.append(d0 + state_bytes * n / d2h_Bps)
    return d_end[-1] if d_end else 0.0


@pytest.mark.parametrize("h2d,d2h,ug", [(60e9, 40e9, 200e9), (40e9, 60e9, 200e9), (50e9, 50e9, 2e9),
                                        (55e9, 48e9, 230e9)])
@pytest.mark.parametrize("n_slots", [1, 2, 3, 5])
def test_lane_estimate_against_an_event_by_event_timeline(h2d, d2h, ug, n_slots):
    """The closed form is a bound from below on what a pipeline with these stage times can do, and it
    is tight: the timeline ends no earlier, and no later than the closed form plus the stages of one
    piece (fill and drain), whichever stage is the slow one.  With one slot the two agree exactly."""
    rate = dict(h2d_Bps=h2d, d2h_Bps=d2h, gpu_params_per_s=ug, launch_overhead_s=10e-6)
    piece = 16 << 20
    for n_staged in (1, 2, 7, 24):
        pieces = [piece] * n_staged
        got = simulate_pipeline(pieces, n_slots, **rate)
        model, _ = ref.phase_cost(pieces, [1] * n_staged, n_slots=n_slots, cpu_params_per_s=1e30, **rate)
        one = 12.0 * piece / h2d + piece / ug + 10e-6 + 12.0 * piece / d2h
        if n_slots == 1:
            assert got == pytest.approx(model, rel=1e-12)
        else:
            assert model <= got * (1 + 1e-12)
            slack = one if n_slots >= 3 else one * n_staged   # two slots stall on every other piece
            assert got <= model + slack * (1 + 1e-12)
