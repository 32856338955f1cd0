"""The interleaved update phase (dos_run_update_phase through the C ABI) must be
bit-identical to running every subgroup through the oracle, for every plan,
slot count, piece size and order."""
import ctypes as C
import random

import numpy as np
import pytest
import torch

import dos_synth as S
import paper_2410_21316_amd as dos

from gpu_util import OffloadedState, make_context

pytestmark = pytest.mark.gpu

SIZES = [300_001, 262_144, 100_000, 65, 0, 500_003, 1_000_000, 64, 131_073]


def run_phase_case(sizes, targets, order, n_slots, slot_params, hp, steps=3, resident=None,
                   grad_on_device=None, host_threads=4, chunk_params=1 << 16, ring_chunks=6, flags=0,
                   seed=S.BASE_SEED, optimizer="adamw", **gkw):
    st = OffloadedState(sizes, seed, resident=resident, grad_on_device=grad_on_device, **gkw)
    ctx = make_context(n_slots, slot_params, host_threads, chunk_params, ring_chunks, flags=flags)
    plan = dos.Plan.manual(targets, order, n_slots, slot_params, resident)
    stats = None
    try:
        for step in range(1, steps + 1):
            st.set_grads(step)
            stats = ctx.dos_run_update_phase(st.sgs, plan, dos.hparams(step=step, optimizer=optimizer, **hp))
            st.oracle_step(hp, step, optimizer=optimizer)
            st.check(f"{optimizer} step {step} targets {targets} slots {n_slots}x{slot_params}")
    finally:
        ctx.close()
        if ctx._keep[1] is not None:
            ctx._keep[1].free()
        st.free()
    return stats


def test_alternate_subgroups_on_gpu_like_stride_two(hp):
    """k = 2: every alternate subgroup on the GPU (Sections 5.3, 5.4)."""
    targets = [(i + 1) % 2 == 0 for i in range(len(SIZES))]
    stats = run_phase_case(SIZES, targets, None, 2, 1 << 20, hp, zero_pct=1.0)
    n_g = sum(n for n, t in zip(SIZES, targets) if t)
    n_c = sum(n for n, t in zip(SIZES, targets) if not t)
    assert stats.params_gpu == n_g and stats.params_cpu == n_c
    assert stats.d2h_bytes == 12.0 * n_g
    assert stats.h2d_bytes == 12.0 * n_g + 2.0 * n_c + 2.0 * n_g     # gradients staged too here
    assert stats.n_gpu == sum(1 for n, t in zip(SIZES, targets) if t and n)


@pytest.mark.parametrize("case", range(8))
def test_random_plans_slots_pieces_and_orders(case, hp):
    rng = random.Random(1000 + case)
    sizes = SIZES[:]
    rng.shuffle(sizes)
    targets = [rng.random() < 0.5 for _ in sizes]
    order = list(range(len(sizes)))
    rng.shuffle(order)
    n_slots = rng.choice([1, 2, 3, 4])
    slot_params = rng.choice([1 << 16, 3 << 16, 1 << 20])       # smaller than some subgroups: pieces
    grad_dev = [t and rng.random() < 0.5 for t in targets]
    run_phase_case(sizes, targets, order, n_slots, slot_params, hp, steps=2, grad_on_device=grad_dev,
                   host_threads=rng.choice([1, 3, 8]), chunk_params=rng.choice([1 << 12, 1 << 16]),
                   ring_chunks=rng.choice([2, 3, 9]), seed=S.BASE_SEED + case, zero_pct=5.0, heavy_tail=True)


@pytest.mark.parametrize("case", range(6))
def test_direct_uploads_through_the_bar(case, hp):
    """DOS_CTX_UPLOAD_DIRECT: the host workers write the 16-bit parameters of CPU-planned subgroups
    straight into the device model (host stores through the PCIe BAR), with or without an upload ring
    in the context; same bits as the oracle, and the device sees them as soon as the phase returns."""
    if not dos.dos_device_large_bar(0):
        pytest.skip("the device memory is not mapped into the host's address space")
    rng = random.Random(2000 + case)
    sizes = SIZES[:]
    rng.shuffle(sizes)
    targets = [rng.random() < 0.4 for _ in sizes]
    order = list(range(len(sizes)))
    rng.shuffle(order)
    optimizer = ["adamw", "adagrad", "rmsprop"][case % 3]
    stats = run_phase_case(sizes, targets, order, rng.choice([1, 3]), rng.choice([1 << 16, 1 << 20]), hp, steps=3,
                           grad_on_device=[t and rng.random() < 0.5 for t in targets],
                           host_threads=rng.choice([1, 4, 8]), chunk_params=rng.choice([1 << 12, 1 << 16]),
                           ring_chunks=rng.choice([0, 3]), seed=S.BASE_SEED + 50 + case, optimizer=optimizer,
                           flags=dos.DOS_CTX_UPLOAD_DIRECT | (dos.DOS_CTX_PROFILE if case % 2 else 0),
                           zero_pct=5.0, heavy_tail=True)
    assert stats.params_cpu == sum(n for n, t in zip(sizes, targets) if not t)
    assert stats.cpu_wait_s == 0.0 and stats.cpu_enqueue_s == 0.0        # no ring, no upload kernels


def test_direct_uploads_are_visible_to_kernels_that_cached_the_old_model(hp):
    """A kernel reads the 16-bit model (its lines may sit in the GPU's caches), the phase then rewrites it
    from the host cores through the BAR, and a kernel launched afterwards must read the new values."""
    if not dos.dos_device_large_bar(0):
        pytest.skip("the device memory is not mapped into the host's address space")
    sizes = [300_000, 150_016]
    st = OffloadedState(sizes, S.BASE_SEED + 60)
    ctx = make_context(0, 1 << 16, 4, ring_chunks=0, flags=dos.DOS_CTX_UPLOAD_DIRECT)
    plan = dos.Plan.manual([0, 0], None, 0, 0)
    try:
        for step in range(1, 6):
            before = [st.dev[i]["lp"].view(torch.int16).to(torch.int64).sum().item() for i in range(2)]  # caches it
            st.set_grads(step)
            ctx.dos_run_update_phase(st.sgs, plan, dos.hparams(step=step, **hp))
            st.oracle_step(hp, step)
            for i in range(2):
                # a reduction kernel, not a copy engine, reads the model right after the phase
                got = st.dev[i]["lp"].view(torch.int16).to(torch.int64).sum().item()
                want = int(st.ref[i][3].view(np.int16).astype(np.int64).sum())
                assert got == want and (step == 1 or got != before[i])
            st.check(f"direct step {step}")
    finally:
        ctx.close()
        st.free()


def test_direct_uploads_next_to_gpu_written_ranges_of_a_large_model(hp):
    """Direct uploads at a size no cache holds: one contiguous 16-bit model of 137M parameters (274 MB, beyond
    the GPU's L2 and its memory-side cache) cut into four subgroups whose boundaries fall inside cache
    lines.  Two subgroups are updated by the host cores, which store their part of the model through the
    PCIe BAR; the two between them are staged and their kernels write the neighbouring ranges of the same
    model -- partial lines from both sides -- in the same phase.  A reduction kernel on a side stream reads
    the whole model before every phase (so that the old lines sit wherever the GPU caches them) and right
    after it; the model must then equal the oracle's, bit for bit."""
    if not dos.dos_device_large_bar(0):
        pytest.skip("the device memory is not mapped into the host's address space")
    from gpu_util import Pinned, assert_parity, oracle_step, round_up
    sizes = [60_000_008, 4_000_024, 70_000_040, 3_000_008]        # 16-byte aligned slices, not line-aligned
    targets = [0, 1, 0, 1]
    total = sum(sizes)
    assert total * 2 >= 256 * 10**6
    seed = S.BASE_SEED + 61
    model = torch.zeros(total, dtype=torch.bfloat16, device="cuda:0")
    grads = torch.zeros(total, dtype=torch.bfloat16, device="cuda:0")
    pin = Pinned(sum(3 * round_up(4 * n, 256) + round_up(2 * n, 256) for n in sizes))
    host, ref, sgs, offs = [], [], [], []
    off_b, off_e = 0, 0
    for i, n in enumerate(sizes):
        h = {}
        for name in "pmv":
            h[name] = pin.view(np.float32, off_b, n); off_b += round_up(4 * n, 256)
        h["g"] = pin.view(np.uint16, off_b, n); off_b += round_up(2 * n, 256)
        tmp = torch.empty(n, dtype=torch.float32, device="cuda:0")
        S.fill_chunked(lambda start, count: S.params(seed, i, start, count, "cuda:0"), tmp)
        h["p"][:] = tmp.cpu().numpy(); h["m"][:] = 0; h["v"][:] = 0
        del tmp
        host.append(h)
        ref.append([h["p"].copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)])
        lp = model[off_e:off_e + n]
        gd = grads[off_e:off_e + n]
        g_ptr = gd.data_ptr() if targets[i] else h["g"].ctypes.data
        sgs.append(dos.subgroup(h["p"].ctypes.data, h["m"].ctypes.data, h["v"].ctypes.data, g_ptr, lp.data_ptr(), n,
                                dos.DOS_HOST_PINNED, dos.DOS_DEVICE if targets[i] else dos.DOS_HOST_PINNED))
        offs.append(off_e)
        off_e += n
    ctx = make_context(3, 1 << 20, 8, chunk_params=1 << 20, ring_chunks=0, flags=dos.DOS_CTX_UPLOAD_DIRECT)
    plan = dos.Plan.manual(targets, None, 3, 1 << 20)
    side = torch.cuda.Stream()
    try:
        for step in (1, 2, 3):
            gbits = []
            for i, n in enumerate(sizes):
                gd = grads[offs[i]:offs[i] + n]
                S.fill_chunked(lambda start, count: S.grads_bf16(seed, step, i, start, count, "cuda:0", zero_pct=1.0), gd)
                bits = gd.view(torch.int16).cpu().numpy().view(np.uint16)
                gbits.append(bits)
                if not targets[i]:
                    host[i]["g"][:] = bits
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                before = model.view(torch.int16).to(torch.int64).sum()       # reads (and may cache) the old model
            side.synchronize()
            st = ctx.dos_run_update_phase(sgs, plan, dos.hparams(step=step, **hp))
            with torch.cuda.stream(side):
                after = model.view(torch.int16).to(torch.int64).sum()        # a kernel, on a stream of its own
            side.synchronize()
            want_sum = 0
            for i, n in enumerate(sizes):
                oracle_step(ref[i], gbits[i], hp, step)
                want_sum += int(ref[i][3].view(np.int16).astype(np.int64).sum())
            assert int(after.item()) == want_sum and int(after.item()) != int(before.item()), f"step {step}"
            assert st.params_cpu == sizes[0] + sizes[2] and st.params_gpu == sizes[1] + sizes[3]
        got_model = model.view(torch.int16).cpu().numpy().view(np.uint16)
        for i, n in enumerate(sizes):
            assert_parity(f"large direct model, subgroup {i}", (host[i]["p"], host[i]["m"], host[i]["v"]), ref[i][:3],
                          got_model[offs[i]:offs[i] + n], ref[i][3])
    finally:
        ctx.close()
        host = None
        pin.free()


@pytest.mark.parametrize("optimizer", ["adagrad", "rmsprop"])
def test_other_rules_through_the_phase(optimizer, hp):
    """Adagrad and RMSProp: mixed plan with a resident, device and host gradients, pieces smaller than
    the subgroups; only p and v cross the link (8 bytes per parameter each way), m is left alone."""
    n = len(SIZES)
    targets = [1, 0, 1, 1, 0, 0, 1, 1, 1]
    resident = [0, 0, 0, 0, 0, 0, 0, 0, 1]
    grad_dev = [1, 0, 0, 1, 0, 0, 1, 0, 1]
    stats = run_phase_case(SIZES, targets, list(reversed(range(n))), 3, 1 << 17, hp, resident=resident,
                           grad_on_device=grad_dev, optimizer=optimizer, zero_pct=5.0, heavy_tail=True)
    staged = sum(s for s, t, r in zip(SIZES, targets, resident) if t and not r)
    on_cpu = sum(s for s, t in zip(SIZES, targets) if not t)
    spilled = sum(s for s, t, r, gd in zip(SIZES, targets, resident, grad_dev) if t and not r and not gd)
    assert stats.d2h_bytes == 8.0 * staged
    assert stats.h2d_bytes == 8.0 * staged + 2.0 * on_cpu + 2.0 * spilled


@pytest.mark.parametrize("flags", ["dma", "spin", "dma+spin", "spin+direct", "profile+dma"])
def test_upload_and_wait_modes_give_the_same_bits(flags, hp):
    """The other ways a context can be told to work -- 16-bit uploads by hipMemcpyAsync instead of the copy
    kernel, spinning instead of sleeping waits -- change timing only: a mixed plan with pieces, host and device
    gradients stays bit-identical to the oracle."""
    f = 0
    if "dma" in flags:
        f |= dos.DOS_CTX_UPLOAD_DMA
    if "spin" in flags:
        f |= dos.DOS_CTX_SPIN_WAIT
    if "profile" in flags:
        f |= dos.DOS_CTX_PROFILE
    if "direct" in flags:
        if not dos.dos_device_large_bar(0):
            pytest.skip("the device memory is not mapped into the host's address space")
        f |= dos.DOS_CTX_UPLOAD_DIRECT
    targets = [1, 0, 1, 0, 0, 1, 0, 1, 0]
    stats = run_phase_case(SIZES, targets, list(reversed(range(len(SIZES)))), 3, 1 << 17, hp, steps=2,
                           grad_on_device=[1, 0, 0, 0, 0, 1, 0, 0, 0], host_threads=3, chunk_params=1 << 14,
                           ring_chunks=5, flags=f, zero_pct=5.0, heavy_tail=True, seed=S.BASE_SEED + 33)
    assert stats.params_gpu == sum(n for n, t in zip(SIZES, targets) if t)


def test_all_gpu_and_all_cpu_plans(hp):
    run_phase_case(SIZES, [1] * len(SIZES), None, 3, 1 << 18, hp, steps=2)
    run_phase_case(SIZES, [0] * len(SIZES), None, 0, 1 << 18, hp, steps=2)


def test_static_residents_placed_last_update_in_place(hp):
    """Update figure of Section 4.1: residents are the trailing subgroups; their
    state never crosses the link."""
    sizes = [200_000, 150_001, 300_000, 120_000, 250_007, 99_999, 180_000, 210_000]
    resident = [0, 0, 0, 0, 0, 0, 1, 1]
    targets = [0, 0, 1, 0, 0, 1, 1, 1]          # stride 3 plus the two residents
    stats = run_phase_case(sizes, targets, None, 2, 1 << 18, hp, resident=resident,
                           grad_on_device=[0, 0, 1, 0, 0, 1, 1, 1], flags=dos.DOS_CTX_PROFILE)
    assert stats.n_resident == 2 and stats.params_resident == 390_000
    assert stats.d2h_bytes == 12.0 * (300_000 + 99_999)
    assert stats.h2d_bytes == 12.0 * (300_000 + 99_999) + 2.0 * (200_000 + 150_001 + 120_000 + 250_007)
    assert stats.h2d_busy_s > 0 and stats.d2h_busy_s > 0 and stats.gpu_busy_s > 0


def test_placement_does_not_change_results(hp):
    """Subgroups update independently: any placement gives the same bits
    (Section 4.1: out-of-order updates do not affect the result)."""
    sizes = [100_000, 70_001, 130_000, 65_536]
    results = []
    for targets in ([0, 0, 0, 0], [1, 1, 1, 1], [1, 0, 1, 0], [0, 1, 0, 1]):
        st = OffloadedState(sizes, S.BASE_SEED + 3)
        ctx = make_context(2, 1 << 16)
        plan = dos.Plan.manual(targets, None, 2, 1 << 16)
        for step in (1, 2):
            st.set_grads(step)
            ctx.dos_run_update_phase(st.sgs, plan, dos.hparams(step=step, **hp))
        results.append(st.snapshot())
        ctx.close(); st.free()
    for other in results[1:]:
        for a, b in zip(results[0], other):
            for x, y in zip(a, b):
                assert x.tobytes() == y.tobytes()


def test_validation_errors_leave_state_untouched(hp):
    sizes = [100_000, 50_000]
    st = OffloadedState(sizes, S.BASE_SEED, grad_on_device=[1, 0])
    st.set_grads(1)
    ctx = make_context(2, 1 << 16, stage_grads=False)
    lib = dos.load()
    before = st.snapshot()
    arr = (dos.dos_subgroup * 2)(*st.sgs)
    stats = dos.dos_phase_stats()
    good = dos.hparams(step=1, **hp)

    def call(plan, hp_=good, n=2):
        return lib.dos_run_update_phase(ctx._h, arr, n, C.byref(plan.c), C.byref(hp_), C.byref(stats))

    assert call(dos.Plan.manual([1, 0])) == dos.DOS_OK                       # the valid call
    st.oracle_step(hp, 1); st.check("valid call")
    before = st.snapshot()
    assert call(dos.Plan.manual([0, 0])) == dos.DOS_ESTATE                   # CPU plan, device grads
    assert call(dos.Plan.manual([1, 1])) == dos.DOS_EBUDGET                  # host grads, 12-byte slots
    assert call(dos.Plan.manual([1, 0], order=[0, 0])) == dos.DOS_EINVAL     # not a permutation
    assert call(dos.Plan.manual([1, 0]), dos.hparams(step=0, **hp)) == dos.DOS_EINVAL
    assert call(dos.Plan.manual([1, 0, 0]), n=2) == dos.DOS_EINVAL           # plan length mismatch
    assert call(dos.Plan.manual([2, 0])) == dos.DOS_EINVAL
    arr[1].p += 4
    assert call(dos.Plan.manual([1, 0])) == dos.DOS_EALIGN
    arr[1].p -= 4
    for a, b in zip(before, st.snapshot()):
        for x, y in zip(a, b):
            assert x.tobytes() == y.tobytes()
    ctx.close(); st.free()


def test_transfers_overlap_full_duplex(hp):
    """Prefetch of the next piece and flush of the previous one run at the same
    time (Section 4.1); measured with the context's profiling events."""
    from paper_2410_21316_amd import workloads as W
    sizes = [32 << 20] * 6
    state = W.OffloadedState(sizes, S.BASE_SEED + 8)
    ctx = W.make_context(3, 16 << 20, 4, flags=dos.DOS_CTX_PROFILE)
    plan = dos.Plan.manual([1] * 6, None, 3, 16 << 20)
    state.place([1] * 6)
    try:
        for step in (1, 2):
            stats = ctx.dos_run_update_phase(state.sgs, plan, dos.hparams(step=step, **hp))
        timeline = ctx.dos_ctx_last_timeline()
    finally:
        ctx.close()
        ctx._keep[1].free()
        state.free()
    assert stats.n_pieces == 12
    # the per-piece timeline: prefetch, kernel and flush of a piece follow each other, pieces of one
    # direction do not overlap, a slot is refilled only after its flush, and the spans cover the busy times
    assert len(timeline) == 12
    for j, (p0, p1, k0, k1, f0, f1) in enumerate(timeline):
        assert 0.0 <= p0 < p1 <= k0 < k1 <= f0 < f1, (j, timeline[j])
        if j:
            assert timeline[j - 1][1] <= p0 and timeline[j - 1][5] <= f0
        if j >= 3:
            assert timeline[j - 3][5] <= p0, "slot refilled before its flush had landed"
    assert stats.h2d_span_s == pytest.approx((timeline[-1][1] - timeline[0][0]) * 1e-3, rel=1e-3)
    assert stats.h2d_span_s >= stats.h2d_busy_s * 0.999 and stats.d2h_span_s >= stats.d2h_busy_s * 0.999
    assert stats.gpu_lane_s >= stats.d2h_span_s
    print({k: v for k, v in stats.asdict().items() if k.endswith("_s")})
    # a good part of the flush time runs concurrently with prefetches
    assert stats.duplex_overlap_s > stats.d2h_busy_s / 4 > 0.0


def test_pageable_subgroups_are_updated_by_the_host_cores_only(hp):
    """State the machine cannot pin stays in ordinary host memory: the host lane
    updates it in place; planning it for the GPU is refused before anything runs."""
    from paper_2410_21316_amd import workloads as W
    from oracle import adamw_oracle as ref
    sizes = [300_001, 200_000, 250_003, 100_000, 65]
    state = W.OffloadedState(sizes, S.BASE_SEED + 10, pageable_rest=True, pin_at_most=2)
    assert state.cpu_only == [False, False, True, True, True]
    cm = dos.cost_model(50e9, 50e9, 150e9, 0.2e9)            # slow host: the planner wants the GPU
    plan = dos.dos_plan_subgroups(cm, sizes, 64 << 20, cpu_only=state.cpu_only)
    assert plan.targets[:2] == [1, 1] and plan.targets[2:] == [0, 0, 0]
    ctx = W.make_context(plan.c.n_slots, plan.c.slot_params, 4, chunk_params=1 << 16, ring_chunks=6)
    want = [[state.hp[i].numpy().copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)]
            for i, n in enumerate(sizes)]
    try:
        for step in (1, 2, 3):
            state.place(plan.targets, plan.residents)
            assert [sg.state_loc for sg in state.sgs] == [0, 0, 2, 2, 2]
            state.fill_grads(step, zero_pct=1.0)
            state.sync_host_grads()
            ctx.dos_run_update_phase(state.sgs, plan, dos.hparams(step=step, **hp))
            for i in range(len(sizes)):
                g = state.g[i].view(torch.int16).cpu().numpy().view(np.uint16)
                ref.adamw_step(want[i][0], want[i][1], want[i][2], g, want[i][3], step=step, **hp)
        for i in range(len(sizes)):
            for t, w in zip((state.hp[i], state.hm[i], state.hv[i]), want[i][:3]):
                assert t.numpy().tobytes() == w.tobytes()
            assert state.lp[i].view(torch.int16).cpu().numpy().view(np.uint16).tobytes() == want[i][3].tobytes()
        # a GPU plan for a pageable subgroup is refused and nothing is touched
        before = state.hp[2].numpy().copy()
        bad = dos.Plan.manual([1, 1, 1, 0, 0], None, plan.c.n_slots, plan.c.slot_params)
        lib = dos.load()
        good_hp = dos.hparams(step=4, **hp)
        rc = lib.dos_run_update_phase(ctx._h, state.sgs, len(sizes), C.byref(bad.c), C.byref(good_hp), None)
        assert rc == dos.DOS_ESTATE
        assert state.hp[2].numpy().tobytes() == before.tobytes()
    finally:
        ctx.close()
        ctx._keep[1].free()
        state.free()


def test_phase_allocates_no_device_memory(hp):
    """Section 4.1: interleaving must not allocate; slots, ring, streams and events
    are the context's.  Free device memory is the same before and after phases."""
    from paper_2410_21316_amd import workloads as W
    sizes = [3_000_000, 2_000_001, 4_000_000, 1_000_000]
    state = W.OffloadedState(sizes, S.BASE_SEED + 9)
    ctx = W.make_context(3, 1 << 20, 4, chunk_params=1 << 18, ring_chunks=8)
    plan = dos.Plan.manual([1, 0, 1, 0], None, 3, 1 << 20)
    state.place(plan.targets)
    state.sync_host_grads()
    try:
        ctx.dos_run_update_phase(state.sgs, plan, dos.hparams(step=1, **hp))     # first call loads the kernels
        torch.cuda.synchronize()
        free_before, _ = torch.cuda.mem_get_info()
        for step in (2, 3, 4):
            ctx.dos_run_update_phase(state.sgs, plan, dos.hparams(step=step, **hp))
        torch.cuda.synchronize()
        free_after, _ = torch.cuda.mem_get_info()
    finally:
        ctx.close()
        ctx._keep[1].free()
        state.free()
    assert free_after == free_before


def _plausible(cm):
    assert 5e9 < cm.h2d_Bps < 130e9 and 5e9 < cm.d2h_Bps < 130e9
    assert 20e9 < cm.gpu_params_per_s < 400e9
    assert 0.05e9 < cm.cpu_params_per_s < 100e9
    assert 0 < cm.launch_overhead_s < 1e-3
    assert cm.downscale_params_per_s == 0.0


def test_calibration_reports_plausible_rates():
    ctx = make_context(2, 4 << 20, host_threads=8, chunk_params=1 << 20, ring_chunks=16)
    cm = ctx.dos_calibrate()
    ctx.close()
    ctx._keep[1].free()
    _plausible(cm)


def test_calibration_of_a_direct_context_without_a_ring(hp):
    """A context whose host lane stores through the BAR needs no upload ring; its calibration measures the
    host update through that same path (16-bit output into device memory) and the link with pinned memory
    of its own, and leaves the context fit for phases."""
    if not dos.dos_device_large_bar(0):
        pytest.skip("the device memory is not mapped into the host's address space")
    ctx = make_context(3, 4 << 20, host_threads=8, chunk_params=1 << 20, ring_chunks=0,
                       flags=dos.DOS_CTX_UPLOAD_DIRECT)
    st = OffloadedState([600_000, 300_008, 400_000], S.BASE_SEED + 70)
    try:
        cm = ctx.dos_calibrate()
        _plausible(cm)
        plan = dos.Plan.manual([0, 1, 0], None, 3, 4 << 20)
        for step in (1, 2):
            st.set_grads(step)
            ctx.dos_run_update_phase(st.sgs, plan, dos.hparams(step=step, **hp))
            st.oracle_step(hp, step)
            st.check(f"after calibration, step {step}")
    finally:
        ctx.close()
        st.free()
    # no slot at all: nothing to measure the link or the kernel with
    ctx = make_context(0, 1 << 16, 2, ring_chunks=0, flags=dos.DOS_CTX_UPLOAD_DIRECT)
    with pytest.raises(dos.DosError) as e:
        ctx.dos_calibrate()
    assert e.value.status == dos.DOS_EBUDGET
    ctx.close()
