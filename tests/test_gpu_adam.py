"""GPU parity of the fused AdamW kernel (dos_adam_step through the C ABI)
against the scalar oracle, element by element, on the same seeded inputs."""
import ctypes as C

import numpy as np
import pytest
import torch

import dos_synth as S
import paper_2410_21316_amd as dos
from oracle import adamw_oracle as ref

from gpu_util import DEV, DeviceSubgroup, assert_parity, oracle_step

pytestmark = pytest.mark.gpu


def run_steps(n, seed, steps, hp, launch=None, optimizer="adamw", **gkw):
    sg = DeviceSubgroup(n, seed)
    st = list(sg.host_copy())
    state = [st[0], st[1], st[2], st[4]]
    for step in range(1, steps + 1):
        sg.set_grads(step, **gkw)
        h = dos.hparams(step=step, optimizer=optimizer, **hp)
        if launch is None:
            dos.dos_adam_step(sg.desc, h, torch.cuda.current_stream().cuda_stream)
        else:
            dos.dos_adam_step_cfg(sg.desc, h, torch.cuda.current_stream().cuda_stream, **launch)
        torch.cuda.synchronize()
        p, m, v, g, lp = sg.host_copy()
        oracle_step(state, g, hp, step, optimizer=optimizer)
        assert_parity(f"{optimizer} n={n} step={step} launch={launch}", (p, m, v), state[:3], lp, state[3])


def test_config1_one_mebi_subgroup_ten_steps(hp):
    """Configuration 1: 1,048,576 parameters, p ~ N(0, 0.02), m = v = 0, fresh
    gradients ~ N(0, 1e-3) per step, 10 steps; full comparison after every step."""
    run_steps(1 << 20, S.BASE_SEED, 10, hp)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 7, 8, 9, 63, 64, 65, 1023, 1025, 4099, 262_147, (1 << 21) + 5])
def test_ragged_sizes(n, hp):
    run_steps(n, S.BASE_SEED + n, 2, hp, zero_pct=1.0)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 0x10, 0x21, 0x32, 0x33])
@pytest.mark.parametrize("threads,blocks", [(0, 0), (64, 7), (512, 256), (256, 1)])
def test_every_launch_shape_gives_the_same_bits(variant, threads, blocks, hp):
    run_steps(300_007, S.BASE_SEED + variant, 2, hp,
              launch=dict(variant=variant, block_threads=threads, grid_blocks=blocks),
              zero_pct=5.0, heavy_tail=True)


@pytest.mark.parametrize("variant", [4, 0x14, 0x24, 0x34, 0x54, 0x74])
@pytest.mark.parametrize("threads,lds", [(0, 0), (64, -1), (128, 20480), (512, 65536), (256, 1)])
def test_untiled_layout_and_wave_cap_give_the_same_bits(variant, threads, lds, hp):
    """The layout without a tile loop (the default of dos_adam_step) under every
    cache policy, block size and cap on resident waves."""
    run_steps(300_007, S.BASE_SEED + variant, 2, hp,
              launch=dict(variant=variant, block_threads=threads, grid_blocks=0, lds_bytes=lds),
              zero_pct=5.0, heavy_tail=True)


@pytest.mark.parametrize("variant", [5, 0x35, 0x75, 6, 0x56, 0x76])
@pytest.mark.parametrize("n,threads,lds,group", [(300_007, 0, 0, 0), (5, 64, -1, 0), (1023, 128, 20480, 2),
                                                 ((1 << 21) + 5, 256, 65536, 0), (262_147, 64, 27000, 16)])
def test_untiled_layouts_with_two_and_four_quads_per_lane_give_the_same_bits(variant, n, threads, lds, group, hp):
    """Layouts 5 and 6: a block owns two or four 1 KiB bursts per array instead of one."""
    run_steps(n, S.BASE_SEED + variant + n, 2, hp,
              launch=dict(variant=variant, block_threads=threads, grid_blocks=0, lds_bytes=lds, xcd_group=group),
              zero_pct=5.0, heavy_tail=True)


@pytest.mark.parametrize("n", [5, 300_007, (1 << 21) + 5])
@pytest.mark.parametrize("group", [1, 2, 16, 1024, 1 << 20])
def test_xcd_grouped_tile_order_gives_the_same_bits(n, group, hp):
    """Each XCD taking `group` consecutive tiles at a time is only another order of the same tiles."""
    run_steps(n, S.BASE_SEED + group, 2, hp, launch=dict(variant=0x74, xcd_group=group), zero_pct=5.0,
              heavy_tail=True)


# ---- Adagrad and RMSProp (Section 4.1 names them next to Adam): p and one accumulator

@pytest.mark.parametrize("optimizer", ["adagrad", "rmsprop"])
def test_other_rules_one_mebi_subgroup_ten_steps(optimizer, hp):
    run_steps(1 << 20, S.BASE_SEED + 40, 10, hp, optimizer=optimizer)


@pytest.mark.parametrize("optimizer", ["adagrad", "rmsprop"])
@pytest.mark.parametrize("n", [1, 3, 4, 5, 63, 257, 1025, 262_147, (1 << 21) + 5])
def test_other_rules_ragged_sizes(optimizer, n, hp):
    run_steps(n, S.BASE_SEED + n, 2, hp, optimizer=optimizer, zero_pct=1.0)


@pytest.mark.parametrize("optimizer", ["adagrad", "rmsprop"])
@pytest.mark.parametrize("variant,threads,lds", [(4, 0, 0), (0x34, 64, -1), (0x74, 128, 20480), (0x54, 512, 65536)])
def test_other_rules_launch_shapes(optimizer, variant, threads, lds, hp):
    run_steps(300_007, S.BASE_SEED + variant, 2, hp, optimizer=optimizer,
              launch=dict(variant=variant, block_threads=threads, grid_blocks=0, lds_bytes=lds),
              zero_pct=5.0, heavy_tail=True)


@pytest.mark.parametrize("optimizer", ["adagrad", "rmsprop"])
def test_other_rules_extremes_null_m_and_errors(optimizer, hp):
    """Extreme values go through the same IEEE operations on both sides; the first-moment
    array is never touched (a NULL pointer is accepted); tiled layouts are refused."""
    n = 4096
    sg = DeviceSubgroup(n, S.BASE_SEED + 6)
    sg.set_grads(1, heavy_tail=True, zero_pct=5.0, scale=10.0)
    p, m, v, g, lp = (x.copy() for x in sg.host_copy())
    g[:8] = ref.f32_to_bf16(np.array([1e-30, -1e-25, 3e38, -3e38, 0.0, -0.0, np.inf, np.nan], np.float32))
    v[8:12] = np.array([1e-45, 1e-40, 0.0, 1e30], np.float32)
    p[12:16] = np.array([1e-45, -1e-38, 3e38, -0.0], np.float32)
    m[:] = 7.0                                  # must come back untouched
    sg.p.copy_(torch.from_numpy(p)); sg.m.copy_(torch.from_numpy(m)); sg.v.copy_(torch.from_numpy(v))
    sg.g.view(torch.int16).copy_(torch.from_numpy(g.view(np.int16)))
    desc = dos.subgroup(sg.p.data_ptr(), None, sg.v.data_ptr(), sg.g.data_ptr(), sg.lp.data_ptr(), n,
                        dos.DOS_DEVICE, dos.DOS_DEVICE)
    state = [p, m, v, lp]
    for step in (1, 2, 3):
        dos.dos_adam_step(desc, dos.hparams(step=step, optimizer=optimizer, **hp), 0)
        torch.cuda.synchronize()
        oracle_step(state, g, hp, step, optimizer=optimizer)
        gp, gm, gv, _, glp = sg.host_copy()
        assert_parity(f"{optimizer} extremes step={step}", (gp, gm, gv), state[:3], glp, state[3])
        assert np.all(gm == 7.0)
    lib = dos.load()
    before = sg.host_copy()
    h = dos.hparams(step=1, optimizer=optimizer, **hp)
    cfg = dos.dos_launch_cfg(1, 64, 0)          # a tiled layout
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(h), None, C.byref(cfg)) == dos.DOS_EINVAL
    bad = dos.hparams(step=1, optimizer=7, **hp)
    assert lib.dos_adam_step(C.byref(sg.desc), C.byref(bad), None) == dos.DOS_EINVAL
    adam = dos.hparams(step=1, **hp)            # AdamW needs m
    assert lib.dos_adam_step(C.byref(desc), C.byref(adam), None) == dos.DOS_EINVAL
    torch.cuda.synchronize()
    for a, b in zip(before, sg.host_copy()):
        assert a.tobytes() == b.tobytes()


def test_extreme_values_match_the_oracle(hp):
    """Underflowing squares, huge gradients, denormal state, infinities and NaN go
    through the same IEEE operations on both sides."""
    n = 4096
    sg = DeviceSubgroup(n, S.BASE_SEED + 5)
    sg.set_grads(1, heavy_tail=True, zero_pct=5.0, scale=10.0)
    p, m, v, g, lp = (x.copy() for x in sg.host_copy())
    g[:8] = ref.f32_to_bf16(np.array([1e-30, -1e-25, 3e38, -3e38, 0.0, -0.0, np.inf, np.nan], np.float32))
    v[8:12] = np.array([1e-45, 1e-40, 0.0, 1e30], np.float32)
    m[8:12] = np.array([1e-45, -1e-40, 1e-38, 1e20], np.float32)
    p[12:16] = np.array([1e-45, -1e-38, 3e38, -0.0], np.float32)
    sg.p.copy_(torch.from_numpy(p)); sg.m.copy_(torch.from_numpy(m)); sg.v.copy_(torch.from_numpy(v))
    sg.g.view(torch.int16).copy_(torch.from_numpy(g.view(np.int16)))
    state = [p, m, v, lp]
    for step in (1, 2, 3):
        dos.dos_adam_step(sg.desc, dos.hparams(step=step, **hp), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        oracle_step(state, g, hp, step)
        gp, gm, gv, _, glp = sg.host_copy()
        assert_parity(f"extremes step={step}", (gp, gm, gv), state[:3], glp, state[3])


def test_other_hyperparameters_and_late_steps():
    hp = dict(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-5, weight_decay=0.1)
    n = 70_001
    sg = DeviceSubgroup(n, S.BASE_SEED + 9)
    st = sg.host_copy()
    state = [st[0], st[1], st[2], st[4]]
    for step in (1, 2, 17, 1000, 250_000):
        sg.set_grads(step, scale=3.0)
        dos.dos_adam_step(sg.desc, dos.hparams(step=step, **hp), 0)
        torch.cuda.synchronize()
        p, m, v, g, lp = sg.host_copy()
        oracle_step(state, g, hp, step)
        assert_parity(f"late step={step}", (p, m, v), state[:3], lp, state[3])


def test_errors_leave_device_state_untouched(hp):
    sg = DeviceSubgroup(1000, S.BASE_SEED)
    before = sg.host_copy()
    lib = dos.load()
    bad = dos.hparams(step=0, **hp)
    assert lib.dos_adam_step(C.byref(sg.desc), C.byref(bad), None) == dos.DOS_EINVAL
    cfg = dos.dos_launch_cfg(7, 0, 0)
    good = dos.hparams(step=1, **hp)
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(good), None, C.byref(cfg)) == dos.DOS_EINVAL
    cfg = dos.dos_launch_cfg(0, 100, 0)
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(good), None, C.byref(cfg)) == dos.DOS_EINVAL
    cfg = dos.dos_launch_cfg(0x51, 64, 0)       # system-scope stores exist in the untiled layout only
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(good), None, C.byref(cfg)) == dos.DOS_EINVAL
    cfg = dos.dos_launch_cfg(4, 64, 8)          # the untiled layout takes no grid size
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(good), None, C.byref(cfg)) == dos.DOS_EINVAL
    cfg = dos.dos_launch_cfg(0x74, 64, 0, 0, 3)  # XCD groups are powers of two
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(good), None, C.byref(cfg)) == dos.DOS_EINVAL
    cfg = dos.dos_launch_cfg(1, 64, 0, 0, 4)     # and exist in the untiled layout only
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(good), None, C.byref(cfg)) == dos.DOS_EINVAL
    cfg = dos.dos_launch_cfg(1, 64, 0, 65537)   # more LDS than a block may request
    assert lib.dos_adam_step_cfg(C.byref(sg.desc), C.byref(good), None, C.byref(cfg)) == dos.DOS_EINVAL
    torch.cuda.synchronize()
    for a, b in zip(before, sg.host_copy()):
        assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("optimizer", ["adamw", "adagrad"])
def test_can_be_captured_in_a_hip_graph_and_replayed(optimizer, hp):
    """dos_adam_step allocates nothing and synchronises nothing, so a stream that is being captured
    records just the kernel launch.  The graph is replayed four times with fresh gradients copied into
    the same buffer and eager work between the replays; every replay is checked against the oracle (the
    per-step scalars are kernel arguments, so each replay is the captured step number again)."""
    n = 300_007
    sg = DeviceSubgroup(n, S.BASE_SEED + 21)
    st = list(sg.host_copy())
    state = [st[0], st[1], st[2], st[4]]
    h = dos.hparams(step=5, optimizer=optimizer, **hp)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    sg.set_grads(1)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        dos.dos_adam_step(sg.desc, h, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    # capture records, it does not run: the state is still the initial one
    assert sg.host_copy()[0].tobytes() == state[0].tobytes()
    scratch = torch.zeros(1 << 20, device=DEV)
    for replay in range(1, 5):
        sg.set_grads(replay, zero_pct=1.0)
        scratch.add_(1.0)                                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        p, m, v, g, lp = sg.host_copy()
        oracle_step(state, g, hp, 5, optimizer=optimizer)
        assert_parity(f"{optimizer} graph replay {replay}", (p, m, v), state[:3], lp, state[3])
    assert float(scratch[0]) == 4.0


def test_runs_on_a_side_stream_without_synchronising(hp):
    side = torch.cuda.Stream()
    sg = DeviceSubgroup(1 << 18, S.BASE_SEED + 1)
    sg.set_grads(1)
    st = sg.host_copy()
    state = [st[0], st[1], st[2], st[4]]
    torch.cuda.synchronize()
    dos.dos_adam_step(sg.desc, dos.hparams(step=1, **hp), side.cuda_stream)
    side.synchronize()
    oracle_step(state, st[3], hp, 1)
    p, m, v, _, lp = sg.host_copy()
    assert_parity("side stream", (p, m, v), state[:3], lp, state[3])
