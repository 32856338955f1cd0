#!/usr/bin/env python3
"""Benchmark of the update-phase hot path on one MI355X.

One JSON line on stdout.  Primary workload (`value`): the device-resident AdamW
update over a GPT-2-small-sized flat partition, 4 subgroups of 31,000,000
parameters (fp32 p/m/v, bf16 gradients with 1 % exact zeros, bf16 parameter copy
out); a step is one pass over all four subgroups through dos_adam_step.  Extra
workloads ride in the same line under "extra": the single 1Mi-parameter subgroup,
the 7B-parameter resident state (70 x 100M), the 13B-parameter host-offloaded
state (130 x 100M, 40 GB GPU budget) run through dos_plan_subgroups +
dos_run_update_phase (with the host lane's 16-bit output stored straight into
device memory where the machine allows; then the pinned part of it through the
GPU lane alone and with 2 and 4 host threads, the whole once more through the
pinned ring, and under six schedules), the corners of the subgroup-size x budget
grid, and Adagrad / RMSProp on the primary workload's shape.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--extra c1,c3,c4,c5,rules|none] [--upload auto|direct|pull|dma]
                    [--rule adamw|adagrad|rmsprop] [--schedule balanced|stride|all_cpu|all_gpu|fixed:N]
                    [--c4-legs gpu_lane,ring,ablation|none] [--host-threads T] [--ablation] [--sweep] [--full-size]
                    [--ceilings]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
LINK_NOMINAL_GBPS = 64.0        # PCIe Gen5 x16 per direction, nominal
BYTES_PER_PARAM = 28            # reads 4+4+4+2, writes 4+4+4+2


UPLOAD_FLAGS = 0                # set in main(): how the host lane sends the 16-bit parameters to the device


def profiled_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 counter summary (None if absent)."""
    try:
        with open(os.path.join(ROOT, "profiles", name)) as f:
            for ln in f:
                if ln.strip().startswith("traffic_bytes_per_launch"):
                    return int(ln.split("=")[1].strip())
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def timed_resident(state, dos, torch, hp_kw, steps, warmup, stream, optimizer="adamw"):
    """W warm-up steps then exactly K timed steps; returns (wall_s, event_s, launches)."""
    sh = stream.cuda_stream
    n_sets = state.n_grad_sets

    def one_step(step):
        h = dos.hparams(step=step, optimizer=optimizer, **hp_kw)
        for sg in state.descs[(step - 1) % n_sets]:
            dos.dos_adam_step(sg, h, sh)

    for s in range(1, warmup + 1):
        one_step(s)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for s in range(warmup + 1, warmup + steps + 1):
        one_step(s)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, e0.elapsed_time(e1) * 1e-3, steps * len(state.sizes)


def oracle_leg(state, torch, np, ref, hp_kw, total_steps, grad_sets_host, check_against_gpu=True):
    """The oracle over the same inputs on the host cores: timed (all cores, and one
    core on a bounded sample) and compared with the GPU result."""
    out = {}
    n_sg = len(state.sizes)
    # initial state is regenerated on the GPU from the seed and copied to the host
    import dos_synth as S
    init = []
    for i, n in enumerate(state.sizes):
        p = torch.empty(n, dtype=torch.float32, device=state.device)
        S.fill_chunked(lambda start, count: S.params(state.seed, i, start, count, state.device), p)
        init.append([p.cpu().numpy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)])
        for a in init[-1][1:]:
            a.fill(0)                      # touch the pages outside the timed region
        del p
    # one core: one subgroup, three steps (bounded sample)
    one = [x.copy() for x in init[0]]
    t0 = time.perf_counter()
    for step in (1, 2, 3):
        ref.adamw_step(one[0], one[1], one[2], grad_sets_host[(step - 1) % len(grad_sets_host)][0], one[3],
                       step=step, threads=1, **hp_kw)
    t_one = time.perf_counter() - t0
    out["single_core_params_per_s"] = 3 * state.sizes[0] / t_one
    # all cores: the whole job
    t0 = time.perf_counter()
    used = 1
    for step in range(1, total_steps + 1):
        gs = grad_sets_host[(step - 1) % len(grad_sets_host)]
        for i in range(n_sg):
            used = ref.adamw_step(init[i][0], init[i][1], init[i][2], gs[i], init[i][3], step=step, threads=0, **hp_kw)
    t_all = time.perf_counter() - t0
    out["value"] = sum(state.sizes) * total_steps / t_all
    out["cores"] = used
    out["seconds"] = t_all + t_one
    if check_against_gpu:
        bad = 0
        for i in range(n_sg):
            for dev_t, host_a in ((state.p[i], init[i][0]), (state.m[i], init[i][1]), (state.v[i], init[i][2])):
                bad += int(np.count_nonzero(dev_t.cpu().numpy().view(np.uint32) != host_a.view(np.uint32)))
            bad += int(np.count_nonzero(state.lp[i].view(torch.int16).cpu().numpy().view(np.uint16) != init[i][3]))
        out["gpu_mismatches_vs_oracle"] = bad
    return out


def bench_c2(args, dos, torch, np):
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    hp_kw = dict(S.HPARAMS)
    sizes = [31_000_000] * 4
    n_sets = 4
    log("[c2] building 4 x 31,000,000 resident state")
    state = W.ResidentState(sizes, S.BASE_SEED, "cuda:0", n_grad_sets=n_sets)
    for k in range(n_sets):
        state.fill_grads(k, k + 1, zero_pct=1.0)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    if args.copy_probe:
        # known-size copy kernel for scaling the profiler's traffic counters: 1 GiB read + 1 GiB written
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        b = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
        from paper_2410_21316_amd import probe
        for _ in range(3):
            probe.dos_probe_copy(a.data_ptr(), b.data_ptr(), 1 << 30, stream.cuda_stream)
        stream.synchronize()
        del a, b
    wall, ev_s, launches = timed_resident(state, dos, torch, hp_kw, args.steps, args.warmup, stream)
    params_per_step = state.total
    value = params_per_step * args.steps / wall
    launch_s = ev_s / launches
    achieved = BYTES_PER_PARAM * sizes[0] / launch_s / 1e9
    log(f"[c2] {value/1e9:.1f} G params/s, kernel {launch_s*1e6:.1f} us/launch, {achieved:.0f} GB/s")
    res = {
        "metric": "adam_update_params_per_s", "value": value, "unit": "params/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "c2: 124M-param flat partition, 4 device-resident subgroups of 31,000,000; "
                               "fp32 p/m/v, bf16 grads ~N(0,1e-3) with 1% exact zeros, bf16 params out; "
                               "AdamW lr=1e-4 b1=0.9 b2=0.999 eps=1e-8 wd=0.01",
                   "subgroups": 4, "subgroup_params": sizes[0], "grad_sets_cycled": n_sets},
        "hbm_GBps": BYTES_PER_PARAM * value / 1e9,
        "hbm_frac_of_peak": BYTES_PER_PARAM * value / 1e9 / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": profiled_traffic("adam_kernel_c2.md"),
                     "traffic_source": "profiles/adam_kernel_c2.md: FETCH_SIZE and WRITE_SIZE of rocprofv3 --pmc runs of "
                                       "this command, scaled by a copy kernel of known size; not measured in this run",
                     "kernel": "dos::adam_kernel_tile (fused AdamW)", "bytes_per_launch": BYTES_PER_PARAM * sizes[0],
                     "avg_launch_us": launch_s * 1e6},
    }
    if not args.no_cpu_baseline:
        from oracle import adamw_oracle as ref
        log("[c2] oracle leg on the host cores")
        grads_host = [[state.g[i][k].view(torch.int16).cpu().numpy().view(np.uint16) for i in range(len(sizes))]
                      for k in range(n_sets)]
        o = oracle_leg(state, torch, np, ref, hp_kw, args.warmup + args.steps, grads_host)
        res["cpu_baseline"] = {"value": o["value"], "unit": "params/s", "cores": o["cores"], "kind": "oracle",
                               "sample": f"the whole c2 job ({args.warmup + args.steps} steps x 124M params) under "
                                         f"the oracle's static parallel-for; single core on one 31M subgroup x 3 steps: "
                                         f"{o['single_core_params_per_s']:.3e} params/s",
                               "single_core_value": o["single_core_params_per_s"],
                               "seconds": o["seconds"],
                               "gpu_mismatches_vs_oracle": o["gpu_mismatches_vs_oracle"]}
        log(f"[c2] oracle {o['value']/1e9:.2f} G params/s on {o['cores']} cores; "
            f"GPU-vs-oracle mismatching words: {o['gpu_mismatches_vs_oracle']}")
    del state
    torch.cuda.empty_cache()
    return res


def bench_other_rules(args, dos, torch, np):
    """Adagrad and RMSProp (the other adaptive optimizers the paper's Section 4.1 names) on the c2 shape:
    p and one accumulator, 20 bytes per parameter (reads 4+4+2, writes 4+4+2); whole state compared with
    the oracle's rule of the same name."""
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    from oracle import adamw_oracle as ref
    hp_kw = dict(S.HPARAMS)
    sizes = [31_000_000] * 4
    n_sets = 4
    out = {}
    for rule in ("adagrad", "rmsprop"):
        state = W.ResidentState(sizes, S.BASE_SEED + 3, "cuda:0", n_grad_sets=n_sets)
        for k in range(n_sets):
            state.fill_grads(k, k + 1, zero_pct=1.0)
        torch.cuda.synchronize()
        stream = torch.cuda.Stream()
        stream.wait_stream(torch.cuda.current_stream())
        wall, ev_s, launches = timed_resident(state, dos, torch, hp_kw, args.steps, args.warmup, stream, rule)
        value = state.total * args.steps / wall
        launch_s = ev_s / launches
        r = {"params_per_s": value, "ms_per_step": wall / args.steps * 1e3, "bytes_per_param": 20,
             "kernel_avg_launch_us": launch_s * 1e6, "kernel_GBps": 20 * sizes[0] / launch_s / 1e9,
             "hbm_frac_of_peak": 20 * sizes[0] / launch_s / 1e9 / HBM_PEAK_GBPS}
        if not args.no_cpu_baseline:
            bad = 0
            t_or = 0.0
            for i, n in enumerate(sizes):
                p = torch.empty(n, dtype=torch.float32, device="cuda:0")
                S.fill_chunked(lambda start, count: S.params(state.seed, i, start, count, "cuda:0"), p)
                want = [p.cpu().numpy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)]
                del p
                gs = [state.g[i][k].view(torch.int16).cpu().numpy().view(np.uint16) for k in range(n_sets)]
                t0 = time.perf_counter()
                for step in range(1, args.warmup + args.steps + 1):
                    ref.optimizer_step(rule, want[0], want[1], want[2], gs[(step - 1) % n_sets], want[3], step=step,
                                       threads=0, **hp_kw)
                t_or += time.perf_counter() - t0
                for dev_t, host_a in ((state.p[i], want[0]), (state.m[i], want[1]), (state.v[i], want[2])):
                    bad += int(np.count_nonzero(dev_t.cpu().numpy().view(np.uint32) != host_a.view(np.uint32)))
                bad += int(np.count_nonzero(state.lp[i].view(torch.int16).cpu().numpy().view(np.uint16) != want[3]))
            r["gpu_mismatches_vs_oracle"] = bad
            r["oracle_params_per_s"] = state.total * (args.warmup + args.steps) / t_or
        log(f"[rules] {rule}: {value/1e9:.1f} G params/s, kernel {launch_s*1e6:.1f} us/launch, "
            f"{r['kernel_GBps']:.0f} GB/s at 20 B/param, mismatches {r.get('gpu_mismatches_vs_oracle')}")
        out[rule] = r
        del state
        torch.cuda.empty_cache()
    out["workload"] = "c2 shape (4 x 31,000,000 resident, 1% zero grads) under Adagrad and RMSProp"
    return out


def bench_ceilings(args, dos, torch, np):
    """What bounds the AdamW kernel: its own launch with only the loads, only the stores, both without the
    arithmetic, and the full kernel, on 4 x 100M-parameter subgroups (rotated, so nothing is reused from a cache)."""
    from paper_2410_21316_amd import probe, workloads as W
    import dos_synth as S
    n = 100_000_000
    state = W.ResidentState([n] * 4, S.BASE_SEED + 7, "cuda:0")
    state.fill_grads(0, 1)
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    sh = stream.cuda_stream
    hp = dos.hparams(step=1, **S.HPARAMS)

    def rate(fn, bytes_per_param):
        for sg in state.descs[0]:
            fn(sg)
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(4):
            for sg in state.descs[0]:
                fn(sg)
        e1.record(stream)
        stream.synchronize()
        return bytes_per_param * n * 16 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    out = {"params_per_launch": n,
           "note": "same launch shape as dos_adam_step: 16 B per lane, non-temporal, 64-thread blocks; "
                   "'capped' = its cap on resident waves per compute unit, 'uncapped' = none"}
    out["adamw_capped_GBps"] = rate(lambda sg: dos.dos_adam_step(sg, hp, sh), 28)
    out["adamw_uncapped_GBps"] = rate(lambda sg: dos.dos_adam_step_cfg(sg, hp, sh, variant=0x74, lds_bytes=-1), 28)
    for name, lds in (("capped", probe.DEFAULT_LDS_CAP), ("uncapped", 0)):
        rd = rate(lambda sg: probe.dos_probe_adam_traffic(sg, 0, sh, lds), 14)
        both = rate(lambda sg: probe.dos_probe_adam_traffic(sg, 2, sh, lds), 28)
        out[f"loads_only_{name}_GBps"] = rd
        out[f"loads_and_stores_no_math_{name}_GBps"] = both
    for name, lds in (("capped", probe.DEFAULT_LDS_CAP), ("uncapped", 0)):   # last: these zero the state
        out[f"stores_only_{name}_GBps"] = rate(lambda sg: probe.dos_probe_adam_traffic(sg, 1, sh, lds), 14)
    rd = max(out["loads_only_capped_GBps"], out["loads_only_uncapped_GBps"])
    wr = max(out["stores_only_capped_GBps"], out["stores_only_uncapped_GBps"])
    out["time_shared_mix_GBps"] = 1.0 / (0.5 / rd + 0.5 / wr)
    log("[ceilings] " + ", ".join(f"{k} {v:.0f}" for k, v in out.items() if k.endswith("GBps")))
    return out


def bench_c1(args, dos, torch, np):
    """Single device-resident subgroup of 1,048,576 parameters, fresh gradients per step, 10 steps: a parity
    configuration (29 MB per step fits the on-die caches and one launch is a few microseconds: launch-bound)."""
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    from oracle import adamw_oracle as ref
    hp_kw = dict(S.HPARAMS)
    n = 1 << 20
    state = W.ResidentState([n], S.BASE_SEED + 1, "cuda:0", n_grad_sets=10)
    for k in range(10):
        state.fill_grads(k, k + 1)
    want = [state.p[0].cpu().numpy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)]
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for step in range(1, 11):
        dos.dos_adam_step(state.descs[step - 1][0], dos.hparams(step=step, **hp_kw), stream.cuda_stream)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for step in range(1, 11):
        g = state.g[0][step - 1].view(torch.int16).cpu().numpy().view(np.uint16)
        ref.adamw_step(want[0], want[1], want[2], g, want[3], step=step, **hp_kw)
    mism = sum(int(np.count_nonzero(t.cpu().numpy().view(np.uint32) != w.view(np.uint32)))
               for t, w in ((state.p[0], want[0]), (state.m[0], want[1]), (state.v[0], want[2])))
    mism += int(np.count_nonzero(state.lp[0].view(torch.int16).cpu().numpy().view(np.uint16) != want[3]))
    ev = e0.elapsed_time(e1) * 1e-3
    out = {"workload": "c1: one device-resident subgroup of 1,048,576 params, fresh grads ~N(0,1e-3) per step, 10 steps",
           "us_per_step_wall": wall / 10 * 1e6, "us_per_step_on_stream": ev / 10 * 1e6,
           "params_per_s": n * 10 / ev, "effective_GBps": BYTES_PER_PARAM * n * 10 / ev / 1e9,
           "note": "launch- and cache-dominated; not a roofline configuration",
           "mismatches_vs_oracle": mism}
    log(f"[c1] {out['us_per_step_on_stream']:.1f} us/step on the stream, mismatches {mism}")
    return out


def bench_c3(args, dos, torch, np):
    """7B-parameter optimizer state fully on the GPU: 70 subgroups of 100M."""
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    from oracle import adamw_oracle as ref
    hp_kw = dict(S.HPARAMS)
    sizes = [100_000_000] * 70
    steps, warmup = 5, 1
    log("[c3] building 70 x 100,000,000 resident state (112 GB)")
    t0 = time.perf_counter()
    state = W.ResidentState(sizes, S.BASE_SEED + 3, "cuda:0", n_grad_sets=1)
    scales = [S.subgroup_scale(S.BASE_SEED + 3, i) for i in range(len(sizes))]
    idx = torch.from_numpy(W.sample_index(sizes[0])).to("cuda:0")
    samp = [[state.p[i][idx].cpu().numpy(), np.zeros(idx.numel(), np.float32), np.zeros(idx.numel(), np.float32),
             np.zeros(idx.numel(), np.uint16)] for i in range(len(sizes))]
    log(f"[c3] built in {time.perf_counter()-t0:.1f}s")
    stream = torch.cuda.Stream()
    sh = stream.cuda_stream
    times, ev_times = [], []
    mism = 0
    for step in range(1, warmup + steps + 1):
        state.fill_grads(0, step, scales=scales)
        torch.cuda.synchronize()
        h = dos.hparams(step=step, **hp_kw)
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for sg in state.descs[0]:
            dos.dos_adam_step(sg, h, sh)
        e1.record(stream)
        torch.cuda.synchronize()
        if step > warmup:
            times.append(time.perf_counter() - t0)
            ev_times.append(e0.elapsed_time(e1) * 1e-3)
        # oracle on the index subset
        for i in range(len(sizes)):
            gs = state.g[i][0][idx].view(torch.int16).cpu().numpy().view(np.uint16)
            ref.adamw_step(samp[i][0], samp[i][1], samp[i][2], gs, samp[i][3], step=step, threads=0, **hp_kw)
    for i in range(len(sizes)):
        for dev_t, host_a in ((state.p[i], samp[i][0]), (state.m[i], samp[i][1]), (state.v[i], samp[i][2])):
            mism += int(np.count_nonzero(dev_t[idx].cpu().numpy().view(np.uint32) != host_a.view(np.uint32)))
        mism += int(np.count_nonzero(state.lp[i][idx].view(torch.int16).cpu().numpy().view(np.uint16) != samp[i][3]))
    wall = sum(times)
    value = state.total * steps / wall
    launch_s = sum(ev_times) / (steps * len(sizes))
    out = {"workload": "c3: 7B params resident, 70 subgroups of 100,000,000; grads ~N(0,1e-3) x per-subgroup "
                       "log-uniform[0.1,10] scale; 5 steps",
           "params_per_s": value, "ms_per_step": wall / steps * 1e3, "hbm_GBps": BYTES_PER_PARAM * value / 1e9,
           "hbm_frac_of_peak": BYTES_PER_PARAM * value / 1e9 / HBM_PEAK_GBPS,
           "kernel_avg_launch_us": launch_s * 1e6,
           "kernel_GBps": BYTES_PER_PARAM * sizes[0] / launch_s / 1e9,
           "oracle_sample": "first 65,536 of every 1,048,576 elements of every subgroup, every step",
           "sample_mismatches_vs_oracle": mism}
    log(f"[c3] {value/1e9:.1f} G params/s, {out['hbm_GBps']:.0f} GB/s, {out['ms_per_step']:.2f} ms/step, "
        f"sample mismatches {mism}")
    del state
    torch.cuda.empty_cache()
    return out


def make_plan(dos, schedule, cm, sizes, budget_bytes, residents_max, bpp=12, cpu_only=None):
    """schedule: 'balanced' (this library's planner), 'stride' (Eq. 1 + Algorithm 1), 'all_cpu' (every update
    on the host cores, as a fully offloaded optimizer does), 'static' (a fixed set of residents that fits the
    budget, everything else on the host cores: static hybrid placement without interleaving), 'all_gpu'
    (every stageable subgroup through the GPU lane), 'fixed:<n>' (n stageable subgroups, evenly spread,
    through the GPU lane -- a plan that does not move, for profiling)."""
    if schedule == "balanced":
        return dos.dos_plan_subgroups(cm, sizes, budget_bytes, dos.DOS_PLAN_BALANCED, residents_max, bpp, cpu_only)
    if schedule == "stride":
        return dos.dos_plan_subgroups(cm, sizes, budget_bytes, dos.DOS_PLAN_STRIDE, residents_max, bpp, cpu_only)
    base = dos.dos_plan_subgroups(cm, sizes, budget_bytes, dos.DOS_PLAN_BALANCED,
                                  len(sizes) if schedule == "static" else 0, bpp, cpu_only)
    if schedule == "all_cpu":
        return dos.Plan.manual([dos.DOS_ON_CPU] * len(sizes), None, base.c.n_slots, base.c.slot_params)
    if schedule == "static":
        res = base.residents
        return dos.Plan.manual([dos.DOS_ON_GPU if r else dos.DOS_ON_CPU for r in res], None, base.c.n_slots,
                               base.c.slot_params, res)
    movable = [i for i in range(len(sizes)) if not (cpu_only and cpu_only[i])]
    if schedule == "all_gpu":
        chosen = set(movable)
    elif schedule.startswith("fixed:"):
        c = min(int(schedule.split(":")[1]), len(movable))
        chosen = {movable[q] for q in range(len(movable)) if (q + 1) * c // len(movable) > q * c // len(movable)}
    else:
        raise ValueError(schedule)
    return dos.Plan.manual([dos.DOS_ON_GPU if i in chosen else dos.DOS_ON_CPU for i in range(len(sizes))], None,
                           base.c.n_slots, base.c.slot_params)


class OracleShare:
    """The oracle's share of a host-offloaded state: the first `take` of every 1,048,576 elements of every
    subgroup (elements are independent, so the oracle is exact on its share).  It follows the state through
    every phase that is run on it, whatever leg of the benchmark runs it."""

    def __init__(self, state, torch, np, take=1 << 16):
        from paper_2410_21316_amd import workloads as W
        self.W, self.torch, self.np, self.take = W, torch, np, take
        self.samp = [[W.sample_take(t, take=take).cpu().numpy().copy() for t in state.state(i)]
                     + [np.zeros(W.sample_take(state.state(i)[0], take=take).numel(), np.uint16)]
                     for i in range(len(state.sizes))]
        self.touched = [False] * len(state.sizes)

    def describe(self):
        return f"first {self.take:,} of every 1,048,576 elements of every subgroup, every step"

    def step(self, state, rule, step, hp_kw, only=None):
        from oracle import adamw_oracle as ref
        for i in (range(len(state.sizes)) if only is None else only):
            gs = self.W.sample_take(state.g[i], take=self.take).view(self.torch.int16).cpu().numpy().view(self.np.uint16)
            s = self.samp[i]
            ref.optimizer_step(rule, s[0], s[1], s[2], gs, s[3], step=step, threads=0, **hp_kw)
            self.touched[i] = True

    def mismatches(self, state):
        np = self.np
        bad = 0
        for i in range(len(state.sizes)):
            for t, want in zip(state.state(i), self.samp[i][:3]):
                got = self.W.sample_take(t, take=self.take).cpu().numpy()
                bad += int(np.count_nonzero(got.view(np.uint32) != want.view(np.uint32)))
            if self.touched[i]:                 # the 16-bit copy exists once the subgroup has been updated
                got = self.W.sample_take(state.lp[i], take=self.take).view(self.torch.int16).cpu().numpy().view(np.uint16)
                bad += int(np.count_nonzero(got != self.samp[i][3]))
        return bad


def host_stream_ceiling(dos, torch, np, host_threads, direct):
    """Host-memory stream with the host update's access pattern and (almost) no arithmetic, in the same
    run, measured the way dos_calibrate measures the update itself: chunks from a shared counter over a buffer
    of 16 Mi parameters per thread (7.5 GB for 16 threads, far beyond the host's caches), about a quarter of a
    second per measurement, best of three, for the phase's thread count and for three quarters and half of it.
    Reads p, m, v, g and rewrites p, m, v; the 16-bit output goes through the PCIe BAR into device memory
    (direct uploads) or into host memory (ring uploads)."""
    from paper_2410_21316_amd import probe
    n = max(64 << 20, min(512 << 20, host_threads << 24))
    arrs = [torch.empty(n, dtype=torch.float32) for _ in range(3)] + [torch.empty(n, dtype=torch.int16)]
    for t in arrs:
        dos.dos_host_advise_hugepages(t.data_ptr(), t.numel() * t.element_size())
        dos.dos_host_prefault(t.data_ptr(), t.numel() * t.element_size(), host_threads)
        t.zero_()
    out_n = 64 << 20
    if direct:
        out = torch.zeros(out_n, dtype=torch.int16, device="cuda:0")
        torch.cuda.synchronize()
        dos.dos_host_prefault(out.data_ptr(), out_n * 2, host_threads)      # map the device pages for the host
    else:
        out, out_n = torch.zeros(n, dtype=torch.int16), n
    ptrs = [t.data_ptr() for t in arrs]
    bpp = 26 if direct else 28
    by_threads = {}
    for T in sorted({max(1, host_threads // 2), max(1, host_threads * 3 // 4), host_threads}):
        t1 = probe.dos_probe_host_stream(*ptrs, out.data_ptr(), n, out_n, T, 1, direct)         # warm-up, and its time
        reps = max(1, min(400, int(0.25 / t1)))
        best = min(probe.dos_probe_host_stream(*ptrs, out.data_ptr(), n, out_n, T, reps, direct) / reps
                   for _ in range(3))
        by_threads[T] = bpp * n / best / 1e9
    top = max(by_threads, key=by_threads.get)
    return {"GBps": by_threads[top], "threads_at_best": top, "GBps_by_threads": by_threads, "bytes_per_param": bpp,
            "what": "plain stream of the host update's access pattern (read p, m, v, g; rewrite p, m, v; 16-bit output "
                    + ("stored through the PCIe BAR" if direct else "to host memory") + f"), {n >> 20} Mi parameters in "
                    "1 Mi chunks from a shared counter, best of three quarter-second measurements per thread count, same run"}


class HostMemoryLoad:
    """The plain stream of host_stream_ceiling (host memory only: 28 B per parameter), kept running on
    `threads` threads in the background between start() and stop(): what the host lane of a ring-upload phase
    does to the host's memory while the link is working.  stop() returns the stream's own rate in GB/s."""

    def __init__(self, dos, torch, threads):
        from paper_2410_21316_amd import probe
        self.probe, self.threads = probe, threads
        self.n = n = max(64 << 20, min(512 << 20, threads << 24))
        self.arrs = [torch.empty(n, dtype=torch.float32) for _ in range(3)] + [torch.empty(n, dtype=torch.int16)
                                                                                for _ in range(2)]
        for t in self.arrs:
            dos.dos_host_advise_hugepages(t.data_ptr(), t.numel() * t.element_size())
            dos.dos_host_prefault(t.data_ptr(), t.numel() * t.element_size(), threads)
            t.zero_()
        self.ptrs = [t.data_ptr() for t in self.arrs]
        t1 = self._sweeps(1)
        self.reps = max(1, min(400, int(0.1 / t1)))
        self.thread = None

    def _sweeps(self, reps):
        return self.probe.dos_probe_host_stream(*self.ptrs, self.n, self.n, self.threads, reps, 0)

    def start(self):
        import threading
        self.halt, self.sweeps, self.busy_s = False, 0, 0.0

        def loop():
            while not self.halt:
                self.busy_s += self._sweeps(self.reps)
                self.sweeps += self.reps
        self.thread = threading.Thread(target=loop, daemon=True)
        self.thread.start()

    def stop(self):
        self.halt = True
        self.thread.join()
        self.thread = None
        return 28.0 * self.n * self.sweeps / max(self.busy_s, 1e-9) / 1e9


def calibrate_peaks(ctx, log, tag, rule):
    """dos_calibrate twice; each rate keeps the better of the two (they are peaks: bounds are priced with them)."""
    cms = [ctx.dos_calibrate() for _ in range(2)]
    cm = cms[0]
    for f in ("h2d_Bps", "d2h_Bps", "gpu_params_per_s", "cpu_params_per_s"):
        setattr(cm, f, max(getattr(c, f) for c in cms))
    cm.launch_overhead_s = min(c.launch_overhead_s for c in cms)
    cm.fp32_arrays = 3 if rule == "adamw" else 2    # Adagrad, RMSProp stage p and v only
    log(f"[{tag}] calibrated: H2D {cm.h2d_Bps/1e9:.1f} GB/s, D2H {cm.d2h_Bps/1e9:.1f} GB/s (duplex), "
        f"U_g {cm.gpu_params_per_s/1e9:.1f} G/s, U_c {cm.cpu_params_per_s/1e9:.2f} G/s (stand-alone, through the "
        f"upload path in use)")
    return cm


def run_interleaved(dos, torch, np, sizes, budget_bytes, steps, warmup, host_threads, gkw, seed, check=True,
                    cm=None, residents_max=0, tag="c4", state=None, adapt=True, schedule="balanced",
                    fresh_grads=True, spill_grads=False, pageable_rest=False, rule="adamw", upload_flags=None,
                    share=None, only=None, keep_steps=True, peaks=None):
    """Plan + run the interleaved phase on a host-offloaded state; returns a dict.
    fresh_grads=False generates the gradients once and reuses them for every step, fresh_grads="keep" uses
    the gradients the state already holds (the caller generated them);
    spill_grads=True keeps every gradient in pinned host memory (GPU-planned subgroups fetch theirs
    with p, m, v through 14-byte slots); pageable_rest=True keeps the subgroups the machine cannot pin in
    ordinary host memory (CPU-only) instead of dropping them; `only` restricts the phase to a subset of the
    subgroups (the others are not part of the phase at all); `share` is the oracle's share of the state;
    `peaks` are the calibrated stand-alone rates that price the bounds when `cm` is a cost model that earlier
    phases have already adapted."""
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    hp_kw = dict(S.HPARAMS)
    own_state = state is None
    if upload_flags is None:
        upload_flags = UPLOAD_FLAGS
    t0 = time.perf_counter()
    if own_state:
        # leave room for the context's pinned upload ring
        state = W.OffloadedState(sizes, seed, "cuda:0", pinned_reserve_bytes=1 << 30, pageable_rest=pageable_rest)
        if state.truncated:
            log(f"[{tag}] this machine pins only {len(state.sizes)} of the {len(sizes)} subgroups "
                f"(hipHostMalloc limit); running the scaled-down state")
        elif state.n_pinned < len(sizes):
            log(f"[{tag}] this machine pins only {state.n_pinned} of the {len(sizes)} subgroups (hipHostMalloc "
                f"limit); the other {len(sizes) - state.n_pinned} live in pageable host memory and stay on the host cores")
        sizes = list(state.sizes)
        log(f"[{tag}] built {sum(sizes)*12/1e9:.0f} GB of host state in {time.perf_counter()-t0:.1f}s")
        if upload_flags & dos.DOS_CTX_UPLOAD_DIRECT:
            t0 = time.perf_counter()
            state.map_model_for_host_writes(host_threads)
            log(f"[{tag}] mapped the 16-bit model ({sum(sizes)*2/1e9:.0f} GB) for host writes in {time.perf_counter()-t0:.1f}s")
    all_sizes = list(state.sizes)
    members = list(range(len(all_sizes))) if only is None else list(only)
    sizes = [all_sizes[i] for i in members]
    cpu_only_all = state.cpu_only
    cpu_only = [cpu_only_all[i] for i in members]
    cpu_only = cpu_only if any(cpu_only) else None
    # slots first (they decide what the context can do), then calibration, then the plan
    probe_cm = cm or dos.cost_model(50e9, 50e9, 180e9, 5e9)
    bpp = 14 if spill_grads else 12
    plan = dos.dos_plan_subgroups(probe_cm, sizes, budget_bytes, dos.DOS_PLAN_BALANCED, residents_max, bpp, cpu_only)
    ctx = W.make_context(plan.c.n_slots, plan.c.slot_params, host_threads, flags=dos.DOS_CTX_PROFILE | upload_flags,
                         stage_grads=spill_grads)
    if cm is None:
        cm = calibrate_peaks(ctx, log, tag, rule)
    calibrated = tuple(peaks) if peaks else (cm.h2d_Bps, cm.d2h_Bps, cm.gpu_params_per_s, cm.cpu_params_per_s,
                                             cm.downscale_params_per_s, cm.launch_overhead_s)
    link = (calibrated[0], calibrated[1])
    results = []
    if check and share is None:
        share = OracleShare(state, torch, np)
    sb = 12.0 if rule == "adamw" else 8.0
    for step in range(1, warmup + steps + 1):
        # with feedback on, the first warm-up phase runs on the host cores alone: together with the staged
        # phases that follow it tells the cost model what staging takes away from the host lane
        probe_all_cpu = adapt and schedule == "balanced" and step == 1 and warmup >= 2 and not residents_max
        plan = make_plan(dos, "all_cpu" if probe_all_cpu else schedule, cm, sizes, budget_bytes, residents_max, bpp,
                         cpu_only)
        # the plan covers the members; everybody else keeps its place and takes no part
        tg_all, res_all = [dos.DOS_ON_CPU] * len(all_sizes), [0] * len(all_sizes)
        for k, i in enumerate(members):
            tg_all[i], res_all[i] = plan.targets[k], plan.residents[k]
        state.place(tg_all, res_all, spill_all_grads=spill_grads)
        if fresh_grads is True or (step == 1 and fresh_grads != "keep"):
            state.fill_grads(step, **gkw)
        state.sync_host_grads()
        sgs = state.sgs if only is None else (dos.dos_subgroup * len(members))(*[state.sgs[i] for i in members])
        st = ctx.dos_run_update_phase(sgs, plan, dos.hparams(step=step, optimizer=rule, **hp_kw))
        lb_plan = max(st.h2d_bytes / link[0], st.d2h_bytes / link[1])
        lb_nominal = max(st.h2d_bytes, st.d2h_bytes) / (LINK_NOMINAL_GBPS * 1e9)
        staged = sb * st.params_gpu
        r = {"step": step, "wall_s": st.wall_s, "n_gpu": st.n_gpu, "n_cpu": st.n_cpu, "n_resident": st.n_resident,
             "gpu_fraction": (st.params_gpu + st.params_resident) / max(1, sum(sizes)),
             "h2d_GBps": st.h2d_bytes / st.wall_s / 1e9, "d2h_GBps": st.d2h_bytes / st.wall_s / 1e9,
             "h2d_busy_s": st.h2d_busy_s, "d2h_busy_s": st.d2h_busy_s, "gpu_busy_s": st.gpu_busy_s,
             "h2d_span_s": st.h2d_span_s, "d2h_span_s": st.d2h_span_s,
             "duplex_overlap_s": st.duplex_overlap_s, "cpu_lane_s": st.cpu_lane_s, "gpu_lane_s": st.gpu_lane_s,
             "host_update_params_per_s": st.params_cpu / st.cpu_lane_s if st.cpu_lane_s > 0 else None,
             # host memory traffic of the phase: 26 B per host-updated parameter (18 for the rules without a
             # first moment; 2 more through the ring), and every staged byte is read from or written to host
             # memory once
             "host_dram_GBps": (((26.0 if rule == "adamw" else 18.0)
                                 + (0.0 if upload_flags & dos.DOS_CTX_UPLOAD_DIRECT else 2.0)) * st.params_cpu
                                + 2.0 * staged) / st.wall_s / 1e9,
             "lower_bound_s": lb_plan, "ratio_to_lower_bound": st.wall_s / lb_plan if lb_plan > 0 else None,
             "ratio_to_nominal_link_bound": st.wall_s / lb_nominal if lb_nominal > 0 else None,
             "predicted_s": plan.c.predicted_s, "timed": step > warmup}
        if st.params_gpu and st.h2d_busy_s > 0:
            # where the GPU lane's time went: the prefetches at the calibrated rate, what they lost to the
            # uploads and the host update sharing the direction and the host's memory, the gaps between
            # copies, and the tail behind the last prefetch (its kernel and flush)
            ideal = staged / link[0]
            uploads = 2.0 * st.params_cpu
            share_busy = min(1.0, st.h2d_busy_s / st.cpu_lane_s) if st.cpu_lane_s > 0 else 0.0
            combined = (staged + uploads * share_busy) / st.h2d_busy_s          # uploads are spread over the host lane
            r["gpu_lane_accounting"] = {
                "h2d_combined_rate_while_prefetches_busy_GBps": combined / 1e9,
                "link_bound_of_plan_s": lb_plan,
                "excess_over_link_bound_s": st.wall_s - lb_plan,
                "excess_from_link_rate_shortfall_s": (st.h2d_bytes / combined - st.h2d_bytes / link[0])
                                                     if st.h2d_bytes / link[0] >= st.d2h_bytes / link[1] else None,
                "prefetches_at_calibrated_rate_s": ideal, "prefetch_slowdown_s": st.h2d_busy_s - ideal,
                "h2d_idle_between_copies_s": st.h2d_span_s - st.h2d_busy_s,
                "d2h_idle_between_copies_s": st.d2h_span_s - st.d2h_busy_s,
                "lead_and_tail_s": st.gpu_lane_s - st.h2d_span_s,
                "sum_s": ideal + (st.h2d_busy_s - ideal) + (st.h2d_span_s - st.h2d_busy_s)
                         + (st.gpu_lane_s - st.h2d_span_s),
                "gpu_lane_s": st.gpu_lane_s,
                "h2d_rate_while_busy_GBps": staged / st.h2d_busy_s / 1e9,
                "d2h_rate_while_busy_GBps": staged / st.d2h_busy_s / 1e9 if st.d2h_busy_s > 0 else None,
                "uploads_share_of_h2d_bytes": 2.0 * st.params_cpu / st.h2d_bytes if st.h2d_bytes else 0.0}
        results.append(r)
        log(f"[{tag}] step {step}: {st.wall_s:.3f}s gpu {st.n_gpu}+{st.n_resident}r cpu {st.n_cpu} "
            f"lanes cpu {st.cpu_lane_s:.3f} gpu {st.gpu_lane_s:.3f} LB {lb_plan:.3f} ratio "
            f"{r['ratio_to_lower_bound'] if r['ratio_to_lower_bound'] is None else round(r['ratio_to_lower_bound'], 3)}")
        if adapt:
            # feed the measured lane rates back into the cost model (the plan is
            # re-derived every iteration, as a training loop would)
            dos.dos_cost_model_observe(cm, st)
        if check:
            share.step(state, rule, step, hp_kw, only=members)
    mism = share.mismatches(state) if check else None
    timed = [r for r in results if r["timed"]]
    best = min(timed, key=lambda r: r["wall_s"])
    mean_wall = sum(r["wall_s"] for r in timed) / len(timed)
    res_params = sum(n for n, r in zip(sizes, plan.residents or [0] * len(sizes)) if r)
    pinned_ok = [not c for c in (cpu_only or [0] * len(sizes))]
    movable = [ok and not r for ok, r in zip(pinned_ok, plan.residents or [0] * len(sizes))]
    # a bound must be priced with peaks: where a phase beat a calibrated rate, the phase's own rate is the peak
    seen_u_cpu = max([r["host_update_params_per_s"] or 0.0 for r in results])
    u_cpu_peak = max(calibrated[3], seen_u_cpu)
    lb_opt, k_opt = lower_bound_opt(sizes, movable, link, calibrated[2], u_cpu_peak, sb, res_params)
    lb_free, k_free = lower_bound_opt(sizes, [not r for r in (plan.residents or [0] * len(sizes))], link,
                                      calibrated[2], u_cpu_peak, sb, res_params)
    walls = sorted(r["wall_s"] for r in timed)
    out = {"update_phase_s_per_iter": mean_wall, "best_s": best["wall_s"], "median_s": walls[len(walls) // 2],
           "lower_bound_opt_s": lb_opt, "lower_bound_opt_gpu_subgroups": k_opt,
           "ratio_to_lower_bound_opt": mean_wall / lb_opt,
           "lower_bound_opt_all_pinnable_s": lb_free, "ratio_to_lower_bound_opt_all_pinnable": mean_wall / lb_free,
           "lower_bound_note": "ratio_to_lower_bound prices the executed plan's link bytes at the measured duplex "
                               "link rates; lower_bound_opt is the best any split could reach with link, host "
                               "update and GPU update all at their stand-alone peaks (the calibrated rates, or a "
                               "phase's own rate where it beat them; over the subgroups this machine can pin; "
                               "_all_pinnable: if it could pin all of them)",
           "host_rate_peak_used_for_bounds": u_cpu_peak, "host_rate_calibrated": calibrated[3],
           "host_rate_best_phase": seen_u_cpu, "phase_beat_calibrated_host_rate": seen_u_cpu > calibrated[3],
           "params": sum(sizes), "n_subgroups": len(sizes), "n_subgroups_pinned": sum(pinned_ok),
           "params_per_s": sum(sizes) / mean_wall,
           "ratio_to_lower_bound": sum(r["ratio_to_lower_bound"] for r in timed) / len(timed),
           "ratio_to_nominal_link_bound": sum(r["ratio_to_nominal_link_bound"] for r in timed) / len(timed),
           "link_duplex_GBps": {"h2d": link[0] / 1e9, "d2h": link[1] / 1e9, "nominal": LINK_NOMINAL_GBPS},
           "h2d_GBps": best["h2d_GBps"], "d2h_GBps": best["d2h_GBps"],
           "h2d_frac_of_measured_link": best["h2d_GBps"] * 1e9 / link[0],
           "d2h_frac_of_measured_link": best["d2h_GBps"] * 1e9 / link[1],
           "host_update_params_per_s": best["host_update_params_per_s"],
           "host_dram_GBps": best["host_dram_GBps"],
           "gpu_fraction": best["gpu_fraction"], "n_slots": plan.c.n_slots, "slot_params": plan.c.slot_params,
           "host_threads": host_threads, "uploads": {0: "pull", 2: "dma", 8: "direct"}[upload_flags],
           "sample_mismatches_vs_oracle": mism, "oracle_sample": share.describe() if check else None,
           "calibrated": calibrated}
    out["_cost_model"] = cm                      # as adapted by the phases of this leg (not JSON: popped by callers)
    if "gpu_lane_accounting" in best:
        out["gpu_lane_accounting"] = best["gpu_lane_accounting"]
    if keep_steps:
        out["steps"] = results
    ctx.close()
    ctx._keep[1].free()          # the pinned upload ring
    if own_state:
        state.place([dos.DOS_ON_CPU] * len(all_sizes), [0] * len(all_sizes))
        state.free()
    return out


def lower_bound_opt(sizes, movable, link, u_gpu, u_cpu, state_bytes, resident_params=0):
    """The best any CPU/GPU split could do with every resource at its calibrated peak:
    min over GPU sets of max(H2D time, D2H time, host update time, GPU update time).  Subgroups
    are taken in decreasing size among the movable ones (those the link can reach); residents cost GPU
    time only.  An all-GPU or all-CPU plan cannot game this bound the way it can a bound that prices
    only the executed plan's link traffic."""
    total = float(sum(sizes))
    order = sorted((n for n, mv in zip(sizes, movable) if mv), reverse=True)
    best = None
    n_g = 0.0
    for k in range(len(order) + 1):
        if k:
            n_g += order[k - 1]
        n_c = total - n_g - resident_params
        t = max((state_bytes * n_g + 2.0 * n_c) / link[0], state_bytes * n_g / link[1], n_c / u_cpu,
                (n_g + resident_params) / u_gpu)
        if best is None or t < best[0]:
            best = (t, k)
    return best


ABLATION_ROWS = (
    ("all updates on host cores (fully offloaded optimizer)", "all_cpu", 0, False),
    ("static residents only (fixed hybrid placement)", "static", 1, False),
    ("stride from Eq. 1 + Algorithm 1 placement", "stride", 0, False),
    ("balanced plan with feedback (default)", "balanced", 0, False),
    ("balanced plan, all gradients spilled to the host and fetched with the state", "balanced", 0, True),
    ("balanced plan + static residents placed last", "balanced", 1, False))


def schedule_ablation(args, dos, torch, np, state, share, budget, warmup, steps, tag="abl", calibrated=None,
                      grads=False):
    """The same host-offloaded state under different schedules, all through dos_run_update_phase: the
    schedules the paper compares against are degenerate plans of the same pipeline."""
    sizes = list(state.sizes)
    rows = []
    for name, schedule, res, spill in ABLATION_ROWS:
        r = run_interleaved(dos, torch, np, sizes, budget, steps=steps, warmup=warmup, host_threads=args.host_threads,
                            gkw={}, seed=None, check=share is not None, share=share,
                            tag=f"{tag} " + schedule + ("+res" if res else "") + ("+spill" if spill else ""),
                            state=state, residents_max=len(sizes) if res else 0, schedule=schedule, spill_grads=spill,
                            fresh_grads=grads, cm=dos.cost_model(*calibrated) if calibrated else None)
        r.pop("_cost_model", None)
        last = r.pop("steps")[-1]
        rows.append({"schedule": name, "s_per_iter": r["update_phase_s_per_iter"], "best_s": r["best_s"],
                     "params_per_s": r["params_per_s"], "n_gpu": last["n_gpu"], "n_cpu": last["n_cpu"],
                     "n_resident": last["n_resident"], "ratio_to_lower_bound": r["ratio_to_lower_bound"],
                     "host_dram_GBps": r["host_dram_GBps"],
                     "sample_mismatches_vs_oracle": r["sample_mismatches_vs_oracle"]})
    base = rows[0]["s_per_iter"]
    for r in rows:
        r["speedup_vs_all_cpu"] = base / r["s_per_iter"]
    return rows


def bench_c4(args, dos, torch, np):
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    sizes = [100_000_000] * 130
    legs = set(args.c4_legs.split(","))
    t0 = time.perf_counter()
    state = W.OffloadedState(sizes, S.BASE_SEED + 4, "cuda:0", pinned_reserve_bytes=1 << 30, pageable_rest=True)
    if state.n_pinned < len(sizes):
        log(f"[c4] this machine pins only {state.n_pinned} of the {len(sizes)} subgroups (hipHostMalloc limit); the "
            f"other {len(sizes) - state.n_pinned} live in pageable host memory and stay on the host cores")
    log(f"[c4] built {sum(sizes)*12/1e9:.0f} GB of host state in {time.perf_counter()-t0:.1f}s")
    direct = bool(UPLOAD_FLAGS & dos.DOS_CTX_UPLOAD_DIRECT)
    if direct:
        t0 = time.perf_counter()
        state.map_model_for_host_writes(args.host_threads)
        log(f"[c4] mapped the 16-bit model ({sum(sizes)*2/1e9:.0f} GB) for host writes in {time.perf_counter()-t0:.1f}s")
    share = OracleShare(state, torch, np)
    budget = 40 * 10**9
    out = run_interleaved(dos, torch, np, sizes, budget, steps=5, warmup=3, host_threads=args.host_threads,
                          gkw={}, seed=S.BASE_SEED + 4, check=True, share=share, tag="c4", state=state, rule=args.rule,
                          schedule=args.schedule, adapt=args.schedule == "balanced")
    out["workload"] = ("c4: 13B params, fp32 p/m/v (156 GB) in host memory, 130 subgroups of 100,000,000, "
                       "40 GB GPU budget, " + ("balanced plan re-derived per iteration" if args.schedule == "balanced"
                                               else f"schedule {args.schedule}")
                       + "; bf16 grads ~N(0,1e-3); 5 steps")
    if args.rule != "adamw":
        out["workload"] += f"; update rule {args.rule}: only p and v are updated and staged (8 B/param each way)"
    if out["n_subgroups_pinned"] < out["n_subgroups"]:
        out["workload"] += (f"; hipHostMalloc pins only {out['n_subgroups_pinned']} subgroups on this machine, the "
                            "others are in pageable host memory and are planned CPU-only")
    # the roofline that governs the executed plan when it keeps (most of) the work on the host cores:
    # host memory bandwidth, against a plain stream of the same access pattern measured in this run
    # (the plain stream has AdamW's access pattern; with another rule only the stand-alone update is a ceiling)
    ceil = (host_stream_ceiling(dos, torch, np, args.host_threads, direct) if args.rule == "adamw"
            else {"GBps": 0.0, "threads_at_best": None, "what": "not measured for this rule"})
    bpp_host = (26.0 if args.rule == "adamw" else 18.0) + (0.0 if direct else 2.0)
    same_kernel = out["host_rate_calibrated"] * bpp_host / 1e9
    ceiling = max(ceil["GBps"], same_kernel)
    out["host_dram"] = {"bound": "host memory bandwidth", "achieved_GBps": out["host_dram_GBps"],
                        "ceiling_GBps": ceiling, "frac": out["host_dram_GBps"] / ceiling,
                        "ceiling_plain_stream": ceil,
                        "ceiling_same_kernel_standalone_GBps": same_kernel,
                        "ceiling_note": "the higher of two same-run measurements: a plain stream of the same access "
                                        "pattern, and the host update itself with all threads over a buffer of 470 MB "
                                        "per thread (dos_calibrate)",
                        "traffic_model": "26 B per host-updated parameter with direct uploads (reads 4+4+4+2, writes "
                                         "4+4+4; the 16-bit output leaves through the BAR), 28 B through the ring; "
                                         "24 B per staged parameter (read by the prefetch, written by the flush)"}
    if args.rule != "adamw":
        # dos_calibrate and the plain stream both measure AdamW's access pattern: no ceiling for other rules
        out["host_dram"].update({"ceiling_GBps": None, "frac": None, "ceiling_same_kernel_standalone_GBps": None,
                                 "ceiling_note": "the ceilings are measured with AdamW's access pattern only"})
    log(f"[c4] host memory: phase {out['host_dram_GBps']:.0f} GB/s; ceilings: plain stream {ceil['GBps']:.0f} GB/s "
        f"({ceil['threads_at_best']} threads), the update itself stand-alone {same_kernel:.0f} GB/s")
    out.pop("_cost_model", None)
    cm_cal = dos.cost_model(*out["calibrated"])
    if "gpu_lane" in legs:
        # The staging pipeline by itself: every subgroup this machine can pin goes through the GPU lane
        # (prefetch, kernel, flush; Section 4.1's full-duplex overlap), the host lane has nothing to do.
        pinned = [i for i in range(len(sizes)) if not state.cpu_only[i]]
        lane = run_interleaved(dos, torch, np, sizes, budget, steps=3, warmup=1, host_threads=args.host_threads,
                               gkw={}, seed=None, check=True, share=share, tag="c4 gpu lane only", state=state,
                               rule=args.rule, schedule="all_gpu", adapt=False, only=pinned, fresh_grads="keep",
                               cm=dos.cost_model(*out["calibrated"]))
        best = min((r for r in lane["steps"] if r["timed"]), key=lambda r: r["wall_s"])
        out_lane = {k: lane[k] for k in (
            "update_phase_s_per_iter", "best_s", "params", "n_subgroups", "params_per_s", "ratio_to_lower_bound",
            "ratio_to_nominal_link_bound", "link_duplex_GBps", "h2d_GBps", "d2h_GBps", "h2d_frac_of_measured_link",
            "d2h_frac_of_measured_link", "n_slots", "slot_params", "sample_mismatches_vs_oracle")}
        out_lane["workload"] = (f"the {len(pinned)} subgroups of c4 that this machine can pin, all GPU-planned: "
                                "prefetch, fused kernel and flush of 16 Mi-parameter pieces through 3 slots; host "
                                "lane idle; 1 warm-up + 3 timed phases")
        out_lane["duplex_overlap_frac_of_phase"] = best["duplex_overlap_s"] / best["wall_s"]
        out_lane["gpu_kernel_busy_s"] = best["gpu_busy_s"]
        out_lane["gpu_lane_accounting"] = best.get("gpu_lane_accounting")
        out_lane["steps"] = [{k: r[k] for k in ("wall_s", "h2d_GBps", "d2h_GBps", "ratio_to_lower_bound",
                                                "duplex_overlap_s", "h2d_busy_s", "d2h_busy_s", "h2d_span_s",
                                                "d2h_span_s", "timed")} for r in lane["steps"]]
        # The same lane once more while all host threads stream through host memory (the access pattern of the
        # host lane with ring uploads, on buffers of its own): what a saturated host memory leaves of the link.
        load = HostMemoryLoad(dos, torch, args.host_threads)
        load.start()
        try:
            loaded = run_interleaved(dos, torch, np, sizes, budget, steps=2, warmup=1, host_threads=args.host_threads,
                                     gkw={}, seed=None, check=True, share=share, tag="c4 gpu lane, host memory busy",
                                     state=state, rule=args.rule, schedule="all_gpu", adapt=False, only=pinned,
                                     fresh_grads="keep", cm=dos.cost_model(*out["calibrated"]))
        finally:
            stream_GBps = load.stop()
        del load
        out_lane["with_host_memory_busy"] = {
            "what": f"the same phases while {args.host_threads} other threads stream through host memory (read p, m, v, g; "
                    "rewrite p, m, v; 16-bit output to host memory; 1 warm-up + 2 timed phases)",
            "update_phase_s_per_iter": loaded["update_phase_s_per_iter"], "h2d_GBps": loaded["h2d_GBps"],
            "d2h_GBps": loaded["d2h_GBps"], "ratio_to_lower_bound": loaded["ratio_to_lower_bound"],
            "host_stream_GBps_meanwhile": stream_GBps,
            "sample_mismatches_vs_oracle": loaded["sample_mismatches_vs_oracle"]}
        log(f"[c4 gpu lane, host memory busy] {loaded['update_phase_s_per_iter']:.3f} s per phase, H2D "
            f"{loaded['h2d_GBps']:.1f} GB/s, D2H {loaded['d2h_GBps']:.1f} GB/s, the host stream at {stream_GBps:.0f} GB/s meanwhile")
        out["gpu_lane_only"] = out_lane
    if "few_cores" in legs:
        # The regime the paper works in: host cores that update far less than the link can stage (its testbed:
        # about 2 G params/s of host update per GPU against a 55 GB/s link).  The same library with 2 and 4 host
        # threads on the subgroups this machine can pin: every update on the host cores against the interleaved
        # plan, and how close the interleaved phase comes to the link bound of its plan.
        pinned = [i for i in range(len(sizes)) if not state.cpu_only[i]]
        sub_budget = int(budget * len(pinned) / len(sizes))
        rows = []
        for T in (2, 4):
            pair = {}
            for schedule, wu in (("all_cpu", 1), ("balanced", 3)):
                r = run_interleaved(dos, torch, np, sizes, sub_budget, steps=3, warmup=wu, host_threads=T, gkw={},
                                    seed=None, check=True, share=share, tag=f"c4 {T} host threads {schedule}",
                                    state=state, rule=args.rule, schedule=schedule, only=pinned, fresh_grads="keep")
                r.pop("_cost_model", None)
                pair[schedule] = r
            b = pair["balanced"]
            rows.append({"host_threads": T, "all_cpu_s": pair["all_cpu"]["update_phase_s_per_iter"],
                         "all_cpu_host_params_per_s": pair["all_cpu"]["host_update_params_per_s"],
                         "interleaved_s": b["update_phase_s_per_iter"], "gpu_fraction": b["gpu_fraction"],
                         "speedup": pair["all_cpu"]["update_phase_s_per_iter"] / b["update_phase_s_per_iter"],
                         "ratio_to_lower_bound": b["ratio_to_lower_bound"],
                         "ratio_to_lower_bound_opt": b["ratio_to_lower_bound_opt"],
                         "h2d_GBps": b["h2d_GBps"], "d2h_GBps": b["d2h_GBps"],
                         "gpu_lane_accounting": b.get("gpu_lane_accounting"),
                         "sample_mismatches_vs_oracle": (pair["all_cpu"]["sample_mismatches_vs_oracle"] or 0)
                                                        + (b["sample_mismatches_vs_oracle"] or 0)})
        out["few_host_cores"] = {
            "workload": f"the {len(pinned)} pinnable subgroups of c4 ({sum(sizes[i] for i in pinned)/1e9:.1f} B parameters), GPU budget "
                        f"{sub_budget/1e9:.1f} GB, 2 and 4 host threads: all updates on the host cores against the balanced "
                        "interleaved plan (3 warm-up + 3 timed phases); the paper's testbed had about 2 G params/s of "
                        "host update per GPU",
            "rows": rows}
    if direct and "ring" in legs:
        # The same state with the 16-bit parameters going through the pinned ring and the copy kernel: the
        # configuration in which this host leaves something for the link to do, i.e. the staged, link-bound
        # regime the interleaving is made for.
        ring = run_interleaved(dos, torch, np, sizes, budget, steps=3, warmup=3, host_threads=args.host_threads,
                               gkw={}, seed=S.BASE_SEED + 4, check=True, share=share, tag="c4 ring uploads",
                               state=state, rule=args.rule, upload_flags=0, fresh_grads="keep")
        out["with_ring_uploads"] = {k: ring[k] for k in (
            "update_phase_s_per_iter", "best_s", "params_per_s", "ratio_to_lower_bound", "ratio_to_lower_bound_opt",
            "h2d_GBps", "d2h_GBps", "h2d_frac_of_measured_link", "d2h_frac_of_measured_link", "gpu_fraction",
            "host_dram_GBps", "uploads", "sample_mismatches_vs_oracle") if k in ring}
        out["with_ring_uploads"]["gpu_lane_accounting"] = ring.get("gpu_lane_accounting")
    if "ablation" in legs:
        rows = schedule_ablation(args, dos, torch, np, state, share, budget, warmup=2, steps=3,
                                 calibrated=out["calibrated"], grads="keep")
        out["schedule_ablation"] = {
            "workload": "the c4 state under six schedules, all through dos_run_update_phase; gradients generated "
                        "once; 2 warm-up + 3 timed phases each; residents are moved to the device before timing",
            "rows": rows}
    state.place([dos.DOS_ON_CPU] * len(sizes), [0] * len(sizes))
    state.free()
    return out


def bench_ablation(args, dos, torch, np):
    """The schedule table on its own state, plus the host-threads sweep (the paper's CPU-cores-per-GPU study)."""
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    sizes = [100_000_000] * 130
    state = W.OffloadedState(sizes, S.BASE_SEED + 4, "cuda:0", pinned_reserve_bytes=1 << 30,
                             pageable_rest=args.full_size)
    if UPLOAD_FLAGS & dos.DOS_CTX_UPLOAD_DIRECT:
        state.map_model_for_host_writes(args.host_threads)
    sizes = list(state.sizes)
    scale = sum(sizes) / 13e9
    budget = int(40 * 10**9 * scale)
    share = OracleShare(state, torch, np)
    rows = schedule_ablation(args, dos, torch, np, state, share, budget, warmup=3, steps=4)
    # host cores per GPU (the paper's CPU-cores-per-GPU study, Section 5.4): fewer host threads make the
    # all-CPU schedule slower and the interleaved one comparatively better
    thread_rows = []
    for T in sorted({2, 4, 8, 12, args.host_threads}):
        if T > args.host_threads:
            continue
        pair = {}
        for schedule in ("all_cpu", "balanced"):
            r = run_interleaved(dos, torch, np, sizes, budget, steps=3, warmup=3, host_threads=T, gkw={},
                                seed=S.BASE_SEED + 4, check=False, tag=f"threads {T} {schedule}", state=state,
                                schedule=schedule, fresh_grads=False)
            r.pop("_cost_model", None)
            pair[schedule] = r
        thread_rows.append({"host_threads": T, "all_cpu_s": pair["all_cpu"]["update_phase_s_per_iter"],
                            "balanced_s": pair["balanced"]["update_phase_s_per_iter"],
                            "gpu_fraction": pair["balanced"]["gpu_fraction"],
                            "speedup": pair["all_cpu"]["update_phase_s_per_iter"]
                            / pair["balanced"]["update_phase_s_per_iter"]})
    state.place([dos.DOS_ON_CPU] * len(sizes), [0] * len(sizes))
    state.free()
    return {"workload": f"{len(sizes)} x 100M-parameter subgroups in host memory ({state.n_pinned} pinned), GPU "
                        f"budget {budget/1e9:.1f} GB (40 GB scaled by {scale:.3f}), grads ~N(0,1e-3), 4 timed steps",
            "rows": rows, "host_threads_sweep": thread_rows}


def bench_c5(args, dos, torch, np, sg_sizes_m, budgets_gb, full_size, steps=3, warmup=2, take=1 << 16):
    """Interleaving sweep: subgroup size x GPU budget, heavy-tailed gradients with 5 % zeros, 3 steps per cell.
    Each cell is run twice: state entirely host-resident (budget = staging only), and with the budget's
    remainder used for static residents placed last.  One host state per subgroup size serves all its cells."""
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    total_nominal = 13_000_000_000
    cells = []
    scale = None
    cm = peaks = None
    for sg_params in [int(x) * 1_000_000 for x in sg_sizes_m]:
        n_sg = -(-total_nominal // sg_params)
        sizes = [sg_params] * (n_sg - 1) + [total_nominal - sg_params * (n_sg - 1)]
        if scale is not None and scale < 1:        # same parameter count for every subgroup size
            keep = int(round(scale * total_nominal))
            n_keep = max(1, keep // sg_params)
            sizes = [sg_params] * n_keep
        t0 = time.perf_counter()
        state = W.OffloadedState(sizes, S.BASE_SEED + 5, "cuda:0", pinned_reserve_bytes=1 << 30,
                                 pageable_rest=full_size)
        if UPLOAD_FLAGS & dos.DOS_CTX_UPLOAD_DIRECT:
            state.map_model_for_host_writes(args.host_threads)
        sizes = list(state.sizes)
        log(f"[c5] S={sg_params//10**6}M: {len(sizes)} subgroups ({state.n_pinned} pinned) built in "
            f"{time.perf_counter()-t0:.1f}s")
        if scale is None:
            scale = sum(sizes) / total_nominal
            if scale < 1:
                log(f"[c5] this machine pins {sum(sizes)/1e9:.1f}B of the 13B parameters; budgets are scaled "
                    f"by {scale:.3f}")
        share = OracleShare(state, torch, np, take=take)
        state.fill_grads(1, heavy_tail=True, zero_pct=5.0)          # one set of gradients serves every cell
        for budget_gb in budgets_gb:
            budget = int(budget_gb * 10**9 * scale)
            for residents in (0, len(sizes)):
                tag = f"c5 S={sg_params//10**6}M B={budget_gb}GB{' +res' if residents else ''}"
                try:
                    # the first cell calibrates and lets the planner's feedback settle (3 warm-up phases); the
                    # cost model it ends with is carried from cell to cell, as a training run carries it from
                    # iteration to iteration
                    r = run_interleaved(dos, torch, np, sizes, budget, steps=steps, warmup=warmup if cm else 3,
                                        host_threads=args.host_threads, gkw={}, seed=S.BASE_SEED + 5,
                                        check=True, share=share, tag=tag, state=state, residents_max=residents,
                                        cm=cm, peaks=peaks, fresh_grads="keep", keep_steps=False)
                    cm = r.pop("_cost_model")
                    peaks = r["calibrated"]
                except dos.DosError as e:
                    r = {"error": str(e)}
                for k in ("calibrated", "lower_bound_note", "gpu_lane_accounting"):
                    r.pop(k, None)
                r.update({"subgroup_params": sg_params, "budget_GB_nominal": budget_gb,
                          "budget_bytes_scaled": budget, "static_residents": bool(residents)})
                cells.append(r)
        state.place([dos.DOS_ON_CPU] * len(sizes), [0] * len(sizes))   # residents back to the host
        state.free()
        del state, share
        torch.cuda.empty_cache()
    return {"workload": f"c5: subgroup size {{{','.join(str(x) for x in sg_sizes_m)}}}M x GPU budget "
                        f"{{{','.join(str(b) for b in budgets_gb)}}} GB on 13B parameters of host-resident state "
                        f"(what cannot be pinned is pageable and CPU-only), grads Student-t(3) x 1e-3 with 5% zeros, "
                        f"generated once, {warmup} warm-up + {steps} timed steps per cell, each cell with and without "
                        "static residents placed last",
            "scale": scale, "cells": cells}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--extra", default="c1,c3,c4,c5,rules",
                    help="comma list of extra workloads (c1, c3, c4, c5 = the reduced subgroup-size x budget grid, "
                         "rules = Adagrad and RMSProp on the c2 shape) or 'none'")
    ap.add_argument("--host-threads", type=int, default=0)
    ap.add_argument("--upload", default="auto", choices=["auto", "direct", "pull", "dma"],
                    help="how the host lane of the interleaved workloads sends the 16-bit parameters to the device: "
                         "direct = host stores through the PCIe BAR (auto picks it when the device memory is mapped "
                         "into the host's address space), pull = copy kernel reading a pinned ring, dma = hipMemcpyAsync")
    ap.add_argument("--rule", default="adamw", choices=["adamw", "adagrad", "rmsprop"],
                    help="update rule of the interleaved workload c4 (the primary workload is always AdamW)")
    ap.add_argument("--schedule", default="balanced",
                    help="schedule of c4's main leg: balanced (planner with feedback), stride (Eq. 1), all_cpu, all_gpu, "
                         "or fixed:<n> (n subgroups staged in every phase: a plan that does not move, for profiling "
                         "the staged regime)")
    ap.add_argument("--c4-legs", default="gpu_lane,few_cores,ring,ablation",
                    help="what c4 runs after its main leg: gpu_lane (the pinned subgroups through the GPU lane alone), "
                         "few_cores (the same subgroups with 2 and 4 host threads, all-CPU against interleaved), ring (the "
                         "main leg again with ring uploads), ablation (six schedules); 'none' for none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ablation", action="store_true",
                    help="the schedule table on a state of its own, longer, plus the host-threads sweep")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure the AdamW launch with only its loads / only its stores (HBM ceilings)")
    ap.add_argument("--sweep", action="store_true", help="the full c5 grid (4 sizes x 4 budgets) instead of the reduced one")
    ap.add_argument("--sweep-sizes", default="50,100,200,400", help="subgroup sizes of the full sweep, in millions")
    ap.add_argument("--full-size", action="store_true",
                    help="--ablation on the full 13B parameters: what cannot be pinned lives in pageable host "
                         "memory and is planned CPU-only (default: only the part that can be pinned)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB copy kernel three times (reference for traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the update phase needs no inter-GPU exchange; "
              "each GPU would run its own context). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2410_21316_amd as dos
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dos.load()
    global UPLOAD_FLAGS
    upload = args.upload
    if upload == "auto":
        upload = "direct" if dos.dos_device_large_bar(0) else "pull"
    UPLOAD_FLAGS = {"direct": dos.DOS_CTX_UPLOAD_DIRECT, "dma": dos.DOS_CTX_UPLOAD_DMA, "pull": 0}[upload]
    log(f"[bench] 16-bit uploads of the host lane: {upload}")
    if args.host_threads <= 0:
        args.host_threads = len(os.sched_getaffinity(0))
    t_start = time.perf_counter()
    res = bench_c2(args, dos, torch, np)
    extra = {}
    wanted = [] if args.extra == "none" else [w.strip() for w in args.extra.split(",") if w.strip()]
    if "c1" in wanted:
        extra["c1_single_subgroup_1m"] = bench_c1(args, dos, torch, np)
    if "c3" in wanted:
        extra["c3_resident_7b"] = bench_c3(args, dos, torch, np)
    if "rules" in wanted:
        extra["other_update_rules"] = bench_other_rules(args, dos, torch, np)
    if args.ceilings:
        extra["hbm_stream_ceilings"] = bench_ceilings(args, dos, torch, np)
    if "c4" in wanted:
        log(f"[bench] {time.perf_counter()-t_start:.0f}s so far; c4")
        extra["c4_interleaved_13b"] = bench_c4(args, dos, torch, np)
        if "schedule_ablation" in extra["c4_interleaved_13b"]:
            extra["schedule_ablation"] = extra["c4_interleaved_13b"].pop("schedule_ablation")
        if "gpu_lane_only" in extra["c4_interleaved_13b"]:
            extra["c4_gpu_lane_only"] = extra["c4_interleaved_13b"].pop("gpu_lane_only")
        if "few_host_cores" in extra["c4_interleaved_13b"]:
            extra["c4_few_host_cores"] = extra["c4_interleaved_13b"].pop("few_host_cores")
    if args.ablation:
        extra["schedule_ablation_long"] = bench_ablation(args, dos, torch, np)
    if args.sweep:
        extra["c5_interleaving_sweep"] = bench_c5(args, dos, torch, np, args.sweep_sizes.split(","), (8, 16, 32, 64),
                                                  full_size=True)
    elif "c5" in wanted:
        log(f"[bench] {time.perf_counter()-t_start:.0f}s so far; c5 (reduced grid)")
        extra["c5_interleaving_sweep"] = bench_c5(args, dos, torch, np, ("50", "400"), (8, 64), full_size=True,
                                                  steps=3, warmup=1, take=1 << 14)
        extra["c5_interleaving_sweep"]["grid"] = ("reduced: the corners of the 4 x 4 grid (subgroup size 50M and 400M, "
                                                  "budget 8 and 64 GB); --sweep runs all 16 cells")
    if extra:
        res["extra"] = extra
    res["bench_wall_s"] = time.perf_counter() - t_start
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
