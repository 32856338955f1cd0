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
device memory where the machine allows, and once more through the pinned ring),
and Adagrad / RMSProp on the primary workload's shape.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--extra c1,c3,c4,rules|none] [--upload auto|direct|pull|dma]
                    [--rule adamw|adagrad|rmsprop] [--host-threads T] [--ablation] [--sweep] [--full-size] [--ceilings]
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
                     "kernel": "dos::adam_kernel (fused AdamW)", "bytes_per_launch": BYTES_PER_PARAM * sizes[0],
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
    budget, everything else on the host cores: static hybrid placement without interleaving)."""
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
    raise ValueError(schedule)


def run_interleaved(dos, torch, np, sizes, budget_bytes, steps, warmup, host_threads, gkw, seed, check=True,
                    cm=None, residents_max=0, tag="c4", state=None, adapt=True, schedule="balanced",
                    fresh_grads=True, spill_grads=False, pageable_rest=False, rule="adamw", upload_flags=None):
    """Plan + run the interleaved phase on a host-offloaded state; returns a dict.
    fresh_grads=False generates the gradients once and reuses them for every step;
    spill_grads=True keeps every gradient in pinned host memory (GPU-planned subgroups fetch theirs
    with p, m, v through 14-byte slots); pageable_rest=True keeps the subgroups the machine cannot pin in
    ordinary host memory (CPU-only) instead of dropping them."""
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
    if upload_flags & dos.DOS_CTX_UPLOAD_DIRECT and own_state:
        t0 = time.perf_counter()
        state.map_model_for_host_writes(host_threads)
        log(f"[{tag}] mapped the 16-bit model ({sum(sizes)*2/1e9:.0f} GB) for host writes in {time.perf_counter()-t0:.1f}s")
    cpu_only = state.cpu_only if any(state.cpu_only) else None
    # slots first (they decide what the context can do), then calibration, then the plan
    probe_cm = cm or dos.cost_model(50e9, 50e9, 180e9, 5e9)
    bpp = 14 if spill_grads else 12
    plan = dos.dos_plan_subgroups(probe_cm, sizes, budget_bytes, dos.DOS_PLAN_BALANCED, residents_max, bpp, cpu_only)
    ctx = W.make_context(plan.c.n_slots, plan.c.slot_params, host_threads, flags=dos.DOS_CTX_PROFILE | upload_flags,
                         stage_grads=spill_grads)
    if cm is None:
        cm = ctx.dos_calibrate()
        cm.fp32_arrays = 3 if rule == "adamw" else 2    # Adagrad, RMSProp stage p and v only
        log(f"[{tag}] calibrated: H2D {cm.h2d_Bps/1e9:.1f} GB/s, D2H {cm.d2h_Bps/1e9:.1f} GB/s (duplex), "
            f"U_g {cm.gpu_params_per_s/1e9:.1f} G/s, U_c {cm.cpu_params_per_s/1e9:.2f} G/s (stand-alone)")
    link = (cm.h2d_Bps, cm.d2h_Bps)
    calibrated = (cm.h2d_Bps, cm.d2h_Bps, cm.gpu_params_per_s, cm.cpu_params_per_s, cm.downscale_params_per_s,
                  cm.launch_overhead_s)
    results = []
    samp = None
    if check:
        from oracle import adamw_oracle as ref
        idxs = [torch.from_numpy(W.sample_index(n)) for n in sizes]

        def take(t, idx):
            return (t[idx.to(t.device)].cpu() if t.is_cuda else t[idx]).numpy().copy()

        # the oracle's share starts from the state as it is now (wherever it lives)
        samp = [[take(t, idxs[i]) for t in state.state(i)] + [np.zeros(idxs[i].numel(), np.uint16)]
                for i in range(len(sizes))]
    for step in range(1, warmup + steps + 1):
        # with feedback on, the first warm-up phase runs on the host cores alone: together with the staged
        # phases that follow it tells the cost model what staging takes away from the host lane
        probe_all_cpu = adapt and schedule == "balanced" and step == 1 and warmup >= 2 and not residents_max
        plan = make_plan(dos, "all_cpu" if probe_all_cpu else schedule, cm, sizes, budget_bytes, residents_max, bpp,
                         cpu_only)
        state.place(plan.targets, plan.residents, spill_all_grads=spill_grads)
        if fresh_grads or step == 1:
            state.fill_grads(step, **gkw)
        state.sync_host_grads()
        st = ctx.dos_run_update_phase(state.sgs, plan, dos.hparams(step=step, optimizer=rule, **hp_kw))
        lb_plan = max(st.h2d_bytes / link[0], st.d2h_bytes / link[1])
        r = {"step": step, "wall_s": st.wall_s, "n_gpu": st.n_gpu, "n_cpu": st.n_cpu, "n_resident": st.n_resident,
             "gpu_fraction": (st.params_gpu + st.params_resident) / max(1, sum(sizes)),
             "h2d_GBps": st.h2d_bytes / st.wall_s / 1e9, "d2h_GBps": st.d2h_bytes / st.wall_s / 1e9,
             "h2d_busy_s": st.h2d_busy_s, "d2h_busy_s": st.d2h_busy_s, "gpu_busy_s": st.gpu_busy_s,
             "duplex_overlap_s": st.duplex_overlap_s, "cpu_lane_s": st.cpu_lane_s, "gpu_lane_s": st.gpu_lane_s,
             "host_update_params_per_s": st.params_cpu / st.cpu_lane_s if st.cpu_lane_s > 0 else None,
             "lower_bound_s": lb_plan, "ratio_to_lower_bound": st.wall_s / lb_plan if lb_plan > 0 else None,
             "predicted_s": plan.c.predicted_s, "timed": step > warmup}
        results.append(r)
        log(f"[{tag}] step {step}: {st.wall_s:.3f}s gpu {st.n_gpu}+{st.n_resident}r cpu {st.n_cpu} "
            f"lanes cpu {st.cpu_lane_s:.3f} gpu {st.gpu_lane_s:.3f} LB {lb_plan:.3f} ratio {r['ratio_to_lower_bound']}")
        if adapt:
            # feed the measured lane rates back into the cost model (the plan is
            # re-derived every iteration, as a training loop would)
            dos.dos_cost_model_observe(cm, st)
        if check:
            for i in range(len(sizes)):
                gs = state.g[i][idxs[i].to("cuda:0")].view(torch.int16).cpu().numpy().view(np.uint16)
                ref.optimizer_step(rule, samp[i][0], samp[i][1], samp[i][2], gs, samp[i][3], step=step, threads=0,
                                   **hp_kw)
    mism = None
    if check:
        mism = 0
        for i in range(len(sizes)):
            cur = state.state(i)
            for t, host_a in zip(cur, samp[i][:3]):
                got = t[idxs[i].to(t.device)].cpu().numpy() if t.is_cuda else t[idxs[i]].numpy()
                mism += int(np.count_nonzero(got.view(np.uint32) != host_a.view(np.uint32)))
            got = state.lp[i][idxs[i].to("cuda:0")].view(torch.int16).cpu().numpy().view(np.uint16)
            mism += int(np.count_nonzero(got != samp[i][3]))
    timed = [r for r in results if r["timed"]]
    best = min(timed, key=lambda r: r["wall_s"])
    mean_wall = sum(r["wall_s"] for r in timed) / len(timed)
    sb = 12.0 if rule == "adamw" else 8.0
    res_params = sum(n for n, r in zip(sizes, plan.residents or [0] * len(sizes)) if r)
    movable = [not c and not r for c, r in zip(state.cpu_only, plan.residents or [0] * len(sizes))]
    lb_opt, k_opt = lower_bound_opt(sizes, movable, link, calibrated[2], calibrated[3], sb, res_params)
    lb_free, k_free = lower_bound_opt(sizes, [not r for r in (plan.residents or [0] * len(sizes))], link,
                                      calibrated[2], calibrated[3], sb, res_params)
    out = {"update_phase_s_per_iter": mean_wall, "best_s": best["wall_s"],
           "lower_bound_opt_s": lb_opt, "lower_bound_opt_gpu_subgroups": k_opt,
           "ratio_to_lower_bound_opt": mean_wall / lb_opt,
           "lower_bound_opt_all_pinnable_s": lb_free, "ratio_to_lower_bound_opt_all_pinnable": mean_wall / lb_free,
           "lower_bound_note": "ratio_to_lower_bound prices the executed plan's link bytes at the measured duplex "
                               "link rates; lower_bound_opt is the best any split could reach with link, host "
                               "update and GPU update all at their calibrated stand-alone peaks (over the "
                               "subgroups this machine can pin; _all_pinnable: if it could pin all of them)",
           "params": sum(sizes), "n_subgroups": len(sizes), "n_subgroups_pinned": state.n_pinned,
           "params_per_s": sum(sizes) / mean_wall,
           "ratio_to_lower_bound": sum(r["ratio_to_lower_bound"] for r in timed) / len(timed),
           "link_duplex_GBps": {"h2d": link[0] / 1e9, "d2h": link[1] / 1e9, "nominal": LINK_NOMINAL_GBPS},
           "h2d_GBps": best["h2d_GBps"], "d2h_GBps": best["d2h_GBps"],
           "h2d_frac_of_measured_link": best["h2d_GBps"] * 1e9 / link[0],
           "d2h_frac_of_measured_link": best["d2h_GBps"] * 1e9 / link[1],
           "host_update_params_per_s": best["host_update_params_per_s"],
           "gpu_fraction": best["gpu_fraction"], "n_slots": plan.c.n_slots, "slot_params": plan.c.slot_params,
           "host_threads": host_threads, "uploads": {0: "pull", 2: "dma", 8: "direct"}[upload_flags],
           "sample_mismatches_vs_oracle": mism, "steps": results,
           "calibrated": calibrated}
    ctx.close()
    ctx._keep[1].free()          # the pinned upload ring
    if own_state:
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


def bench_c4(args, dos, torch, np):
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    sizes = [100_000_000] * 130
    t0 = time.perf_counter()
    state = W.OffloadedState(sizes, S.BASE_SEED + 4, "cuda:0", pinned_reserve_bytes=1 << 30, pageable_rest=True)
    if state.n_pinned < len(sizes):
        log(f"[c4] this machine pins only {state.n_pinned} of the {len(sizes)} subgroups (hipHostMalloc limit); the "
            f"other {len(sizes) - state.n_pinned} live in pageable host memory and stay on the host cores")
    log(f"[c4] built {sum(sizes)*12/1e9:.0f} GB of host state in {time.perf_counter()-t0:.1f}s")
    if UPLOAD_FLAGS & dos.DOS_CTX_UPLOAD_DIRECT:
        t0 = time.perf_counter()
        state.map_model_for_host_writes(args.host_threads)
        log(f"[c4] mapped the 16-bit model ({sum(sizes)*2/1e9:.0f} GB) for host writes in {time.perf_counter()-t0:.1f}s")
    out = run_interleaved(dos, torch, np, sizes, 40 * 10**9, steps=5, warmup=3, host_threads=args.host_threads,
                          gkw={}, seed=S.BASE_SEED + 4, check=True, tag="c4", state=state, rule=args.rule)
    out["workload"] = ("c4: 13B params, fp32 p/m/v (156 GB) in host memory, 130 subgroups of 100,000,000, "
                       "40 GB GPU budget, balanced plan re-derived per iteration; bf16 grads ~N(0,1e-3); 5 steps")
    if args.rule != "adamw":
        out["workload"] += f"; update rule {args.rule}: only p and v are updated and staged (8 B/param each way)"
    if out["n_subgroups_pinned"] < out["n_subgroups"]:
        out["workload"] += (f"; hipHostMalloc pins only {out['n_subgroups_pinned']} subgroups on this machine, the "
                            "others are in pageable host memory and are planned CPU-only")
    if UPLOAD_FLAGS & dos.DOS_CTX_UPLOAD_DIRECT:
        # The same state with the 16-bit parameters going through the pinned ring and the copy kernel: the
        # configuration in which this host leaves something for the link to do, i.e. the staged, link-bound
        # regime the interleaving is made for.
        ring = run_interleaved(dos, torch, np, sizes, 40 * 10**9, steps=3, warmup=3, host_threads=args.host_threads,
                               gkw={}, seed=S.BASE_SEED + 4, check=True, tag="c4 ring uploads", state=state,
                               rule=args.rule, upload_flags=0)
        out["with_ring_uploads"] = {k: ring[k] for k in (
            "update_phase_s_per_iter", "best_s", "params_per_s", "ratio_to_lower_bound", "ratio_to_lower_bound_opt",
            "h2d_GBps", "d2h_GBps", "h2d_frac_of_measured_link", "d2h_frac_of_measured_link", "gpu_fraction",
            "uploads", "sample_mismatches_vs_oracle")}
    state.place([dos.DOS_ON_CPU] * len(sizes), [0] * len(sizes))
    state.free()
    return out


def bench_ablation(args, dos, torch, np):
    """The same host-offloaded state under different schedules, all through dos_run_update_phase."""
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
    rows = []
    for name, schedule, res, spill in (
            ("all updates on host cores (fully offloaded optimizer)", "all_cpu", 0, False),
            ("static residents only (fixed hybrid placement)", "static", len(sizes), False),
            ("stride from Eq. 1 + Algorithm 1 placement", "stride", 0, False),
            ("balanced plan with feedback (default)", "balanced", 0, False),
            ("balanced plan, all gradients spilled to the host and fetched with the state", "balanced", 0, True),
            ("balanced plan + static residents placed last", "balanced", len(sizes), False)):
        r = run_interleaved(dos, torch, np, sizes, budget, steps=4, warmup=3, host_threads=args.host_threads, gkw={},
                            seed=S.BASE_SEED + 4, check=True,
                            tag="abl " + schedule + ("+res" if res else "") + ("+spill" if spill else ""),
                            state=state, residents_max=res, schedule=schedule, spill_grads=spill)
        last = r.pop("steps")[-1]
        rows.append({"schedule": name, "s_per_iter": r["update_phase_s_per_iter"], "best_s": r["best_s"],
                     "params_per_s": r["params_per_s"], "n_gpu": last["n_gpu"], "n_cpu": last["n_cpu"],
                     "n_resident": last["n_resident"], "sample_mismatches_vs_oracle": r["sample_mismatches_vs_oracle"]})
    base = rows[0]["s_per_iter"]
    for r in rows:
        r["speedup_vs_all_cpu"] = base / r["s_per_iter"]
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


def bench_c5(args, dos, torch, np):
    """Interleaving sweep: subgroup size x GPU budget, heavy-tailed gradients with 5 % zeros, 3 steps per cell.
    Each cell is run twice: state entirely host-resident (budget = staging only), and with the budget's
    remainder used for static residents placed last."""
    from paper_2410_21316_amd import workloads as W
    import dos_synth as S
    total_nominal = 13_000_000_000
    cells = []
    scale = None
    for sg_params in [int(x) * 1_000_000 for x in args.sweep_sizes.split(",")]:
        n_sg = -(-total_nominal // sg_params)
        sizes = [sg_params] * (n_sg - 1) + [total_nominal - sg_params * (n_sg - 1)]
        if scale is not None and scale < 1:        # same parameter count for every subgroup size
            keep = int(round(scale * total_nominal))
            n_keep = max(1, keep // sg_params)
            sizes = [sg_params] * n_keep
        state = W.OffloadedState(sizes, S.BASE_SEED + 5, "cuda:0", pinned_reserve_bytes=1 << 30,
                                 pageable_rest=args.full_size)
        if UPLOAD_FLAGS & dos.DOS_CTX_UPLOAD_DIRECT:
            state.map_model_for_host_writes(args.host_threads)
        sizes = list(state.sizes)
        if scale is None:
            scale = sum(sizes) / total_nominal
            if scale < 1:
                log(f"[c5] this machine pins {sum(sizes)/1e9:.1f}B of the 13B parameters; budgets are scaled "
                    f"by {scale:.3f}")
            else:
                log(f"[c5] full size; {state.n_pinned} of {len(sizes)} subgroups pinned, the rest pageable (CPU-only)")
        cm = None
        for budget_gb in (8, 16, 32, 64):
            budget = int(budget_gb * 10**9 * scale)
            for residents in (0, len(sizes)):
                tag = f"c5 S={sg_params//10**6}M B={budget_gb}GB{' +res' if residents else ''}"
                try:
                    r = run_interleaved(dos, torch, np, sizes, budget, steps=3, warmup=2,
                                        host_threads=args.host_threads,
                                        gkw=dict(heavy_tail=True, zero_pct=5.0), seed=S.BASE_SEED + 5,
                                        check=True, tag=tag, state=state, residents_max=residents,
                                        cm=(dos.cost_model(*cm) if cm else None), fresh_grads=False)
                    if cm is None:
                        cm = r.get("calibrated")
                except dos.DosError as e:
                    r = {"error": str(e)}
                r.pop("steps", None)
                r.pop("calibrated", None)
                r.update({"subgroup_params": sg_params, "budget_GB_nominal": budget_gb,
                          "budget_bytes_scaled": budget, "static_residents": bool(residents)})
                cells.append(r)
        state.place([dos.DOS_ON_CPU] * len(sizes), [0] * len(sizes))   # residents back to the host
        state.free()
        del state
        torch.cuda.empty_cache()
    return {"workload": "c5: subgroup size {50,100,200,400}M x GPU budget {8,16,32,64} GB on host-resident state, "
                        "grads Student-t(3) x 1e-3 with 5% zeros, 3 timed steps per cell; parameter count and "
                        "budgets scaled by the fraction of 13B this machine can pin",
            "scale": scale, "cells": cells}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--extra", default="c1,c3,c4,rules",
                    help="comma list of extra workloads (c1, c3, c4, rules = Adagrad and RMSProp on the c2 shape) "
                         "or 'none'")
    ap.add_argument("--host-threads", type=int, default=0)
    ap.add_argument("--upload", default="auto", choices=["auto", "direct", "pull", "dma"],
                    help="how the host lane of the interleaved workloads sends the 16-bit parameters to the device: "
                         "direct = host stores through the PCIe BAR (auto picks it when the device memory is mapped "
                         "into the host's address space), pull = copy kernel reading a pinned ring, dma = hipMemcpyAsync")
    ap.add_argument("--rule", default="adamw", choices=["adamw", "adagrad", "rmsprop"],
                    help="update rule of the interleaved workload c4 (the primary workload is always AdamW)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ablation", action="store_true", help="also compare schedules on the host-offloaded state")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure the AdamW launch with only its loads / only its stores (HBM ceilings)")
    ap.add_argument("--sweep", action="store_true", help="also run the c5 subgroup-size x budget sweep")
    ap.add_argument("--sweep-sizes", default="50,100,200,400", help="subgroup sizes of the sweep, in millions")
    ap.add_argument("--full-size", action="store_true",
                    help="ablation / sweep on the full 13B parameters: what cannot be pinned lives in pageable host "
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
    res = bench_c2(args, dos, torch, np)
    extra = {}
    wanted = [] if args.extra == "none" else [w.strip() for w in args.extra.split(",") if w.strip()]
    if "c1" in wanted:
        extra["c1_single_subgroup_1m"] = bench_c1(args, dos, torch, np)
    if "c3" in wanted:
        extra["c3_resident_7b"] = bench_c3(args, dos, torch, np)
    if "c4" in wanted:
        extra["c4_interleaved_13b"] = bench_c4(args, dos, torch, np)
    if "rules" in wanted:
        extra["other_update_rules"] = bench_other_rules(args, dos, torch, np)
    if args.ceilings:
        extra["hbm_stream_ceilings"] = bench_ceilings(args, dos, torch, np)
    if args.ablation:
        extra["schedule_ablation"] = bench_ablation(args, dos, torch, np)
    if args.sweep:
        extra["c5_interleaving_sweep"] = bench_c5(args, dos, torch, np)
    if extra:
        res["extra"] = extra
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
