"""Synthetic optimizer-state workloads shaped like the paper's models (Table 2:
7B-20B parameters; 100M-parameter subgroups as in its evaluation set-up), for the
benchmark and the full-size tests.  Memory plumbing only: torch allocates device
memory, libdos allocates pinned host memory, the seeded generator fills both.
No optimizer arithmetic lives here."""
from __future__ import annotations

import ctypes

import numpy as np
import torch

import dos_synth as S

from . import binding as dos


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


class ResidentState:
    """All five arrays of every subgroup in device memory (configurations with
    device-resident optimizer state)."""

    def __init__(self, sizes, seed=S.BASE_SEED, device="cuda:0", n_grad_sets=1):
        self.sizes, self.seed, self.device = list(sizes), seed, device
        self.p, self.m, self.v, self.lp, self.g = [], [], [], [], []
        for i, n in enumerate(self.sizes):
            p = torch.empty(n, dtype=torch.float32, device=device)
            S.fill_chunked(lambda start, count: S.params(seed, i, start, count, device), p)
            self.p.append(p)
            self.m.append(torch.zeros(n, dtype=torch.float32, device=device))
            self.v.append(torch.zeros(n, dtype=torch.float32, device=device))
            self.lp.append(torch.zeros(n, dtype=torch.bfloat16, device=device))
            self.g.append([torch.zeros(n, dtype=torch.bfloat16, device=device) for _ in range(n_grad_sets)])
        self.n_grad_sets = n_grad_sets
        self.descs = [[dos.subgroup_from_tensors(self.p[i], self.m[i], self.v[i], self.g[i][k], self.lp[i])
                       for i in range(len(self.sizes))] for k in range(n_grad_sets)]

    def fill_grads(self, k: int, step: int, scales=None, **gkw):
        """Generate gradient set k for `step` (set k is used by steps = k mod n_grad_sets)."""
        for i in range(len(self.sizes)):
            sc = 1.0 if scales is None else scales[i]
            S.fill_chunked(lambda start, count: S.grads_bf16(self.seed, step, i, start, count, self.device,
                                                             scale=sc, **gkw), self.g[i][k])

    @property
    def total(self):
        return sum(self.sizes)


class PinnedBlock:
    def __init__(self, nbytes: int):
        self.nbytes = max(int(nbytes), 256)
        self.ptr = dos.dos_pinned_alloc(self.nbytes)
        self._buf = (ctypes.c_uint8 * self.nbytes).from_address(self.ptr)

    def tensor(self, dtype, offset_bytes: int, count: int) -> torch.Tensor:
        """A torch CPU tensor viewing part of the block (no copy)."""
        t = torch.frombuffer(self._buf, dtype=torch.uint8, count=self.nbytes)
        nb = count * torch.empty((), dtype=dtype).element_size()
        return t[offset_bytes:offset_bytes + nb].view(dtype)

    def free(self):
        if self.ptr:
            self._buf = None
            dos.dos_pinned_free(self.ptr)
            self.ptr = 0


class OffloadedState:
    """FP32 p, m, v of every subgroup in pinned host memory (one pinned block per
    subgroup: p | m | v | g), the bf16 model and a full set of bf16 gradients on
    the device.  `place(plan)` points each descriptor's gradient at the device copy
    (GPU-planned) or at the pinned copy (CPU-planned) and moves static residents'
    state to the device, following the plan as Section 4.1 describes."""

    def __init__(self, sizes, seed=S.BASE_SEED, device="cuda:0", fill=True, pinned_reserve_bytes=0,
                 pageable_rest=False, pin_at_most=None, hugepages=True):
        """If the machine cannot pin all of it (leaving `pinned_reserve_bytes` for
        the caller's own pinned buffers), the subgroups that do not fit either
        live in ordinary pageable host memory (`pageable_rest=True`: they can then
        only be updated by the host cores, `self.cpu_only` marks them) or are
        dropped (`self.truncated`, `self.sizes` tells what was built).
        `pin_at_most` caps the number of pinned subgroups (for tests)."""
        self.sizes, self.seed, self.device = list(sizes), seed, device
        self.blocks, self.hp, self.hm, self.hv, self.hg = [], [], [], [], []
        self.truncated = False
        try:
            reserve = PinnedBlock(pinned_reserve_bytes) if pinned_reserve_bytes else None
            for n in self.sizes[:pin_at_most]:
                fb, gb = _round_up(4 * n, 4096), _round_up(2 * n, 4096)
                self.blocks.append(PinnedBlock(3 * fb + gb))
        except dos.DosError as e:
            if e.status != dos.DOS_EHIP or not self.blocks:
                raise
            if not pageable_rest:
                self.truncated = True
                self.sizes = self.sizes[:len(self.blocks)]
        finally:
            if pinned_reserve_bytes and reserve is not None:
                reserve.free()
        if pin_at_most is not None and not pageable_rest:
            self.sizes = self.sizes[:len(self.blocks)]
        n_sg = len(self.sizes)
        self.n_pinned = len(self.blocks)
        self.cpu_only = [i >= self.n_pinned for i in range(n_sg)]
        self.lp = [torch.zeros(n, dtype=torch.bfloat16, device=device) for n in self.sizes]
        self.g = [torch.zeros(n, dtype=torch.bfloat16, device=device) for n in self.sizes]
        self.res = [None] * n_sg                      # device p, m, v of static residents
        zeros = torch.zeros(max(self.sizes), dtype=torch.float32, device=device)
        tmp = torch.empty(max(self.sizes), dtype=torch.float32, device=device)
        for i, n in enumerate(self.sizes):
            fb = _round_up(4 * n, 4096)
            if i < self.n_pinned:
                blk = self.blocks[i]
                self.hp.append(blk.tensor(torch.float32, 0, n))
                self.hm.append(blk.tensor(torch.float32, fb, n))
                self.hv.append(blk.tensor(torch.float32, 2 * fb, n))
                self.hg.append(blk.tensor(torch.bfloat16, 3 * fb, n))
            else:                                     # ordinary host memory, 64-byte aligned by torch
                self.hp.append(torch.empty(n, dtype=torch.float32))
                self.hm.append(torch.empty(n, dtype=torch.float32))
                self.hv.append(torch.empty(n, dtype=torch.float32))
                self.hg.append(torch.empty(n, dtype=torch.bfloat16))
                for t in (self.hp[i], self.hm[i], self.hv[i], self.hg[i]):
                    if hugepages:                     # before the first touch
                        dos.dos_host_advise_hugepages(t.data_ptr(), t.numel() * t.element_size())
                    dos.dos_host_prefault(t.data_ptr(), t.numel() * t.element_size(), 16)
                self.hm[i].zero_()
                self.hv[i].zero_()
            if fill:
                S.fill_chunked(lambda start, count: S.params(seed, i, start, count, device), tmp[:n])
                self.hp[i].copy_(tmp[:n])
                if i < self.n_pinned:
                    self.hm[i].copy_(zeros[:n])
                    self.hv[i].copy_(zeros[:n])
                    # the fill came in by DMA: map the pages for the host cores too
                    dos.dos_host_prefault(self.blocks[i].ptr, self.blocks[i].nbytes, 16)
        del zeros, tmp
        self.targets = [dos.DOS_ON_CPU] * n_sg
        self.grads_on_host = [True] * n_sg
        self.host_grads_current = [False] * n_sg      # the pinned / pageable copy equals the device copy
        self.sgs = None

    def fill_grads(self, step: int, scales=None, **gkw):
        """Fresh gradients on the device for every subgroup (the backward pass'
        output); `place` / `sync_host_grads` then spill the CPU-planned ones."""
        for i in range(len(self.sizes)):
            sc = 1.0 if scales is None else scales[i]
            S.fill_chunked(lambda start, count: S.grads_bf16(self.seed, step, i, start, count, self.device,
                                                             scale=sc, **gkw), self.g[i])
            self.host_grads_current[i] = False

    def place(self, targets, residents=None, spill_all_grads=False):
        """Build the descriptor array for a plan; move resident state as needed.
        spill_all_grads: gradients of GPU-planned (non-resident) subgroups live in
        pinned host memory too and are fetched with p, m, v (Section 4.1, the case
        where freed GPU memory cannot hold them)."""
        n_sg = len(self.sizes)
        residents = residents if residents is not None else [0] * n_sg
        arr = (dos.dos_subgroup * max(n_sg, 1))()
        for i, n in enumerate(self.sizes):
            if residents[i] and self.res[i] is None:      # host -> device, once
                self.res[i] = [t.to(self.device) for t in (self.hp[i], self.hm[i], self.hv[i])]
            if not residents[i] and self.res[i] is not None:  # device -> host
                for h, d in zip((self.hp[i], self.hm[i], self.hv[i]), self.res[i]):
                    h.copy_(d)
                self.res[i] = None
            st = self.res[i] if residents[i] else (self.hp[i], self.hm[i], self.hv[i])
            on_gpu = targets[i] == dos.DOS_ON_GPU and (residents[i] or not spill_all_grads)
            g = self.g[i] if on_gpu else self.hg[i]
            host = dos.DOS_HOST_PAGEABLE if self.cpu_only[i] else dos.DOS_HOST_PINNED
            assert not (self.cpu_only[i] and targets[i] == dos.DOS_ON_GPU and not residents[i])
            arr[i] = dos.dos_subgroup(st[0].data_ptr(), st[1].data_ptr(), st[2].data_ptr(), g.data_ptr(),
                                      self.lp[i].data_ptr(), n,
                                      dos.DOS_DEVICE if residents[i] else host,
                                      dos.DOS_DEVICE if on_gpu else host)
        self.targets = list(targets)
        self.grads_on_host = [not (targets[i] == dos.DOS_ON_GPU and (residents[i] or not spill_all_grads))
                              for i in range(n_sg)]
        self.sgs = arr
        return arr

    def map_model_for_host_writes(self, threads: int = 1):
        """Touches every page of the device-resident 16-bit model from the host, so that the first phase
        with direct uploads (host stores through the PCIe BAR) does not pay for mapping those pages."""
        torch.cuda.synchronize()
        for lp in self.lp:
            if lp.numel():
                dos.dos_host_prefault(lp.data_ptr(), lp.numel() * 2, threads)

    def sync_host_grads(self):
        """Spill the gradients the descriptors expect in host memory (those whose host copy is stale)."""
        for i in range(len(self.sizes)):
            if self.grads_on_host[i] and not self.host_grads_current[i]:
                self.hg[i].copy_(self.g[i], non_blocking=True)
                self.host_grads_current[i] = True
        torch.cuda.synchronize()

    def state(self, i):
        """Current (p, m, v) tensors of subgroup i wherever they live."""
        return self.res[i] if self.res[i] is not None else (self.hp[i], self.hm[i], self.hv[i])

    @property
    def total(self):
        return sum(self.sizes)

    def free(self):
        self.hp = self.hm = self.hv = self.hg = None
        for b in self.blocks:
            b.free()
        self.blocks = []


def make_context(n_slots: int, slot_params: int, host_threads: int, *, device="cuda:0", stage_grads=False,
                 chunk_params: int = 4 << 20, ring_chunks: int = 0, flags: int = 0):
    """dos_ctx with torch-allocated slot memory and a libdos-pinned upload ring."""
    bpp = 14 if stage_grads else 12
    ring_chunks = ring_chunks or max(4, 3 * host_threads)
    slot_mem = torch.empty(max(n_slots, 1) * bpp * slot_params + 256, dtype=torch.uint8, device=device)
    base = _round_up(slot_mem.data_ptr(), 256)
    stage = PinnedBlock(ring_chunks * chunk_params * 2)
    cfg = dos.dos_ctx_config()
    cfg.slot_mem = base if n_slots else None
    cfg.slot_bytes = n_slots * bpp * slot_params
    cfg.slot_params = slot_params
    cfg.n_slots = n_slots
    cfg.host_threads = host_threads
    cfg.pinned_stage = stage.ptr
    cfg.pinned_stage_bytes = stage.nbytes
    cfg.upload_chunk_params = chunk_params
    cfg.flags = flags
    cfg.device = torch.device(device).index or 0
    ctx = dos.Context(cfg)
    ctx._keep = (slot_mem, stage)
    return ctx


def sample_take(t: torch.Tensor, every: int = 1 << 20, take: int = 1 << 16) -> torch.Tensor:
    """The elements of the flat tensor `t` at sample_index(len(t), every, take), in that order, gathered
    with strided views instead of an index list (the sample is runs of `take` consecutive elements)."""
    n = t.numel()
    full = n // every
    parts = []
    if full:
        parts.append(t[:full * every].view(full, every)[:, :take].reshape(-1))
    tail = n - full * every
    if tail:
        parts.append(t[full * every:full * every + min(take, tail)])
    return torch.cat(parts) if len(parts) != 1 else parts[0].clone()


def sample_index(n: int, every: int = 1 << 20, take: int = 1 << 16) -> np.ndarray:
    """Deterministic index subset the oracle owns at full size: the first `take`
    of every `every` elements (elements are independent, so the oracle is exact on
    the subset)."""
    base = np.arange(0, n, every, dtype=np.int64)
    idx = (base[:, None] + np.arange(take, dtype=np.int64)[None, :]).ravel()
    return idx[idx < n]
