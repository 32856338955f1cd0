"""Helpers shared by the GPU parity tests (no test logic of their own)."""
import numpy as np
import torch

import dos_synth as S
import paper_2410_21316_amd as dos
from oracle import adamw_oracle as ref

DEV = "cuda:0"


def ordered(bits16: np.ndarray) -> np.ndarray:
    """Map bf16 bit patterns to integers that are monotone in the value (both
    zeros map to the same integer)."""
    b = bits16.astype(np.int32)
    mag = b & 0x7FFF
    return np.where(b & 0x8000, 0x8000 - mag, 0x8000 + mag)


def assert_parity(tag, got_f32, want_f32, got_lp=None, want_lp=None, bitwise=True):
    """The bar: FP32 p, m, v within 1e-6 relative of the oracle, the bf16 copy
    within 1 bf16 ULP; and (design goal) bit-identical."""
    for name, g, w in zip("pmv", got_f32, want_f32):
        g = np.asarray(g); w = np.asarray(w)
        if g.shape == w.shape and np.array_equal(g.view(np.uint32), w.view(np.uint32)):
            continue                      # bit-identical: both bars hold
        both_nan = np.isnan(g) & np.isnan(w)
        fin = ~both_nan
        with np.errstate(invalid="ignore", divide="ignore", over="ignore"):
            err = np.abs(g[fin].astype(np.float64) - w[fin].astype(np.float64))
            den = np.abs(w[fin].astype(np.float64))
            same = g[fin].view(np.uint32) == w[fin].view(np.uint32)
            rel = np.where(same, 0.0, err / np.maximum(den, 1e-300))
        worst = float(np.max(rel)) if rel.size else 0.0
        assert worst <= 1e-6, f"{tag}: {name} max relative error {worst:.3e} > 1e-6"
        if bitwise:
            nbad = int(np.count_nonzero(g.view(np.uint32) != w.view(np.uint32)) - np.count_nonzero(
                both_nan & (g.view(np.uint32) != w.view(np.uint32))))
            assert nbad == 0, f"{tag}: {name} differs from the oracle in {nbad} of {g.size} bit patterns"
    if got_lp is not None:
        g = np.asarray(got_lp).view(np.uint16); w = np.asarray(want_lp).view(np.uint16)
        if g.shape == w.shape and np.array_equal(g, w):
            return
        nan = ((w & 0x7F80) == 0x7F80) & ((w & 0x7F) != 0)
        d = np.abs(ordered(g[~nan]) - ordered(w[~nan]))
        worst = int(d.max()) if d.size else 0
        assert worst <= 1, f"{tag}: bf16 copy off by {worst} ULP"
        if bitwise:
            assert np.array_equal(g[~nan], w[~nan]), f"{tag}: bf16 copy not bit-identical"
        assert np.all(((g[nan] & 0x7F80) == 0x7F80) & ((g[nan] & 0x7F) != 0))


class DeviceSubgroup:
    """Five device tensors and their descriptor."""

    def __init__(self, n, seed, index=0, device=DEV):
        self.n, self.seed, self.index = n, seed, index
        self.p = torch.empty(n, dtype=torch.float32, device=device)
        if n:
            S.fill_chunked(lambda start, count: S.params(seed, index, start, count, device), self.p)
        self.m = torch.zeros(n, dtype=torch.float32, device=device)
        self.v = torch.zeros(n, dtype=torch.float32, device=device)
        self.g = torch.zeros(n, dtype=torch.bfloat16, device=device)
        self.lp = torch.zeros(n, dtype=torch.bfloat16, device=device)
        self.desc = dos.subgroup_from_tensors(self.p, self.m, self.v, self.g, self.lp)

    def set_grads(self, step, **kw):
        if self.n:
            S.fill_chunked(lambda start, count: S.grads_bf16(self.seed, step, self.index, start, count,
                                                             self.g.device, **kw), self.g)

    def host_copy(self, sl=slice(None)):
        return (self.p[sl].cpu().numpy(), self.m[sl].cpu().numpy(), self.v[sl].cpu().numpy(),
                self.g[sl].view(torch.int16).cpu().numpy().view(np.uint16),
                self.lp[sl].view(torch.int16).cpu().numpy().view(np.uint16))


def oracle_step(state, g_bits, hp, step, threads=0, optimizer="adamw"):
    """state = [p, m, v, lp] numpy arrays, updated in place by the oracle's rule
    of that name (Adagrad and RMSProp leave m alone)."""
    ref.optimizer_step(optimizer, state[0], state[1], state[2], np.ascontiguousarray(g_bits), state[3], step=step,
                       threads=threads, **hp)


class Pinned:
    """A block of pinned host memory from dos_pinned_alloc, viewed as numpy."""

    def __init__(self, nbytes):
        import ctypes
        self.nbytes = max(int(nbytes), 256)
        self.ptr = dos.dos_pinned_alloc(self.nbytes)
        self._buf = (ctypes.c_uint8 * self.nbytes).from_address(self.ptr)
        self.u8 = np.frombuffer(self._buf, dtype=np.uint8)

    def view(self, dtype, offset_bytes, count):
        nb = count * np.dtype(dtype).itemsize
        return self.u8[offset_bytes:offset_bytes + nb].view(dtype)

    def free(self):
        if self.ptr:
            self.u8 = None
            self._buf = None
            dos.dos_pinned_free(self.ptr)
            self.ptr = 0


def round_up(x, a):
    return (x + a - 1) // a * a


class OffloadedState:
    """Optimizer state of several subgroups laid out as the interleaved phase
    expects it: p, m, v in pinned host memory (or on the device for static
    residents), gradients where ``grad_on_device[i]`` says, the bf16 model on the
    device.  Also keeps the oracle's copy of everything."""

    def __init__(self, sizes, seed, resident=None, grad_on_device=None, device=DEV, **gkw):
        self.sizes, self.seed, self.gkw, self.device = list(sizes), seed, gkw, device
        n_sg = len(sizes)
        self.resident = list(resident) if resident is not None else [0] * n_sg
        self.grad_on_device = list(grad_on_device) if grad_on_device is not None else [0] * n_sg
        total = sum(round_up(4 * n, 256) * 3 + round_up(2 * n, 256) for n in sizes) + 256
        self.pin = Pinned(total)
        self.sgs, self.host, self.dev, self.ref = [], [], [], []
        off = 0
        for i, n in enumerate(sizes):
            h = {}
            for name in "pmv":
                h[name] = self.pin.view(np.float32, off, n); off += round_up(4 * n, 256)
            h["g"] = self.pin.view(np.uint16, off, n); off += round_up(2 * n, 256)
            d = {"lp": torch.zeros(max(n, 1), dtype=torch.bfloat16, device=device)[:n]}
            p0 = S.params(seed, i, 0, n).numpy() if n else np.zeros(0, np.float32)
            if self.resident[i]:
                for name in "pmv":
                    d[name] = torch.zeros(max(n, 1), dtype=torch.float32, device=device)[:n]
                d["p"].copy_(torch.from_numpy(p0))
            else:
                h["p"][:] = p0; h["m"][:] = 0; h["v"][:] = 0
            if self.grad_on_device[i] or self.resident[i]:
                d["g"] = torch.zeros(max(n, 1), dtype=torch.bfloat16, device=device)[:n]
            self.host.append(h); self.dev.append(d)
            self.ref.append([p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)])
            st = d if self.resident[i] else h
            addr = lambda x: (x.data_ptr() if torch.is_tensor(x) else x.ctypes.data) if n else 0
            gsrc = d["g"] if "g" in d else h["g"]
            self.sgs.append(dos.subgroup(addr(st["p"]), addr(st["m"]), addr(st["v"]), addr(gsrc), addr(d["lp"]), n,
                                         dos.DOS_DEVICE if self.resident[i] else dos.DOS_HOST_PINNED,
                                         dos.DOS_DEVICE if "g" in d else dos.DOS_HOST_PINNED))

    def set_grads(self, step):
        self.gbits = []
        for i, n in enumerate(self.sizes):
            g = S.grads_bf16(self.seed, step, i, 0, n, **self.gkw) if n else torch.zeros(0, dtype=torch.bfloat16)
            bits = g.view(torch.int16).numpy().view(np.uint16)
            self.gbits.append(bits.copy())
            if "g" in self.dev[i]:
                self.dev[i]["g"].copy_(g)
            else:
                self.host[i]["g"][:] = bits
        torch.cuda.synchronize()

    def oracle_step(self, hp, step, optimizer="adamw"):
        for i, n in enumerate(self.sizes):
            if n:
                oracle_step(self.ref[i], self.gbits[i], hp, step, optimizer=optimizer)

    def current(self, i):
        if self.resident[i]:
            d = self.dev[i]
            return d["p"].cpu().numpy(), d["m"].cpu().numpy(), d["v"].cpu().numpy()
        h = self.host[i]
        return h["p"], h["m"], h["v"]

    def lp(self, i):
        return self.dev[i]["lp"].view(torch.int16).cpu().numpy().view(np.uint16)

    def check(self, tag):
        torch.cuda.synchronize()
        for i, n in enumerate(self.sizes):
            if n:
                assert_parity(f"{tag} subgroup {i}", self.current(i), self.ref[i][:3], self.lp(i), self.ref[i][3])

    def snapshot(self):
        return [tuple(np.array(x, copy=True) for x in self.current(i)) + (self.lp(i).copy(),)
                for i in range(len(self.sizes))]

    def free(self):
        self.host = None
        self.pin.free()


def make_context(n_slots, slot_params, host_threads=4, chunk_params=1 << 16, ring_chunks=6, stage_grads=True,
                 flags=0, device=DEV):
    """dos_ctx with torch-allocated slot memory and a pinned upload ring."""
    bpp = 14 if stage_grads else 12
    slot_mem = torch.empty(max(n_slots, 1) * bpp * slot_params + 256, dtype=torch.uint8, device=device)
    base = round_up(slot_mem.data_ptr(), 256)
    stage = Pinned(ring_chunks * chunk_params * 2) if ring_chunks else None     # 0: no upload ring at all
    cfg = dos.dos_ctx_config()
    cfg.slot_mem = base if n_slots else None
    cfg.slot_bytes = n_slots * bpp * slot_params
    cfg.slot_params = slot_params
    cfg.n_slots = n_slots
    cfg.host_threads = host_threads
    cfg.pinned_stage = stage.ptr if stage else None
    cfg.pinned_stage_bytes = stage.nbytes if stage else 0
    cfg.upload_chunk_params = chunk_params
    cfg.flags = flags
    cfg.device = 0
    ctx = dos.Context(cfg)
    ctx._keep = (slot_mem, stage)
    return ctx
