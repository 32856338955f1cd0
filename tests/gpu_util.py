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


def oracle_step(state, g_bits, hp, step, threads=0):
    """state = [p, m, v, lp] numpy arrays, updated in place by the oracle."""
    ref.adamw_step(state[0], state[1], state[2], np.ascontiguousarray(g_bits), state[3], step=step,
                   threads=threads, **hp)
