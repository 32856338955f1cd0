"""Seeded synthetic optimizer state and gradients.

This module serves both the HIP library's callers and the CPU oracle's callers
and holds none of the optimizer's arithmetic: it only produces inputs.  Every
value is a pure function of (seed, tensor id, step, subgroup, element index),
built from 64-bit integer mixing and exactly rounded float operations, so the
same call yields the same bits on the CPU and on the GPU and any index range can
be regenerated on its own (the oracle can own a sample of a state that is far
too large to hold twice).

Recipe (stands in for the flattened FP32 optimizer partitions and 16-bit
gradients of the paper's 7B-20B models, cut into ~100M-parameter subgroups as in
its evaluation setup; the training corpus itself is not needed because the
update depends on the data only through gradient values):

* standard normal Z: twelve 16-bit uniform fields (from three hashes) summed,
  centred and scaled by 2^-16 -- an Irwin-Hall(12) variate, exact in float32,
  tails end at +-6 sigma;
* parameters p = 0.02 * Z; moments start at zero;
* gradients g = bf16(scale * 1e-3 * X) with X = Z, or a Student-t with 3 degrees
  of freedom Z0 / sqrt((Z1^2+Z2^2+Z3^2)/3) for the heavy-tailed workloads;
* an exact-zero mask with probability ``zero_pct`` percent;
* a per-subgroup gradient scale drawn log-uniform in [0.1, 10].
"""
from __future__ import annotations

import torch

BASE_SEED = 241021316
TENSOR_P, TENSOR_G, TENSOR_MASK, TENSOR_SCALE = 0, 1, 2, 3

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(x: int) -> int:
    """Python int -> the same 64 bits as a signed value torch.int64 accepts."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_scalar(x: int) -> int:
    """splitmix64 finaliser on a Python int."""
    x &= _M64
    x = ((x ^ (x >> 30)) * _C1) & _M64
    x = ((x ^ (x >> 27)) * _C2) & _M64
    return x ^ (x >> 31)


def stream_key(seed: int, tensor_id: int, step: int, subgroup: int) -> int:
    k = _mix_scalar(seed + _GOLDEN)
    for word in (tensor_id, step, subgroup):
        k = _mix_scalar(k ^ ((word + 1) * _GOLDEN))
    return k


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 tensors (wrapping arithmetic)."""
    x = (x ^ _lsr(x, 30)) * _s64(_C1)
    x = (x ^ _lsr(x, 27)) * _s64(_C2)
    return x ^ _lsr(x, 31)


def _hashes(key: int, start: int, count: int, lane: int, device) -> torch.Tensor:
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(idx * _s64(_GOLDEN) + _s64(key + lane * _C2))


def _sum_fields(h: torch.Tensor) -> torch.Tensor:
    return (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)


def std_normal(key: int, start: int, count: int, device="cpu", lane0: int = 0) -> torch.Tensor:
    """float32 Irwin-Hall(12) standard normal for indices [start, start+count)."""
    s = _sum_fields(_hashes(key, start, count, lane0, device))
    s = s + _sum_fields(_hashes(key, start, count, lane0 + 1, device))
    s = s + _sum_fields(_hashes(key, start, count, lane0 + 2, device))
    # |s - 393210| < 2^24: the conversion and the power-of-two scale are exact.
    return (s - 393210).to(torch.float32) * (2.0 ** -16)


def student_t3(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    z0 = std_normal(key, start, count, device, 0)
    q = std_normal(key, start, count, device, 3) ** 2
    q = q + std_normal(key, start, count, device, 6) ** 2
    q = q + std_normal(key, start, count, device, 9) ** 2
    q = torch.clamp(q, min=2.0 ** -30)          # the three normals can all be 0
    return z0 / torch.sqrt(q / 3.0)


def subgroup_scale(seed: int, subgroup: int) -> float:
    """Log-uniform in [0.1, 10], one draw per subgroup (host-side double)."""
    u = (stream_key(seed, TENSOR_SCALE, 0, subgroup) >> 11) * (2.0 ** -53)
    return 10.0 ** (2.0 * u - 1.0)


def params(seed: int, subgroup: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """FP32 master parameters ~ N(0, 0.02^2)."""
    z = std_normal(stream_key(seed, TENSOR_P, 0, subgroup), start, count, device)
    return z * 0.02


def grads_bf16(seed: int, step: int, subgroup: int, start: int, count: int, device="cpu", *,
               sigma: float = 1e-3, scale: float = 1.0, zero_pct: float = 0.0,
               heavy_tail: bool = False) -> torch.Tensor:
    """bf16 gradients for one step (torch.bfloat16 tensor)."""
    key = stream_key(seed, TENSOR_G, step, subgroup)
    x = student_t3(key, start, count, device) if heavy_tail else std_normal(key, start, count, device)
    x = x * float(torch.tensor(scale * sigma, dtype=torch.float32))
    if zero_pct > 0.0:
        h = _hashes(stream_key(seed, TENSOR_MASK, step, subgroup), start, count, 0, device)
        keep = (_lsr(h, 32) % 10000) >= int(round(zero_pct * 100))
        x = torch.where(keep, x, torch.zeros_like(x))
    return x.to(torch.bfloat16)


def bits16(t: torch.Tensor) -> torch.Tensor:
    """Reinterpret a bf16 tensor as its 16-bit patterns (int16 view, no copy)."""
    assert t.dtype == torch.bfloat16
    return t.view(torch.int16)


def fill_chunked(fn, out: torch.Tensor, chunk: int = 1 << 24, **kw) -> torch.Tensor:
    """Fill the flat tensor ``out`` from ``fn(start=..., count=...)`` chunk by
    chunk (bounds the int64 temporaries to a few hundred MB)."""
    n = out.numel()
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        out[s:s + c].copy_(fn(start=s, count=c, **kw), non_blocking=False)
    return out


# Hyper-parameters every workload of the benchmark configuration list uses.
HPARAMS = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


__all__ = ["BASE_SEED", "HPARAMS", "params", "grads_bf16", "std_normal", "student_t3",
           "subgroup_scale", "stream_key", "bits16", "fill_chunked"]
