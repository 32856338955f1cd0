"""ctypes front end of the scalar AdamW reference in ``adamw_ref.c``.

TEST INFRASTRUCTURE ONLY.  Only the tests, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module; the HIP library and
its Python binding never do, and this module never imports them.

The arithmetic lives in the C file (textbook bias-corrected AdamW in binary32,
paper Sections 1, 2 and 4.1 name the state and the precisions); this file only
builds it with gcc and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adamw_ref.c")
_LIB = os.path.join(_HERE, "libadamw_ref.so")
_lock = threading.Lock()
_lib = None

# No fast-math, no contraction: every C statement of the reference is one
# correctly rounded binary32 operation.
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-math-errno", "-fopenmp"]


def build(force: bool = False) -> str:
    """Compile the reference with gcc.  Returns the path of the shared object."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + ".tmp.%d" % os.getpid()
            subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", tmp, "-lm"])
            os.replace(tmp, _LIB)
    return _LIB


def _bind(lib):
    """Declare the C signatures on a loaded copy of the reference."""
    f32p = ctypes.POINTER(ctypes.c_float)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    hp = [ctypes.c_float] * 5 + [ctypes.c_int64]
    lib.ref_adamw_step.argtypes = [f32p, f32p, f32p, u16p, u16p, ctypes.c_uint64, *hp]
    lib.ref_adamw_step.restype = ctypes.c_int
    lib.ref_adamw_step_parallel.argtypes = [f32p, f32p, f32p, u16p, u16p, ctypes.c_uint64, *hp, ctypes.c_int]
    lib.ref_adamw_step_parallel.restype = ctypes.c_int
    lib.ref_adagrad_step.argtypes = [f32p, f32p, u16p, u16p, ctypes.c_uint64] + [ctypes.c_float] * 3 + [ctypes.c_int]
    lib.ref_adagrad_step.restype = ctypes.c_int
    lib.ref_rmsprop_step.argtypes = [f32p, f32p, u16p, u16p, ctypes.c_uint64] + [ctypes.c_float] * 4 + [ctypes.c_int]
    lib.ref_rmsprop_step.restype = ctypes.c_int
    lib.ref_adamw_scalars.argtypes = [*hp, f32p]
    lib.ref_adamw_scalars.restype = None
    lib.ref_bf16_to_f32_n.argtypes = [u16p, f32p, ctypes.c_uint64]
    lib.ref_bf16_to_f32_n.restype = None
    lib.ref_f32_to_bf16_n.argtypes = [f32p, u16p, ctypes.c_uint64]
    lib.ref_f32_to_bf16_n.restype = None
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(ctypes.CDLL(build()))
    return _lib


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous and a.flags.writeable
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _u16(a: np.ndarray, writeable: bool):
    assert a.dtype == np.uint16 and a.flags.c_contiguous and (a.flags.writeable or not writeable)
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def adamw_step(p, m, v, g, p_lp, *, lr, beta1, beta2, eps, weight_decay, step, threads=1):
    """Update ``p, m, v`` (float32 numpy, in place) with bf16 gradient bits ``g``
    (uint16) and write the bf16 bits of the new parameters into ``p_lp``.

    ``threads=1`` runs the plain scalar loop; ``threads>1`` (or 0 = all cores)
    runs the same loop body under a static parallel-for.  Returns the number of
    threads used."""
    n = p.shape[0]
    assert p.ndim == 1 and m.shape == v.shape == g.shape == p_lp.shape == (n,)
    lib = _load()
    args = (_f32(p), _f32(m), _f32(v), _u16(g, False), _u16(p_lp, True), n,
            lr, beta1, beta2, eps, weight_decay, int(step))
    if threads == 1:
        rc = lib.ref_adamw_step(*args)
        used = 1
    else:
        rc = used = lib.ref_adamw_step_parallel(*args, int(threads))
    if rc < 0:
        raise ValueError("AdamW is not defined for these hyper-parameters / step")
    return used


def adagrad_step(p, v, g, p_lp, *, lr, eps, weight_decay, threads=1):
    """Adagrad over ``p`` and its accumulator ``v`` (float32 numpy, in place) with
    bf16 gradient bits ``g``; writes the bf16 bits of the new parameters into
    ``p_lp``.  Returns the number of threads used (``threads`` as in adamw_step)."""
    n = p.shape[0]
    assert p.ndim == 1 and v.shape == g.shape == p_lp.shape == (n,)
    used = _load().ref_adagrad_step(_f32(p), _f32(v), _u16(g, False), _u16(p_lp, True), n, lr, eps, weight_decay,
                                    int(threads))
    if used < 0:
        raise ValueError("Adagrad is not defined for these hyper-parameters")
    return used


def rmsprop_step(p, v, g, p_lp, *, lr, alpha, eps, weight_decay, threads=1):
    """RMSProp (uncentred, no momentum) over ``p`` and its running mean of squared
    gradients ``v``; arguments as adagrad_step plus the smoothing constant."""
    n = p.shape[0]
    assert p.ndim == 1 and v.shape == g.shape == p_lp.shape == (n,)
    used = _load().ref_rmsprop_step(_f32(p), _f32(v), _u16(g, False), _u16(p_lp, True), n, lr, alpha, eps,
                                    weight_decay, int(threads))
    if used < 0:
        raise ValueError("RMSProp is not defined for these hyper-parameters")
    return used


def optimizer_step(name, p, m, v, g, p_lp, *, lr, beta1, beta2, eps, weight_decay, step, threads=1):
    """One step of the named rule ("adamw", "adagrad", "rmsprop") with the
    hyper-parameter set of adamw_step: Adagrad ignores the betas and the step,
    RMSProp takes beta2 as its smoothing constant; neither touches ``m``."""
    if name == "adamw":
        return adamw_step(p, m, v, g, p_lp, lr=lr, beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay,
                          step=step, threads=threads)
    if name == "adagrad":
        return adagrad_step(p, v, g, p_lp, lr=lr, eps=eps, weight_decay=weight_decay, threads=threads)
    if name == "rmsprop":
        return rmsprop_step(p, v, g, p_lp, lr=lr, alpha=beta2, eps=eps, weight_decay=weight_decay, threads=threads)
    raise ValueError(name)


def scalars(*, lr, beta1, beta2, eps, weight_decay, step) -> dict:
    """The eight binary32 per-step scalars the reference loop uses."""
    out = np.zeros(8, dtype=np.float32)
    _load().ref_adamw_scalars(lr, beta1, beta2, eps, weight_decay, int(step), _f32(out))
    names = ["beta1", "beta2", "omb1", "omb2", "step_size", "inv_sqrt_bc2", "eps", "decay"]
    return dict(zip(names, out))


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    src = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    out = np.empty(src.size, dtype=np.float32)
    _load().ref_bf16_to_f32_n(_u16(src, False), _f32(out), src.size)
    return out.reshape(np.shape(bits))


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even.  The input
    is read as raw bits, so NaN payloads reach the C helper unchanged."""
    src = np.ascontiguousarray(x, dtype=np.float32).ravel()
    out = np.empty(src.size, dtype=np.uint16)
    src_w = src if src.flags.writeable else src.copy()
    _load().ref_f32_to_bf16_n(_f32(src_w), _u16(out, True), src.size)
    return out.reshape(np.shape(x))
