"""ctypes binding of libdos.so: the same names as include/dos.h, argument
marshalling only.  Every step of the update path runs inside the library; there
is no Python or CPU fallback -- if the library cannot be loaded this module
raises."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdos.so")

DOS_OK, DOS_EINVAL, DOS_EALIGN, DOS_EBUDGET, DOS_EHIP, DOS_ESTATE, DOS_ENOMEM = 0, -1, -2, -3, -4, -5, -6
DOS_STAGED_MAX_PARAMS = 2097152
DOS_HOST_PINNED, DOS_DEVICE, DOS_HOST_PAGEABLE = 0, 1, 2
DOS_ON_CPU, DOS_ON_GPU = 0, 1
DOS_OPT_ADAMW, DOS_OPT_ADAGRAD, DOS_OPT_RMSPROP = 0, 1, 2
DOS_PLAN_STRIDE, DOS_PLAN_BALANCED = 0, 1
DOS_CTX_PROFILE = 1
DOS_CTX_UPLOAD_DMA = 2
DOS_CTX_SPIN_WAIT = 4
DOS_CTX_UPLOAD_DIRECT = 8


class dos_subgroup(C.Structure):
    _fields_ = [("p", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p), ("g", C.c_void_p),
                ("p_lp", C.c_void_p), ("n", C.c_uint64), ("state_loc", C.c_int32),
                ("grad_loc", C.c_int32)]


class dos_hparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_int64), ("optimizer", C.c_int32)]


class dos_launch_cfg(C.Structure):
    _fields_ = [("variant", C.c_int32), ("block_threads", C.c_int32), ("grid_blocks", C.c_int32),
                ("lds_bytes", C.c_int32), ("xcd_group", C.c_int32)]


class dos_cost_model(C.Structure):
    _fields_ = [("h2d_Bps", C.c_double), ("d2h_Bps", C.c_double), ("gpu_params_per_s", C.c_double),
                ("cpu_params_per_s", C.c_double), ("downscale_params_per_s", C.c_double),
                ("launch_overhead_s", C.c_double), ("fp32_arrays", C.c_int32),
                ("cpu_cost_per_dma_byte", C.c_double), ("fit", C.c_double * 5)]


class dos_plan(C.Structure):
    _fields_ = [("n_sg", C.c_int32), ("n_slots", C.c_int32), ("slot_params", C.c_uint64),
                ("target", C.POINTER(C.c_uint8)), ("order", C.POINTER(C.c_int32)),
                ("resident", C.POINTER(C.c_uint8)), ("stride_k", C.c_int32),
                ("stride_k_real", C.c_double), ("predicted_s", C.c_double),
                ("lower_bound_s", C.c_double)]


class dos_ctx_config(C.Structure):
    _fields_ = [("slot_mem", C.c_void_p), ("slot_bytes", C.c_uint64), ("slot_params", C.c_uint64),
                ("n_slots", C.c_int32), ("host_threads", C.c_int32), ("h2d_stream", C.c_void_p),
                ("compute_stream", C.c_void_p), ("d2h_stream", C.c_void_p),
                ("upload_stream", C.c_void_p), ("pinned_stage", C.c_void_p),
                ("pinned_stage_bytes", C.c_uint64), ("upload_chunk_params", C.c_uint64),
                ("flags", C.c_int32), ("device", C.c_int32)]


class dos_phase_stats(C.Structure):
    _fields_ = [("wall_s", C.c_double), ("h2d_bytes", C.c_double), ("d2h_bytes", C.c_double),
                ("h2d_busy_s", C.c_double), ("d2h_busy_s", C.c_double), ("gpu_busy_s", C.c_double),
                ("duplex_overlap_s", C.c_double), ("cpu_lane_s", C.c_double),
                ("gpu_lane_s", C.c_double), ("cpu_compute_s", C.c_double), ("cpu_wait_s", C.c_double),
                ("cpu_enqueue_s", C.c_double), ("params_gpu", C.c_uint64), ("params_cpu", C.c_uint64),
                ("params_resident", C.c_uint64), ("n_gpu", C.c_int32), ("n_cpu", C.c_int32),
                ("n_resident", C.c_int32), ("n_slots", C.c_int32), ("n_pieces", C.c_int32),
                ("host_threads", C.c_int32), ("h2d_span_s", C.c_double), ("d2h_span_s", C.c_double)]

    def asdict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


# name -> (restype, argtypes); the list the symbol test checks against dos.h
SIGNATURES = {
    "dos_adam_step": (C.c_int, [C.POINTER(dos_subgroup), C.POINTER(dos_hparams), C.c_void_p]),
    "dos_adam_step_cfg": (C.c_int, [C.POINTER(dos_subgroup), C.POINTER(dos_hparams), C.c_void_p,
                                    C.POINTER(dos_launch_cfg)]),
    "dos_adam_step_host": (C.c_int, [C.POINTER(dos_subgroup), C.POINTER(dos_hparams), C.c_int32]),
    "dos_plan_subgroups": (C.c_int, [C.POINTER(dos_cost_model), C.POINTER(C.c_uint64), C.POINTER(C.c_uint8), C.c_int32,
                                     C.c_uint64, C.c_int32, C.c_int32, C.c_int32,
                                     C.POINTER(dos_plan)]),
    "dos_plan_cost": (C.c_int, [C.POINTER(dos_cost_model), C.POINTER(C.c_uint64),
                                C.POINTER(C.c_uint8), C.POINTER(C.c_uint8), C.c_int32, C.c_int32,
                                C.c_uint64, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "dos_ctx_create": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(dos_ctx_config)]),
    "dos_ctx_destroy": (None, [C.c_void_p]),
    "dos_run_update_phase": (C.c_int, [C.c_void_p, C.POINTER(dos_subgroup), C.c_int32,
                                       C.POINTER(dos_plan), C.POINTER(dos_hparams),
                                       C.POINTER(dos_phase_stats)]),
    "dos_calibrate": (C.c_int, [C.c_void_p, C.POINTER(dos_cost_model)]),
    "dos_ctx_last_timeline": (C.c_int, [C.c_void_p, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_int32)]),
    "dos_cost_model_observe": (C.c_int, [C.POINTER(dos_cost_model), C.POINTER(dos_phase_stats)]),
    "dos_device_large_bar": (C.c_int, [C.c_int32, C.POINTER(C.c_int32)]),
    "dos_pinned_alloc": (C.c_int, [C.POINTER(C.c_void_p), C.c_uint64]),
    "dos_pinned_free": (C.c_int, [C.c_void_p]),
    "dos_gpu_update_staged": (C.c_int, [C.POINTER(dos_subgroup), C.POINTER(dos_hparams), C.c_void_p]),
    "dos_host_advise_hugepages": (C.c_int, [C.c_void_p, C.c_uint64]),
    "dos_host_prefault": (C.c_int, [C.c_void_p, C.c_uint64, C.c_int32]),
    "dos_strerror": (C.c_char_p, [C.c_int]),
    "dos_last_hip_error": (C.c_char_p, []),
    "dos_version": (C.c_int32, []),
}

_lib = None


def load():
    """Load libdos.so (building it first only if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build_library()
    # Streams and device pointers come from PyTorch, so libdos must bind to the
    # HIP runtime PyTorch ships: load torch's runtime first, then the library
    # (same soname, the loader then shares one copy), and refuse two runtimes.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    with open("/proc/self/maps") as f:
        runtimes = {ln.split()[-1] for ln in f if "libamdhip64" in ln}
    if len(runtimes) > 1:
        raise ImportError("two HIP runtimes are mapped (%s): import torch before anything that loads "
                          "libamdhip64" % ", ".join(sorted(runtimes)))
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError = a declared symbol is missing
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


class DosError(RuntimeError):
    def __init__(self, status: int, where: str):
        lib = load()
        msg = lib.dos_strerror(status).decode()
        hip = lib.dos_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({status})" + (f" [{hip}]" if status == DOS_EHIP and hip else ""))
        self.status = status


def check(status: int, where: str) -> None:
    if status != DOS_OK:
        raise DosError(status, where)


# ------------------------------------------------------------- marshalling helpers

OPTIMIZERS = {"adamw": DOS_OPT_ADAMW, "adagrad": DOS_OPT_ADAGRAD, "rmsprop": DOS_OPT_RMSPROP}


def hparams(lr, beta1, beta2, eps, weight_decay, step, optimizer=DOS_OPT_ADAMW) -> dos_hparams:
    """optimizer: a dos_optimizer value or one of "adamw", "adagrad", "rmsprop"."""
    return dos_hparams(lr, beta1, beta2, eps, weight_decay, int(step), int(OPTIMIZERS.get(optimizer, optimizer)))


def subgroup(p, m, v, g, p_lp, n, state_loc, grad_loc) -> dos_subgroup:
    """Build a descriptor from raw addresses (ints)."""
    return dos_subgroup(p, m, v, g, p_lp, int(n), int(state_loc), int(grad_loc))


def subgroup_from_tensors(p, m, v, g, p_lp) -> dos_subgroup:
    """Descriptor over torch tensors (device or pinned host); the tensors must
    stay alive while the descriptor is in use."""
    n = p.numel()
    assert m.numel() == v.numel() == g.numel() == p_lp.numel() == n
    assert g.element_size() == 2 and p_lp.element_size() == 2 and p.element_size() == 4
    for t in (p, m, v, g, p_lp):
        assert t.is_contiguous()
    st = DOS_DEVICE if p.is_cuda else DOS_HOST_PINNED
    gl = DOS_DEVICE if g.is_cuda else DOS_HOST_PINNED
    return dos_subgroup(p.data_ptr(), m.data_ptr(), v.data_ptr(), g.data_ptr(), p_lp.data_ptr(), n, st, gl)


def dos_adam_step(sg: dos_subgroup, hp: dos_hparams, stream: int = 0) -> None:
    check(load().dos_adam_step(C.byref(sg), C.byref(hp), C.c_void_p(stream)), "dos_adam_step")


def dos_adam_step_cfg(sg, hp, stream=0, variant=0, block_threads=0, grid_blocks=0, lds_bytes=0, xcd_group=0) -> None:
    cfg = dos_launch_cfg(variant, block_threads, grid_blocks, lds_bytes, xcd_group)
    check(load().dos_adam_step_cfg(C.byref(sg), C.byref(hp), C.c_void_p(stream), C.byref(cfg)),
          "dos_adam_step_cfg")


def dos_adam_step_host(sg: dos_subgroup, hp: dos_hparams, threads: int = 1) -> None:
    check(load().dos_adam_step_host(C.byref(sg), C.byref(hp), int(threads)), "dos_adam_step_host")


class Plan:
    """Owns the arrays a dos_plan points to."""

    def __init__(self, n_sg: int):
        self.n_sg = n_sg
        self.target = (C.c_uint8 * max(n_sg, 1))()
        self.order = (C.c_int32 * max(n_sg, 1))()
        self.resident = (C.c_uint8 * max(n_sg, 1))()
        self.c = dos_plan(n_sg, 0, 0, C.cast(self.target, C.POINTER(C.c_uint8)),
                          C.cast(self.order, C.POINTER(C.c_int32)),
                          C.cast(self.resident, C.POINTER(C.c_uint8)), 0, 0.0, 0.0, 0.0)

    @property
    def targets(self):
        return list(self.target[:self.n_sg])

    @property
    def orders(self):
        return list(self.order[:self.n_sg])

    @property
    def residents(self):
        return list(self.resident[:self.n_sg])

    @classmethod
    def manual(cls, targets, order=None, n_slots=2, slot_params=0, residents=None):
        pl = cls(len(targets))
        for i, t in enumerate(targets):
            pl.target[i] = int(t)
            pl.order[i] = i if order is None else int(order[i])
            pl.resident[i] = 0 if residents is None else int(residents[i])
        pl.c.n_slots = n_slots
        pl.c.slot_params = slot_params
        return pl


def cost_model(h2d_Bps, d2h_Bps, gpu_params_per_s, cpu_params_per_s, downscale_params_per_s=0.0,
               launch_overhead_s=0.0, fp32_arrays=3, cpu_cost_per_dma_byte=0.0) -> dos_cost_model:
    return dos_cost_model(h2d_Bps, d2h_Bps, gpu_params_per_s, cpu_params_per_s,
                          downscale_params_per_s, launch_overhead_s, int(fp32_arrays), float(cpu_cost_per_dma_byte))


def dos_plan_subgroups(cm: dos_cost_model, sizes, gpu_budget_bytes: int, mode: int = DOS_PLAN_BALANCED,
                       n_resident_max: int = 0, bytes_per_param_slot: int = 12, cpu_only=None) -> Plan:
    n = len(sizes)
    arr = (C.c_uint64 * max(n, 1))(*[int(s) for s in sizes])
    mask = (C.c_uint8 * max(n, 1))(*[int(bool(x)) for x in cpu_only]) if cpu_only is not None else None
    pl = Plan(n)
    check(load().dos_plan_subgroups(C.byref(cm), arr, mask, n, int(gpu_budget_bytes),
                                    int(bytes_per_param_slot), int(mode), int(n_resident_max),
                                    C.byref(pl.c)), "dos_plan_subgroups")
    return pl


def dos_plan_cost(cm: dos_cost_model, sizes, targets, n_slots: int, residents=None, slot_params: int = 0):
    n = len(sizes)
    arr = (C.c_uint64 * max(n, 1))(*[int(s) for s in sizes])
    tg = (C.c_uint8 * max(n, 1))(*[int(t) for t in targets])
    rs = (C.c_uint8 * max(n, 1))(*[int(r) for r in residents]) if residents is not None else None
    pred, low = C.c_double(), C.c_double()
    check(load().dos_plan_cost(C.byref(cm), arr, tg, rs, n, int(n_slots), int(slot_params), C.byref(pred),
                               C.byref(low)),
          "dos_plan_cost")
    return pred.value, low.value


def dos_cost_model_observe(cm: dos_cost_model, st: dos_phase_stats) -> None:
    check(load().dos_cost_model_observe(C.byref(cm), C.byref(st)), "dos_cost_model_observe")


def dos_device_large_bar(device: int = 0) -> bool:
    yes = C.c_int32()
    check(load().dos_device_large_bar(int(device), C.byref(yes)), "dos_device_large_bar")
    return bool(yes.value)


def dos_pinned_alloc(nbytes: int) -> int:
    out = C.c_void_p()
    check(load().dos_pinned_alloc(C.byref(out), int(nbytes)), "dos_pinned_alloc")
    return out.value


def dos_pinned_free(ptr: int) -> None:
    check(load().dos_pinned_free(C.c_void_p(ptr)), "dos_pinned_free")


def dos_gpu_update_staged(sg: dos_subgroup, hp: dos_hparams, stream: int = 0) -> None:
    check(load().dos_gpu_update_staged(C.byref(sg), C.byref(hp), C.c_void_p(stream)), "dos_gpu_update_staged")


def dos_host_advise_hugepages(ptr: int, nbytes: int) -> bool:
    """True when the kernel accepted the advice."""
    return load().dos_host_advise_hugepages(C.c_void_p(ptr), int(nbytes)) == DOS_OK


def dos_host_prefault(ptr: int, nbytes: int, threads: int = 1) -> None:
    check(load().dos_host_prefault(C.c_void_p(ptr), int(nbytes), int(threads)), "dos_host_prefault")


class Context:
    """dos_ctx handle (dos_ctx_create / dos_ctx_destroy)."""

    def __init__(self, cfg: dos_ctx_config):
        self._h = C.c_void_p()
        self.cfg = cfg
        check(load().dos_ctx_create(C.byref(self._h), C.byref(cfg)), "dos_ctx_create")

    def close(self):
        if self._h:
            load().dos_ctx_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def dos_run_update_phase(self, sgs, plan: Plan, hp: dos_hparams) -> dos_phase_stats:
        n = len(sgs)
        arr = sgs if isinstance(sgs, C.Array) else (dos_subgroup * max(n, 1))(*sgs)
        st = dos_phase_stats()
        check(load().dos_run_update_phase(self._h, arr, n, C.byref(plan.c), C.byref(hp), C.byref(st)),
              "dos_run_update_phase")
        return st

    def dos_ctx_last_timeline(self):
        """Rows of (prefetch start, end, kernel start, end, flush start, end) in ms, one per staged piece."""
        n = C.c_int32()
        check(load().dos_ctx_last_timeline(self._h, None, 0, C.byref(n)), "dos_ctx_last_timeline")
        buf = (C.c_float * (6 * max(1, n.value)))()
        check(load().dos_ctx_last_timeline(self._h, buf, n.value, C.byref(n)), "dos_ctx_last_timeline")
        return [tuple(buf[6 * j:6 * j + 6]) for j in range(n.value)]

    def dos_calibrate(self) -> dos_cost_model:
        cm = dos_cost_model()
        check(load().dos_calibrate(self._h, C.byref(cm)), "dos_calibrate")
        return cm


def dos_version() -> int:
    return load().dos_version()
