"""The C-ABI library loads and exports every symbol include/dos.h declares; argument
validation (which precedes any GPU work) returns the documented codes."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

import paper_2410_21316_amd as dos

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dos.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dos_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    lib = dos.load()
    names = declared_functions()
    assert "dos_adam_step" in names and "dos_plan_subgroups" in names and "dos_run_update_phase" in names
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(dos.binding.SIGNATURES) == names
    assert dos.dos_version() >= 100


def test_struct_layouts_match_the_header(tmp_path):
    """Compile the header with gcc and compare every field offset and struct size
    with the ctypes mirror."""
    structs = ["dos_subgroup", "dos_hparams", "dos_launch_cfg", "dos_cost_model", "dos_plan",
               "dos_ctx_config", "dos_phase_stats"]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "dos.h"', 'int main(void){']
    for st in structs:
        lines.append(f'printf("{st} %zu\\n", sizeof({st}));')
        for name, _ in getattr(dos, st)._fields_:
            lines.append(f'printf("{st}.{name} %zu\\n", offsetof({st}, {name}));')
    lines.append("return 0;}")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = dict(ln.split() for ln in subprocess.check_output([str(exe)], text=True).splitlines())
    for st in structs:
        cls = getattr(dos, st)
        assert int(got[st]) == C.sizeof(cls), st
        for name, _ in cls._fields_:
            assert int(got[f"{st}.{name}"]) == getattr(cls, name).offset, (st, name)


def test_strerror():
    lib = dos.load()
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert lib.dos_strerror(code)
    assert lib.dos_strerror(-2) == b"array not 16-byte aligned"


def _host_sg(n=64, offset=0):
    buf = [np.zeros(n + 8, np.float32) for _ in range(3)] + [np.zeros(n + 16, np.uint16) for _ in range(2)]
    ptrs = [b.ctypes.data + offset for b in buf]
    return buf, dos.subgroup(*ptrs, n, dos.DOS_DEVICE, dos.DOS_DEVICE)


GOOD = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1)


@pytest.mark.parametrize("bad", [dict(step=0), dict(step=-1), dict(beta1=1.0), dict(beta1=-0.5),
                                 dict(beta2=1.5), dict(eps=-1.0), dict(lr=float("nan")),
                                 dict(weight_decay=float("inf"))])
def test_adam_step_rejects_bad_hyperparameters_before_touching_the_gpu(bad):
    _, sg = _host_sg()
    lib = dos.load()
    hp = dos.hparams(**{**GOOD, **bad})
    assert lib.dos_adam_step(C.byref(sg), C.byref(hp), None) == dos.DOS_EINVAL
    sg.state_loc = sg.grad_loc = dos.DOS_HOST_PINNED
    assert lib.dos_adam_step_host(C.byref(sg), C.byref(hp), 1) == dos.DOS_EINVAL


def test_adam_step_rejects_null_misaligned_and_misplaced():
    lib = dos.load()
    hp = dos.hparams(**GOOD)
    _, sg = _host_sg()
    assert lib.dos_adam_step(None, C.byref(hp), None) == dos.DOS_EINVAL
    assert lib.dos_adam_step(C.byref(sg), None, None) == dos.DOS_EINVAL
    for field in ("p", "m", "v", "g", "p_lp"):
        _, bad = _host_sg()
        setattr(bad, field, None)
        assert lib.dos_adam_step(C.byref(bad), C.byref(hp), None) == dos.DOS_EINVAL
        _, bad = _host_sg()
        setattr(bad, field, getattr(bad, field) + 4)
        assert lib.dos_adam_step(C.byref(bad), C.byref(hp), None) == dos.DOS_EALIGN
    # host pointers handed to the device entry point (and the reverse) are refused
    _, sg = _host_sg()
    sg.state_loc = dos.DOS_HOST_PINNED
    assert lib.dos_adam_step(C.byref(sg), C.byref(hp), None) == dos.DOS_ESTATE
    _, sg = _host_sg()
    assert lib.dos_adam_step_host(C.byref(sg), C.byref(hp), 1) == dos.DOS_ESTATE
    # n == 0 is a no-op even with NULL arrays
    empty = dos.subgroup(None, None, None, None, None, 0, dos.DOS_DEVICE, dos.DOS_DEVICE)
    assert lib.dos_adam_step(C.byref(empty), C.byref(hp), None) == dos.DOS_OK
    cfg = dos.dos_launch_cfg(99, 0, 0)
    # (launch shape is validated only when there is work; checked on the GPU)
    assert lib.dos_adam_step_cfg(C.byref(empty), C.byref(hp), None, C.byref(cfg)) == dos.DOS_OK


def test_ctx_create_rejects_bad_configs_without_a_gpu():
    lib = dos.load()
    h = C.c_void_p()
    assert lib.dos_ctx_create(C.byref(h), None) == dos.DOS_EINVAL
    cfg = dos.dos_ctx_config()
    cfg.host_threads = 0
    assert lib.dos_ctx_create(C.byref(h), C.byref(cfg)) == dos.DOS_EINVAL
    cfg.host_threads = 2
    cfg.n_slots = 2
    cfg.slot_mem = 4096
    cfg.slot_params = 100            # not a multiple of 64
    cfg.slot_bytes = 1 << 20
    assert lib.dos_ctx_create(C.byref(h), C.byref(cfg)) == dos.DOS_EINVAL
    cfg.slot_params = 1 << 20        # 2 slots x 12 MiB do not fit 1 MiB
    assert lib.dos_ctx_create(C.byref(h), C.byref(cfg)) == dos.DOS_EBUDGET
    cfg.slot_mem = 4096 + 16
    assert lib.dos_ctx_create(C.byref(h), C.byref(cfg)) == dos.DOS_EALIGN
    assert not h.value
