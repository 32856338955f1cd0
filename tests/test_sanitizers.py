"""Host-only translation units of libdos (planner, host AdamW and its thread
split) under AddressSanitizer + UndefinedBehaviorSanitizer, and the threaded host
update under ThreadSanitizer.  CPU only: built with g++, no HIP involved."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2410_21316_amd", "csrc")
SOURCES = [os.path.join(ROOT, "tests", "native", "host_driver.cpp"), os.path.join(CSRC, "plan.cpp"),
           os.path.join(CSRC, "adam_host.cpp")]
COMMON = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", "-pthread",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


PHASE_SOURCES = [os.path.join(ROOT, "tests", "native", "phase_driver.cpp"), os.path.join(CSRC, "phase.cpp"),
                 os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "adam_host.cpp")]
STUB = ["-I", os.path.join(ROOT, "tests", "native", "hip_stub"), "-DDOS_NO_TARGET_CLONES"]
SAN = [
    ("asan_ubsan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"],
     {"ASAN_OPTIONS": "detect_leaks=0", "UBSAN_OPTIONS": "print_stacktrace=1"}),
    ("tsan", ["-fsanitize=thread"], {"TSAN_OPTIONS": "halt_on_error=1"}),
]


@pytest.mark.parametrize("name,flags,env", SAN)
def test_update_phase_host_logic_under_sanitizers(name, flags, env, tmp_path):
    """The interleaved phase (validation, pieces, chunks, worker pool, upload ring)
    built against a stand-in HIP runtime whose copies are memcpy and whose kernels
    are the library's host update: results must equal the direct host update, and
    the sanitizers must stay silent.  (Streams created once per device are kept
    for the life of the process by design, so leak checking is off here.)"""
    exe = tmp_path / f"phase_driver_{name}"
    subprocess.check_call([*COMMON, *STUB, *flags, *PHASE_SOURCES, "-o", str(exe)])
    r = subprocess.run([str(exe)], capture_output=True, text=True, env={**os.environ, **env}, timeout=900)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "phase_driver ok" in r.stdout


def test_update_phase_allocates_no_host_memory(tmp_path):
    """Section 4.1: the interleaved update must not pay for allocations.  The same driver with every
    heap allocation of the process counted -- operator new replaced, malloc / calloc / realloc /
    aligned_alloc / posix_memalign wrapped by the linker: the count must not move across any
    dos_run_update_phase call, profiling statistics included (half of the driver's contexts profile)."""
    exe = tmp_path / "phase_driver_allocs"
    wraps = ["-Wl,--wrap=" + f for f in ("malloc", "calloc", "realloc", "aligned_alloc", "posix_memalign")]
    subprocess.check_call([*COMMON, *STUB, "-DDOS_COUNT_ALLOCS", *PHASE_SOURCES, *wraps, "-o", str(exe)])
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "phase_driver ok" in r.stdout


@pytest.mark.parametrize("name,flags,env", [
    ("asan_ubsan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"],
     {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1"}),
    ("tsan", ["-fsanitize=thread", "-DDOS_NO_TARGET_CLONES"], {"TSAN_OPTIONS": "halt_on_error=1"}),
])
def test_host_units_are_clean_under_sanitizers(name, flags, env, tmp_path):
    exe = tmp_path / f"host_driver_{name}"
    subprocess.check_call([*COMMON, *flags, *SOURCES, "-o", str(exe)])
    r = subprocess.run([str(exe)], capture_output=True, text=True, env={**os.environ, **env}, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "host_driver ok" in r.stdout
