"""Host-only helpers the benchmark and the full-size tests rely on: the strided gather of the oracle's share
must pick exactly the elements of the index list it stands for, and the benchmark's bound over all CPU/GPU
splits must be a bound (brute force on small cases)."""
import importlib.util
import itertools
import os

import numpy as np
import pytest
import torch

from paper_2410_21316_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("n", [0, 1, 5, 100, 1 << 10, (1 << 10) + 7, 3 * (1 << 10) + 700, 5 * (1 << 10)])
@pytest.mark.parametrize("every,take", [(1 << 10, 1 << 4), (1 << 10, 1 << 10), (64, 3)])
def test_sample_take_is_the_gather_of_sample_index(n, every, take):
    t = torch.arange(n, dtype=torch.int64) * 3 + 1
    got = W.sample_take(t, every, take).numpy() if n else np.zeros(0, np.int64)
    idx = W.sample_index(n, every, take)
    assert np.array_equal(got, t.numpy()[idx])
    # the sample is the first `take` of every `every`
    assert all(i % every < take for i in idx)
    assert len(idx) == sum(min(take, n - b) for b in range(0, n, every))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_lower_bound_opt_is_below_every_split_of_equal_subgroups():
    """With equal subgroups the bound tries every count of staged subgroups, so no assignment of them can
    have a smaller max(H2D time, D2H time, host update time, GPU update time)."""
    bench = _bench()
    sizes = [100_000_000] * 7
    link = (56e9, 48e9)
    for u_cpu in (2e9, 6e9, 16e9):
        for movable in ([True] * 7, [True, True, False, False, True, False, False]):
            lb, k = bench.lower_bound_opt(sizes, movable, link, 230e9, u_cpu, 12.0)
            best = None
            for bits in itertools.product((0, 1), repeat=7):
                if any(b and not mv for b, mv in zip(bits, movable)):
                    continue
                ng = sum(n for n, b in zip(sizes, bits) if b)
                nc = sum(sizes) - ng
                t = max((12.0 * ng + 2.0 * nc) / link[0], 12.0 * ng / link[1], nc / u_cpu, ng / 230e9)
                best = t if best is None else min(best, t)
            assert lb == pytest.approx(best, rel=1e-12)
            assert 0 <= k <= sum(movable)
    # residents cost GPU time only and take no part in the split
    lb, _ = bench.lower_bound_opt(sizes, [True] * 5 + [False] * 2, link, 1e9, 16e9, 12.0, resident_params=200_000_000)
    assert lb >= 200_000_000 / 1e9
