"""Reference for the CPU/GPU subgroup planner.  TEST INFRASTRUCTURE ONLY: pure
Python, shares nothing with the HIP library, imported only by the tests.

Three pieces:

* ``stride_k``      -- the closed form of the performance model (Section 4.2, Eq. 1).
* ``stride_targets`` / ``run_update_trace`` -- the placement rule and the action
  order of the scheduling algorithm (Section 4.3, Algorithm 1).
* ``phase_cost`` / ``brute_force_plan`` -- a makespan estimate for an arbitrary
  CPU/GPU assignment and its exhaustive minimiser, used to bound the gap of the
  library's "balanced" planner.  The estimate is this build's own reading of the
  performance model, not a formula the paper prints: it keeps Eq. 1's terms
  (3S/B per staged subgroup and direction, S/(2B) per CPU-updated subgroup,
  S/U_g, S/U_c) and writes them per lane instead of per stride period, so that
  unequal subgroup sizes, separate link rates per direction, a fused host
  downscale, static residents (Section 4.1), slots smaller than a subgroup,
  the two-array update rules and the contention between the lanes that
  Section 5.4 reports can be priced.

Pins (tests/test_plan_pins.py): the paper's second-machine worked example
(Section 5.4: B=3, U_g=35, U_c=2, D_c=8.7 G params/s gives stride 2), "k=2 means
every alternate subgroup" (Sections 5.3, 5.4), the 8-subgroup timeline of the
update figure (33 % on the GPU, two static residents placed last; Section 4.1),
independence of k from the subgroup size (Section 4.2), and the balance identity
of Eq. 1 itself.  ``phase_cost``: every branch against numbers worked out by
hand from the terms above, the balance of Eq. 1 recovered from it (at the
paper's k both lanes end together), and an event-by-event timeline of the
three-stage pipeline that brackets the closed form.  The rounding of k is a
reading (the paper's one example fits rounding down and to nearest alike) and
is pinned as such.  tests/test_oracle_mutants.py plants mistakes in this file,
each caught by a pin.
"""
from __future__ import annotations

import itertools
from typing import Iterable, List, Sequence, Tuple

ON_CPU, ON_GPU = 0, 1


def stride_k_real(B: float, U_g: float, U_c: float, D_c: float) -> float:
    """Eq. 1 solved for k.  All four rates are in FP32 parameters per second:
    B the host link (each direction), U_g / U_c the GPU / CPU update rates, D_c
    the host FP32->16-bit downscale rate."""
    return (3.0 / B + 1.0 / U_g) / (1.0 / U_c + 1.0 / D_c - 1.0 / (2.0 * B))


def stride_k(B: float, U_g: float, U_c: float, D_c: float) -> int:
    """The integer stride handed to Algorithm 1.  The paper rounds its worked
    example 2.294 to 2; this build reads that as round-to-nearest, at least 1.
    A non-positive denominator means the host never becomes the bottleneck in
    the model: everything stays on the CPU except as forced, expressed here as
    an infinite stride (0 is returned as the 'no GPU subgroup' marker)."""
    den = 1.0 / U_c + 1.0 / D_c - 1.0 / (2.0 * B)
    if den <= 0.0:
        return 0
    k = stride_k_real(B, U_g, U_c, D_c)
    return max(1, int(k + 0.5))


def stride_targets(n_sg: int, k: int, residents: Iterable[int] = ()) -> List[int]:
    """Algorithm 1's test: subgroup i (0-based) goes to the GPU if it is a
    static resident or if (i+1) is a multiple of the stride k."""
    R = set(residents)
    return [ON_GPU if (i in R or (k >= 1 and (i + 1) % k == 0)) else ON_CPU for i in range(n_sg)]


def run_update_trace(n_sg: int, k: int, residents: Iterable[int] = ()) -> List[Tuple]:
    """Algorithm 1 as a list of actions, in issue order.  Actions:
    ("gpu_update", i), ("cpu_downscale", [subgroups queued so far]),
    ("flush_out", j), ("prefetch_in", j), ("cpu_update", i).
    prev_on_gpu / next_on_gpu are the nearest GPU-scheduled, non-resident
    subgroups before / after i; when none exists the action is omitted."""
    R = set(residents)
    tgt = stride_targets(n_sg, k, R)
    trace: List[Tuple] = []
    queue: List[int] = []
    for i in range(n_sg):
        if i in R or (k >= 1 and (i + 1) % k == 0):
            trace.append(("gpu_update", i))
            trace.append(("cpu_downscale", list(queue)))
            continue
        elif i not in R and k >= 1 and i % k == 0:
            prev = [j for j in range(i - 1, -1, -1) if tgt[j] == ON_GPU and j not in R]
            nxt = [j for j in range(i + 1, n_sg) if tgt[j] == ON_GPU and j not in R]
            if prev:
                trace.append(("flush_out", prev[0]))
            if nxt:
                trace.append(("prefetch_in", nxt[0]))
        trace.append(("cpu_update", i))
        queue.append(i)
    return trace


# --------------------------------------------------------------------------
# This build's makespan estimate for an arbitrary assignment.
# --------------------------------------------------------------------------

def phase_cost(sizes: Sequence[int], target: Sequence[int], *, h2d_Bps: float, d2h_Bps: float,
               gpu_params_per_s: float, cpu_params_per_s: float, launch_overhead_s: float,
               n_slots: int, resident: Sequence[int] = (), slot_params: int = 0,
               fp32_arrays: int = 3, cpu_cost_per_dma_byte: float = 0.0) -> Tuple[float, float]:
    """(predicted_s, lower_bound_s) of one update phase.

    The terms are those of the performance model (Section 4.2), written per lane
    instead of per stride period.  With A = ``fp32_arrays`` FP32 state arrays
    (3 for Adam: p, m, v -- the "3" of Eq. 1; 2 for the rules that keep p and one
    accumulator), a GPU-planned subgroup of n parameters moves 4*A*n bytes each
    way (Eq. 1's 3S/B) and costs n/U_g + one launch on the GPU; a CPU-planned one
    costs n/U_c on the host and 2n bytes of H2D for its refreshed 16-bit
    parameters (Eq. 1's S/(2B)).  Static residents (indices in ``resident``, all
    GPU-planned) never cross the link: they only add GPU time (Section 4.1).

    GPU lane.  With two or more staging slots prefetch, kernel and flush of
    consecutive pieces overlap, so the lane takes as long as its slowest stage:
    all H2D traffic, or all kernels, or the D2H traffic behind the lead of the
    first piece (its prefetch and its kernel; a piece is a whole subgroup, or
    ``slot_params`` parameters when subgroups stream through smaller slots).  With
    a single slot prefetch, kernel and flush of every staged subgroup run back to
    back, next to the 16-bit uploads.

    Host lane.  Both lanes share the host's memory system (Section 5.4, CPU cores
    per GPU): every staged byte, in either direction, takes
    ``cpu_cost_per_dma_byte`` parameters of update work away from the host cores,
    so the host lane takes (N_C + cost * 2 * 4*A*N_G) / U_c.

    predicted = max(host lane, GPU lane); lower = max(link time per direction)."""
    assert len(sizes) == len(target)
    assert fp32_arrays in (2, 3)
    R = set(resident)
    assert all(target[i] == ON_GPU for i in R)
    n_g = [n for i, (n, t) in enumerate(zip(sizes, target)) if t == ON_GPU and i not in R]
    n_r = [sizes[i] for i in R]
    n_c = [n for n, t in zip(sizes, target) if t == ON_CPU]
    N_G, N_C, N_R = float(sum(n_g)), float(sum(n_c)), float(sum(n_r))
    state_bytes = 4.0 * fp32_arrays
    h2d_bytes = state_bytes * N_G + 2.0 * N_C
    d2h_bytes = state_bytes * N_G
    t_h2d = h2d_bytes / h2d_Bps
    t_d2h = d2h_bytes / d2h_Bps
    staged_bytes = 2.0 * state_bytes * N_G
    t_cpu = (N_C + cpu_cost_per_dma_byte * staged_bytes) / cpu_params_per_s
    t_gpu = (N_G + N_R) / gpu_params_per_s + launch_overhead_s * (len(n_g) + len(n_r))
    if not n_g:
        lane = max(t_h2d, t_gpu)
    elif n_slots >= 2:
        first = n_g[0]
        if slot_params:                      # subgroups stream through the slots in pieces
            first = min(first, slot_params)
        lead = state_bytes * first / h2d_Bps + first / gpu_params_per_s + launch_overhead_s
        lane = max(t_h2d, lead + t_d2h, t_gpu)
    else:
        lane = state_bytes * N_G / h2d_Bps + t_gpu + t_d2h
        lane = max(lane, t_h2d)
    predicted = max(t_cpu, lane)
    lower = max(t_h2d, t_d2h)
    return predicted, lower


def brute_force_plan(sizes: Sequence[int], **cost) -> Tuple[float, List[int]]:
    """Exhaustive minimum of ``phase_cost`` over all 2^n assignments (n <= ~14)."""
    best, best_t = None, None
    for bits in itertools.product((ON_CPU, ON_GPU), repeat=len(sizes)):
        c, _ = phase_cost(sizes, bits, **cost)
        if best is None or c < best:
            best, best_t = c, list(bits)
    return best, best_t
