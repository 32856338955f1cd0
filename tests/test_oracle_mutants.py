"""The pins must notice a plausible mistake anywhere in the oracle.  Each case
plants one mistake in a copy of oracle/adamw_ref.c (on the CPU, in a temporary
file), builds it, points the oracle's Python front end at the mutant and runs
the pin checks: at least one of them has to fail."""
import ctypes
import os
import subprocess

import pytest

import test_oracle_pins as pins
import test_oracle_pins_accum as acc
from oracle import adamw_oracle as ref

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "adamw_ref.c")

PIN_CHECKS = [
    lambda: pins.test_first_step_is_sign_step(0.0),
    lambda: pins.test_first_step_is_sign_step(0.3),
    pins.test_zero_gradients_give_pure_decoupled_decay,
    lambda: pins.test_constant_gradient_recurrences(3e-3),
    lambda: pins.test_constant_gradient_recurrences(-7e-4),
    lambda: pins.test_against_double_precision_textbook(1e-8, 0.01, 1e-4),
    lambda: pins.test_against_double_precision_textbook(1e-3, 0.0, 1e-2),
    lambda: pins.test_against_double_precision_textbook(1e-5, 0.2, 3e-3),
    pins.test_eps_sits_outside_the_root_and_is_not_bias_corrected,
    pins.test_against_torch_adamw,
    pins.test_elements_are_independent_brute_force,
    pins.test_parallel_loop_is_bit_identical_to_scalar_loop,
    pins.test_step_scalars_match_their_definitions,
    pins.test_bf16_widening_is_exact_and_roundtrips_exhaustively,
    pins.test_bf16_rounding_hand_built_cases,
    pins.test_bf16_rounding_is_nearest_value_with_even_ties,
    # Adagrad and RMSProp
    lambda: acc.test_adagrad_first_step_is_sign_step(0.3),
    lambda: acc.test_rmsprop_first_step_is_scaled_sign_step(0.3),
    lambda: acc.test_adagrad_constant_gradient(-7e-4),
    lambda: acc.test_rmsprop_constant_gradient(3e-3),
    lambda: acc.test_zero_gradients_give_pure_decoupled_decay("adagrad"),
    lambda: acc.test_zero_gradients_give_pure_decoupled_decay("rmsprop"),
    lambda: acc.test_eps_sits_outside_the_root("adagrad"),
    lambda: acc.test_eps_sits_outside_the_root("rmsprop"),
    lambda: acc.test_against_double_precision_textbook("adagrad", 1e-5, 0.2, 3e-3),
    lambda: acc.test_against_double_precision_textbook("rmsprop", 1e-3, 0.0, 1e-2),
    lambda: acc.test_against_torch("adagrad"),
    lambda: acc.test_against_torch("rmsprop"),
    lambda: acc.test_elements_are_independent_and_loops_agree("adagrad"),
    lambda: acc.test_elements_are_independent_and_loops_agree("rmsprop"),
]

# (name, [(text in the reference, planted replacement), ...])
MUTANTS = [
    ("beta2 used for the first moment", [("float a = s->beta1 * *m;", "float a = s->beta2 * *m;")]),
    ("first moment terms subtracted", [("float mt = a + b;", "float mt = a - b;")]),
    ("gradient not squared", [("float f = e * g;", "float f = e;")]),
    ("second moment terms subtracted", [("float vt = c + f;", "float vt = c - f;")]),
    ("square root dropped", [("float r = sqrtf(vt);", "float r = vt;")]),
    ("eps dropped", [("float d = q + s->eps;", "float d = q;")]),
    ("eps inside the root", [("float r = sqrtf(vt);", "float r = sqrtf(vt + s->eps);"),
                             ("float d = q + s->eps;", "float d = q;")]),
    ("second bias correction dropped", [("float q = r * s->inv_sqrt_bc2;", "float q = r;")]),
    ("second bias correction inverted", [("s.inv_sqrt_bc2 = (float)(1.0 / sqrt(bc2));",
                                          "s.inv_sqrt_bc2 = (float)(sqrt(bc2));")]),
    ("first bias correction dropped", [("s.step_size = (float)((double)lr / bc1);",
                                        "s.step_size = (float)((double)lr);")]),
    ("bias corrections use the wrong beta", [("double bc2 = 1.0 - pow((double)beta2, (double)step);",
                                              "double bc2 = 1.0 - pow((double)beta1, (double)step);")]),
    ("step counted from zero", [("double bc1 = 1.0 - pow((double)beta1, (double)step);",
                                 "double bc1 = 1.0 - pow((double)beta1, (double)step + 1.0);")]),
    ("weight decay dropped", [("float pd = *p * s->decay;", "float pd = *p;")]),
    ("decay without the learning rate", [("s.decay = (float)(1.0 - (double)lr * (double)weight_decay);",
                                          "s.decay = (float)(1.0 - (double)weight_decay);")]),
    ("decay applied after the step", [("float pt = pd - w;", "float pt = (*p - w) * s->decay;")]),
    ("update added instead of subtracted", [("float pt = pd - w;", "float pt = pd + w;")]),
    ("quotient transposed", [("float u = mt / d;", "float u = d / mt;")]),
    ("old momentum in the update", [("float u = mt / d;", "float u = *m / d;")]),
    ("one minus beta1 replaced by beta1", [("s.omb1 = 1.0f - beta1;", "s.omb1 = beta1;")]),
    ("one minus beta2 replaced by one minus beta1", [("s.omb2 = 1.0f - beta2;", "s.omb2 = 1.0f - beta1;")]),
    ("gradient index reversed", [("ref_adamw_element(&s, &p[i], &m[i], &v[i], g[i], &p_lp[i]);\n  return 0;",
                                  "ref_adamw_element(&s, &p[i], &m[i], &v[i], g[n - 1 - i], &p_lp[i]);\n  return 0;")]),
    ("state arrays swapped", [("ref_adamw_element(&s, &p[i], &m[i], &v[i], g[i], &p_lp[i]);\n  return 0;",
                               "ref_adamw_element(&s, &p[i], &v[i], &m[i], g[i], &p_lp[i]);\n  return 0;")]),
    ("bf16 widening shifted wrongly", [("uint32_t u = (uint32_t)h << 16;", "uint32_t u = (uint32_t)h << 15;")]),
    ("bf16 rounding truncates", [("keep += 1u;", "keep += 0u;")]),
    ("bf16 ties round up", [("if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1u;",
                             "if (rest >= 0x8000u) keep += 1u;")]),
    ("bf16 NaN not kept", [("if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);", "")]),
    ("low-precision copy of the old parameter", [("*p_lp = ref_f32_to_bf16(pt);", "*p_lp = ref_f32_to_bf16(pd);")]),
    ("parallel loop skips the last element", [("for (int64_t i = 0; i < (int64_t)n; ++i)",
                                               "for (int64_t i = 0; i < (int64_t)n - 1; ++i)")]),
    # Adagrad and RMSProp
    ("adagrad: gradient not squared", [("float f = g * g;", "float f = g;")]),
    ("adagrad: accumulator overwritten", [("float vt = *v + f;", "float vt = f;")]),
    ("adagrad: accumulator decreases", [("float vt = *v + f;", "float vt = *v - f;")]),
    ("accumulators: eps dropped", [("float d = r + eps;", "float d = r;")]),
    ("accumulators: eps inside the root", [("float r = sqrtf(vt);\n  float d = r + eps;",
                                            "float r = sqrtf(vt + eps);\n  float d = r;")]),
    ("accumulators: quotient transposed", [("float u = g / d;", "float u = d / g;")]),
    ("accumulators: learning rate dropped", [("float w = lr * u;", "float w = u;")]),
    ("accumulators: update added", [("float pt = pd - w;\n  *v = vt;", "float pt = pd + w;\n  *v = vt;")]),
    ("accumulators: weight decay dropped", [("float pd = *p * decay;", "float pd = *p;")]),
    ("accumulators: new accumulator not stored", [("float pt = pd - w;\n  *v = vt;", "float pt = pd - w;")]),
    ("accumulators: 16-bit copy of the decayed old parameter",
     [("*p = pt;\n  *p_lp = ref_f32_to_bf16(pt);\n}\n\nstatic inline void ref_adagrad_element",
       "*p = pt;\n  *p_lp = ref_f32_to_bf16(pd);\n}\n\nstatic inline void ref_adagrad_element")]),
    ("adagrad: decay without the learning rate",
     [("const float decay = (float)(1.0 - (double)lr * (double)weight_decay);",
       "const float decay = (float)(1.0 - (double)weight_decay);")]),
    ("adagrad: gradient index reversed",
     [("ref_adagrad_element(lr, eps, decay, &p[i], &v[i], g[i], &p_lp[i]);\n    return 1;",
       "ref_adagrad_element(lr, eps, decay, &p[i], &v[i], g[n - 1 - i], &p_lp[i]);\n    return 1;")]),
    ("rmsprop: old mean not discounted", [("float c = alpha * *v;", "float c = *v;")]),
    ("rmsprop: new term weighted by alpha", [("const float oma = 1.0f - alpha;", "const float oma = alpha;")]),
    ("rmsprop: gradient not squared", [("float e = oma * g;\n  float f = e * g;", "float e = oma * g;\n  float f = e;")]),
    ("rmsprop: parallel loop skips the last element",
     [("for (int64_t i = 0; i < (int64_t)n; ++i)\n      ref_rmsprop_element",
       "for (int64_t i = 0; i < (int64_t)n - 1; ++i)\n      ref_rmsprop_element")]),
]


@pytest.mark.parametrize("name,edits", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, edits, tmp_path, monkeypatch):
    text = open(SRC).read()
    for old, new in edits:
        assert text.count(old) >= 1, f"reference text changed: {old!r}"
        text = text.replace(old, new, 1)
    c_file = tmp_path / "mutant.c"
    c_file.write_text(text)
    so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", *ref.CFLAGS, str(c_file), "-o", str(so), "-lm"])
    ref._load()                                           # make sure the real one is built and bound
    monkeypatch.setattr(ref, "_lib", ref._bind(ctypes.CDLL(str(so))))
    failed = []
    for check in PIN_CHECKS:
        try:
            check()
        except AssertionError:
            failed.append(check)
            break
    assert failed, f"no pin noticed: {name}"


def test_unmodified_reference_passes_every_pin():
    for check in PIN_CHECKS:
        check()


# ---- the planner reference (oracle/plan_ref.py) -----------------------------------------------------

import importlib.util

import test_plan_pins as plan_pins

PLAN_SRC = os.path.join(os.path.dirname(SRC), "plan_ref.py")

PLAN_PIN_CHECKS = [
    plan_pins.test_second_machine_worked_example,
    plan_pins.test_eq1_balances_host_time_against_link_plus_gpu_time,
    plan_pins.test_faster_host_means_larger_stride_and_faster_link_smaller,
    plan_pins.test_stride_rounding_follows_the_reading_taken,
    plan_pins.test_stride_two_is_every_alternate_subgroup,
    plan_pins.test_update_figure_timeline,
    plan_pins.test_every_subgroup_is_updated_exactly_once,
    plan_pins.test_cost_function_limits,
    plan_pins.test_brute_force_beats_both_extremes,
    plan_pins.test_overlapped_lane_waits_for_the_flushes_behind_the_first_piece,
    plan_pins.test_pieces_shorten_the_lead,
    plan_pins.test_single_slot_serialises_the_staged_subgroups_next_to_the_uploads,
    plan_pins.test_residents_cost_gpu_time_only,
    plan_pins.test_two_array_rules_move_eight_bytes_per_parameter,
    plan_pins.test_staged_traffic_is_charged_to_the_host_lane,
    plan_pins.test_eq1_balance_is_the_models_balance,
    lambda: plan_pins.test_lane_estimate_against_an_event_by_event_timeline(60e9, 40e9, 200e9, 3),
    lambda: plan_pins.test_lane_estimate_against_an_event_by_event_timeline(40e9, 60e9, 200e9, 2),
    lambda: plan_pins.test_lane_estimate_against_an_event_by_event_timeline(50e9, 50e9, 2e9, 3),
    lambda: plan_pins.test_lane_estimate_against_an_event_by_event_timeline(55e9, 48e9, 230e9, 1),
]

PLAN_MUTANTS = [
    ("Eq. 1: link term counted once instead of three times", [("(3.0 / B + 1.0 / U_g)", "(1.0 / B + 1.0 / U_g)")]),
    ("Eq. 1: upload term added instead of subtracted", [("return (3.0 / B + 1.0 / U_g) / (1.0 / U_c + 1.0 / D_c - 1.0 / (2.0 * B))",
                                                         "return (3.0 / B + 1.0 / U_g) / (1.0 / U_c + 1.0 / D_c + 1.0 / (2.0 * B))")]),
    ("Eq. 1: downscale term dropped", [("return (3.0 / B + 1.0 / U_g) / (1.0 / U_c + 1.0 / D_c - 1.0 / (2.0 * B))",
                                        "return (3.0 / B + 1.0 / U_g) / (1.0 / U_c - 1.0 / (2.0 * B))")]),
    ("Eq. 1: GPU term dropped", [("(3.0 / B + 1.0 / U_g)", "(3.0 / B)")]),
    ("stride rounds down", [("return max(1, int(k + 0.5))", "return max(1, int(k))")]),
    ("stride rounds up", [("return max(1, int(k + 0.5))", "return max(1, int(k + 0.999))")]),
    ("stride test off by one", [("(k >= 1 and (i + 1) % k == 0)) else ON_CPU", "(k >= 1 and i % k == 0)) else ON_CPU")]),
    ("residents ignored by the placement", [("[ON_GPU if (i in R or (k >= 1", "[ON_GPU if ((k >= 1")]),
    ("trace: flush and prefetch swapped", [('trace.append(("flush_out", prev[0]))', 'trace.append(("prefetch_in", prev[0]))'),
                                           ('trace.append(("prefetch_in", nxt[0]))', 'trace.append(("flush_out", nxt[0]))')]),
    ("trace: prefetch looks backwards", [("nxt = [j for j in range(i + 1, n_sg)", "nxt = [j for j in range(i - 1, -1, -1)")]),
    ("trace: downscale queue not handed over", [('trace.append(("cpu_downscale", list(queue)))', 'trace.append(("cpu_downscale", []))')]),
    ("cost: flushes priced at the prefetch rate in the overlapped lane", [("lane = max(t_h2d, lead + t_d2h, t_gpu)",
                                                                           "lane = max(t_h2d, lead + t_h2d, t_gpu)")]),
    ("cost: lead of the first piece dropped", [("lane = max(t_h2d, lead + t_d2h, t_gpu)", "lane = max(t_h2d, t_d2h, t_gpu)")]),
    ("cost: lead priced at the flush rate", [("lead = state_bytes * first / h2d_Bps", "lead = state_bytes * first / d2h_Bps")]),
    ("cost: lead without its kernel", [("lead = state_bytes * first / h2d_Bps + first / gpu_params_per_s + launch_overhead_s",
                                        "lead = state_bytes * first / h2d_Bps")]),
    ("cost: slot size ignored", [("first = min(first, slot_params)", "first = first")]),
    ("cost: the largest staged subgroup leads", [("first = n_g[0]", "first = max(n_g)")]),
    ("cost: residents dropped from the GPU time", [("t_gpu = (N_G + N_R) / gpu_params_per_s + launch_overhead_s * (len(n_g) + len(n_r))",
                                                    "t_gpu = N_G / gpu_params_per_s + launch_overhead_s * len(n_g)")]),
    ("cost: residents cross the link", [("h2d_bytes = state_bytes * N_G + 2.0 * N_C", "h2d_bytes = state_bytes * (N_G + N_R) + 2.0 * N_C"),
                                        ("d2h_bytes = state_bytes * N_G", "d2h_bytes = state_bytes * (N_G + N_R)")]),
    ("cost: residents-only lane forgets the kernels", [("lane = max(t_h2d, t_gpu)\n    elif", "lane = t_h2d\n    elif")]),
    ("cost: uploads dropped from H2D", [("h2d_bytes = state_bytes * N_G + 2.0 * N_C", "h2d_bytes = state_bytes * N_G")]),
    ("cost: uploads priced at four bytes", [("h2d_bytes = state_bytes * N_G + 2.0 * N_C", "h2d_bytes = state_bytes * N_G + 4.0 * N_C")]),
    ("cost: three arrays whatever the rule", [("state_bytes = 4.0 * fp32_arrays", "state_bytes = 12.0")]),
    ("cost: contention charged for one direction only", [("staged_bytes = 2.0 * state_bytes * N_G", "staged_bytes = state_bytes * N_G")]),
    ("cost: contention term dropped", [("t_cpu = (N_C + cpu_cost_per_dma_byte * staged_bytes) / cpu_params_per_s",
                                        "t_cpu = N_C / cpu_params_per_s")]),
    ("cost: contention charged for the uploads too", [("staged_bytes = 2.0 * state_bytes * N_G", "staged_bytes = 2.0 * state_bytes * N_G + 2.0 * N_C")]),
    ("cost: single slot overlaps the flushes", [("lane = state_bytes * N_G / h2d_Bps + t_gpu + t_d2h", "lane = state_bytes * N_G / h2d_Bps + t_gpu")]),
    ("cost: single slot forgets the uploads", [("        lane = max(lane, t_h2d)\n", "")]),
    ("cost: launches not counted", [("launch_overhead_s * (len(n_g) + len(n_r))", "0.0")]),
    ("cost: host lane not part of the makespan", [("predicted = max(t_cpu, lane)", "predicted = lane")]),
    ("cost: lower bound prices one direction", [("lower = max(t_h2d, t_d2h)", "lower = t_h2d")]),
    ("brute force keeps the worst", [("if best is None or c < best:", "if best is None or c > best:")]),
]


@pytest.mark.parametrize("name,edits", PLAN_MUTANTS, ids=[m[0] for m in PLAN_MUTANTS])
def test_planted_mistake_in_the_planner_reference_is_caught(name, edits, tmp_path, monkeypatch):
    text = open(PLAN_SRC).read()
    for old, new in edits:
        assert text.count(old) >= 1, f"reference text changed: {old!r}"
        text = text.replace(old, new, 1)
    py = tmp_path / "plan_ref_mutant.py"
    py.write_text(text)
    spec = importlib.util.spec_from_file_location("plan_ref_mutant", str(py))
    mutant = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mutant)
    monkeypatch.setattr(plan_pins, "ref", mutant)
    failed = False
    for check in PLAN_PIN_CHECKS:
        try:
            check()
        except AssertionError:
            failed = True
            break
    assert failed, f"no pin noticed: {name}"


def test_unmodified_planner_reference_passes_every_pin():
    for check in PLAN_PIN_CHECKS:
        check()
