"""Pins for the scalar AdamW oracle (oracle/adamw_ref.c).

The paper prints no numeric example of an update (it cites Adam and names the
FP32 state and 16-bit gradients/parameters; Sections 1, 2, 4.1), so the oracle is
pinned to what the mathematics fixes: closed forms, an independent evaluation in
double of the textbook formulas in a different grouping, a library optimizer,
brute-force element independence and exhaustive checks of the bf16 helpers.
None of these tests touches the HIP library.
"""
import numpy as np
import pytest
import torch

from oracle import adamw_oracle as ref


def bf16_bits_of(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns of float32 values, via torch (library conversion)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16) \
        .view(torch.int16).numpy().view(np.uint16).copy()


def widen(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def fresh(n, seed, gscale=1e-3):
    rng = np.random.default_rng(seed)
    p = (0.02 * rng.standard_normal(n)).astype(np.float32)
    g = bf16_bits_of((gscale * rng.standard_normal(n)).astype(np.float32))
    return p, np.zeros(n, np.float32), np.zeros(n, np.float32), g, np.zeros(n, np.uint16)


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.max(np.abs(a - b) / np.maximum(np.abs(b), 1e-30))


def scaled_err(a, b):
    """max |a-b| / max |b|.  For m (a sum of terms of mixed sign) the rounding
    error of one FP32 step is half an ulp of the *terms*, so it does not shrink
    when the sum cancels: an element-wise relative error is not bounded by FP32
    epsilon, the error relative to the size of the array is."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.max(np.abs(a - b)) / np.max(np.abs(b))


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("wd", [0.0, 0.01, 0.3])
def test_first_step_is_sign_step(wd):
    """t=1, m=v=0, eps -> 0: m1/(sqrt(v1)/sqrt(1-b2)) = (1-b1) sign(g), so
    p1 = p0 (1 - lr wd) - lr sign(g)."""
    n, lr = 4096, 1e-2
    p, m, v, g, lp = fresh(n, 1)
    p0 = p.astype(np.float64)
    gf = widen(g).astype(np.float64)
    assert np.all(gf != 0)
    ref.adamw_step(p, m, v, g, lp, lr=lr, beta1=0.9, beta2=0.999, eps=1e-30, weight_decay=wd, step=1)
    lr32 = float(np.float32(lr))
    want = p0 * (1.0 - lr32 * float(np.float32(wd))) - lr32 * np.sign(gf)
    assert np.max(np.abs(p - want)) <= 4 * np.spacing(np.float32(np.max(np.abs(want))))
    # moments after one step from zero
    assert relerr(m, (1 - float(np.float32(0.9))) * gf) < 3e-7
    assert relerr(v, (1 - float(np.float32(0.999))) * gf * gf) < 3e-7


def test_zero_gradients_give_pure_decoupled_decay():
    n, T, lr, wd = 1000, 25, 1e-3, 0.1
    p, m, v, g, lp = fresh(n, 2)
    g[:] = 0
    p0 = p.astype(np.float64)
    for t in range(1, T + 1):
        ref.adamw_step(p, m, v, g, lp, lr=lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=wd, step=t)
        assert not m.any() and not v.any()
        want = p0 * (1.0 - float(np.float32(lr)) * float(np.float32(wd))) ** t
        assert relerr(p, want) < (t + 1) * 6e-8
    # the decay must be relative to p (decoupled), not a constant shift
    assert np.all(np.sign(p) == np.sign(p0))
    assert np.array_equal(lp, bf16_bits_of(p))


def test_negative_zero_and_zero_state_stay_finite():
    p = np.array([0.0, -0.0, 1.0], np.float32)
    m = np.zeros(3, np.float32); v = np.zeros(3, np.float32)
    g = np.zeros(3, np.uint16); lp = np.zeros(3, np.uint16)
    ref.adamw_step(p, m, v, g, lp, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1)
    assert np.all(np.isfinite(p)) and p[2] == 1.0 and p[0] == 0.0


@pytest.mark.parametrize("gval", [3e-3, -7e-4, 0.5])
def test_constant_gradient_recurrences(gval):
    """Constant g: m_t = g (1 - b1^t), v_t = g^2 (1 - b2^t); the bias-corrected
    ratio is g/|g|, so each step moves p by lr g / (|g| + eps) after the decay."""
    b1, b2, lr, eps, wd, T = 0.9, 0.999, 1e-3, 1e-8, 0.01, 40
    gb = bf16_bits_of(np.array([gval], np.float32))
    gd = float(widen(gb)[0])
    p = np.array([0.75], np.float32); m = np.zeros(1, np.float32); v = np.zeros(1, np.float32)
    lp = np.zeros(1, np.uint16)
    b1d, b2d, lrd, wdd, epsd = (float(np.float32(x)) for x in (b1, b2, lr, wd, eps))
    pd = 0.75
    for t in range(1, T + 1):
        ref.adamw_step(p, m, v, gb, lp, lr=lr, beta1=b1, beta2=b2, eps=eps, weight_decay=wd, step=t)
        assert abs(m[0] - gd * (1 - b1d ** t)) <= 1e-6 * abs(gd * (1 - b1d ** t))
        assert abs(v[0] - gd * gd * (1 - b2d ** t)) <= 1e-6 * gd * gd * (1 - b2d ** t)
        pd = pd * (1 - lrd * wdd) - lrd * gd / (abs(gd) + epsd)
        assert abs(p[0] - pd) <= 1e-6 * abs(pd)


# ------------------------------------------------- independent double evaluation

def textbook_adamw_f64(p, m, v, g, lr, b1, b2, eps, wd, t):
    """Kingma & Ba's update with explicit bias-corrected moments and additive
    decoupled decay, all in double: a different grouping from the oracle's."""
    m = b1 * m + (1 - b1) * g
    v = b2 * v + (1 - b2) * g * g
    mhat = m / (1 - b1 ** t)
    vhat = v / (1 - b2 ** t)
    p = p - lr * wd * p - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


@pytest.mark.parametrize("eps,wd,lr", [(1e-8, 0.01, 1e-4), (1e-3, 0.0, 1e-2), (1e-5, 0.2, 3e-3)])
def test_against_double_precision_textbook(eps, wd, lr):
    n, T = 64, 10
    rng = np.random.default_rng(7)
    p, m, v, _, lp = fresh(n, 3)
    f = lambda x: float(np.float32(x))
    pd, md, vd = p.astype(np.float64), m.astype(np.float64), v.astype(np.float64)
    for t in range(1, T + 1):
        g = bf16_bits_of((1e-3 * rng.standard_normal(n)).astype(np.float32))
        ref.adamw_step(p, m, v, g, lp, lr=lr, beta1=0.9, beta2=0.999, eps=eps, weight_decay=wd, step=t)
        pd, md, vd = textbook_adamw_f64(pd, md, vd, widen(g).astype(np.float64), f(lr), f(0.9),
                                        f(0.999), f(eps), f(wd), t)
        assert scaled_err(m, md) < 1e-6
        assert relerr(v, vd) < 1e-6
        # p: compare the step taken, relative to the size of p, to FP32 accuracy
        assert np.max(np.abs(p - pd)) < 1e-6 * np.max(np.abs(pd))
        # element-wise: a few FP32 ulps of max(|p|, lr) per step taken
        ulp = np.spacing(np.maximum(np.abs(pd), f(lr)).astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(p - pd) <= 2 * t * ulp)


def test_eps_sits_outside_the_root_and_is_not_bias_corrected():
    """With v = 0 after the step (g = 0, v = 0) and m != 0 the denominator is
    exactly eps: p moves by step_size * m1 / eps."""
    p = np.array([0.0], np.float32); m = np.array([1e-3], np.float32); v = np.zeros(1, np.float32)
    g = np.zeros(1, np.uint16); lp = np.zeros(1, np.uint16)
    ref.adamw_step(p, m, v, g, lp, lr=1e-3, beta1=0.5, beta2=0.5, eps=1e-2, weight_decay=0.0, step=3)
    m1 = 0.5 * float(np.float32(1e-3))
    want = -(float(np.float32(1e-3)) / (1 - 0.5 ** 3)) * m1 / float(np.float32(1e-2))
    assert abs(p[0] - want) < 1e-6 * abs(want)


# ----------------------------------------------------------- library optimizer

def test_against_torch_adamw():
    """torch.optim.AdamW takes its hyper-parameters as Python doubles; the oracle
    (like the C ABI) takes binary32.  With dyadic values both see the same
    numbers, so the two must agree to FP32 rounding."""
    n, T = 2048, 10
    hp = dict(lr=2.0 ** -13, beta1=0.875, beta2=1 - 2.0 ** -9, eps=2.0 ** -27, weight_decay=2.0 ** -7)
    rng = np.random.default_rng(11)
    p, m, v, _, lp = fresh(n, 5)
    tp = torch.nn.Parameter(torch.from_numpy(p.copy()))
    opt = torch.optim.AdamW([tp], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                            weight_decay=hp["weight_decay"], foreach=False, fused=False)
    for t in range(1, T + 1):
        g = bf16_bits_of((1e-3 * rng.standard_normal(n)).astype(np.float32))
        ref.adamw_step(p, m, v, g, lp, step=t, **hp)
        tp.grad = torch.from_numpy(widen(g).copy())
        opt.step()
        st = opt.state[tp]
        assert scaled_err(m, st["exp_avg"].numpy()) < 1e-6
        assert relerr(v, st["exp_avg_sq"].numpy()) < 1e-6
        tpn = tp.detach().numpy().astype(np.float64)
        ulp = np.spacing(np.maximum(np.abs(tpn), hp["lr"]).astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(p - tpn) <= 2 * t * ulp)
    assert np.array_equal(lp, bf16_bits_of(p))


# -------------------------------------------------------- element independence

def test_elements_are_independent_brute_force():
    n = 257
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    p, m, v, g, lp = fresh(n, 9)
    rng = np.random.default_rng(9)
    m[:] = (1e-3 * rng.standard_normal(n)).astype(np.float32)
    v[:] = (1e-6 * rng.random(n)).astype(np.float32)
    whole = [x.copy() for x in (p, m, v, lp)]
    ref.adamw_step(*whole[:3], g, whole[3], step=4, **hp)
    # one element at a time
    for i in range(n):
        one = [x[i:i + 1].copy() for x in (p, m, v, lp)]
        ref.adamw_step(*one[:3], g[i:i + 1].copy(), one[3], step=4, **hp)
        for w, o in zip(whole, one):
            assert w[i:i + 1].tobytes() == o.tobytes()
    # permuted copy
    perm = rng.permutation(n)
    per = [x[perm].copy() for x in (p, m, v, lp)]
    ref.adamw_step(*per[:3], g[perm].copy(), per[3], step=4, **hp)
    for w, o in zip(whole, per):
        assert w[perm].tobytes() == o.tobytes()


def test_parallel_loop_is_bit_identical_to_scalar_loop():
    n = 100_003
    hp = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    a = fresh(n, 21)
    b = [x.copy() for x in a]
    for t in (1, 2, 3):
        ref.adamw_step(*a, step=t, threads=1, **hp)
        used = ref.adamw_step(*b, step=t, threads=4, **hp)
        assert used >= 1
    for x, y in zip(a, b):
        assert x.tobytes() == y.tobytes()


# ------------------------------------------------------------------ scalars

def test_step_scalars_match_their_definitions():
    for t in (1, 2, 10, 1000, 100000):
        s = ref.scalars(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=t)
        b1, b2, lr, wd = (float(np.float32(x)) for x in (0.9, 0.999, 1e-4, 0.01))
        assert abs(s["step_size"] * (1 - b1 ** t) / lr - 1) < 2e-7
        assert abs(s["inv_sqrt_bc2"] ** 2 * (1 - b2 ** t) - 1) < 4e-7
        assert abs(float(s["decay"]) - (1 - lr * wd)) < 6e-8
        assert float(s["omb1"]) == float(np.float32(1) - np.float32(0.9))
        assert float(s["omb2"]) == float(np.float32(1) - np.float32(0.999))


def test_rejects_undefined_arguments():
    a = fresh(4, 1)
    ok = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1)
    for bad in (dict(step=0), dict(step=-3), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1e-8)):
        before = [x.copy() for x in a]
        with pytest.raises(ValueError):
            ref.adamw_step(*a, **{**ok, **bad})
        for x, y in zip(a, before):
            assert x.tobytes() == y.tobytes()


# ------------------------------------------------------------------ bf16 helpers

def test_bf16_widening_is_exact_and_roundtrips_exhaustively():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = ref.bf16_to_f32(bits)
    assert np.array_equal(f.view(np.uint32), bits.astype(np.uint32) << 16)
    back = ref.f32_to_bf16(f)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], bits[~nan])
    # NaN stays NaN, sign kept, quiet bit set
    assert np.all((back[nan] & 0x7F80) == 0x7F80) and np.all(back[nan] & 0x0040)
    assert np.array_equal(back[nan] & 0x8000, bits[nan] & 0x8000)


def test_bf16_rounding_hand_built_cases():
    def one(u32):
        return int(ref.f32_to_bf16(np.array([u32], np.uint32).view(np.float32))[0])
    assert one(0x3F808000) == 0x3F80          # tie, even keeps
    assert one(0x3F818000) == 0x3F82          # tie, odd rounds up
    assert one(0x3F808001) == 0x3F81          # just above the tie
    assert one(0x3F807FFF) == 0x3F80          # just below the tie
    assert one(0x7F7FFFFF) == 0x7F80          # largest float32 -> +inf
    assert one(0xFF7FFFFF) == 0xFF80
    assert one(0x7F800000) == 0x7F80 and one(0xFF800000) == 0xFF80
    assert one(0x00000000) == 0x0000 and one(0x80000000) == 0x8000
    assert one(0x00008000) == 0x0000          # denormal tie to even (zero)
    assert one(0x00018000) == 0x0002          # denormal tie, odd -> up
    assert one(0x007FFFFF) == 0x0080          # largest denormal -> smallest normal
    assert one(0x7FC00001) & 0x7FC0 == 0x7FC0 and one(0x7F800001) & 0x7FC0 == 0x7FC0


def test_bf16_rounding_is_nearest_value_with_even_ties():
    """Value-based check: among the two neighbouring bf16 values the result is
    the nearer one in exact (double) arithmetic; at equal distance the one with
    an even last bit."""
    rng = np.random.default_rng(5)
    u = rng.integers(0, 1 << 32, size=200_000, dtype=np.uint64).astype(np.uint32)
    ties = (rng.integers(0, 1 << 16, size=50_000, dtype=np.uint64).astype(np.uint32) << 16) | 0x8000
    u = np.concatenate([u, ties, ties + 1, ties - 1])
    x = u.view(np.float32)
    fin = np.isfinite(x)
    u, x = u[fin], x[fin]
    got = ref.f32_to_bf16(x)
    lo = (u >> 16).astype(np.uint16)                       # truncation toward zero
    hi = (lo + 1).astype(np.uint16)                        # next bf16 away from zero
    xl = widen(lo).astype(np.float64); xh = widen(hi).astype(np.float64)
    xd = x.astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        # past the largest finite bf16 the upper neighbour counts as 2^128
        xh = np.where(np.isinf(xh), np.sign(xh) * 2.0 ** 128, xh)
        dl, dh = np.abs(xd - xl), np.abs(xh - xd)
    want = np.where(dl < dh, lo, np.where(dh < dl, hi, np.where(lo & 1, hi, lo))).astype(np.uint16)
    assert np.array_equal(got, want)


def test_bf16_rounding_matches_torch_conversion():
    rng = np.random.default_rng(6)
    u = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    x = u.view(np.float32)
    x = x[~np.isnan(x)]
    assert np.array_equal(ref.f32_to_bf16(x), bf16_bits_of(x))
