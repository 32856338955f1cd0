"""Pins for the Adagrad and RMSProp references at the end of oracle/adamw_ref.c.

Section 4.1 of the paper names Adam, Adagrad and RMSProp as the adaptive
optimizers whose per-element independence the interleaving relies on and prints
no equations for any of them, so these are pinned like the AdamW reference: to
closed forms, to an independent evaluation in double with a different grouping,
to torch's optimizers, and to brute-force element independence.  None of these
tests touches the HIP library.
"""
import numpy as np
import pytest
import torch

from oracle import adamw_oracle as ref

from test_oracle_pins import bf16_bits_of, fresh, relerr, widen

f32 = lambda x: float(np.float32(x))


def step(name, p, v, g, lp, **hp):
    if name == "adagrad":
        hp.pop("alpha", None)
        return ref.adagrad_step(p, v, g, lp, **hp)
    return ref.rmsprop_step(p, v, g, lp, **hp)


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("wd", [0.0, 0.3])
def test_adagrad_first_step_is_sign_step(wd):
    """v = 0, eps -> 0: v1 = g^2 and p1 = p0 (1 - lr wd) - lr g/|g|."""
    n, lr = 4096, 1e-2
    p, _, v, g, lp = fresh(n, 31)
    p0, gf = p.astype(np.float64), widen(g).astype(np.float64)
    assert np.all(gf != 0)
    ref.adagrad_step(p, v, g, lp, lr=lr, eps=1e-30, weight_decay=wd)
    want = p0 * (1.0 - f32(lr) * f32(wd)) - f32(lr) * np.sign(gf)
    assert np.max(np.abs(p - want)) <= 4 * np.spacing(np.float32(np.max(np.abs(want))))
    assert relerr(v, gf * gf) < 1e-7
    assert np.array_equal(lp, bf16_bits_of(p))


@pytest.mark.parametrize("wd", [0.0, 0.3])
def test_rmsprop_first_step_is_scaled_sign_step(wd):
    """v = 0, eps -> 0: v1 = (1-alpha) g^2 and the step is lr sign(g) / sqrt(1-alpha)."""
    n, lr, alpha = 4096, 1e-2, 0.75
    p, _, v, g, lp = fresh(n, 32)
    p0, gf = p.astype(np.float64), widen(g).astype(np.float64)
    ref.rmsprop_step(p, v, g, lp, lr=lr, alpha=alpha, eps=1e-30, weight_decay=wd)
    want = p0 * (1.0 - f32(lr) * f32(wd)) - f32(lr) * np.sign(gf) / np.sqrt(1.0 - alpha)
    assert np.max(np.abs(p - want)) <= 4 * np.spacing(np.float32(np.max(np.abs(want))))
    assert relerr(v, (1.0 - alpha) * gf * gf) < 2e-7
    assert np.array_equal(lp, bf16_bits_of(p))


@pytest.mark.parametrize("gval", [3e-3, -7e-4, 0.5])
def test_adagrad_constant_gradient(gval):
    """Constant g: v_T = T g^2, so step t moves p by lr g / (sqrt(t) |g| + eps)."""
    lr, eps, wd, T = 1e-3, 1e-10, 0.01, 40
    gb = bf16_bits_of(np.array([gval], np.float32))
    gd = float(widen(gb)[0])
    p = np.array([0.75], np.float32); v = np.zeros(1, np.float32); lp = np.zeros(1, np.uint16)
    pd = 0.75
    for t in range(1, T + 1):
        ref.adagrad_step(p, v, gb, lp, lr=lr, eps=eps, weight_decay=wd)
        assert abs(v[0] - t * gd * gd) <= 1e-6 * t * gd * gd
        pd = pd * (1 - f32(lr) * f32(wd)) - f32(lr) * gd / (np.sqrt(t) * abs(gd) + f32(eps))
        assert abs(p[0] - pd) <= 1e-6 * abs(pd)
    # without decay the distance travelled is lr * sum 1/sqrt(t)
    p = np.array([0.0], np.float32); v = np.zeros(1, np.float32)
    for t in range(1, T + 1):
        ref.adagrad_step(p, v, gb, lp, lr=lr, eps=0.0, weight_decay=0.0)
    want = -np.sign(gd) * f32(lr) * sum(1.0 / np.sqrt(t) for t in range(1, T + 1))
    assert abs(p[0] - want) <= 1e-5 * abs(want)


@pytest.mark.parametrize("gval", [3e-3, -7e-4, 0.5])
def test_rmsprop_constant_gradient(gval):
    """Constant g: v_t = g^2 (1 - alpha^t), so step t moves p by lr g / (|g| sqrt(1-alpha^t) + eps)."""
    lr, alpha, eps, wd, T = 1e-3, 0.99, 1e-10, 0.01, 40
    gb = bf16_bits_of(np.array([gval], np.float32))
    gd = float(widen(gb)[0])
    a = f32(alpha)
    p = np.array([0.75], np.float32); v = np.zeros(1, np.float32); lp = np.zeros(1, np.uint16)
    pd = 0.75
    for t in range(1, T + 1):
        ref.rmsprop_step(p, v, gb, lp, lr=lr, alpha=alpha, eps=eps, weight_decay=wd)
        assert abs(v[0] - gd * gd * (1 - a ** t)) <= 2e-6 * gd * gd * (1 - a ** t)
        pd = pd * (1 - f32(lr) * f32(wd)) - f32(lr) * gd / (abs(gd) * np.sqrt(1 - a ** t) + f32(eps))
        assert abs(p[0] - pd) <= 2e-6 * abs(pd)


@pytest.mark.parametrize("name", ["adagrad", "rmsprop"])
def test_zero_gradients_give_pure_decoupled_decay(name):
    """g = 0: Adagrad's accumulator stays, RMSProp's decays geometrically, and p
    only decays, in proportion to itself (also from v = 0, where 0/eps = 0)."""
    n, T, lr, wd, alpha = 1000, 25, 1e-3, 0.1, 0.9
    for v0 in (0.0, 4e-6):
        p, _, v, g, lp = fresh(n, 33)
        g[:] = 0
        v[:] = v0
        p0 = p.astype(np.float64)
        for t in range(1, T + 1):
            step(name, p, v, g, lp, lr=lr, alpha=alpha, eps=1e-8, weight_decay=wd)
            want_v = f32(v0) if name == "adagrad" else f32(v0) * f32(alpha) ** t
            assert relerr(v, np.full(n, want_v)) < (t + 1) * 6e-8 if v0 else not v.any()
            assert relerr(p, p0 * (1.0 - f32(lr) * f32(wd)) ** t) < (t + 1) * 6e-8


@pytest.mark.parametrize("name", ["adagrad", "rmsprop"])
def test_eps_sits_outside_the_root(name):
    """With eps far above sqrt(v) the step is lr g / eps, not lr g / sqrt(eps)."""
    gb = bf16_bits_of(np.array([2.0 ** -20], np.float32))
    p = np.zeros(1, np.float32); v = np.zeros(1, np.float32); lp = np.zeros(1, np.uint16)
    step(name, p, v, gb, lp, lr=2.0 ** -3, alpha=0.5, eps=2.0 ** -4, weight_decay=0.0)
    root = 2.0 ** -20 if name == "adagrad" else 2.0 ** -20 * np.sqrt(0.5)
    want = -(2.0 ** -3) * 2.0 ** -20 / (root + 2.0 ** -4)
    assert abs(p[0] - want) < 1e-6 * abs(want)


# ------------------------------------------------- independent double evaluation

def textbook_f64(name, p, v, g, lr, alpha, eps, wd):
    """The rules in double with additive decay and the step formed as
    (lr / denominator) * g: a different grouping from the reference's."""
    v = v + g * g if name == "adagrad" else v + (1 - alpha) * (g * g - v)
    p = p - lr * wd * p - (lr / (np.sqrt(v) + eps)) * g
    return p, v


@pytest.mark.parametrize("name", ["adagrad", "rmsprop"])
@pytest.mark.parametrize("eps,wd,lr", [(1e-8, 0.01, 1e-4), (1e-3, 0.0, 1e-2), (1e-5, 0.2, 3e-3)])
def test_against_double_precision_textbook(name, eps, wd, lr):
    n, T, alpha = 64, 10, 0.99
    rng = np.random.default_rng(37)
    p, _, v, _, lp = fresh(n, 34)
    pd, vd = p.astype(np.float64), v.astype(np.float64)
    size = np.full(n, f32(lr))
    for t in range(1, T + 1):
        g = bf16_bits_of((1e-3 * rng.standard_normal(n)).astype(np.float32))
        step(name, p, v, g, lp, lr=lr, alpha=alpha, eps=eps, weight_decay=wd)
        before = pd
        pd, vd = textbook_f64(name, pd, vd, widen(g).astype(np.float64), f32(lr), f32(alpha), f32(eps), f32(wd))
        assert relerr(v, vd) < 1e-6
        assert np.max(np.abs(p - pd)) < 1e-6 * np.max(np.abs(pd))
        # element-wise: each step rounds the decayed p, the quotient, the step and the difference once, so
        # it adds a few FP32 ulps of the larger of |p| and the step taken (RMSProp's first steps are
        # lr / sqrt(1 - alpha), ten times lr here); errors of earlier steps stay, so the size is the
        # largest seen so far
        size = np.maximum(size, np.maximum(np.abs(pd), np.abs(pd - before)))
        ulp = np.spacing(size.astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(p - pd) <= 3 * t * ulp)
        assert np.array_equal(lp, bf16_bits_of(p))


# ----------------------------------------------------------- library optimizers

@pytest.mark.parametrize("name", ["adagrad", "rmsprop"])
def test_against_torch(name):
    """torch.optim.Adagrad / RMSprop (no momentum, not centred, no weight decay:
    torch's is the coupled kind) with dyadic hyper-parameters, which are the same
    numbers in binary32 and in double."""
    n, T = 2048, 10
    lr, alpha, eps = 2.0 ** -9, 1 - 2.0 ** -6, 2.0 ** -27
    rng = np.random.default_rng(41)
    p, _, v, _, lp = fresh(n, 35)
    tp = torch.nn.Parameter(torch.from_numpy(p.copy()))
    if name == "adagrad":
        opt = torch.optim.Adagrad([tp], lr=lr, lr_decay=0, weight_decay=0, initial_accumulator_value=0, eps=eps,
                                  foreach=False)
        key = "sum"
    else:
        opt = torch.optim.RMSprop([tp], lr=lr, alpha=alpha, eps=eps, weight_decay=0, momentum=0, centered=False,
                                  foreach=False)
        key = "square_avg"
    size = np.full(n, lr)
    for t in range(1, T + 1):
        g = bf16_bits_of((1e-3 * rng.standard_normal(n)).astype(np.float32))
        before = tp.detach().numpy().astype(np.float64)
        step(name, p, v, g, lp, lr=lr, alpha=alpha, eps=eps, weight_decay=0.0)
        tp.grad = torch.from_numpy(widen(g).copy())
        opt.step()
        assert relerr(v, opt.state[tp][key].numpy()) < 1e-6
        tpn = tp.detach().numpy().astype(np.float64)
        # both sides round a handful of FP32 operations per step: a few ulps of the larger of |p| and
        # the step taken, accumulated over the steps so far
        size = np.maximum(size, np.maximum(np.abs(tpn), np.abs(tpn - before)))
        ulp = np.spacing(size.astype(np.float32)).astype(np.float64)
        assert np.all(np.abs(p - tpn) <= 3 * t * ulp)
    assert np.array_equal(lp, bf16_bits_of(p))


# -------------------------------------------------------- element independence

@pytest.mark.parametrize("name", ["adagrad", "rmsprop"])
def test_elements_are_independent_and_loops_agree(name):
    n = 257
    hp = dict(lr=1e-3, alpha=0.99, eps=1e-8, weight_decay=0.01)
    p, _, v, g, lp = fresh(n, 36)
    rng = np.random.default_rng(36)
    v[:] = (1e-6 * rng.random(n)).astype(np.float32)
    whole = [x.copy() for x in (p, v, lp)]
    step(name, whole[0], whole[1], g, whole[2], **hp)
    for i in range(n):
        one = [x[i:i + 1].copy() for x in (p, v, lp)]
        step(name, one[0], one[1], g[i:i + 1].copy(), one[2], **hp)
        for w, o in zip(whole, one):
            assert w[i:i + 1].tobytes() == o.tobytes()
    perm = rng.permutation(n)
    per = [x[perm].copy() for x in (p, v, lp)]
    step(name, per[0], per[1], g[perm].copy(), per[2], **hp)
    for w, o in zip(whole, per):
        assert w[perm].tobytes() == o.tobytes()
    # the parallel-for is the same loop body
    par = [x.copy() for x in (p, v, lp)]
    assert step(name, par[0], par[1], g, par[2], threads=4, **hp) >= 1
    for w, o in zip(whole, par):
        assert w.tobytes() == o.tobytes()


def test_optimizer_step_dispatch_and_rejections():
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.01, step=3)
    p, m, v, g, lp = fresh(100, 38)
    for name in ("adagrad", "rmsprop"):
        a = [x.copy() for x in (p, m, v, lp)]
        b = [x.copy() for x in (p, v, lp)]
        ref.optimizer_step(name, a[0], a[1], a[2], g, a[3], **hp)
        step(name, b[0], b[1], g, b[2], lr=1e-3, alpha=0.99, eps=1e-8, weight_decay=0.01)
        assert a[0].tobytes() == b[0].tobytes() and a[2].tobytes() == b[1].tobytes() and not a[1].any()
    a = [x.copy() for x in (p, m, v, lp)]
    b = [x.copy() for x in (p, m, v, lp)]
    ref.optimizer_step("adamw", a[0], a[1], a[2], g, a[3], **hp)
    ref.adamw_step(b[0], b[1], b[2], g, b[3], **hp)
    assert all(x.tobytes() == y.tobytes() for x, y in zip(a, b))
    with pytest.raises(ValueError):
        ref.adagrad_step(p, v, g, lp, lr=1e-3, eps=-1.0, weight_decay=0.0)
    with pytest.raises(ValueError):
        ref.rmsprop_step(p, v, g, lp, lr=1e-3, alpha=1.0, eps=1e-8, weight_decay=0.0)
    with pytest.raises(ValueError):
        ref.optimizer_step("sgd", p, m, v, g, lp, **hp)
