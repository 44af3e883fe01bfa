"""Pins for the CPU oracle: everything here checks oracle/ against something other than itself.

  - hand-worked exact-rational examples (tests/golden/worked_examples.txt);
  - torch.optim's SGD / Adam / AdamW run in fp64 on the CPU: an independent library routine that
    Alg. 1 (tau-damped momentum with a pre-existing buffer) and App. A's SGD / Adam / AdamW (alpha = 1)
    reduce to;
  - closed forms and symmetries of the update lines;
  - round trips undo(step(s)) = s: bit-exact where every operation is exact in binary64
    (dyadic hyper-parameters), ~1e-13 otherwise;
  - the digest against stored vectors, an explicit inverse of its mixer, and shard invariants.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from oracle import Hyper
from golden_io import read_worked_examples, read_digest_vectors

F64 = np.float64


def _close(a, b, rtol=1e-13, atol=1e-300):
    a, b = np.asarray(a, F64), np.asarray(b, F64)
    assert a.shape == b.shape
    bad = np.abs(a - b) > np.maximum(rtol * np.abs(b), atol)
    assert not bad.any(), f"mismatch at {np.nonzero(bad)[0][:5]}: {a[bad][:5]} vs {b[bad][:5]}"


# --------------------------------------------------------------------------- worked examples
@pytest.mark.parametrize("case", read_worked_examples(), ids=lambda c: c["name"])
def test_worked_example_step_and_undo(case):
    hp = Hyper(kind=case["kind"], eta=float(case["eta"]), lam=float(case["lam"]),
               mu=float(case.get("mu", 0)), tau=float(case.get("tau", 0)),
               beta1=float(case.get("beta1", 0.9)), beta2=float(case.get("beta2", 0.999)),
               eps=float(case.get("eps", 0)), t=int(case.get("t", 1)))
    f = lambda k: None if k not in case else np.array([float(q) for q in case[k]], F64)
    x, g, m, v = f("x"), f("g"), f("m"), f("v")
    if case["kind"] == "lamb":
        xn, mn, vn, norms = oracle.lamb_step(hp, x, g, m, v)
        _close(norms, f("norms"), rtol=4e-16)
        _close(xn, f("x_new"), rtol=4e-16, atol=1e-16)
        _close(mn, f("m_new"), rtol=4e-16)
        _close(vn, f("v_new"), rtol=4e-16)
        xo, mo, vo = oracle.lamb_undo(hp, f("x_new"), g, f("m_new"), f("v_new"), f("norms"))
        _close(xo, x, rtol=1e-15, atol=1e-15)
        _close(mo, m, rtol=1e-15, atol=1e-15)
        _close(vo, v, rtol=1e-15, atol=1e-15)
        return
    xn, mn, vn = oracle.opt_step(hp, x, g, m, v)
    _close(xn, f("x_new"), rtol=4e-16, atol=1e-16)
    if m is not None:
        _close(mn, f("m_new"), rtol=4e-16, atol=1e-16)
    else:
        assert mn is None and vn is None          # App. A's plain SGD keeps no state
    if v is not None:
        _close(vn, f("v_new"), rtol=4e-16, atol=1e-16)
    # undo from the stored (not the computed) new state
    xo, mo, vo = oracle.opt_undo(hp, f("x_new"), g, f("m_new"), f("v_new"))
    _close(xo, x, rtol=1e-15, atol=1e-15)
    if m is not None:
        _close(mo, m, rtol=1e-15, atol=1e-15)
    if v is not None:
        _close(vo, v, rtol=1e-15, atol=1e-15)


# --------------------------------------------------------------------------- torch.optim (fp64)
def _rand_state(seed, n=257):
    r = np.random.default_rng(seed)
    x = r.normal(0, 0.02, n)
    g = r.normal(0, 1e-3, n)
    m = r.normal(0, 1e-4, n)
    v = np.abs(r.normal(0, 1e-6, n))
    g[::7] = 0.0
    g[3::31] *= 1e3
    return x, g, m, v


@pytest.mark.parametrize("mu,tau,lam", [(0.9, 0.0, 1e-4), (0.5, 0.25, 0.1), (0.0, 0.0, 0.01), (0.9, 0.5, 0.0)])
def test_sgdm_step_matches_torch_sgd(mu, tau, lam):
    x, g, m, _ = _rand_state(1)
    p = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    p.grad = torch.tensor(g, dtype=torch.float64)
    opt = torch.optim.SGD([p], lr=0.1, momentum=mu, dampening=tau, weight_decay=lam, foreach=False)
    if mu != 0.0:
        # a pre-existing buffer makes torch apply the damped recurrence of Alg. 1 from the start
        opt.state[p]["momentum_buffer"] = torch.tensor(m, dtype=torch.float64)
    opt.step()
    xn, mn, _ = oracle.opt_step(Hyper("sgdm", eta=0.1, lam=lam, mu=mu, tau=tau), x, g, m)
    _close(xn, p.detach().numpy(), rtol=1e-14, atol=1e-18)
    if mu != 0.0:
        _close(mn, opt.state[p]["momentum_buffer"].numpy(), rtol=1e-14, atol=1e-20)
    else:
        # App. A's plain SGD: x_new = x - eta (g + lam x); the oracle keeps (1-tau) g' in m
        _close(xn, x - 0.1 * (g + lam * x), rtol=1e-14, atol=1e-18)
        _close(mn, (1 - tau) * (g + lam * x), rtol=1e-14, atol=1e-20)


@pytest.mark.parametrize("kind,lam,t,betas", [
    ("adam", 0.0, 1000, (0.9, 0.999)), ("adam", 0.01, 7, (0.9, 0.999)), ("adam", 0.1, 1, (0.5, 0.75)),
    ("adamw", 0.01, 10000, (0.9, 0.999)), ("adamw", 0.1, 3, (0.9, 0.95)), ("adamw", 0.0, 50000, (0.9, 0.95))])
def test_adam_step_matches_torch(kind, lam, t, betas):
    x, g, m, v = _rand_state(2)
    p = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    p.grad = torch.tensor(g, dtype=torch.float64)
    cls = torch.optim.Adam if kind == "adam" else torch.optim.AdamW
    opt = cls([p], lr=1e-3, betas=betas, eps=1e-8, weight_decay=lam, foreach=False, fused=False,
              capturable=False, amsgrad=False)
    opt.state[p]["step"] = torch.tensor(float(t - 1))
    opt.state[p]["exp_avg"] = torch.tensor(m, dtype=torch.float64)
    opt.state[p]["exp_avg_sq"] = torch.tensor(v, dtype=torch.float64)
    opt.step()
    hp = Hyper(kind, eta=1e-3, lam=lam, beta1=betas[0], beta2=betas[1], eps=1e-8, t=t)
    xn, mn, vn = oracle.opt_step(hp, x, g, m, v)
    # torch forms m by lerp, m + (1-beta1)(g' - m): a different rounding order, so where the two
    # terms cancel the results differ by a few ulps of the larger term
    _close(mn, opt.state[p]["exp_avg"].numpy(), rtol=1e-14, atol=4e-16 * np.abs(mn).max())
    _close(vn, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-14, atol=4e-16 * np.abs(vn).max())
    # torch folds the bias corrections differently (sqrt(v)/sqrt(bc2), lr/bc1): a few ulps apart
    _close(xn, p.detach().numpy(), rtol=1e-13, atol=1e-18)


# --------------------------------------------------------------------------- closed forms
def test_first_adam_step_is_sign_like():
    # m = v = 0, lam = 0, t = 1: m^ = g, v^ = g^2, so x_new = x - eta g / (|g| + eps) for any betas
    x, g, _, _ = _rand_state(3)
    z = np.zeros_like(x)
    for kind in ("adam", "adamw"):
        for b1, b2 in ((0.9, 0.999), (0.5, 0.75), (0.1, 0.3)):
            xn, mn, vn = oracle.opt_step(Hyper(kind, eta=0.01, lam=0.0, beta1=b1, beta2=b2, eps=1e-8, t=1), x, g, z, z)
            _close(xn, x - 0.01 * g / (np.abs(g) + 1e-8), rtol=1e-12, atol=1e-16)
            _close(mn, (1 - b1) * g, rtol=1e-15)
            _close(vn, (1 - b2) * g * g, rtol=1e-15)


def test_adamw_zero_grad_zero_moment_is_pure_decay():
    x, _, _, v = _rand_state(4)
    z = np.zeros_like(x)
    xn, mn, vn = oracle.opt_step(Hyper("adamw", eta=0.25, lam=0.5, t=9), x, z, z, v)
    _close(xn, (1 - 0.25 * 0.5) * x, rtol=1e-15)
    assert not mn.any()
    _close(vn, 0.999 * v, rtol=1e-15)
    # coupled Adam with the same inputs is NOT a pure decay: g' = lam x feeds the moments
    xa, ma, _ = oracle.opt_step(Hyper("adam", eta=0.25, lam=0.5, t=9), x, z, z, v)
    _close(ma, 0.1 * 0.5 * x, rtol=1e-14)
    assert np.abs(xa - xn).max() > 1e-3


def test_sgdm_zero_learning_rate_moves_only_the_buffer():
    x, g, m, _ = _rand_state(5)
    hp = Hyper("sgdm", eta=0.0, lam=0.01, mu=0.9, tau=0.1)
    xn, mn, _ = oracle.opt_step(hp, x, g, m)
    assert np.array_equal(xn, x)
    _close(mn, 0.9 * m + 0.9 * (g + 0.01 * x), rtol=1e-15, atol=1e-22)
    xo, mo, _ = oracle.opt_undo(hp, xn, g, mn)
    assert np.array_equal(xo, x)
    _close(mo, m, rtol=1e-12, atol=1e-15 * np.abs(mn).max())


def test_adam_fixed_point_of_moments():
    # m = g and v = g^2 (lam = 0) are reproduced by the two recurrences
    _, g, _, _ = _rand_state(6)
    x = np.ones_like(g)
    for kind in ("adam", "adamw"):
        _, mn, vn = oracle.opt_step(Hyper(kind, eta=1e-3, lam=0.0, t=5), x, g, g, g * g)
        _close(mn, g, rtol=1e-15, atol=1e-300)
        _close(vn, g * g, rtol=1e-15, atol=1e-300)


@pytest.mark.parametrize("kind", ["sgdm", "adam", "adamw"])
def test_odd_symmetry(kind):
    # negating (x, g, m) negates (x_new, m_new) and leaves v_new: bit-exact, IEEE negation is exact
    x, g, m, v = _rand_state(7)
    hp = Hyper(kind, eta=0.01, lam=0.05, mu=0.9, tau=0.1, t=11)
    vv = None if kind == "sgdm" else v
    a = oracle.opt_step(hp, x, g, m, vv)
    b = oracle.opt_step(hp, -x, -g, -m, vv)
    assert np.array_equal(a[0], -b[0]) and np.array_equal(a[1], -b[1])
    if vv is not None:
        assert np.array_equal(a[2], b[2])
    a = oracle.opt_undo(hp, x, g, m, vv)
    b = oracle.opt_undo(hp, -x, -g, -m, vv)
    assert np.array_equal(a[0], -b[0]) and np.array_equal(a[1], -b[1])
    if vv is not None:
        assert np.array_equal(a[2], b[2])


@pytest.mark.parametrize("kind", ["adam", "adamw"])
def test_scale_invariance_without_eps(kind):
    # eps = 0, lam = 0: g -> c g, m -> c m, v -> c^2 v leaves the parameter update unchanged;
    # c a power of two makes the scaling exact, so the results agree bit for bit
    x, g, m, v = _rand_state(8)
    v = v + 1e-12
    hp = Hyper(kind, eta=1e-3, lam=0.0, eps=0.0, t=4)
    a = oracle.opt_step(hp, x, g, m, v)
    b = oracle.opt_step(hp, x, 8 * g, 8 * m, 64 * v)
    assert np.array_equal(a[0], b[0])
    assert np.array_equal(8 * a[1], b[1]) and np.array_equal(64 * a[2], b[2])


def test_bias_correction_uses_t():
    # t enters only through 1 - beta^t; compare with a scalar evaluation at two different t
    x, g, m, v = (np.array([0.3]), np.array([-0.2]), np.array([0.05]), np.array([0.01]))
    for t in (1, 2, 10):
        xn, mn, vn = oracle.opt_step(Hyper("adam", eta=0.1, lam=0.0, beta1=0.5, beta2=0.25, eps=0.0, t=t), x, g, m, v)
        mt = 0.5 * 0.05 + 0.5 * -0.2
        vt = 0.25 * 0.01 + 0.75 * 0.04
        want = 0.3 - 0.1 * (mt / (1 - 0.5 ** t)) / np.sqrt(vt / (1 - 0.25 ** t))
        _close(xn, [want], rtol=1e-15)


# --------------------------------------------------------------------------- round trips
_DYADIC = [0.0, 0.5, -0.5, 1.0, -1.0, 0.375, -2.25, 3.0]


def test_sgdm_round_trip_is_bit_exact_on_dyadic_grid():
    # eta = 1/8, lam = 1/4, mu = 1/2, tau = 1/4 and dyadic inputs: every product, sum and the
    # division by mu is exact in binary64, so Alg. 2 must return the inputs of Alg. 1 exactly
    grid = np.array(list(itertools.product(_DYADIC, repeat=3)), F64)
    x, g, m = (np.ascontiguousarray(grid[:, k]) for k in range(3))
    hp = Hyper("sgdm", eta=0.125, lam=0.25, mu=0.5, tau=0.25)
    xn, mn, _ = oracle.opt_step(hp, x, g, m)
    # exact forward values too
    assert np.array_equal(mn, 0.5 * m + 0.75 * (g + 0.25 * x))
    assert np.array_equal(xn, x - 0.125 * mn)
    xo, mo, _ = oracle.opt_undo(hp, xn, g, mn)
    assert np.array_equal(xo, x) and np.array_equal(mo, m)
    # the undo must feed the *recovered* x into the decay term: with x_new instead, m would be off
    wrong = (mn - 0.75 * (g + 0.25 * xn)) / 0.5
    assert not np.array_equal(wrong, m)


@pytest.mark.parametrize("kind", ["adam", "adamw"])
def test_adam_round_trip_moments_bit_exact_on_dyadic_grid(kind):
    # beta1 = 1/2, beta2 = 3/4, lam = 1/4 (adamw: eta*lam = 1/32) and dyadic inputs: the moment
    # recurrences and their inverses are exact; only x passes through sqrt and a division
    vals_v = [0.0, 0.25, 1.0, 2.5]
    grid = np.array(list(itertools.product(_DYADIC, _DYADIC, _DYADIC[:6], vals_v)), F64)
    x, g, m, v = (np.ascontiguousarray(grid[:, k]) for k in range(4))
    hp = Hyper(kind, eta=0.125, lam=0.25, beta1=0.5, beta2=0.75, eps=2.0 ** -20, t=3)
    xn, mn, vn = oracle.opt_step(hp, x, g, m, v)
    xo, mo, vo = oracle.opt_undo(hp, xn, g, mn, vn)
    _close(xo, x, rtol=1e-15, atol=1e-15)
    if kind == "adamw":
        assert np.array_equal(mo, m) and np.array_equal(vo, v)
    else:
        # g' = g + lam x_old is rebuilt from the recovered x (a few ulps off), so m, v follow to ~1e-15
        _close(mo, m, rtol=1e-14, atol=1e-14)
        _close(vo, v, rtol=1e-14, atol=1e-13)
        # and it must be the recovered x, not x_new, that enters g'
        gp_wrong = g + 0.25 * xn
        wrong = (mn - 0.5 * gp_wrong) / 0.5
        assert np.abs(wrong - m).max() > 1e-3


@pytest.mark.parametrize("kind,lam", [("sgdm", 1e-4), ("adam", 0.01), ("adamw", 0.1)])
def test_round_trip_random_fp64(kind, lam):
    x, g, m, v = _rand_state(9, n=4099)
    vv = None if kind == "sgdm" else v
    hp = Hyper(kind, eta=1e-3 if kind != "sgdm" else 0.1, lam=lam, mu=0.9, tau=0.0, t=1000)
    new = oracle.opt_step(hp, x, g, m, vv)
    old = oracle.opt_undo(hp, new[0], g, new[1], new[2])
    _close(old[0], x, rtol=1e-13, atol=1e-17)
    # the inverse recurrences cancel: absolute error scales with the new moment, not the old one
    _close(old[1], m, rtol=1e-12, atol=1e-15 * np.abs(new[1]).max())
    if vv is not None:
        _close(old[2], v, rtol=1e-12, atol=1e-15 * np.abs(new[2]).max())


@pytest.mark.parametrize("kind", ["adam", "adamw"])
def test_zero_grad_moments_return_to_fp32_originals(kind):
    # g = 0 (and lam = 0 for coupled Adam): m_old = m_new/beta1, v_old = v_new/beta2; started from
    # fp32 values, the recovered moments round back to exactly those fp32 values
    x, _, m, v = _rand_state(10)
    x32, m32, v32 = x.astype(np.float32), m.astype(np.float32), v.astype(np.float32)
    z = np.zeros_like(x32)
    hp = Hyper(kind, eta=1e-3, lam=0.0 if kind == "adam" else 0.1, t=77)
    xn, mn, vn = oracle.opt_step(hp, x32, z, m32, v32)
    _close(mn, 0.9 * m32.astype(F64), rtol=1e-15)
    xo, mo, vo = oracle.opt_undo(hp, xn, z, mn, vn)
    assert np.array_equal(mo.astype(np.float32), m32)
    assert np.array_equal(vo.astype(np.float32), v32)
    assert np.array_equal(xo.astype(np.float32), x32)


def test_k_steps_then_k_undos_in_reverse():
    x, _, m, v = _rand_state(11, n=513)
    r = np.random.default_rng(12)
    grads = [r.normal(0, 1e-3, x.size) for _ in range(5)]
    for kind in ("sgdm", "adam", "adamw"):
        s = (x, m, None if kind == "sgdm" else v)
        hps = [Hyper(kind, eta=0.01 * (k + 1), lam=0.01, mu=0.9, tau=0.1, t=k + 1) for k in range(5)]
        for hp, g in zip(hps, grads):
            s = oracle.opt_step(hp, s[0], g, s[1], s[2])
        for hp, g in zip(reversed(hps), reversed(grads)):
            s = oracle.opt_undo(hp, s[0], g, s[1], s[2])
        _close(s[0], x, rtol=1e-12, atol=1e-16)
        _close(s[1], m, rtol=1e-10, atol=1e-16)
        if s[2] is not None:
            _close(s[2], v, rtol=1e-9, atol=1e-18)


def test_momentum_zero_is_plain_sgd_and_its_undo():
    # App. A "SGD"/"Undo SGD": x_old = (x_new + eta g)/(1 - eta lam); with the damped g' kept in m,
    # Alg. 2's first line gives the same parameter and the buffer comes back untouched
    x, g, m, _ = _rand_state(13)
    hp = Hyper("sgdm", eta=0.1, lam=0.01, mu=0.0, tau=0.0)
    xn, mn, _ = oracle.opt_step(hp, x, g, m)
    xo, mo, _ = oracle.opt_undo(hp, xn, g, mn)
    # (outlier gradients move x by ~0.1, so agreement is to ulps of that, not of x)
    _close(xo, (xn + 0.1 * g) / (1 - 0.1 * 0.01), rtol=1e-13, atol=1e-16)
    _close(xo, x, rtol=1e-14, atol=1e-16)
    assert np.array_equal(mo, mn)


# --------------------------------------------------------------------------- App. A "SGD" / "Undo SGD"
@pytest.mark.parametrize("lam", [0.0, 0.01, 0.5])
def test_plain_sgd_step_matches_torch_sgd_without_momentum(lam):
    x, g, _, _ = _rand_state(21)
    p = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    p.grad = torch.tensor(g, dtype=torch.float64)
    torch.optim.SGD([p], lr=0.1, momentum=0.0, weight_decay=lam, foreach=False).step()
    xn, mn, vn = oracle.opt_step(Hyper("sgd", eta=0.1, lam=lam), x, g)
    assert mn is None and vn is None
    _close(xn, p.detach().numpy(), rtol=1e-14, atol=1e-18)


def test_plain_sgd_equals_momentum_sgd_with_mu_zero_bit_for_bit():
    # Alg. 1 with mu = 0, tau = 0 performs the same operations on x as App. A's "SGD" (0 * m + g' = g' exactly)
    x, g, m, _ = _rand_state(22)
    a, _, _ = oracle.opt_step(Hyper("sgd", eta=0.1, lam=0.01), x, g)
    b, _, _ = oracle.opt_step(Hyper("sgdm", eta=0.1, lam=0.01, mu=0.0, tau=0.0), x, g, m)
    assert np.array_equal(a, b)


def test_plain_sgd_undo_is_the_printed_closed_form_and_round_trips():
    x, g, _, _ = _rand_state(23)
    hp = Hyper("sgd", eta=0.1, lam=0.01)
    xn, _, _ = oracle.opt_step(hp, x, g)
    xo, mo, vo = oracle.opt_undo(hp, xn, g)
    assert mo is None and vo is None
    # solving x_new = x - eta (g + lam x) for x, digit by digit in exact rational arithmetic
    from fractions import Fraction as Fr
    eta, lam = Fr(0.1), Fr(0.01)                 # the binary64 values the oracle received
    for i in (0, 3, 7, 100, 256):
        exact = (Fr(float(xn[i])) + eta * Fr(float(g[i]))) / (1 - eta * lam)
        assert abs(Fr(float(xo[i])) - exact) <= abs(exact) * Fr(1, 2 ** 50) + Fr(1, 10 ** 30)
    # (outlier gradients move x by ~0.1, so agreement with the originals is to ulps of that)
    _close(xo, x, rtol=1e-14, atol=1e-16)
    # dyadic values: every operation is exact, the round trip returns the original bits
    r = np.random.default_rng(24)
    xd = r.integers(-2 ** 20, 2 ** 20, 64).astype(F64) / 2 ** 10
    gd = r.integers(-2 ** 20, 2 ** 20, 64).astype(F64) / 2 ** 12
    hd = Hyper("sgd", eta=0.5, lam=0.0)
    back, _, _ = oracle.opt_undo(hd, oracle.opt_step(hd, xd, gd)[0], gd)
    assert np.array_equal(back, xd)
    # the sign of the gradient term and the side the divisor is on: a step with g = 0 scales by (1 - eta lam),
    # the undo by its reciprocal
    z = np.zeros_like(x)
    _close(oracle.opt_step(hp, x, z)[0], x * (1 - 0.1 * 0.01), rtol=1e-15, atol=1e-300)
    _close(oracle.opt_undo(hp, x, z)[0], x / (1 - 0.1 * 0.01), rtol=1e-15, atol=1e-300)
    # and with lam = 0 the undo adds back exactly what the step took away
    h0 = Hyper("sgd", eta=0.25, lam=0.0)
    # (the difference is taken off values of size 0.02-0.1: good to their ulp, 1e-17)
    _close(oracle.opt_undo(h0, x, g)[0] - x, 0.25 * g, rtol=1e-12, atol=3e-17)
    _close(oracle.opt_step(h0, x, g)[0] - x, -0.25 * g, rtol=1e-12, atol=3e-17)


def test_not_invertible_settings_raise():
    x, g, m, v = _rand_state(14, n=8)
    with pytest.raises(ZeroDivisionError):
        oracle.opt_undo(Hyper("adam", eta=1e-3, beta1=0.0), x, g, m, v)
    with pytest.raises(ZeroDivisionError):
        oracle.opt_undo(Hyper("adamw", eta=1e-3, beta2=0.0), x, g, m, v)
    with pytest.raises(ZeroDivisionError):
        oracle.opt_undo(Hyper("adamw", eta=0.5, lam=2.0), x, g, m, v)
    with pytest.raises(ZeroDivisionError):
        oracle.opt_undo(Hyper("sgd", eta=0.5, lam=2.0), x, g)


def test_list_walk_respects_mask_and_leaves_inputs_alone():
    r = np.random.default_rng(15)
    xs = [r.normal(size=n).astype(np.float32) for n in (5, 0, 17)]
    gs = [r.normal(size=a.size).astype(np.float32) for a in xs]
    ms = [r.normal(size=a.size).astype(np.float32) for a in xs]
    keep = [a.copy() for a in xs + gs + ms]
    hp = Hyper("sgdm", eta=0.1, lam=0.0, mu=0.9)
    out = oracle.step_list(hp, xs, gs, ms, None, mask=[1, 1, 0])
    assert all(np.array_equal(a, b) for a, b in zip(keep, xs + gs + ms))
    assert np.array_equal(out[2][0], xs[2].astype(F64)) and np.array_equal(out[2][1], ms[2].astype(F64))
    assert not np.array_equal(out[0][0], xs[0].astype(F64))
    assert out[1][0].size == 0
    back = oracle.undo_list(hp, [o[0] for o in out], gs, [o[1] for o in out], None, mask=[1, 1, 0])
    for b, x0 in zip(back, xs):
        _close(b[0], x0.astype(F64), rtol=1e-13, atol=1e-16)


def test_bf16_bits_widen_exactly():
    bits = np.array([0x3F80, 0xBF80, 0x0000, 0x8000, 0x3DCD, 0x0001, 0x7F7F], dtype=np.uint16)
    want = torch.tensor(bits.astype(np.int32).astype(np.int16)).view(torch.bfloat16).double().numpy()
    got = oracle.widen(bits)
    assert np.array_equal(got, want)
    assert np.signbit(got[3]) and got[3] == 0.0


# --------------------------------------------------------------------------- LAMB
def _adamw_direction(hp, x, g, m, v):
    """u = r + lambda x, read off the (already pinned) AdamW step with eta = 1: x_new = x - u."""
    one = Hyper("adamw", eta=1.0, lam=hp.lam, beta1=hp.beta1, beta2=hp.beta2, eps=hp.eps, t=hp.t)
    xn, mn, vn = oracle.opt_step(one, x, g, m, v)
    return x - xn, mn, vn


@pytest.mark.parametrize("lam", [0.0, 0.01, 0.5])
def test_lamb_is_adamw_with_the_trust_ratio_folded_into_the_learning_rate(lam):
    # LAMB(eta) on one tensor = AdamW(eta * q), q = ||x|| / ||u||, with u and the norms taken from
    # the pinned AdamW oracle and numpy, not from the LAMB code
    x, g, m, v = _rand_state(21, n=1001)
    hp = Hyper("lamb", eta=2e-3, lam=lam, beta1=0.9, beta2=0.999, eps=1e-6, t=12)
    u, _, _ = _adamw_direction(hp, x, g, m, v)
    nx, nu = np.sqrt(np.sum(x * x)), np.sqrt(np.sum(u * u))
    xn, mn, vn, norms = oracle.lamb_step(hp, x, g, m, v)
    _close(norms, [nx, nu], rtol=1e-10)          # u from x - x_new carries the subtraction's rounding
    ref = oracle.opt_step(Hyper("adamw", eta=hp.eta * nx / nu, lam=lam, beta1=0.9, beta2=0.999, eps=1e-6, t=12), x, g, m, v)
    _close(xn, ref[0], rtol=1e-11, atol=1e-15)
    assert np.array_equal(mn, ref[1]) and np.array_equal(vn, ref[2])
    # and the undo with the saved norms returns the state
    xo, mo, vo = oracle.lamb_undo(hp, xn, g, mn, vn, norms)
    _close(xo, x, rtol=1e-12, atol=1e-16)
    _close(mo, m, rtol=1e-12, atol=1e-15 * np.abs(mn).max())
    _close(vo, v, rtol=1e-12, atol=1e-15 * np.abs(vn).max())


def test_lamb_zero_norm_falls_back_to_ratio_one():
    _, g, m, v = _rand_state(22, n=64)
    z = np.zeros_like(g)
    hp = Hyper("lamb", eta=1e-3, lam=0.1, t=3)
    xn, mn, vn, norms = oracle.lamb_step(hp, z, g, m, v)          # ||x|| = 0: q = 1, plain AdamW
    ref = oracle.opt_step(Hyper("adamw", eta=1e-3, lam=0.1, t=3), z, g, m, v)
    assert norms[0] == 0.0 and norms[1] > 0.0
    assert np.array_equal(xn, ref[0])
    xo, mo, vo = oracle.lamb_undo(hp, xn, g, mn, vn, norms)      # the undo applies the same fallback
    _close(xo, z, rtol=0, atol=1e-18)
    _close(mo, m, rtol=1e-12, atol=1e-15 * np.abs(mn).max())
    x = np.ones_like(g)
    xn, _, _, norms = oracle.lamb_step(Hyper("lamb", eta=1e-3, lam=0.0, t=3), x, z, z, v)   # u = 0: nothing moves
    assert norms[1] == 0.0 and np.array_equal(xn, x)


def test_lamb_layerwise_scaling():
    # lambda = 0: scaling the parameters of the tensor by a power of two scales the whole update by it,
    # bit for bit (the trust ratio carries the norm of x); scaling g, m, v as c, c, c^2 changes nothing
    x, g, m, v = _rand_state(23, n=333)
    v = v + 1e-12
    hp = Hyper("lamb", eta=1e-2, lam=0.0, eps=0.0, t=5)
    a = oracle.lamb_step(hp, x, g, m, v)
    b = oracle.lamb_step(hp, 4 * x, g, m, v)
    assert np.array_equal(4 * a[0], b[0]) and b[3][0] == 4 * a[3][0] and b[3][1] == a[3][1]
    c = oracle.lamb_step(hp, x, 8 * g, 8 * m, 64 * v)
    assert np.array_equal(a[0], c[0])


# --------------------------------------------------------------------------- digest
M64 = (1 << 64) - 1
K1, K2, K3 = 0x9E3779B97F4A7C15, 0x6A09E667F3BCC909, 0xBB67AE8584CAA73B


def _unmix(z):
    """Inverse of the digest's mixer, step by step in reverse (every step is a bijection)."""
    z ^= z >> 32
    z = (z * pow(K3, -1, 1 << 64)) & M64
    z ^= (z >> 29) ^ (z >> 58)
    z = (z * pow(K2, -1, 1 << 64)) & M64
    z ^= z >> 32
    return (z - K1) & M64


@pytest.mark.parametrize("ws,want", read_digest_vectors(), ids=lambda v: None)
def test_digest_vectors(ws, want):
    got = int(oracle.digest(np.array(ws, dtype=np.uint32))[0])
    assert got == want, f"{got:016X} != {want:016X}"


def test_digest_increments_unmix_to_index_and_word():
    # digest(w[:k+1]) - digest(w[:k]) is the mixed (k, w_k); undoing the mixer must give it back
    r = np.random.default_rng(16)
    w = r.integers(0, 1 << 32, 300, dtype=np.uint64).astype(np.uint32)
    prev = 0
    for k in range(w.size):
        cur = int(oracle.digest(w[:k + 1])[0])
        assert _unmix((cur - prev) & M64) == (k << 32) | int(w[k])
        prev = cur


def test_digest_sees_every_single_bit_flip_and_sign_of_zero():
    w = np.array([0, 0x3F800000, 0xFFFFFFFF, 0x12345678, 0x80000000], dtype=np.uint32)
    base = int(oracle.digest(w)[0])
    seen = {base}
    for i in range(w.size):
        for b in range(32):
            f = w.copy()
            f[i] ^= np.uint32(1 << b)
            seen.add(int(oracle.digest(f)[0]))
    assert len(seen) == 1 + 32 * w.size
    pz, nz = np.array([0.0], np.float32), np.array([-0.0], np.float32)
    assert int(oracle.digest(pz)[0]) != int(oracle.digest(nz)[0])


def test_digest_shards_are_slices_and_order_matters_only_through_the_index():
    r = np.random.default_rng(17)
    buf = r.normal(size=1000).astype(np.float32)
    d = oracle.digest(buf, 256)
    assert d.size == 4
    for k in range(4):
        assert d[k] == oracle.digest(buf[256 * k:256 * (k + 1)])[0]
    assert oracle.digest(buf, 1000)[0] == oracle.digest(buf)[0] == oracle.digest(buf, 4096)[0]
    # permuting the words changes the digest (the index is mixed in) ...
    assert oracle.digest(buf[::-1].copy())[0] != oracle.digest(buf)[0]
    # ... but the sum itself is order-free: summing one-word increments in any order gives the same
    inc = []
    prev = 0
    for k in range(64):
        cur = int(oracle.digest(buf[:k + 1])[0])
        inc.append((cur - prev) & M64)
        prev = cur
    r.shuffle(inc)
    assert sum(inc) & M64 == int(oracle.digest(buf[:64])[0])


def test_digest_list_is_buffer_major_and_empty_cases():
    a = np.arange(10, dtype=np.uint32)
    b = np.arange(3, dtype=np.int32)
    e = np.zeros(0, np.float32)
    d = oracle.digest_list([a, e, b], 4)
    assert d.size == 3 + 0 + 1
    assert d[3] == oracle.digest(b)[0]
    d0 = oracle.digest_list([a, e, b], 0)
    assert d0.size == 3 and d0[1] == 0
    assert oracle.digest_list([], 0).size == 0


# --------------------------------------------------------------------------- bf16 copy
def test_bf16_round_matches_torch_and_the_definition():
    r = np.random.default_rng(31)
    x = np.concatenate([
        r.normal(0, 0.02, 5000).astype(np.float32),
        (r.integers(0, 1 << 32, 20000, dtype=np.uint64).astype(np.uint32)).view(np.float32),   # any bit pattern
        np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 3.4028235e38,
                  1e-40, -1e-45, 65280.0, 65408.0], dtype=np.float32),
    ])
    got = oracle.bf16_round(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], want[~nan])
    assert (got[nan] == 0x7FC0).all()
    # the definition, value by value: the result is a nearest bfloat16, and on a tie the even one
    fin = np.isfinite(x) & (np.abs(x) < 3e38)
    xs = x[fin].astype(np.float64)
    back = (got[fin].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    up = ((got[fin].astype(np.uint32) + 1) << 16).view(np.float32).astype(np.float64)
    dn = ((got[fin].astype(np.uint32) - 1) << 16).view(np.float32).astype(np.float64)
    with np.errstate(invalid="ignore"):
        ok_near = (np.abs(back - xs) <= np.abs(up - xs)) | ~np.isfinite(up)
        ok_near &= (np.abs(back - xs) <= np.abs(dn - xs)) | ~np.isfinite(dn) | (got[fin] == 0) | (got[fin] == 0x8000)
    assert ok_near.all()
    tie = np.array([1.00390625, 1.01171875], dtype=np.float32)    # halfway between neighbours: 0x3F80|0x3F81 and 0x3F81|0x3F82
    assert oracle.bf16_round(tie).tolist() == [0x3F80, 0x3F82]
    assert oracle.bf16_round(np.array([3.4028235e38], np.float32))[0] == 0x7F80   # rounds up to infinity


# ------------------------------------------------------------------------------------------
# Optional clamp of the recovered second moment (not in the paper; off by default).
def test_v_clamp_only_touches_negative_values():
    rng = np.random.default_rng(77)
    n = 4000
    x = rng.normal(0, 0.02, n)
    g = rng.normal(0, 1e-3, n)
    m = rng.normal(0, 1e-4, n)
    v = np.abs(rng.normal(0, 1e-6, n))
    v[::7] = 0.0                                                  # where the step leaves (1-beta2) g^2 only
    for kind in ("adam", "adamw"):
        h = oracle.Hyper(kind, eta=1e-3, lam=0.01, beta1=0.9, beta2=0.999, eps=1e-8, t=10)
        x1, m1, v1 = oracle.opt_step(h, x, g, m, v)
        v1 = v1.astype(np.float32)                                # the stored state is binary32: rounding can push
        xa, ma, va = oracle.opt_undo(h, x1, g, m1, v1)            # the recovered v below zero
        hc = oracle.Hyper(kind, eta=1e-3, lam=0.01, beta1=0.9, beta2=0.999, eps=1e-8, t=10, clamp_v=True)
        xb, mb, vb = oracle.opt_undo(hc, x1, g, m1, v1)
        assert (va < 0).any(), "the case must exercise the clamp"
        assert np.array_equal(xa, xb) and np.array_equal(ma, mb)
        assert np.array_equal(vb, np.where(va < 0, 0.0, va))      # the definition, written out
        assert (vb >= 0).all() and not np.signbit(vb[va < 0]).any()
        # the default stays the paper's formula
        assert np.array_equal(va, (v1.astype(np.float64) - (1 - h.beta2) * (g + (h.lam * xa if kind == "adam" else 0)) ** 2) / h.beta2)


def test_v_clamp_keeps_nan_and_applies_to_lamb():
    h = oracle.Hyper("adamw", eta=1e-3, lam=0.0, beta1=0.5, beta2=0.5, eps=1e-8, t=1, clamp_v=True)
    x = np.array([1.0, 1.0, 1.0]); g = np.array([2.0, 0.0, 1.0]); m = np.array([0.0, 0.0, 0.0])
    v_new = np.array([1.0, np.nan, 3.0])                          # (1 - 0.5*4)/0.5 = -2 -> 0;  NaN;  (3 - 0.5)/0.5 = 5
    _, _, v_old = oracle.opt_undo(h, x, g, m, v_new)
    assert v_old[0] == 0.0 and np.isnan(v_old[1]) and v_old[2] == 5.0
    norms = np.array([1.0, 1.0])
    _, _, vl = oracle.lamb_undo(h, x, g, m, np.array([1.0, 1.0, 3.0]), norms)
    assert vl[0] == 0.0 and vl[1] == 2.0 and vl[2] == 5.0
    h.clamp_v = False
    _, _, vl = oracle.lamb_undo(h, x, g, m, np.array([1.0, 1.0, 3.0]), norms)
    assert vl[0] == -2.0

