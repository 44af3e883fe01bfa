"""Property-based pins of the CPU oracle (hypothesis): algebraic facts that hold for every admissible
hyper-parameter setting, checked on random settings rather than a handful of fixed ones."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from oracle import Hyper

unit = st.floats(min_value=0.05, max_value=0.95)
lr = st.floats(min_value=1e-5, max_value=0.5)
decay = st.floats(min_value=0.0, max_value=0.5)
seeds = st.integers(min_value=0, max_value=2 ** 31 - 1)


def _state(seed, n=64):
    r = np.random.default_rng(seed)
    x, g, m = r.normal(0, 0.02, n), r.normal(0, 1e-3, n), r.normal(0, 1e-4, n)
    v = np.abs(r.normal(0, 1e-6, n)) + 1e-12
    g[::5] = 0.0
    g[1::9] *= 1e3
    return x, g, m, v


def _close(a, b, rtol, atol):
    a, b = np.asarray(a), np.asarray(b)
    assert (np.abs(a - b) <= np.maximum(rtol * np.abs(b), atol)).all(), (np.abs(a - b).max(), atol)


@settings(max_examples=60, deadline=None)
@given(seed=seeds, eta=lr, lam=decay)
def test_plain_sgd_undo_inverts_step(seed, eta, lam):
    x, g, _, _ = _state(seed)
    hp = Hyper("sgd", eta=eta, lam=lam)            # eta * lam <= 0.25: the divisor stays away from zero
    xn, mn, vn = oracle.opt_step(hp, x, g)
    assert mn is None and vn is None
    xo, _, _ = oracle.opt_undo(hp, xn, g)
    scale = max(np.abs(xn).max(), eta * np.abs(g).max())
    _close(xo, x, 1e-12, 1e-14 * scale)
    # App. A's update line by hand, vectorised in numpy
    _close(xn, x - eta * (g + lam * x), 1e-13, 1e-18)
    # the step is affine in (x, g): stepping a sum is the sum of steps minus nothing else
    x2, g2, _, _ = _state(seed + 1)
    both, _, _ = oracle.opt_step(hp, x + x2, g + g2)
    _close(both, xn + oracle.opt_step(hp, x2, g2)[0], 1e-12, 1e-15 * max(scale, 1.0))


@settings(max_examples=60, deadline=None)
@given(seed=seeds, eta=lr, lam=decay, mu=unit, tau=st.floats(min_value=0.0, max_value=0.9))
def test_sgdm_undo_inverts_step(seed, eta, lam, mu, tau):
    x, g, m, _ = _state(seed)
    hp = Hyper("sgdm", eta=eta, lam=lam, mu=mu, tau=tau)
    xn, mn, _ = oracle.opt_step(hp, x, g, m)
    xo, mo, _ = oracle.opt_undo(hp, xn, g, mn)
    scale = max(np.abs(xn).max(), np.abs(mn).max(), np.abs(g).max())
    _close(xo, x, 1e-12, 1e-14 * scale)
    _close(mo, m, 1e-12, 1e-14 * scale / mu)
    # Alg. 1 by hand, vectorised in numpy: a second, independent evaluation of the two update lines
    gp = g + lam * x
    _close(mn, mu * m + (1 - tau) * gp, 1e-14, 1e-300)
    _close(xn, x - eta * (mu * m + (1 - tau) * gp), 1e-13, 1e-18)


@settings(max_examples=60, deadline=None)
@given(seed=seeds, eta=lr, lam=decay, b1=unit, b2=unit, t=st.integers(min_value=1, max_value=100000),
       kind=st.sampled_from(["adam", "adamw"]))
def test_adam_family_undo_inverts_step(seed, eta, lam, b1, b2, t, kind):
    x, g, m, v = _state(seed)
    if kind == "adamw" and abs(1 - eta * lam) < 1e-3:
        return
    hp = Hyper(kind, eta=eta, lam=lam, beta1=b1, beta2=b2, eps=1e-8, t=t)
    xn, mn, vn = oracle.opt_step(hp, x, g, m, v)
    xo, mo, vo = oracle.opt_undo(hp, xn, g, mn, vn)
    _close(xo, x, 1e-11, 1e-13 * max(1.0, np.abs(xn).max()))
    _close(mo, m, 1e-11, 1e-13 * max(np.abs(mn).max(), np.abs(g).max(), lam * np.abs(x).max()) / b1)
    _close(vo, v, 1e-11, 1e-13 * max(np.abs(vn).max(), (np.abs(g).max() + lam * np.abs(x).max()) ** 2) / b2)
    # the moments never depend on the learning rate, the parameter moves by exactly eta * (direction)
    xn2, mn2, vn2 = oracle.opt_step(Hyper(kind, eta=2 * eta, lam=lam, beta1=b1, beta2=b2, eps=1e-8, t=t), x, g, m, v)
    assert np.array_equal(mn, mn2) and np.array_equal(vn, vn2)
    _close(xn2 - x, 2 * (xn - x), 1e-9, 1e-15)


@settings(max_examples=40, deadline=None)
@given(seed=seeds, eta=lr, lam=st.floats(min_value=0.0, max_value=0.05), t=st.integers(min_value=1, max_value=1000))
def test_lamb_undo_inverts_step_and_ratio_is_scale_free(seed, eta, lam, t):
    x, g, m, v = _state(seed, n=200)
    hp = Hyper("lamb", eta=eta, lam=lam, beta1=0.9, beta2=0.999, eps=1e-8, t=t)
    xn, mn, vn, norms = oracle.lamb_step(hp, x, g, m, v)
    q = norms[0] / norms[1]
    if abs(1 - eta * q * lam) < 1e-3:
        return
    xo, mo, vo = oracle.lamb_undo(hp, xn, g, mn, vn, norms)
    _close(xo, x, 1e-10, 1e-13 * max(1.0, np.abs(xn).max()))
    _close(mo, m, 1e-11, 1e-13 * max(np.abs(mn).max(), np.abs(g).max()))
    # the step length is eta * ||x|| whatever the gradients' scale: ||x_new - x|| = eta q ||u|| = eta ||x||
    _close(np.linalg.norm(xn - x), eta * np.linalg.norm(x), 1e-9, 0)


@settings(max_examples=50, deadline=None)
@given(data=st.lists(st.integers(min_value=0, max_value=2 ** 32 - 1), min_size=0, max_size=200),
       cut=st.integers(min_value=1, max_value=64))
def test_digest_is_a_sum_of_independent_word_terms(data, cut):
    w = np.array(data, dtype=np.uint32)
    whole = int(oracle.digest(w)[0])
    # sharding restarts the index: the digest of a shard equals the digest of that slice on its own
    parts = oracle.digest(w, cut)
    assert parts.size == (w.size + cut - 1) // cut
    for k in range(parts.size):
        assert parts[k] == oracle.digest(w[k * cut:(k + 1) * cut])[0]
    # changing one word changes the digest by exactly that word's term: the difference does not depend on the rest
    if w.size >= 2:
        a, b = w.copy(), w.copy()
        a[0] ^= np.uint32(1)
        b[0] ^= np.uint32(1)
        b[1:] = 0
        z = w.copy()
        z[1:] = 0
        M = (1 << 64) - 1
        assert (int(oracle.digest(a)[0]) - whole) & M == (int(oracle.digest(b)[0]) - int(oracle.digest(z)[0])) & M
        assert int(oracle.digest(a)[0]) != whole
