"""Pins of the training-side oracle (Sec. III Eqs. 3-9) against what the paper and the mathematics fix:
hand cases on the interval boundary, exact rational arithmetic on representable inputs, closed forms of
special cases, the reduction of Eq. 3 to Eq. 1 and to the identity, and consistency with the forward
oracle's partition.  No GPU."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import apb_oracle as o
from oracle import apb_train_oracle as t


def f32(x):
    return np.float32(x)


def test_operator_hand_cases_on_the_boundary():
    # alpha = 0.25, delta = 0.5: interval |w| <= 0.75, boundary included (Eq. 3 uses <=); sign(0) = + (Eq. 1)
    W = np.array([0.0, -0.0, 0.1, -0.1, 0.75, -0.75, np.nextafter(f32(0.75), f32(1)), -0.7500001, 2.0, -3.0], dtype=np.float32)
    out = t.apb_operator(W, 0.25, 0.5)
    want = np.array([0.25, 0.25, 0.25, -0.25, 0.25, -0.25, np.nextafter(f32(0.75), f32(1)), f32(-0.7500001), 2.0, -3.0], dtype=np.float32)
    assert np.array_equal(out, want)
    assert t.chi_B(W, 0.25, 0.5).tolist() == [True] * 6 + [False] * 4


def test_operator_limits_reduce_to_bin_and_identity():
    g = np.random.default_rng(1)
    W = g.standard_normal(1000).astype(np.float32)
    # interval covering everything: Eq. 3 becomes Eq. 1, Bin(w) = alpha * sign(w)
    assert np.array_equal(t.apb_operator(W, 0.3, 1e9), np.where(W >= 0, f32(0.3), f32(-0.3)))
    # empty interval (alpha + delta below every |w|): the identity
    assert np.array_equal(t.apb_operator(W + np.where(W >= 0, 1, -1).astype(np.float32), 0.25, 0.25), W + np.where(W >= 0, 1, -1).astype(np.float32))


def test_operator_agrees_with_the_forward_oracle_partition():
    # the dense matrix the forward oracle reconstructs (Eq. 3 through compress) is the same operator
    g = np.random.default_rng(2)
    W = (g.standard_normal((13, 37)) * 0.05).astype(np.float32)
    alpha, delta = f32(0.04), f32(0.06)
    dense = o.apb_dense(W, f32(alpha + delta), alpha)
    assert np.array_equal(t.apb_operator(W, alpha, delta).astype(np.float64), dense)
    assert np.array_equal(t.chi_B(W, alpha, delta), ~o.outlier_mask(W, f32(alpha + delta)))


def _exact(W, G, alpha, delta):
    """Eqs. 7-9 in exact rational arithmetic, term by term as printed."""
    a, d = Fraction(float(f32(alpha))), Fraction(float(f32(delta)))
    lim = Fraction(float(f32(f32(alpha) + f32(delta))))
    n = len(W)
    s_alpha, s_delta = Fraction(0), Fraction(0)
    for w, g in zip(W, G):
        w_, g_ = Fraction(float(w)), Fraction(float(g))
        sign = 1 if w >= 0 else -1
        dL_dwhat = d * sign * g_                       # Eq. 9: dL/dw = (1/delta) dL/dw_hat sign(w)
        chi = 1 if abs(w_) <= lim else 0
        s_delta += dL_dwhat * (a - abs(w_)) * chi      # Eq. 7
        s_alpha += dL_dwhat * chi                      # Eq. 8
    return -s_alpha / (d * n), s_delta / (d * d * n)


def test_gradients_equal_exact_rational_evaluation():
    g = np.random.default_rng(3)
    # dyadic inputs: every product and sum below is exact in float64 as well
    W = (g.integers(-64, 65, 200) / 64.0).astype(np.float32)
    G = (g.integers(-32, 33, 200) / 128.0).astype(np.float32)
    for alpha, delta in ((0.25, 0.25), (0.5, 0.125), (0.125, 0.75)):
        ga, gd = _exact(W, G, alpha, delta)
        assert t.grad_alpha(W, G, alpha, delta) == float(ga)
        assert t.grad_delta(W, G, alpha, delta) == float(gd)


def test_closed_forms():
    g = np.random.default_rng(4)
    W = g.standard_normal(5000).astype(np.float32)
    G = g.standard_normal(5000).astype(np.float32)
    n = W.size
    sgn = np.where(W >= 0, 1.0, -1.0)
    # every weight binarized: Eq. 8 collapses to -(1/n) sum g sign(w), independent of delta
    for delta in (50.0, 70.0):
        assert t.grad_alpha(W, G, 0.5, delta) == pytest.approx(-np.sum(G.astype(np.float64) * sgn) / n, rel=1e-13)
    # no weight binarized: both gradients vanish and the operator is the identity
    big = W + 10 * sgn.astype(np.float32)
    assert t.grad_alpha(big, G, 0.5, 0.5) == 0.0 and t.grad_delta(big, G, 0.5, 0.5) == 0.0
    # every |w| equal to alpha: the factor (alpha - |w|) of Eq. 7 vanishes term by term
    flat = (0.5 * sgn).astype(np.float32)
    assert t.grad_delta(flat, G, 0.5, 0.25) == 0.0
    # Eq. 7 after substituting Eq. 9: (1/(delta n)) sum g sign(w) (alpha - |w|) chi_B
    chi = np.abs(W) <= f32(f32(0.3) + f32(0.4))
    want = np.sum(G.astype(np.float64) * sgn * (float(f32(0.3)) - np.abs(W.astype(np.float64))) * chi) / (float(f32(0.4)) * n)
    assert t.grad_delta(W, G, 0.3, 0.4) == pytest.approx(want, rel=1e-12)


def test_signs_and_scaling_would_be_caught():
    # one binarized positive weight below alpha, positive upstream gradient:
    # dL/dw_hat = delta*g > 0, so Eq. 8 is negative and Eq. 7 positive; n = 2 halves both
    W = np.array([0.25, 9.0], dtype=np.float32)
    G = np.array([2.0, 5.0], dtype=np.float32)
    assert t.grad_alpha(W, G, 0.5, 0.5) == -1.0                  # -(1/(0.5*2)) * (0.5*1*2)
    assert t.grad_delta(W, G, 0.5, 0.5) == 0.5                   # (1/(0.25*2)) * (0.5*2) * (0.5-0.25)
    # mirrored weight: sign(w) flips dL/dw_hat
    W2 = np.array([-0.25, 9.0], dtype=np.float32)
    assert t.grad_alpha(W2, G, 0.5, 0.5) == 1.0 and t.grad_delta(W2, G, 0.5, 0.5) == -0.5
    # straight-through: the latent gradient is the upstream gradient on both branches (Eq. 4, g = id)
    assert np.array_equal(t.grad_latent(G), G)
    b = t.backward(W, G, 0.5, 0.5)
    assert b["n_binarized"] == 1 and b["grad_alpha"] == -1.0 and b["grad_delta"] == 0.5
