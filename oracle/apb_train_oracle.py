"""CPU oracle for the training-side operators of APB -- TEST INFRASTRUCTURE ONLY.

Written from Sec. III of the paper (arXiv 2306.08960), Eqs. 3-9: the APB operator applied to the
latent weights, its straight-through derivative, and the gradients of the loss with respect to the
two learned scalars of a layer, alpha (scale of the binarized weights) and delta (how far the
binarization interval reaches beyond alpha).  Plain numpy in float64, the paper's steps in the
paper's order; nothing here is shared with, or imported by, the HIP library.

  apb_operator      Eq. 3:  APB(w) = sign(w) * alpha  if |w| <= alpha + delta,  w otherwise
                    (sign(0) = +, Eq. 1)
  chi_B             the indicator of the binarized set, 1(w_hat <= 1) with
                    w_hat = (|w| - alpha) / delta  (Eqs. 5-6), evaluated as the equivalent compare
                    |w| <= alpha + delta of Eq. 3
  grad_latent       Eq. 4 with the identity as the surrogate g: dAPB/dw = 1 on both branches, so the
                    gradient of the latent weight is the upstream gradient unchanged
  grad_w_hat        Eq. 9 solved for dL/dw_hat:  dL/dw_hat = delta * sign(w) * dL/dw
  grad_delta        Eq. 7:  dL/ddelta = 1 / (delta^2 n) * sum dL/dw_hat * (alpha - |w|) * chi_B
  grad_alpha        Eq. 8:  dL/dalpha = -1 / (delta n) * sum dL/dw_hat * chi_B

Readings taken (each listed in the design notes):
  * n is the number of weights of the layer (the paper's W in R^n), not the size of the binarized set.
  * dL/dw on the right of Eq. 9 is what backpropagation delivers for the latent weight, which by Eq. 4
    (identity surrogate) equals the gradient with respect to APB(w) on both branches.
  * The interval test is the float32 compare |w| <= fl32(alpha + delta), the same test apb_compress
    applies with its `delta` argument = alpha + delta; everything after the test is float64.
  * Eqs. 7-8 are evaluated as printed (sign and 1/n included), although differentiating
    sign(w) * alpha directly would give +sum(g * sign(w) * chi_B) for alpha: the paper routes both
    scalars through w_hat, and this oracle follows the paper.
"""
from __future__ import annotations

import numpy as np


def _interval(alpha, delta) -> np.float32:
    """Half-width of the binarization interval as the float32 sum alpha + delta."""
    return np.float32(np.float32(alpha) + np.float32(delta))


def sign_pm(W: np.ndarray) -> np.ndarray:
    """+1.0 where w >= 0 (so -0.0 is +), -1.0 elsewhere; float64 (Eq. 1)."""
    return np.where(np.asarray(W, dtype=np.float32) >= np.float32(0), 1.0, -1.0)


def chi_B(W: np.ndarray, alpha, delta) -> np.ndarray:
    """Indicator of the binarized set (Eq. 6), bool."""
    return np.abs(np.asarray(W, dtype=np.float32)) <= _interval(alpha, delta)


def apb_operator(W: np.ndarray, alpha, delta) -> np.ndarray:
    """Eq. 3 element-wise; float32 (either +-alpha as given in float32, or the weight itself)."""
    W = np.asarray(W, dtype=np.float32)
    a = np.float32(alpha)
    return np.where(chi_B(W, alpha, delta), np.where(W >= np.float32(0), a, -a), W).astype(np.float32)


def grad_latent(G: np.ndarray) -> np.ndarray:
    """Eq. 4 with g = id: the straight-through gradient of the latent weights."""
    return np.asarray(G, dtype=np.float32).copy()


def grad_w_hat(W: np.ndarray, G: np.ndarray, delta) -> np.ndarray:
    """Eq. 9 solved for dL/dw_hat; float64."""
    return float(np.float32(delta)) * sign_pm(W) * np.asarray(G, dtype=np.float32).astype(np.float64)


def grad_delta(W: np.ndarray, G: np.ndarray, alpha, delta) -> float:
    """Eq. 7; float64."""
    W = np.asarray(W, dtype=np.float32)
    a, d = float(np.float32(alpha)), float(np.float32(delta))
    n = W.size
    terms = grad_w_hat(W, G, delta) * (a - np.abs(W.astype(np.float64))) * chi_B(W, alpha, delta)
    return float(np.sum(terms, dtype=np.float64) / (d * d * n))


def grad_alpha(W: np.ndarray, G: np.ndarray, alpha, delta) -> float:
    """Eq. 8; float64."""
    W = np.asarray(W, dtype=np.float32)
    d = float(np.float32(delta))
    n = W.size
    terms = grad_w_hat(W, G, delta) * chi_B(W, alpha, delta)
    return float(-np.sum(terms, dtype=np.float64) / (d * n))


def backward(W: np.ndarray, G: np.ndarray, alpha, delta) -> dict:
    """Everything the backward pass of one layer's APB operator produces."""
    return {"grad_w": grad_latent(G), "grad_alpha": grad_alpha(W, G, alpha, delta),
            "grad_delta": grad_delta(W, G, alpha, delta), "n_binarized": int(chi_B(W, alpha, delta).sum())}
