"""The MLP block of Section 3.2 as plain full-matrix arithmetic (oracle; tests only).

Section 3.2 builds the Transformer's MLP block from two 3-D linear layers around an
activation: ``Z = X W1 + b1``, ``H = act(Z)``, ``Y = H W2 + b2``; the first layer
gathers its input in y and leaves its output in z, the second takes that output in
place (directions exchanged, Section 3.1.1 last paragraph).  The activation acts
element by element, so it needs no communication.  The backward pass is the chain
rule through these three steps, with the linear layers' gradients of Section 3.1.2
(first differentiation formula) and the bias gradient of Algorithm 8 (column sums).

Reading: the paper does not name the activation.  Two are written out here: the
rectifier ``max(z, 0)`` (exact on integers) and the Gaussian error linear unit in its
exact form ``z * Phi(z)``, ``Phi`` the standard normal distribution function.

``store`` arguments: where the device keeps an intermediate in a narrower type, the
same single rounding is applied here (a callable fp64 -> fp64; identity by default).
"""
import math

import numpy as np

from . import matmul as _mm

KINDS = ("relu", "gelu")

# The error function is a library primitive here: scipy's vectorised fp64 erf where scipy is
# importable (the full-size cases have 67 million pre-activations), else the C library's through
# Python's math module, element by element.  The two agree to the last bit or two in fp64; the
# tests pin whichever is in use against tabulated values of the normal distribution function.
try:
    from scipy.special import erf as _erf
except ImportError:                      # pragma: no cover
    _erf = np.vectorize(math.erf, otypes=[np.float64])
_erf_scalar = np.vectorize(math.erf, otypes=[np.float64])


def _phi_cdf(z):
    return 0.5 * (1.0 + _erf(np.asarray(z, dtype=np.float64) / math.sqrt(2.0)))


def _phi_pdf(z):
    z = np.asarray(z, dtype=np.float64)
    return np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


def act(z, kind):
    z = np.asarray(z, dtype=np.float64)
    if kind == "relu":
        return np.where(z > 0.0, z, 0.0)
    if kind == "gelu":
        return z * _phi_cdf(z)
    raise ValueError("kind is one of %r" % (KINDS,))


def act_grad(z, kind):
    """d act / d z.  (The rectifier's slope at 0 is taken as 0.)"""
    z = np.asarray(z, dtype=np.float64)
    if kind == "relu":
        return np.where(z > 0.0, 1.0, 0.0)
    if kind == "gelu":
        return _phi_cdf(z) + z * _phi_pdf(z)
    raise ValueError("kind is one of %r" % (KINDS,))


def _same(x):
    return x


def forward(X, W1, b1, W2, b2, kind, store_z=_same, store_h=_same, store_y=_same, threads=1):
    """Returns (Z, H, Y) as the device stores them.  `threads`: host threads of the plain products."""
    Z = store_z(_mm.forward(X, W1, threads) + np.asarray(b1, dtype=np.float64)[None, :])
    H = store_h(act(Z, kind))
    Y = store_y(_mm.forward(H, W2, threads) + np.asarray(b2, dtype=np.float64)[None, :])
    return Z, H, Y


def backward(dY, X, W1, Z, H, W2, kind, store_g=_same, store_dz=_same, threads=1):
    """Gradients of <dY, Y>: returns dict with dX, dW1, db1, dW2, db2 (and dH, dZ as stored)."""
    dY = np.asarray(dY, dtype=np.float64)
    dH = store_g(_mm.backward_dx(dY, W2, threads))         # dH = dY W2^T
    dW2 = _mm.backward_dw(H, dY, threads)                  # dW2 = H^T dY
    db2 = dY.sum(axis=0)
    dZ = store_dz(dH * act_grad(Z, kind))
    dX = _mm.backward_dx(dZ, W1, threads)
    dW1 = _mm.backward_dw(X, dZ, threads)
    db1 = dZ.sum(axis=0)
    return {"dH": dH, "dZ": dZ, "dX": dX, "dW1": dW1, "db1": db1, "dW2": dW2, "db2": db2}
