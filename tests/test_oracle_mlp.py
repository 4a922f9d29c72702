"""Pins for the oracle of the MLP block (two linear layers around an activation; CPU only).

Pinned by: tabulated values of the normal distribution function (golden file) and the
identity gelu(z) - gelu(-z) = z; finite differences (slope of the activation, and every
gradient of the block against central differences of <dY, Y>); exactness of the rectifier
chain on integers; and the storage fact the chain rests on: the output shards of a layer
that gathers in y are, as stored, the input shards of a layer that gathers in z.
"""
import os

import numpy as np
import pytest

from oracle import mlp
from oracle.layout import Cube


def test_tabulated_values_and_symmetry(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "normal_cdf.txt")):
        if line.startswith("#") or not line.strip():
            continue
        z, cdf = [float(v) for v in line.split("|")]
        assert abs(mlp.act(np.array([z]), "gelu")[0] - z * cdf) <= 1e-15 * max(1.0, z)
        assert abs(mlp.act(np.array([-z]), "gelu")[0] + z * (1.0 - cdf)) <= 1e-15 * max(1.0, z)
        n += 1
    assert n == 6
    z = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(mlp.act(z, "gelu") - mlp.act(-z, "gelu"), z, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(mlp.act(np.array([-2.0, 0.0, 3.0]), "relu"), [0.0, 0.0, 3.0])
    np.testing.assert_array_equal(mlp.act_grad(np.array([-2.0, 0.0, 3.0]), "relu"), [0.0, 0.0, 1.0])
    with pytest.raises(ValueError):
        mlp.act(z, "tanh")


def test_the_two_error_function_routines_agree():
    # the vectorised library routine the oracle uses against the C library's, on a fine grid
    z = np.concatenate([np.linspace(-6, 6, 48001), [0.0, 1e-300, -1e-300, 30.0, -30.0]])
    np.testing.assert_allclose(mlp._erf(z), mlp._erf_scalar(z), rtol=0, atol=1e-15)


def test_slope_is_the_derivative():
    z = np.linspace(-5, 5, 101) + 0.013
    h = 1e-5
    fd = (mlp.act(z + h, "gelu") - mlp.act(z - h, "gelu")) / (2 * h)
    np.testing.assert_allclose(mlp.act_grad(z, "gelu"), fd, rtol=0, atol=1e-9)


@pytest.mark.parametrize("kind", mlp.KINDS)
def test_backward_against_central_differences(kind):
    rng = np.random.default_rng(3)
    M, K, N1, N2 = 5, 4, 6, 3
    X, W1, b1 = rng.normal(size=(M, K)), rng.normal(size=(K, N1)), rng.normal(size=N1)
    W2, b2, dY = rng.normal(size=(N1, N2)), rng.normal(size=N2), rng.normal(size=(M, N2))
    if kind == "relu":      # keep pre-activations away from the kink
        b1 = b1 + 0.0
    Z, H, Y = mlp.forward(X, W1, b1, W2, b2, kind)
    if kind == "relu":
        assert np.min(np.abs(Z)) > 1e-3
    g = mlp.backward(dY, X, W1, Z, H, W2, kind)

    def loss(**kw):
        a = dict(X=X, W1=W1, b1=b1, W2=W2, b2=b2)
        a.update(kw)
        return float(np.sum(dY * mlp.forward(a["X"], a["W1"], a["b1"], a["W2"], a["b2"], kind)[2]))

    h = 1e-6
    for name, grad in (("X", g["dX"]), ("W1", g["dW1"]), ("b1", g["db1"]), ("W2", g["dW2"]), ("b2", g["db2"])):
        base = dict(X=X, W1=W1, b1=b1, W2=W2, b2=b2)[name]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            up, dn = base.copy(), base.copy()
            up[it.multi_index] += h
            dn[it.multi_index] -= h
            fd[it.multi_index] = (loss(**{name: up}) - loss(**{name: dn})) / (2 * h)
        np.testing.assert_allclose(grad, fd, rtol=0, atol=2e-7, err_msg=name)


def test_rectifier_chain_is_exact_on_integers():
    rng = np.random.default_rng(9)
    X, W1 = rng.integers(-4, 5, (8, 6)).astype(float), rng.integers(-4, 5, (6, 10)).astype(float)
    W2, dY = rng.integers(-4, 5, (10, 4)).astype(float), rng.integers(-4, 5, (8, 4)).astype(float)
    b1, b2 = rng.integers(-4, 5, 10).astype(float), rng.integers(-4, 5, 4).astype(float)
    Z, H, Y = mlp.forward(X, W1, b1, W2, b2, "relu")
    np.testing.assert_array_equal(Z, X @ W1 + b1)
    np.testing.assert_array_equal(Y, np.maximum(Z, 0) @ W2 + b2)
    g = mlp.backward(dY, X, W1, Z, H, W2, "relu")
    dZ = (dY @ W2.T) * (Z > 0)
    np.testing.assert_array_equal(g["dX"], dZ @ W1.T)
    np.testing.assert_array_equal(g["dW1"], X.T @ dZ)
    np.testing.assert_array_equal(g["db1"], dZ.sum(0))
    np.testing.assert_array_equal(g["dW2"], H.T @ dY)


@pytest.mark.parametrize("q,M,K,N1", [(2, 8, 4, 16), (3, 18, 6, 27)])
def test_output_in_z_is_input_in_z_as_stored(q, M, K, N1):
    """Direction exchange (Section 3.1.1, last paragraph): what a layer that gathers in y leaves on
    each processor is exactly what the next layer, gathering in z, expects there; and the other way round."""
    Z = (np.arange(M)[:, None] * N1 + np.arange(N1)[None, :]).astype(float)
    for first, second in (("y", "z"), ("z", "y")):
        c1, c2 = Cube(q, M, K, N1, first), Cube(q, M, N1, q * q, second)
        np.testing.assert_array_equal(c1.shard_y(Z), c2.shard_x(Z))
