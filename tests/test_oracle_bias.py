"""Pins for the oracle's vector-parameter (bias) layout and Algorithms 7 / 8 (CPU only)."""
import os

import numpy as np
import pytest

from oracle import matmul as om
from oracle.layout import Cube

CASES = [(1, 3, 2, 5, "y"), (2, 8, 4, 8, "y"), (2, 8, 4, 8, "z"), (3, 18, 6, 27, "y"), (3, 18, 6, 27, "z")]


def test_hand_derived_bias_slices(golden_dir):
    cube = Cube(2, 8, 4, 8, "y")
    held = {}
    for line in open(os.path.join(golden_dir, "bias_slices_q2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        (i, j, l), (s0, s1) = ([int(v) for v in p.split()] for p in line.split("|"))
        held[(i, j, l)] = slice(s0, s1)
    assert len(held) == 4
    for i, j, l in cube.ranks():
        assert cube.holds_bias(i, j, l) == ((i, j, l) in held)
        if (i, j, l) in held:
            assert cube.bias_shard_slice(i, j, l) == held[(i, j, l)]
        else:
            with pytest.raises(ValueError):
                cube.bias_shard_slice(i, j, l)


@pytest.mark.parametrize("q,M,K,N,ax", CASES)
def test_bias_pieces_tile_the_vector_and_gather_rebuilds_blocks(q, M, K, N, ax):
    cube = Cube(q, M, K, N, ax)
    b = np.arange(N, dtype=np.float64) + 0.5
    sh = cube.shard_bias(b, fill=np.nan)
    held = sh[~np.isnan(sh)]
    np.testing.assert_array_equal(np.sort(held), b)          # each entry exactly once, on the diagonal
    assert held.size == N and sh.shape == (q, q, q, N // q**2)
    np.testing.assert_array_equal(cube.unshard_bias(np.nan_to_num(sh)), b)
    blocks = cube.gather_bias(sh)
    Nb = N // q
    for i, j, l in cube.ranks():
        a, _ = cube.ab(i, j, l)
        # the block a processor needs is the one its output block's columns fall in
        np.testing.assert_array_equal(blocks[i, j, l], b[cube.y_block_slice(i, j, l)[1]])
        np.testing.assert_array_equal(blocks[i, j, l], b[a * Nb:(a + 1) * Nb])


@pytest.mark.parametrize("q,M,K,N,ax", CASES)
def test_linear_with_bias_end_to_end(q, M, K, N, ax):
    """Algorithm 1 followed by Algorithm 7 equals X W + b; Algorithm 8 equals the column sums of dY."""
    cube = Cube(q, M, K, N, ax)
    rng = np.random.default_rng(23)
    X = rng.integers(-4, 5, size=(M, K)).astype(np.float64)
    W = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    b = rng.integers(-4, 5, size=(N,)).astype(np.float64)
    G = rng.integers(-4, 5, size=(M, N)).astype(np.float64)
    gx, gw = cube.all_gather_x(cube.shard_x(X)), cube.all_gather_w(cube.shard_w(W))
    P = np.stack([om.forward(gx[r], gw[r]) for r in cube.ranks()]).reshape((q, q, q, M // q, N // q))
    ys = cube.add_bias(cube.reduce_scatter_y(P), cube.gather_bias(cube.shard_bias(b)))
    np.testing.assert_array_equal(cube.unshard_y(ys), X @ W + b[None, :])
    db = cube.bias_backward(cube.shard_y(G))
    np.testing.assert_array_equal(cube.unshard_bias(db), G.sum(axis=0))
    for i, j, l in cube.ranks():
        if j != l:
            assert not np.any(db[i, j, l])
    # adjoint of the broadcast add: <dY, 1 b^T> = <db, b>
    assert float(np.sum(G * b[None, :])) == float(np.sum(cube.unshard_bias(db) * b))


def test_bias_backward_closed_form():
    # dY[r, c] = r + 2c  ->  db[c] = S1(M) + 2 c M
    q, M, K, N = 2, 8, 4, 12
    cube = Cube(q, M, K, N, "z")
    r = np.arange(M)[:, None].astype(np.float64)
    c = np.arange(N)[None, :].astype(np.float64)
    db = cube.unshard_bias(cube.bias_backward(cube.shard_y(r + 2 * c)))
    np.testing.assert_array_equal(db, M * (M - 1) / 2 + 2 * np.arange(N) * M)
