"""Pins for the oracle's storage layout and axis collectives (CPU only).

Pinned by: slices worked out by hand from Section 3.1.1's index formulas
(golden file), the symbolic 2x2x2 example of Section 2.3 (golden file), the
facts that shards are a permutation of the matrix and gathers rebuild the
stated blocks, the cost formulas of Sections 3.1.1 / 3.1.2, and the invariant
that the whole 3-D pipeline reproduces the plain products.
"""
import os

import numpy as np
import pytest

from oracle import matmul as om
from oracle.layout import Cube

CASES = [(1, 3, 2, 5, "y"), (2, 8, 4, 8, "y"), (2, 8, 4, 8, "z"), (2, 8, 8, 8, "y"),
         (3, 18, 6, 27, "y"), (3, 18, 6, 27, "z"), (2, 12, 10, 4, "z")]


def _ramp(rows, cols):
    return (np.arange(rows)[:, None] * cols + np.arange(cols)[None, :]).astype(np.float64)


def _slc(vals):
    r0, r1, c0, c1 = vals
    return slice(r0, r1), slice(c0, c1)


def test_hand_derived_slices(golden_dir):
    cube = Cube(2, 8, 4, 8, "y")
    n = 0
    for line in open(os.path.join(golden_dir, "shard_slices_q2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        parts = [[int(v) for v in p.split()] for p in line.split("|")]
        (i, j, l), xs, ws, ys = parts
        assert cube.x_shard_slice(i, j, l) == _slc(xs)
        assert cube.w_shard_slice(i, j, l) == _slc(ws)
        assert cube.y_shard_slice(i, j, l) == _slc(ys)
        n += 1
    assert n == 8


@pytest.mark.parametrize("q,M,K,N,ax", CASES)
def test_shards_are_a_permutation(q, M, K, N, ax):
    cube = Cube(q, M, K, N, ax)
    for full, shard, unshard in ((_ramp(M, K), cube.shard_x, cube.unshard_x),
                                 (_ramp(K, N), cube.shard_w, cube.unshard_w),
                                 (_ramp(M, N), cube.shard_y, cube.unshard_y)):
        sh = shard(full)
        np.testing.assert_array_equal(np.sort(sh.reshape(-1)), full.reshape(-1))
        np.testing.assert_array_equal(unshard(sh), full)
    sizes = cube.shard_x(_ramp(M, K))[0, 0, 0].size + cube.shard_w(_ramp(K, N))[0, 0, 0].size \
        + cube.shard_y(_ramp(M, N))[0, 0, 0].size
    assert sizes == cube.memory_per_rank() == (M // q**2) * (K // q) + (K // q) * (N // q**2) + (M // q**2) * (N // q)
    assert q**3 * cube.memory_per_rank() == M * K + K * N + M * N


@pytest.mark.parametrize("q,M,K,N,ax", CASES)
def test_gathers_rebuild_the_stated_blocks(q, M, K, N, ax):
    cube = Cube(q, M, K, N, ax)
    X, W, Y = _ramp(M, K), _ramp(K, N) + 0.5, _ramp(M, N) + 0.25
    np.testing.assert_array_equal(cube.all_gather_x(cube.shard_x(X)), cube.block_x(X))
    np.testing.assert_array_equal(cube.all_gather_w(cube.shard_w(W)), cube.block_w(W))
    np.testing.assert_array_equal(cube.all_gather_y(cube.shard_y(Y)), cube.block_y(Y))
    # the blocks are the plain q x q partitions, replicated along the gather direction
    Mb, Kb, Nb = M // q, K // q, N // q
    for i, j, l in cube.ranks():
        a, b = cube.ab(i, j, l)
        np.testing.assert_array_equal(cube.block_x(X)[i, j, l], X[i*Mb:(i+1)*Mb, b*Kb:(b+1)*Kb])
        np.testing.assert_array_equal(cube.block_w(W)[i, j, l], W[b*Kb:(b+1)*Kb, a*Nb:(a+1)*Nb])
        np.testing.assert_array_equal(cube.block_y(Y)[i, j, l], Y[i*Mb:(i+1)*Mb, a*Nb:(a+1)*Nb])
    if ax == "y":
        i, j, l = q - 1, 0, q - 1
        assert cube.ab(i, j, l) == (j, l)
    # "gather, then keep your own piece" is the identity
    gx = cube.all_gather_x(cube.shard_x(X))
    Ms = M // q**2
    for i, j, l in cube.ranks():
        a, _ = cube.ab(i, j, l)
        np.testing.assert_array_equal(gx[i, j, l][a*Ms:(a+1)*Ms], cube.shard_x(X)[i, j, l])


def test_worked_example_2x2x2(golden_dir):
    """Each output block is made of exactly the terms the paper's example lists."""
    q, bs = 2, 3
    M = K = N = q * q * bs          # blocks are 6x6, big enough to shard again
    cube = Cube(q, M, K, N, "y")
    Mb = M // q
    rng = np.random.default_rng(4)
    listed = {}
    for line in open(os.path.join(golden_dir, "cube_2x2x2_terms.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, terms = line.split(":")
        i, j = (int(v) for v in head.split())
        listed[(i, j)] = [((int(t[1]), int(t[2])), (int(t[5]), int(t[6]))) for t in terms.split()]
    assert len(listed) == 4
    for (ai, al) in np.ndindex(2, 2):
        for (bl, bj) in np.ndindex(2, 2):
            # one non-zero block in X (at (ai,al)) and one in W (at (bl,bj))
            XA = rng.integers(1, 5, size=(Mb, Mb)).astype(np.float64)
            WB = rng.integers(1, 5, size=(Mb, Mb)).astype(np.float64)
            X = np.zeros((M, K)); X[ai*Mb:(ai+1)*Mb, al*Mb:(al+1)*Mb] = XA
            W = np.zeros((K, N)); W[bl*Mb:(bl+1)*Mb, bj*Mb:(bj+1)*Mb] = WB
            gx = cube.all_gather_x(cube.shard_x(X))
            gw = cube.all_gather_w(cube.shard_w(W))
            P = np.stack([om.forward(gx[r], gw[r]) for r in np.ndindex(2, 2, 2)]).reshape(2, 2, 2, Mb, Mb)
            Y = cube.unshard_y(cube.reduce_scatter_y(P))
            for (i, j), terms in listed.items():
                present = ((ai, al), (bl, bj)) in terms
                blk = Y[i*Mb:(i+1)*Mb, j*Mb:(j+1)*Mb]
                if present:
                    np.testing.assert_array_equal(blk, XA @ WB)
                    # and it was produced on processor (i, j, l = al) alone
                    for l in range(2):
                        assert np.any(P[i, j, l]) == (l == al)
                else:
                    assert not np.any(blk)


@pytest.mark.parametrize("q,M,K,N,ax", CASES)
def test_reduce_scatter_invariants(q, M, K, N, ax):
    cube = Cube(q, M, K, N, ax)
    Mb, Kb, Nb = M // q, K // q, N // q
    rng = np.random.default_rng(q * 100 + M)
    # q equal partials -> q times the kept piece
    base = rng.integers(-4, 5, size=(Mb, Nb)).astype(np.float64)
    same = np.broadcast_to(base, (q, q, q, Mb, Nb)).copy()
    rs = cube.reduce_scatter_y(same)
    Ms = M // q**2
    for i, j, l in cube.ranks():
        _, b = cube.ab(i, j, l)
        np.testing.assert_array_equal(rs[i, j, l], q * base[b*Ms:(b+1)*Ms])
    # reduce-scatter followed by all-gather is the plain sum over the direction
    P = rng.integers(-4, 5, size=(q, q, q, Mb, Nb)).astype(np.float64)
    back = cube.all_gather_y(cube.reduce_scatter_y(P))
    for i, j, l in cube.ranks():
        a, _ = cube.ab(i, j, l)
        total = sum(P[cube.rank_of(i, a, b2)] for b2 in range(q))
        np.testing.assert_array_equal(back[i, j, l], total)
    Q = rng.integers(-4, 5, size=(q, q, q, Mb, Kb)).astype(np.float64)
    back = cube.all_gather_x(cube.reduce_scatter_dx(Q))
    for i, j, l in cube.ranks():
        _, b = cube.ab(i, j, l)
        np.testing.assert_array_equal(back[i, j, l], sum(Q[cube.rank_of(i, a2, b)] for a2 in range(q)))
    R = rng.integers(-4, 5, size=(q, q, q, Kb, Nb)).astype(np.float64)
    back = cube.all_gather_w(cube.reduce_scatter_dw(R))
    for i, j, l in cube.ranks():
        a, b = cube.ab(i, j, l)
        np.testing.assert_array_equal(back[i, j, l], sum(R[cube.rank_of(i2, a, b)] for i2 in range(q)))


@pytest.mark.parametrize("q,M,K,N,ax", CASES)
def test_pipeline_reproduces_the_plain_products(q, M, K, N, ax):
    """Algorithms 1 and 2 end to end on the CPU equal XW, dY W^T and X^T dY."""
    cube = Cube(q, M, K, N, ax)
    rng = np.random.default_rng(17)
    X = rng.integers(-4, 5, size=(M, K)).astype(np.float64)
    W = rng.integers(-4, 5, size=(K, N)).astype(np.float64)
    G = rng.integers(-4, 5, size=(M, N)).astype(np.float64)
    gx = cube.all_gather_x(cube.shard_x(X))
    gw = cube.all_gather_w(cube.shard_w(W))
    gg = cube.all_gather_y(cube.shard_y(G))
    idx = list(cube.ranks())
    shape = (q, q, q)
    P = np.stack([om.forward(gx[r], gw[r]) for r in idx]).reshape(shape + (M // q, N // q))
    Qp = np.stack([om.backward_dx(gg[r], gw[r]) for r in idx]).reshape(shape + (M // q, K // q))
    Rp = np.stack([om.backward_dw(gx[r], gg[r]) for r in idx]).reshape(shape + (K // q, N // q))
    np.testing.assert_array_equal(cube.unshard_y(cube.reduce_scatter_y(P)), om.forward(X, W))
    np.testing.assert_array_equal(cube.unshard_x(cube.reduce_scatter_dx(Qp)), om.backward_dx(G, W))
    np.testing.assert_array_equal(cube.unshard_w(cube.reduce_scatter_dw(Rp)), om.backward_dw(X, G))
    # the l-sum of the per-processor products is the output block
    Y = om.forward(X, W)
    Mb, Nb = M // q, N // q
    for i in range(q):
        for a in range(q):
            tot = sum(P[cube.rank_of(i, a, b)] for b in range(q))
            np.testing.assert_array_equal(tot, Y[i*Mb:(i+1)*Mb, a*Nb:(a+1)*Nb])
    assert cube.multiply_adds_per_rank() * q**3 == M * K * N


def test_direction_exchange_chains_layers_without_data_movement():
    """A layer's output shards are, as stored, the next layer's input shards once
    the input and output directions are exchanged (Section 3.1.1, last paragraph)."""
    q, M, K1, N1, N2 = 2, 8, 4, 12, 8
    first = Cube(q, M, K1, N1, "y")
    second = Cube(q, M, N1, N2, "z")
    H = _ramp(M, N1)
    np.testing.assert_array_equal(first.shard_y(H), second.shard_x(H))
    third = Cube(q, M, N2, K1, "y")
    H2 = _ramp(M, N2)
    np.testing.assert_array_equal(second.shard_y(H2), third.shard_x(H2))


def test_cost_formulas():
    cube = Cube(4, 8192, 2048, 8192)
    assert cube.multiply_adds_per_rank() == 2048 * 512 * 2048
    assert cube.memory_per_rank() == 512 * 512 + 512 * 512 + 512 * 2048
    assert cube.forward_elements_moved_per_rank() == (8192 * 2048 + 2048 * 8192 + 8192 * 8192) // 64
    # what the gathers receive and the reduce-scatter sends, per processor, is q times that minus own part
    assert cube.Mb * cube.Kb + cube.Kb * cube.Nb + cube.Mb * cube.Nb == 4 * cube.memory_per_rank()


def test_bad_shapes_rejected():
    for args in ((2, 6, 4, 8), (2, 8, 3, 8), (2, 8, 4, 6), (0, 8, 4, 8)):
        with pytest.raises(ValueError):
            Cube(*args)
    with pytest.raises(ValueError):
        Cube(2, 8, 4, 8, "x")
