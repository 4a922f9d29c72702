"""Pins for the oracle of the three 3-D matrix products and their backward passes (CPU only).

Pinned by: operand slices worked out by hand in the pattern of Section 3.1.1's formulas
(golden file); the facts that the pieces of every placement tile the matrix exactly once,
that an all-gather rebuilds the stated block and that a reduce-scatter followed by an
all-gather is the plain sum; and the definitions themselves: Algorithms 1, 3, 5 must give
AB, AB^T, A^T B, Algorithms 2, 4, 6 the gradients of the three differentiation formulas
of Section 3.1.2, each checked against the plain product of the whole matrices (on
integers, bit for bit), against numpy's product, and by the adjoint identity.
"""
import os

import numpy as np
import pytest

from oracle import dist3d as d3
from oracle import matmul as om

PLAIN = {"AB": lambda a, b: om.forward(a, b), "ABT": lambda a, b: om.backward_dx(a, b),
         "ATB": lambda a, b: om.backward_dw(a, b)}
NUMPY = {"AB": lambda a, b: a @ b, "ABT": lambda a, b: a @ b.T, "ATB": lambda a, b: a.T @ b}


def _shapes(form, q, scale=1):
    """(A shape, B shape, C shape) with the divisibility each printed placement needs."""
    u = q * q * scale
    if form == "AB":
        return (u, u), (u, u), (u, u)
    if form == "ABT":
        return (u, 2 * u), (3 * u, 2 * u), (u, 3 * u)
    return (2 * u, u), (2 * u, 3 * u), (u, 3 * u)


def _ints(rng, shape):
    return rng.integers(-4, 5, size=shape).astype(np.float64)


def test_hand_derived_slices(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "placement_slices_q2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, rank, want = [p.strip() for p in line.split("|")]
        form, operand = name.split(".")
        pl = d3.PAPER[form]["ABC".index(operand)]
        r0, r1, c0, c1 = [int(v) for v in want.split()]
        assert pl.shard_slice(2, 8, 8, *[int(v) for v in rank.split()]) == (slice(r0, r1), slice(c0, c1)), line
        n += 1
    assert n == 21


@pytest.mark.parametrize("q", [1, 2, 3])
@pytest.mark.parametrize("pl", [d3.Placement(r, c, s) for r in d3.AXES for c in d3.AXES if r != c
                                for s in ("rows", "cols")])
def test_placement_tiles_and_collectives(q, pl):
    R, C = 2 * q * q, 3 * q * q
    T = (np.arange(R)[:, None] * C + np.arange(C)[None, :]).astype(np.float64)
    sh = d3.shard(T, q, pl)
    assert sh[0, 0, 0].size * q ** 3 == R * C                        # every processor holds 1/q^3
    np.testing.assert_array_equal(np.sort(sh.reshape(-1)), T.reshape(-1))
    np.testing.assert_array_equal(d3.unshard(sh, q, pl, R, C), T)
    blocks = d3.all_gather(sh, q, pl)
    for r in d3.ranks(q):
        np.testing.assert_array_equal(blocks[r], T[pl.block_slice(q, R, C, *r)])
    # reduce-scatter of q equal partials is q times the own piece; then the all-gather is the sum
    rs = d3.reduce_scatter(blocks, q, pl)
    np.testing.assert_array_equal(rs, q * sh)
    np.testing.assert_array_equal(d3.all_gather(rs, q, pl), q * blocks)


@pytest.mark.parametrize("form", d3.FORMS)
@pytest.mark.parametrize("q", [1, 2, 3])
def test_forward_is_the_plain_product(form, q):
    rng = np.random.default_rng(10 * q + len(form))
    sa, sb, sc = _shapes(form, q)
    A, B = _ints(rng, sa), _ints(rng, sb)
    C = d3.unshard(d3.forward(form, A, B, q), q, d3.PAPER[form][2], *sc)
    np.testing.assert_array_equal(C, PLAIN[form](A, B))
    np.testing.assert_array_equal(C, NUMPY[form](A, B))


@pytest.mark.parametrize("form", d3.FORMS)
@pytest.mark.parametrize("q", [1, 2, 3])
def test_backward_is_the_plain_gradient(form, q):
    rng = np.random.default_rng(100 * q + len(form))
    sa, sb, sc = _shapes(form, q)
    A, B, dC = _ints(rng, sa), _ints(rng, sb), _ints(rng, sc)
    pa, pb, _ = d3.PAPER[form]
    da, db = d3.backward(form, dC, A, B, q)
    dA, dB = d3.unshard(da, q, pa, *sa), d3.unshard(db, q, pb, *sb)
    # the three differentiation formulas of Section 3.1.2
    want = {"AB": lambda: (dC @ B.T, A.T @ dC), "ABT": lambda: (dC @ B, dC.T @ A),
            "ATB": lambda: (B @ dC.T, A @ dC)}[form]()
    np.testing.assert_array_equal(dA, want[0])
    np.testing.assert_array_equal(dB, want[1])
    # adjoint identity: <dC, f(A, B)> = <dA, A> = <dB, B> for the bilinear f (exact on integers)
    inner = float(np.sum(dC * PLAIN[form](A, B)))
    assert inner == float(np.sum(dA * A)) == float(np.sum(dB * B))


@pytest.mark.parametrize("form", d3.FORMS)
def test_real_data_and_identity(form):
    q = 2
    rng = np.random.default_rng(7)
    sa, sb, sc = _shapes(form, q, scale=2)
    A, B = rng.uniform(-1, 1, sa), rng.uniform(-1, 1, sb)
    C = d3.unshard(d3.forward(form, A, B, q), q, d3.PAPER[form][2], *sc)
    ref = NUMPY[form](A, B)
    assert np.max(np.abs(C - ref)) <= 1e-13 * np.max(np.abs(ref)) * sa[1]
    # a square identity as the second operand returns the first (transposed for A^T B)
    n = sa[1] if form != "ATB" else sa[0]
    if form == "ATB":
        out = d3.unshard(d3.forward(form, A, np.eye(n), q), q, d3.PAPER[form][2], sa[1], n)
        np.testing.assert_array_equal(out, A.T)


def test_single_block_meets_single_block():
    """Which blocks meet (the structure of the worked example of Section 2.3, for C = A B^T):
    with one non-zero block in A and one in B the result has at most one non-zero block, and it
    is there exactly when the two blocks share their contraction index."""
    q, u = 2, 4
    for ia in range(q):
        for la in range(q):
            for jb in range(q):
                for lb in range(q):
                    A, B = np.zeros((2 * u, 2 * u)), np.zeros((2 * u, 2 * u))
                    A[ia * u:(ia + 1) * u, la * u:(la + 1) * u] = 1.0
                    B[jb * u:(jb + 1) * u, lb * u:(lb + 1) * u] = 1.0
                    C = d3.unshard(d3.forward("ABT", A, B, q), q, d3.PAPER["ABT"][2], 2 * u, 2 * u)
                    want = np.zeros((2 * u, 2 * u))
                    if la == lb:
                        want[ia * u:(ia + 1) * u, jb * u:(jb + 1) * u] = u
                    np.testing.assert_array_equal(C, want)


def test_wrong_directions_are_refused():
    pa, pb, pc = d3.PAPER["AB"]
    with pytest.raises(ValueError):
        d3.check_directions("ABT", pa, pb, pc)          # B's contraction index is not along z there
    with pytest.raises(ValueError):
        d3.check_directions("AB", pa, pb, d3.Placement("y", "x", "rows"))   # result rows must stay along x
    with pytest.raises(ValueError):
        d3.Placement("x", "x", "rows")
    with pytest.raises(ValueError):
        d3.shard(np.zeros((6, 8)), 2, pa)               # 4 does not divide 6
