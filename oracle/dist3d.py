"""The three matrix-product forms on the cube, step by step (oracle; test infrastructure only).

Section 3.1.2 gives C = AB, C = AB^T and C = A^T B each as one forward algorithm
(Algorithms 1, 3, 5: all-gather the first operand, all-gather the second, multiply
locally, reduce-scatter the result) and one backward algorithm (Algorithms 2, 4, 6)
whose two lines are again products of these three forms with their directions
permuted.  This module writes those steps out with numpy slicing and the fp64 triple
loops of ``matmul``, for any placement of the three matrices on the cube, so that every
algorithm can be checked against the plain definition of the product it computes.

Readings.  Algorithms 5 and 6 reuse the letters i, j, l for other cube directions than
Algorithms 1-4 do: their A is gathered over its middle index l "in y", their B over j
"in x", their C reduced over i "in z"; so there i runs along z, j along x and l along y
(table ``PAPER`` below).  Algorithm 6 is printed with the caption of Algorithm 4 and
with subscripts that do not match its REQUIRE / ENSURE lines; it is taken as what the
third differentiation formula of Section 3.1.2 says, dA = B dC^T and dB = A dC, each
gradient in the placement of its matrix.

Placement of an ``[R, C]`` matrix (Section 3.1.1, generalised from the three cases
printed there).  The matrix is cut into q x q blocks; ``row_axis`` is the cube
direction whose index picks the row block, ``col_axis`` the direction whose index
picks the column block, and along the remaining direction (``sub_axis``) each block
is cut once more into q pieces, by rows or by columns (``split``).  In the paper's
subscripts the middle index of three cuts rows and the last index cuts columns:
``A_ijl`` is block (i, l) with rows cut by j, ``B_lji`` is block (l, j) with columns
cut by i.  The all-gather of a matrix runs along its ``sub_axis`` and rebuilds the
block; the reduce-scatter of a result runs along its ``sub_axis`` and leaves piece s on
the processor whose index along that direction is s.

Processor ``(i, j, l)`` has index i along x, j along y, l along z.  A cube array has
shape ``[q, q, q, rows, cols]`` indexed ``[i, j, l]``.
"""
import numpy as np

from . import matmul as _mm

AXES = ("x", "y", "z")


class Placement:
    def __init__(self, row_axis, col_axis, split):
        if row_axis not in AXES or col_axis not in AXES or row_axis == col_axis:
            raise ValueError("row_axis and col_axis are two different directions out of x, y, z")
        if split not in ("rows", "cols"):
            raise ValueError("split is 'rows' or 'cols'")
        self.row_axis, self.col_axis, self.split = row_axis, col_axis, split
        self.sub_axis = [a for a in AXES if a not in (row_axis, col_axis)][0]

    def __repr__(self):
        return "Placement(%s, %s, %s)" % (self.row_axis, self.col_axis, self.split)

    def check(self, q, R, C):
        need_r, need_c = (q * q, q) if self.split == "rows" else (q, q * q)
        if R % need_r or C % need_c:
            raise ValueError("%r needs %d | rows and %d | cols" % (self, need_r, need_c))

    def shard_shape(self, q, R, C):
        return (R // (q * q), C // q) if self.split == "rows" else (R // q, C // (q * q))

    def block_slice(self, q, R, C, i, j, l):
        """Block held after the all-gather along ``sub_axis``."""
        idx = {"x": i, "y": j, "z": l}
        rb, cb = idx[self.row_axis], idx[self.col_axis]
        Rb, Cb = R // q, C // q
        return slice(rb * Rb, (rb + 1) * Rb), slice(cb * Cb, (cb + 1) * Cb)

    def shard_slice(self, q, R, C, i, j, l):
        """Piece of the full matrix stored on processor (i, j, l)."""
        idx = {"x": i, "y": j, "z": l}
        rb, cb, s = idx[self.row_axis], idx[self.col_axis], idx[self.sub_axis]
        Rb, Cb = R // q, C // q
        if self.split == "rows":
            Rs = Rb // q
            return slice(rb * Rb + s * Rs, rb * Rb + (s + 1) * Rs), slice(cb * Cb, (cb + 1) * Cb)
        Cs = Cb // q
        return slice(rb * Rb, (rb + 1) * Rb), slice(cb * Cb + s * Cs, cb * Cb + (s + 1) * Cs)


def ranks(q):
    for i in range(q):
        for j in range(q):
            for l in range(q):
                yield i, j, l


def _moved(rank, axis, value):
    """The processor that differs from ``rank`` only in its index along ``axis``."""
    r = list(rank)
    r[AXES.index(axis)] = value
    return tuple(r)


def shard(T, q, pl):
    """Full matrix -> cube array of shards."""
    T = np.asarray(T)
    R, C = T.shape
    pl.check(q, R, C)
    out = np.empty((q, q, q) + pl.shard_shape(q, R, C), dtype=T.dtype)
    for r in ranks(q):
        out[r] = T[pl.shard_slice(q, R, C, *r)]
    return out


def unshard(shards, q, pl, R, C):
    """Cube array of shards -> full matrix; fails unless the pieces tile it exactly once."""
    shards = np.asarray(shards)
    pl.check(q, R, C)
    full = np.zeros((R, C), dtype=shards.dtype)
    count = np.zeros((R, C), dtype=np.int32)
    for r in ranks(q):
        s = pl.shard_slice(q, R, C, *r)
        full[s] = shards[r]
        count[s] += 1
    if not np.all(count == 1):
        raise AssertionError("shards do not tile the matrix exactly once")
    return full


def all_gather(shards, q, pl):
    """Along ``sub_axis``: every processor ends with its whole block (pieces in index order)."""
    shards = np.asarray(shards)
    cat = 0 if pl.split == "rows" else 1
    first = np.concatenate([shards[_moved((0, 0, 0), pl.sub_axis, s)] for s in range(q)], axis=cat)
    out = np.empty((q, q, q) + first.shape, dtype=shards.dtype)
    for r in ranks(q):
        out[r] = np.concatenate([shards[_moved(r, pl.sub_axis, s)] for s in range(q)], axis=cat)
    return out


def reduce_scatter(partials, q, pl):
    """Along ``sub_axis``: fp64 sum of the q partial blocks; the processor with index s keeps piece s."""
    partials = np.asarray(partials, dtype=np.float64)
    Rb, Cb = partials.shape[3:]
    shape = (Rb // q, Cb) if pl.split == "rows" else (Rb, Cb // q)
    out = np.empty((q, q, q) + shape, dtype=np.float64)
    for r in ranks(q):
        s = r[AXES.index(pl.sub_axis)]
        acc = np.zeros((Rb, Cb), dtype=np.float64)
        for s2 in range(q):
            acc += partials[_moved(r, pl.sub_axis, s2)]
        out[r] = acc[s * shape[0]:(s + 1) * shape[0], :] if pl.split == "rows" else \
            acc[:, s * shape[1]:(s + 1) * shape[1]]
    return out


FORMS = ("AB", "ABT", "ATB")


def local_product(form, a, b):
    """One processor's product of its two gathered blocks: the plain fp64 triple loops."""
    if form == "AB":
        return _mm.forward(a, b)
    if form == "ABT":
        return _mm.backward_dx(a, b)      # a b^T
    if form == "ATB":
        return _mm.backward_dw(a, b)      # a^T b
    raise ValueError("form is one of %r" % (FORMS,))


def check_directions(form, pa, pb, pc):
    """The condition under which the four steps below compute the product: the contraction
    index of both operands runs along one direction, which is the direction the result is
    reduce-scattered in; the free index of each operand keeps its direction in the result."""
    a_free, a_con = (pa.row_axis, pa.col_axis) if form != "ATB" else (pa.col_axis, pa.row_axis)
    b_con, b_free = (pb.row_axis, pb.col_axis) if form != "ABT" else (pb.col_axis, pb.row_axis)
    ok = a_con == b_con == pc.sub_axis and a_free == pc.row_axis and b_free == pc.col_axis
    if not ok:
        raise ValueError("placements %r, %r, %r do not form a 3-D %s product" % (pa, pb, pc, form))


def matmul_3d(form, a_shards, b_shards, q, pa, pb, pc):
    """Algorithms 1 / 3 / 5 (and each line of Algorithms 2 / 4 / 6): all-gather the first
    operand, all-gather the second, multiply locally, reduce-scatter the result."""
    check_directions(form, pa, pb, pc)
    a_blocks = all_gather(a_shards, q, pa)                                   # step 1
    b_blocks = all_gather(b_shards, q, pb)                                   # step 2
    first = local_product(form, a_blocks[0, 0, 0], b_blocks[0, 0, 0])
    partial = np.empty((q, q, q) + first.shape, dtype=np.float64)
    for r in ranks(q):
        partial[r] = local_product(form, a_blocks[r], b_blocks[r])           # step 3
    return reduce_scatter(partial, q, pc)                                    # step 4


# ---- the placements the paper's six algorithms print ("directions y, x, z for A, B, C") ------------------
# Algorithm 1 / 2:  A_ijl [M,K], B_lji [K,N], C_ilj [M,N]
# Algorithm 3 / 4:  A_ijl [M,K], B_jli [N,K], C_ilj [M,N]
# Algorithm 5 / 6:  A_ilj [K,M], B_ijl [K,N], C_jli [M,N]; its letters stand for other directions than in
#                   Algorithms 1-4: A is gathered over l "in y", B over j "in x", C reduced over i "in z"
PAPER = {
    "AB": (Placement("x", "z", "rows"), Placement("z", "y", "cols"), Placement("x", "y", "rows")),
    "ABT": (Placement("x", "z", "rows"), Placement("y", "z", "cols"), Placement("x", "y", "rows")),
    "ATB": (Placement("z", "x", "rows"), Placement("z", "y", "rows"), Placement("x", "y", "cols")),
}


def forward(form, A, B, q):
    """Algorithm 1, 3 or 5 on full matrices: shard, run the four steps, return the cube array of C."""
    pa, pb, pc = PAPER[form]
    return matmul_3d(form, shard(A, q, pa), shard(B, q, pb), q, pa, pb, pc)


def backward(form, dC, A, B, q):
    """Algorithm 2, 4 or 6: the two gradient products, each a 3-D product of one of the three
    forms with the placements of its operands as they are stored; gradients come out in the
    placement of the matrix they belong to."""
    pa, pb, pc = PAPER[form]
    a, b, g = shard(A, q, pa), shard(B, q, pb), shard(dC, q, pc)
    if form == "AB":        # dA = dC B^T, dB = A^T dC
        return matmul_3d("ABT", g, b, q, pc, pb, pa), matmul_3d("ATB", a, g, q, pa, pc, pb)
    if form == "ABT":       # dA = dC B, dB = dC^T A
        return matmul_3d("AB", g, b, q, pc, pb, pa), matmul_3d("ATB", g, a, q, pc, pa, pb)
    if form == "ATB":       # dA = B dC^T, dB = A dC
        return matmul_3d("ABT", b, g, q, pb, pc, pa), matmul_3d("AB", a, g, q, pa, pc, pb)
    raise ValueError("form is one of %r" % (FORMS,))
