"""Load-balanced storage and the axis collectives of the 3-D linear layer (oracle).

Follows Section 3.1.1 (which slice of each matrix a processor holds, what the
two all-gathers rebuild, what the reduce-scatter leaves) and the direction
triples of Algorithms 1 and 2.  Everything is numpy slicing and fp64 sums
written from those index formulas; the slice ends, printed inclusive in the
paper, are half-open here.

Notation: ``X [M,K]`` is the paper's A, ``W [K,N]`` its B, ``Y [M,N]`` its C;
``q`` is the cube edge (the paper's p).  ``Mb, Kb, Nb = M/q, K/q, N/q`` are the
block sizes and ``Ms, Ns = M/q^2, N/q^2`` the shard sizes.

Directions.  Processor ``(i, j, l)`` sits at index ``i`` along x, ``j`` along y,
``l`` along z.  Weights always travel along x.  ``in_axis`` is the direction in
which the input is gathered: ``"y"`` for the layout printed in the paper
(input gathered in y, output reduce-scattered in z) and ``"z"`` for a layer
that consumes the previous layer's output, where the two are exchanged
(Section 3.1.1, last paragraph).  ``a`` below is a processor's index along the
input direction and ``b`` its index along the output direction, so the printed
formulas apply with ``(j, l)`` replaced by ``(a, b)``.

A cube array has shape ``[q, q, q, rows, cols]`` indexed ``[i, j, l]``; flattened
in C order it is the buffer convention ``r = (i*q + j)*q + l``, blocks packed
back to back.
"""
import numpy as np


class Cube:
    def __init__(self, q, M, K, N, in_axis="y"):
        if q < 1:
            raise ValueError("q must be positive")
        if M % (q * q) or N % (q * q) or K % q:
            raise ValueError("q^2 must divide M and N, and q must divide K")
        if in_axis not in ("y", "z"):
            raise ValueError("in_axis is 'y' or 'z'")
        self.q, self.M, self.K, self.N = q, M, K, N
        self.in_axis = in_axis
        self.Mb, self.Kb, self.Nb = M // q, K // q, N // q
        self.Ms, self.Ns = M // (q * q), N // (q * q)

    # ---- coordinates -------------------------------------------------------
    def ab(self, i, j, l):
        """Index along the input direction and along the output direction."""
        return (j, l) if self.in_axis == "y" else (l, j)

    def rank_of(self, i, a, b):
        """Physical ``(i, j, l)`` of the processor with input index a, output index b."""
        return (i, a, b) if self.in_axis == "y" else (i, b, a)

    def ranks(self):
        q = self.q
        for i in range(q):
            for j in range(q):
                for l in range(q):
                    yield i, j, l

    # ---- which slice a processor holds (Section 3.1.1) ---------------------
    def x_shard_slice(self, i, j, l):
        a, b = self.ab(i, j, l)
        r0 = i * self.Mb + a * self.Ms
        return slice(r0, r0 + self.Ms), slice(b * self.Kb, (b + 1) * self.Kb)

    def w_shard_slice(self, i, j, l):
        a, b = self.ab(i, j, l)
        c0 = a * self.Nb + i * self.Ns
        return slice(b * self.Kb, (b + 1) * self.Kb), slice(c0, c0 + self.Ns)

    def y_shard_slice(self, i, j, l):
        a, b = self.ab(i, j, l)
        r0 = i * self.Mb + b * self.Ms
        return slice(r0, r0 + self.Ms), slice(a * self.Nb, (a + 1) * self.Nb)

    # ---- what the all-gathers rebuild (Section 3.1.1) ----------------------
    def x_block_slice(self, i, j, l):
        a, b = self.ab(i, j, l)
        return slice(i * self.Mb, (i + 1) * self.Mb), slice(b * self.Kb, (b + 1) * self.Kb)

    def w_block_slice(self, i, j, l):
        a, b = self.ab(i, j, l)
        return slice(b * self.Kb, (b + 1) * self.Kb), slice(a * self.Nb, (a + 1) * self.Nb)

    def y_block_slice(self, i, j, l):
        a, b = self.ab(i, j, l)
        return slice(i * self.Mb, (i + 1) * self.Mb), slice(a * self.Nb, (a + 1) * self.Nb)

    # ---- full matrix -> cube array -----------------------------------------
    def _cut(self, full, shape, slicer):
        full = np.asarray(full)
        if full.shape != shape:
            raise ValueError("matrix has shape %r, expected %r" % (full.shape, shape))
        q = self.q
        first = full[slicer(0, 0, 0)]
        out = np.empty((q, q, q) + first.shape, dtype=full.dtype)
        for i, j, l in self.ranks():
            out[i, j, l] = full[slicer(i, j, l)]
        return out

    def shard_x(self, X):
        return self._cut(X, (self.M, self.K), self.x_shard_slice)

    def shard_w(self, W):
        return self._cut(W, (self.K, self.N), self.w_shard_slice)

    def shard_y(self, Y):
        return self._cut(Y, (self.M, self.N), self.y_shard_slice)

    def block_x(self, X):
        return self._cut(X, (self.M, self.K), self.x_block_slice)

    def block_w(self, W):
        return self._cut(W, (self.K, self.N), self.w_block_slice)

    def block_y(self, Y):
        return self._cut(Y, (self.M, self.N), self.y_block_slice)

    # ---- cube array of shards -> full matrix -------------------------------
    def _paste(self, shards, shape, slicer):
        shards = np.asarray(shards)
        full = np.zeros(shape, dtype=shards.dtype)
        count = np.zeros(shape, dtype=np.int32)
        for i, j, l in self.ranks():
            s = slicer(i, j, l)
            full[s] = shards[i, j, l]
            count[s] += 1
        if not np.all(count == 1):
            raise AssertionError("shards do not tile the matrix exactly once")
        return full

    def unshard_x(self, shards):
        return self._paste(shards, (self.M, self.K), self.x_shard_slice)

    def unshard_w(self, shards):
        return self._paste(shards, (self.K, self.N), self.w_shard_slice)

    def unshard_y(self, shards):
        return self._paste(shards, (self.M, self.N), self.y_shard_slice)

    # ---- all-gathers (Algorithm 1 steps 1-2; Algorithm 2 for dY) ------------
    def all_gather_x(self, shards):
        """Input direction: row-concatenate the q shards of processors ``(i, ., b)``."""
        q = self.q
        out = np.empty((q, q, q, self.Mb, self.Kb), dtype=np.asarray(shards).dtype)
        for i, j, l in self.ranks():
            a, b = self.ab(i, j, l)
            out[i, j, l] = np.concatenate(
                [shards[self.rank_of(i, a2, b)] for a2 in range(q)], axis=0)
        return out

    def all_gather_w(self, shards):
        """Direction x: column-concatenate the q shards of processors ``(., a, b)``."""
        q = self.q
        out = np.empty((q, q, q, self.Kb, self.Nb), dtype=np.asarray(shards).dtype)
        for i, j, l in self.ranks():
            a, b = self.ab(i, j, l)
            out[i, j, l] = np.concatenate(
                [shards[self.rank_of(i2, a, b)] for i2 in range(q)], axis=1)
        return out

    def all_gather_y(self, shards):
        """Output direction: row-concatenate the q shards of processors ``(i, a, .)``."""
        q = self.q
        out = np.empty((q, q, q, self.Mb, self.Nb), dtype=np.asarray(shards).dtype)
        for i, j, l in self.ranks():
            a, b = self.ab(i, j, l)
            out[i, j, l] = np.concatenate(
                [shards[self.rank_of(i, a, b2)] for b2 in range(q)], axis=0)
        return out

    # ---- reduce-scatters (Algorithm 1 step 4; Algorithm 2 third directions) -
    def reduce_scatter_y(self, partials):
        """Sum over the output direction; processor b keeps row panel b."""
        q, Ms = self.q, self.Ms
        out = np.empty((q, q, q, Ms, self.Nb), dtype=np.float64)
        for i, j, l in self.ranks():
            a, b = self.ab(i, j, l)
            acc = np.zeros((Ms, self.Nb), dtype=np.float64)
            for b2 in range(q):
                acc += np.asarray(partials[self.rank_of(i, a, b2)],
                                  dtype=np.float64)[b * Ms:(b + 1) * Ms, :]
            out[i, j, l] = acc
        return out

    def reduce_scatter_dx(self, partials):
        """Sum over the input direction; processor a keeps row panel a."""
        q, Ms = self.q, self.Ms
        out = np.empty((q, q, q, Ms, self.Kb), dtype=np.float64)
        for i, j, l in self.ranks():
            a, b = self.ab(i, j, l)
            acc = np.zeros((Ms, self.Kb), dtype=np.float64)
            for a2 in range(q):
                acc += np.asarray(partials[self.rank_of(i, a2, b)],
                                  dtype=np.float64)[a * Ms:(a + 1) * Ms, :]
            out[i, j, l] = acc
        return out

    def reduce_scatter_dw(self, partials):
        """Sum over direction x; processor i keeps column panel i."""
        q, Ns = self.q, self.Ns
        out = np.empty((q, q, q, self.Kb, Ns), dtype=np.float64)
        for i, j, l in self.ranks():
            a, b = self.ab(i, j, l)
            acc = np.zeros((self.Kb, Ns), dtype=np.float64)
            for i2 in range(q):
                acc += np.asarray(partials[self.rank_of(i2, a, b)],
                                  dtype=np.float64)[:, i * Ns:(i + 1) * Ns]
            out[i, j, l] = acc
        return out

    # ---- vector parameters (Section 3.1.1, the paragraph on vectors; Algorithms 7 and 8) -----
    # A vector b of length N lives on the diagonal of the weight plane: only processors whose
    # y and z indices coincide hold a piece, b[j*Nb + i*Ns : +Ns] on processor (i, j, j).  For the
    # output-side add Y + b the pieces are broadcast along the output direction and all-gathered
    # along x, so that every processor has the Nb entries of its output block.  The printed
    # backward (Algorithm 8) only reduce-scatters along x on the diagonal; the broadcast's own
    # adjoint, a reduce along the broadcast direction onto the diagonal, is needed before it or
    # the rows held off the diagonal would be lost.  Both are taken here.
    def holds_bias(self, i, j, l):
        return j == l

    def bias_shard_slice(self, i, j, l):
        """Slice of b held by the diagonal processor (i, j, l = j)."""
        if j != l:
            raise ValueError("only diagonal processors hold vector parameters")
        s0 = j * self.Nb + i * self.Ns
        return slice(s0, s0 + self.Ns)

    def shard_bias(self, b, fill=0.0):
        """Vector of length N -> cube array [q,q,q,Ns]; processors off the diagonal get `fill`."""
        b = np.asarray(b)
        if b.shape != (self.N,):
            raise ValueError("bias has shape %r, expected (%d,)" % (b.shape, self.N))
        q = self.q
        out = np.full((q, q, q, self.Ns), fill, dtype=b.dtype)
        for i, j, l in self.ranks():
            if j == l:
                out[i, j, l] = b[self.bias_shard_slice(i, j, l)]
        return out

    def unshard_bias(self, shards):
        shards = np.asarray(shards)
        b = np.zeros((self.N,), dtype=shards.dtype)
        count = np.zeros((self.N,), dtype=np.int32)
        for i, j, l in self.ranks():
            if j == l:
                s = self.bias_shard_slice(i, j, l)
                b[s] = shards[i, j, l]
                count[s] += 1
        if not np.all(count == 1):
            raise AssertionError("bias pieces do not tile the vector exactly once")
        return b

    def gather_bias(self, shards):
        """Algorithm 7 steps 1-2 for the output-side add: every processor gets the Nb entries
        of its output block (block index = its index a along the input direction)."""
        q = self.q
        out = np.empty((q, q, q, self.Nb), dtype=np.asarray(shards).dtype)
        for i, j, l in self.ranks():
            a, _ = self.ab(i, j, l)
            out[i, j, l] = np.concatenate([shards[i2, a, a] for i2 in range(q)])
        return out

    def add_bias(self, y_shards, bias_blocks):
        """Algorithm 7 step 3 on the output shards [Ms, Nb]: every row gets the block's bias."""
        return np.asarray(y_shards, dtype=np.float64) + np.asarray(bias_blocks, dtype=np.float64)[:, :, :, None, :]

    def bias_backward(self, dy_shards):
        """Algorithm 8: column sums of every processor's dY shard, reduced along the output
        direction onto the diagonal and reduce-scattered along x; zeros off the diagonal."""
        q, Ns = self.q, self.Ns
        out = np.zeros((q, q, q, Ns), dtype=np.float64)
        for i, j, l in self.ranks():
            if j != l:
                continue
            blk = j                         # the diagonal index is the output-block index
            acc = np.zeros((Ns,), dtype=np.float64)
            for i2 in range(q):
                for b2 in range(q):
                    sh = np.asarray(dy_shards[self.rank_of(i2, blk, b2)], dtype=np.float64)
                    acc += sh[:, i * Ns:(i + 1) * Ns].sum(axis=0)
            out[i, j, l] = acc
        return out

    # ---- cost formulas (Section 3.1.1 memory, Section 3.1.2 compute/comm) ---
    def memory_per_rank(self):
        return self.Ms * self.Kb + self.Kb * self.Ns + self.Ms * self.Nb

    def multiply_adds_per_rank(self):
        return self.Mb * self.Kb * self.Nb

    def forward_elements_moved_per_rank(self):
        return (self.M * self.K + self.K * self.N + self.M * self.N) // self.q ** 3
