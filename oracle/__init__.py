"""CPU oracle for the 3-D parallel linear layer (test infrastructure only).

Nothing under this directory is part of the product path.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import it.  It imports nothing from the HIP package and shares no code with it.

Modules
-------
matmul    the three plain products (Section 3.1.2, first differentiation
          formula), fp64, via the C file ``cube3d_oracle.c``
layout    the load-balanced storage of Section 3.1.1 and the all-gather /
          reduce-scatter steps of Algorithms 1 and 2, as numpy slicing
dist3d    the three matrix-product forms of Section 3.1.2 on the cube, forward and
          backward (Algorithms 1-6), for any placement of the matrices, as numpy
          slicing around the triple loops of ``matmul``
mlp       the MLP block of Section 3.2 (two linear layers around an element-wise
          activation) and its backward pass, as full-matrix fp64 arithmetic
numfmt    decoding of bf16 / fp8-e4m3 bit patterns to fp64 and the single
          round-to-nearest-even of an fp64 result to the compared dtype
"""
