"""MI355X-native hot path of the 3-D model-parallel linear layer.

``binding``  ctypes wrappers with the names of the C entry points in
             ``include/cube3d.h``; the HIP kernels live in ``csrc/``
``build``    compiles ``libcube3d.so`` for gfx950
``synth``    seeded synthetic inputs (no arithmetic of the method)
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
