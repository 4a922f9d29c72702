"""Thin ctypes binding over ``libcube3d.so`` (see ``include/cube3d.h``).

Argument marshalling only: every function takes torch CUDA tensors (device
memory) and forwards raw pointers plus the current HIP stream to the C entry
point of the same name.  There is no fallback: if the library is missing the
import of a function raises, and a non-zero status raises ``Cube3DError``.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcube3d.so")

OK, EINVAL, ESHAPE, EDTYPE, EWORKSPACE, ELAUNCH, ENOTIMPL, ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7
NOALLOC_SCRATCH_BYTES = 16 << 20
F32, BF16, FP8_E4M3 = 0, 1, 2
AXIS_X, AXIS_Y, AXIS_Z = 0, 1, 2
OPERAND_X, OPERAND_W, OPERAND_DY, OPERAND_Y, OPERAND_DX, OPERAND_DW, OPERAND_BIAS = range(7)
OP_FWD, OP_BWD_DX, OP_BWD_DW, OP_BIAS_BWD = 0, 1, 2, 3
SPLIT_ROWS, SPLIT_COLS = 0, 1
FORM_AB, FORM_ABT, FORM_ATB = 0, 1, 2
ACT_RELU, ACT_GELU = 0, 1
ALL_RANKS = (-1, -1, -1)

DTYPE_CODES = {"f32": F32, "bf16": BF16, "fp8_e4m3": FP8_E4M3}
ELEM_SIZE = {F32: 4, BF16: 2, FP8_E4M3: 1}


class Desc(ctypes.Structure):
    """Mirror of ``cube3d_desc``."""
    _fields_ = [("q", ctypes.c_int32), ("in_axis", ctypes.c_int32),
                ("M", ctypes.c_int64), ("K", ctypes.c_int64), ("N", ctypes.c_int64),
                ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("shard_dtype", ctypes.c_int32),
                ("scale_x", ctypes.c_float), ("scale_w", ctypes.c_float),
                ("scale_dy", ctypes.c_float)]


def make_desc(q, M, K, N, in_dtype=BF16, out_dtype=F32, shard_dtype=None, in_axis=AXIS_Y,
              scale_x=1.0, scale_w=1.0, scale_dy=1.0) -> Desc:
    if shard_dtype is None:
        shard_dtype = F32 if in_dtype == F32 else BF16
    return Desc(q, in_axis, M, K, N, in_dtype, out_dtype, shard_dtype, scale_x, scale_w, scale_dy)


class Matrix(ctypes.Structure):
    """Mirror of ``cube3d_matrix``: a [rows, cols] matrix placed on the cube."""
    _fields_ = [("q", ctypes.c_int32), ("row_axis", ctypes.c_int32), ("col_axis", ctypes.c_int32),
                ("split", ctypes.c_int32), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("dtype", ctypes.c_int32)]


class Matmul(ctypes.Structure):
    """Mirror of ``cube3d_matmul``: the batched local product of the q^3 processors."""
    _fields_ = [("q", ctypes.c_int32), ("form", ctypes.c_int32),
                ("m", ctypes.c_int64), ("n", ctypes.c_int64), ("k", ctypes.c_int64),
                ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
                ("scale_a", ctypes.c_float), ("scale_b", ctypes.c_float)]


def make_matrix(q, rows, cols, row_axis, col_axis, split, dtype) -> Matrix:
    return Matrix(q, row_axis, col_axis, split, rows, cols, dtype)


def make_matmul(q, form, m, n, k, in_dtype=BF16, out_dtype=F32, scale_a=1.0, scale_b=1.0) -> Matmul:
    return Matmul(q, form, m, n, k, in_dtype, out_dtype, scale_a, scale_b)


class Cube3DError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))


_lib = None


def load():
    """Load the library (after torch, so both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libcube3d.so is not built: run `python -m paper_2105_14450_amd.build`")
    try:
        import torch  # noqa: F401  (loads the HIP runtime the tensors come from)
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    dp = ctypes.POINTER(Desc)
    for name in ("cube3d_linear_fwd", "cube3d_linear_bwd_dx", "cube3d_linear_bwd_dw"):
        f = getattr(lib, name)
        f.argtypes = [dp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
        f.restype = ci
    lib.cube3d_workspace_bytes.argtypes = [dp, ci, ci]
    lib.cube3d_workspace_bytes.restype = sz
    for name in ("virtual_cube_gather", "virtual_cube_reduce_scatter"):
        f = getattr(lib, name)
        f.argtypes = [dp, ci, ci, vp, vp, vp]
        f.restype = ci
    for name in ("virtual_cube_scatter", "virtual_cube_assemble"):
        f = getattr(lib, name)
        f.argtypes = [dp, ci, vp, vp, vp]
        f.restype = ci
    lib.virtual_cube_bias_gather.argtypes = [dp, vp, vp, vp]
    lib.virtual_cube_bias_gather.restype = ci
    lib.virtual_cube_reduce_scatter_bias.argtypes = [dp, ci, vp, vp, vp, vp]
    lib.virtual_cube_reduce_scatter_bias.restype = ci
    lib.virtual_cube_bias_bwd.argtypes = [dp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.virtual_cube_bias_bwd.restype = ci
    lib.virtual_cube_linear_fwd.argtypes = [dp, vp, vp, vp, vp, vp]
    lib.virtual_cube_linear_fwd.restype = ci
    lib.virtual_cube_linear_bwd_dx.argtypes = [dp, vp, vp, vp, vp]
    lib.virtual_cube_linear_bwd_dx.restype = ci
    lib.virtual_cube_linear_bwd_dw.argtypes = [dp, vp, vp, vp, vp]
    lib.virtual_cube_linear_bwd_dw.restype = ci
    mp, pp = ctypes.POINTER(Matrix), ctypes.POINTER(Matmul)
    for name in ("virtual_cube_matrix_scatter", "virtual_cube_matrix_assemble", "virtual_cube_matrix_gather"):
        f = getattr(lib, name)
        f.argtypes = [mp, vp, vp, vp]
        f.restype = ci
    lib.virtual_cube_matrix_reduce_scatter.argtypes = [mp, ci, vp, vp, vp]
    lib.virtual_cube_matrix_reduce_scatter.restype = ci
    lib.cube3d_matmul_workspace_bytes.argtypes = [pp]
    lib.cube3d_matmul_workspace_bytes.restype = sz
    lib.cube3d_matmul_blocks.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.cube3d_matmul_blocks.restype = ci
    lib.virtual_cube_matmul.argtypes = [ci, mp, mp, mp, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp]
    lib.virtual_cube_matmul.restype = ci
    lib.cube3d_activation_fwd.argtypes = [ci, ci, ci, ctypes.c_int64, vp, vp, vp]
    lib.cube3d_activation_fwd.restype = ci
    lib.cube3d_activation_bwd.argtypes = [ci, ci, ci, ci, ctypes.c_int64, vp, vp, vp, vp]
    lib.cube3d_activation_bwd.restype = ci
    lib.cube3d_status_string.argtypes = [ci]
    lib.cube3d_status_string.restype = ctypes.c_char_p
    lib.cube3d_version.restype = ci
    lib.cube3d_linear_bwd_dw_noalloc.argtypes = [dp, ci, ci, ci, vp, vp, vp, vp]
    lib.cube3d_linear_bwd_dw_noalloc.restype = ci
    lib.cube3d_init.argtypes = []
    lib.cube3d_init.restype = ci
    _lib = lib
    return lib


EXPORTS = ("cube3d_linear_fwd", "cube3d_linear_bwd_dx", "cube3d_linear_bwd_dw", "cube3d_workspace_bytes",
           "virtual_cube_gather", "virtual_cube_reduce_scatter", "virtual_cube_scatter",
           "virtual_cube_assemble", "virtual_cube_bias_gather", "virtual_cube_reduce_scatter_bias",
           "virtual_cube_bias_bwd", "virtual_cube_linear_fwd", "virtual_cube_linear_bwd_dx",
           "virtual_cube_linear_bwd_dw", "virtual_cube_matrix_scatter", "virtual_cube_matrix_assemble",
           "virtual_cube_matrix_gather", "virtual_cube_matrix_reduce_scatter", "cube3d_matmul_workspace_bytes",
           "cube3d_matmul_blocks", "virtual_cube_matmul", "cube3d_activation_fwd", "cube3d_activation_bwd", "cube3d_status_string",
           "cube3d_version", "cube3d_init", "cube3d_linear_bwd_dw_noalloc")


def status_string(status: int) -> str:
    return load().cube3d_status_string(int(status)).decode()


def cube3d_version() -> int:
    return int(load().cube3d_version())


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensors only")
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc, where):
    if rc != OK:
        raise Cube3DError(rc, where)


def cube3d_workspace_bytes(desc: Desc, op: int, batched: bool) -> int:
    return int(load().cube3d_workspace_bytes(ctypes.byref(desc), op, 1 if batched else 0))


def _product(name, desc, rank, a, b, out, workspace, stream):
    i, j, l = rank
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = getattr(load(), name)(ctypes.byref(desc), i, j, l, _ptr(a), _ptr(b), _ptr(out),
                               _ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, name)
    return out


def cube3d_linear_fwd(desc, rank, X_block, W_block, P, workspace=None, stream=None):
    return _product("cube3d_linear_fwd", desc, rank, X_block, W_block, P, workspace, stream)


def cube3d_linear_bwd_dx(desc, rank, dY_block, W_block, Q, workspace=None, stream=None):
    return _product("cube3d_linear_bwd_dx", desc, rank, dY_block, W_block, Q, workspace, stream)


def cube3d_linear_bwd_dw(desc, rank, X_block, dY_block, R, workspace=None, stream=None):
    return _product("cube3d_linear_bwd_dw", desc, rank, X_block, dY_block, R, workspace, stream)


def virtual_cube_gather(desc, which, axis, shards, gathered, stream=None):
    _check(load().virtual_cube_gather(ctypes.byref(desc), which, axis, _ptr(shards), _ptr(gathered),
                                      _stream(stream)), "virtual_cube_gather")
    return gathered


def virtual_cube_reduce_scatter(desc, which, axis, partials, shards, stream=None):
    _check(load().virtual_cube_reduce_scatter(ctypes.byref(desc), which, axis, _ptr(partials), _ptr(shards),
                                              _stream(stream)), "virtual_cube_reduce_scatter")
    return shards


def virtual_cube_scatter(desc, which, full, shards, stream=None):
    _check(load().virtual_cube_scatter(ctypes.byref(desc), which, _ptr(full), _ptr(shards), _stream(stream)),
           "virtual_cube_scatter")
    return shards


def virtual_cube_assemble(desc, which, shards, full, stream=None):
    _check(load().virtual_cube_assemble(ctypes.byref(desc), which, _ptr(shards), _ptr(full), _stream(stream)),
           "virtual_cube_assemble")
    return full


def virtual_cube_bias_gather(desc, bias_diag, bias_blocks, stream=None):
    _check(load().virtual_cube_bias_gather(ctypes.byref(desc), _ptr(bias_diag), _ptr(bias_blocks), _stream(stream)),
           "virtual_cube_bias_gather")
    return bias_blocks


def virtual_cube_reduce_scatter_bias(desc, axis, partials, bias_blocks, shards, stream=None):
    _check(load().virtual_cube_reduce_scatter_bias(ctypes.byref(desc), axis, _ptr(partials), _ptr(bias_blocks),
                                                   _ptr(shards), _stream(stream)), "virtual_cube_reduce_scatter_bias")
    return shards


def virtual_cube_bias_bwd(desc, dY_shards, dbias_diag, workspace, stream=None):
    _check(load().virtual_cube_bias_bwd(ctypes.byref(desc), _ptr(dY_shards), _ptr(dbias_diag), _ptr(workspace),
                                        0 if workspace is None else workspace.numel() * workspace.element_size(),
                                        _stream(stream)), "virtual_cube_bias_bwd")
    return dbias_diag


def virtual_cube_linear_fwd(desc, X_shards, W_shards, bias_diag, Y_shards, stream=None):
    _check(load().virtual_cube_linear_fwd(ctypes.byref(desc), _ptr(X_shards), _ptr(W_shards), _ptr(bias_diag),
                                          _ptr(Y_shards), _stream(stream)), "virtual_cube_linear_fwd")
    return Y_shards


def virtual_cube_linear_bwd_dx(desc, dY_shards, W_shards, dX_shards, stream=None):
    _check(load().virtual_cube_linear_bwd_dx(ctypes.byref(desc), _ptr(dY_shards), _ptr(W_shards), _ptr(dX_shards),
                                             _stream(stream)), "virtual_cube_linear_bwd_dx")
    return dX_shards


def virtual_cube_linear_bwd_dw(desc, X_shards, dY_shards, dW_shards, stream=None):
    _check(load().virtual_cube_linear_bwd_dw(ctypes.byref(desc), _ptr(X_shards), _ptr(dY_shards), _ptr(dW_shards),
                                             _stream(stream)), "virtual_cube_linear_bwd_dw")
    return dW_shards


def virtual_cube_matrix_scatter(m, full, pieces, stream=None):
    _check(load().virtual_cube_matrix_scatter(ctypes.byref(m), _ptr(full), _ptr(pieces), _stream(stream)),
           "virtual_cube_matrix_scatter")
    return pieces


def virtual_cube_matrix_assemble(m, pieces, full, stream=None):
    _check(load().virtual_cube_matrix_assemble(ctypes.byref(m), _ptr(pieces), _ptr(full), _stream(stream)),
           "virtual_cube_matrix_assemble")
    return full


def virtual_cube_matrix_gather(m, pieces, blocks, stream=None):
    _check(load().virtual_cube_matrix_gather(ctypes.byref(m), _ptr(pieces), _ptr(blocks), _stream(stream)),
           "virtual_cube_matrix_gather")
    return blocks


def virtual_cube_matrix_reduce_scatter(m, partial_dtype, partials, pieces, stream=None):
    _check(load().virtual_cube_matrix_reduce_scatter(ctypes.byref(m), partial_dtype, _ptr(partials), _ptr(pieces),
                                                     _stream(stream)), "virtual_cube_matrix_reduce_scatter")
    return pieces


def cube3d_matmul_workspace_bytes(mm: Matmul) -> int:
    return int(load().cube3d_matmul_workspace_bytes(ctypes.byref(mm)))


def cube3d_matmul_blocks(mm, A_blocks, B_blocks, C_blocks, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().cube3d_matmul_blocks(ctypes.byref(mm), _ptr(A_blocks), _ptr(B_blocks), _ptr(C_blocks),
                                       _ptr(workspace), ws_bytes, _stream(stream)), "cube3d_matmul_blocks")
    return C_blocks


def cube3d_activation_fwd(kind, z_dtype, h_dtype, z, h, stream=None):
    _check(load().cube3d_activation_fwd(kind, z_dtype, h_dtype, z.numel(), _ptr(z), _ptr(h), _stream(stream)),
           "cube3d_activation_fwd")
    return h


def cube3d_activation_bwd(kind, z_dtype, dh_dtype, dz_dtype, z, dh, dz, stream=None):
    _check(load().cube3d_activation_bwd(kind, z_dtype, dh_dtype, dz_dtype, z.numel(), _ptr(z), _ptr(dh), _ptr(dz),
                                        _stream(stream)), "cube3d_activation_bwd")
    return dz


def virtual_cube_matmul(form, A, B, C, A_pieces, B_pieces, C_pieces, scale_a=1.0, scale_b=1.0, stream=None):
    _check(load().virtual_cube_matmul(form, ctypes.byref(A), ctypes.byref(B), ctypes.byref(C), scale_a, scale_b,
                                      _ptr(A_pieces), _ptr(B_pieces), _ptr(C_pieces), _stream(stream)),
           "virtual_cube_matmul")
    return C_pieces


def cube3d_init() -> None:
    _check(load().cube3d_init(), "cube3d_init")


def cube3d_linear_bwd_dw_noalloc(desc, rank, X_block, dY_block, R, stream=None):
    i, j, l = rank
    _check(load().cube3d_linear_bwd_dw_noalloc(ctypes.byref(desc), i, j, l, _ptr(X_block), _ptr(dY_block), _ptr(R),
                                               _stream(stream)), "cube3d_linear_bwd_dw_noalloc")
    return R
