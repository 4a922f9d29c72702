"""Host-side tests of the C ABI: the library loads, exports every symbol the header declares,
and every argument error is reported before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2105_14450_amd as c3
from paper_2105_14450_amd.binding import Desc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(c3.binding.LIB_PATH):
        from paper_2105_14450_amd import build
        build.build()
    return c3.binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "cube3d.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:cube3d|virtual_cube)_[a-z0-9_]+)\s*\(", header))
    assert declared == set(c3.binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert c3.cube3d_version() == 100


def test_desc_mirror_matches_the_header_layout():
    # int32 q, in_axis; int64 M, K, N; int32 in/out/shard dtype; float x3
    assert ctypes.sizeof(Desc) == 56
    assert Desc.M.offset == 8 and Desc.in_dtype.offset == 32 and Desc.scale_x.offset == 44


FAKE = ctypes.c_void_p(0x10000)          # aligned, never dereferenced: validation fails first
ODD = ctypes.c_void_p(0x10008)


def good(**kw):
    args = dict(q=2, M=256, K=128, N=128, in_dtype=c3.F32, out_dtype=c3.F32, shard_dtype=c3.F32)
    args.update(kw)
    return c3.make_desc(**args)


def fwd(lib, d, rank=(0, 0, 0), a=FAKE, b=FAKE, c=FAKE, ws=None, ws_bytes=0):
    dp = ctypes.byref(d) if d is not None else None
    return lib.cube3d_linear_fwd(dp, rank[0], rank[1], rank[2], a, b, c, ws, ws_bytes, None)


def test_descriptor_errors(lib):
    assert fwd(lib, None) == c3.EINVAL
    assert fwd(lib, good(q=0)) == c3.EINVAL
    assert fwd(lib, good(q=-3)) == c3.EINVAL
    assert fwd(lib, good(in_axis=c3.AXIS_X)) == c3.EINVAL
    assert fwd(lib, good(in_axis=7)) == c3.EINVAL
    assert fwd(lib, good(M=258)) == c3.ESHAPE       # q^2 does not divide M
    assert fwd(lib, good(N=130)) == c3.ESHAPE
    assert fwd(lib, good(K=127)) == c3.ESHAPE       # q does not divide K
    assert fwd(lib, good(M=0)) == c3.ESHAPE
    assert fwd(lib, good(K=-128)) == c3.ESHAPE
    assert fwd(lib, good(q=64, M=64 * 64, K=64, N=64 * 64)) == c3.ESHAPE   # cube too large for one launch
    assert fwd(lib, good(in_dtype=9)) == c3.EDTYPE
    assert fwd(lib, good(out_dtype=c3.FP8_E4M3)) == c3.EDTYPE
    assert fwd(lib, good(shard_dtype=5)) == c3.EDTYPE
    assert fwd(lib, good(in_dtype=c3.FP8_E4M3, scale_x=0.0)) == c3.EINVAL
    assert fwd(lib, good(in_dtype=c3.FP8_E4M3, scale_w=-1.0)) == c3.EINVAL
    assert fwd(lib, good(in_dtype=c3.FP8_E4M3, scale_dy=float("nan"))) == c3.EINVAL


def test_rank_and_pointer_errors(lib):
    d = good()
    for rank in ((2, 0, 0), (0, -2, 0), (0, 0, 5), (-1, 0, 0), (-1, -1, 0)):
        assert fwd(lib, d, rank) == c3.EINVAL
    assert fwd(lib, d, a=None) == c3.EINVAL
    assert fwd(lib, d, b=None) == c3.EINVAL
    assert fwd(lib, d, c=None) == c3.EINVAL
    assert fwd(lib, d, a=ODD) == c3.EINVAL
    assert fwd(lib, d, c=ODD) == c3.EINVAL
    for f in (lib.cube3d_linear_bwd_dx, lib.cube3d_linear_bwd_dw):
        assert f(ctypes.byref(d), 0, 0, 0, None, FAKE, FAKE, None, 0, None) == c3.EINVAL
        assert f(ctypes.byref(good(M=6)), 0, 0, 0, FAKE, FAKE, FAKE, None, 0, None) == c3.ESHAPE


def test_collective_argument_errors(lib):
    d = good()                       # in_axis = Y, so the output direction is Z
    g = lib.virtual_cube_gather
    assert g(ctypes.byref(d), c3.OPERAND_X, c3.AXIS_Z, FAKE, FAKE, None) == c3.EINVAL
    assert g(ctypes.byref(d), c3.OPERAND_W, c3.AXIS_Y, FAKE, FAKE, None) == c3.EINVAL
    assert g(ctypes.byref(d), c3.OPERAND_DY, c3.AXIS_Y, FAKE, FAKE, None) == c3.EINVAL
    assert g(ctypes.byref(d), c3.OPERAND_Y, c3.AXIS_Z, FAKE, FAKE, None) == c3.EINVAL     # not a gather operand
    assert g(ctypes.byref(d), c3.OPERAND_X, c3.AXIS_Y, None, FAKE, None) == c3.EINVAL
    assert g(ctypes.byref(d), c3.OPERAND_X, c3.AXIS_Y, FAKE, ODD, None) == c3.EINVAL
    assert g(None, c3.OPERAND_X, c3.AXIS_Y, FAKE, FAKE, None) == c3.EINVAL
    r = lib.virtual_cube_reduce_scatter
    assert r(ctypes.byref(d), c3.OPERAND_Y, c3.AXIS_Y, FAKE, FAKE, None) == c3.EINVAL
    assert r(ctypes.byref(d), c3.OPERAND_DX, c3.AXIS_Z, FAKE, FAKE, None) == c3.EINVAL
    assert r(ctypes.byref(d), c3.OPERAND_DW, c3.AXIS_Z, FAKE, FAKE, None) == c3.EINVAL
    assert r(ctypes.byref(d), c3.OPERAND_X, c3.AXIS_Y, FAKE, FAKE, None) == c3.EINVAL     # not a reduce operand
    assert r(ctypes.byref(d), c3.OPERAND_Y, c3.AXIS_Z, FAKE, None, None) == c3.EINVAL
    dz = good(in_axis=c3.AXIS_Z)     # exchanged directions: X travels along z, Y along y
    assert g(ctypes.byref(dz), c3.OPERAND_X, c3.AXIS_Y, FAKE, FAKE, None) == c3.EINVAL
    assert r(ctypes.byref(dz), c3.OPERAND_Y, c3.AXIS_Z, FAKE, FAKE, None) == c3.EINVAL
    for f in (lib.virtual_cube_scatter, lib.virtual_cube_assemble):
        assert f(ctypes.byref(d), 17, FAKE, FAKE, None) == c3.EINVAL
        assert f(ctypes.byref(d), c3.OPERAND_X, None, FAKE, None) == c3.EINVAL
        assert f(ctypes.byref(good(N=6)), c3.OPERAND_X, FAKE, FAKE, None) == c3.ESHAPE


def test_bias_argument_errors(lib):
    d = good()                       # output direction is Z
    g, r, b = lib.virtual_cube_bias_gather, lib.virtual_cube_reduce_scatter_bias, lib.virtual_cube_bias_bwd
    assert g(None, FAKE, FAKE, None) == c3.EINVAL
    assert g(ctypes.byref(d), None, FAKE, None) == c3.EINVAL
    assert g(ctypes.byref(d), FAKE, ODD, None) == c3.EINVAL
    assert g(ctypes.byref(good(N=6)), FAKE, FAKE, None) == c3.ESHAPE
    assert r(ctypes.byref(d), c3.AXIS_Y, FAKE, FAKE, FAKE, None) == c3.EINVAL     # wrong direction
    assert r(ctypes.byref(d), c3.AXIS_X, FAKE, FAKE, FAKE, None) == c3.EINVAL
    assert r(ctypes.byref(d), c3.AXIS_Z, FAKE, None, FAKE, None) == c3.EINVAL
    assert r(ctypes.byref(d), c3.AXIS_Z, None, FAKE, FAKE, None) == c3.EINVAL
    assert r(ctypes.byref(good(in_axis=c3.AXIS_Z)), c3.AXIS_Z, FAKE, FAKE, FAKE, None) == c3.EINVAL
    need = c3.cube3d_workspace_bytes(d, c3.OP_BIAS_BWD, True)
    assert need >= d.q ** 3 * (d.N // d.q) * 4          # at least one fp32 row of partials per processor
    assert need == c3.cube3d_workspace_bytes(d, c3.OP_BIAS_BWD, False)
    assert b(ctypes.byref(d), None, FAKE, FAKE, need, None) == c3.EINVAL
    assert b(ctypes.byref(d), FAKE, ODD, FAKE, need, None) == c3.EINVAL
    assert b(ctypes.byref(d), FAKE, FAKE, ODD, need, None) == c3.EINVAL
    assert b(ctypes.byref(good(in_dtype=11)), FAKE, FAKE, FAKE, need, None) == c3.EDTYPE
    assert b(ctypes.byref(d), FAKE, FAKE, None, 0, None) == c3.EWORKSPACE
    assert b(ctypes.byref(d), FAKE, FAKE, FAKE, need - 1, None) == c3.EWORKSPACE
    for f in (lib.virtual_cube_scatter, lib.virtual_cube_assemble):
        assert f(ctypes.byref(d), c3.OPERAND_BIAS, None, FAKE, None) == c3.EINVAL


def test_cube_linear_argument_errors(lib):
    d = good()
    f, dx, dw = lib.virtual_cube_linear_fwd, lib.virtual_cube_linear_bwd_dx, lib.virtual_cube_linear_bwd_dw
    assert f(None, FAKE, FAKE, None, FAKE, None) == c3.EINVAL
    assert f(ctypes.byref(d), None, FAKE, None, FAKE, None) == c3.EINVAL
    assert f(ctypes.byref(d), FAKE, None, None, FAKE, None) == c3.EINVAL
    assert f(ctypes.byref(d), FAKE, FAKE, None, None, None) == c3.EINVAL
    assert f(ctypes.byref(d), FAKE, FAKE, ODD, FAKE, None) == c3.EINVAL        # misaligned bias
    assert f(ctypes.byref(good(M=7)), FAKE, FAKE, None, FAKE, None) == c3.ESHAPE
    assert f(ctypes.byref(good(in_dtype=11)), FAKE, FAKE, None, FAKE, None) == c3.EDTYPE
    for g in (dx, dw):
        assert g(None, FAKE, FAKE, FAKE, None) == c3.EINVAL
        assert g(ctypes.byref(d), None, FAKE, FAKE, None) == c3.EINVAL
        assert g(ctypes.byref(d), FAKE, ODD, FAKE, None) == c3.EINVAL
        assert g(ctypes.byref(d), FAKE, FAKE, None, None) == c3.EINVAL
        assert g(ctypes.byref(good(N=6)), FAKE, FAKE, FAKE, None) == c3.ESHAPE


def test_matrix_and_matmul_argument_errors(lib):
    def mat(**kw):
        a = dict(q=2, rows=16, cols=8, row_axis=c3.AXIS_X, col_axis=c3.AXIS_Z, split=c3.SPLIT_ROWS, dtype=c3.F32)
        a.update(kw)
        return c3.make_matrix(**a)

    moves = (lib.virtual_cube_matrix_scatter, lib.virtual_cube_matrix_assemble, lib.virtual_cube_matrix_gather)
    for f in moves:
        assert f(None, FAKE, FAKE, None) == c3.EINVAL
        assert f(ctypes.byref(mat()), None, FAKE, None) == c3.EINVAL
        assert f(ctypes.byref(mat()), FAKE, ODD, None) == c3.EINVAL
        assert f(ctypes.byref(mat(q=0)), FAKE, FAKE, None) == c3.EINVAL
        assert f(ctypes.byref(mat(col_axis=c3.AXIS_X)), FAKE, FAKE, None) == c3.EINVAL   # same direction twice
        assert f(ctypes.byref(mat(row_axis=3)), FAKE, FAKE, None) == c3.EINVAL
        assert f(ctypes.byref(mat(split=2)), FAKE, FAKE, None) == c3.EINVAL
        assert f(ctypes.byref(mat(rows=18)), FAKE, FAKE, None) == c3.ESHAPE              # q^2 does not divide rows
        assert f(ctypes.byref(mat(cols=7)), FAKE, FAKE, None) == c3.ESHAPE
        assert f(ctypes.byref(mat(split=c3.SPLIT_COLS, cols=6)), FAKE, FAKE, None) == c3.ESHAPE
        assert f(ctypes.byref(mat(dtype=9)), FAKE, FAKE, None) == c3.EDTYPE
    rs = lib.virtual_cube_matrix_reduce_scatter
    assert rs(None, c3.F32, FAKE, FAKE, None) == c3.EINVAL
    assert rs(ctypes.byref(mat()), c3.FP8_E4M3, FAKE, FAKE, None) == c3.EDTYPE
    assert rs(ctypes.byref(mat(dtype=c3.FP8_E4M3)), c3.F32, FAKE, FAKE, None) == c3.EDTYPE
    assert rs(ctypes.byref(mat()), c3.F32, None, FAKE, None) == c3.EINVAL
    assert rs(ctypes.byref(mat(rows=6)), c3.F32, FAKE, FAKE, None) == c3.ESHAPE

    def mm(**kw):
        a = dict(q=2, form=c3.FORM_ABT, m=64, n=64, k=64, in_dtype=c3.F32, out_dtype=c3.F32)
        a.update(kw)
        return c3.make_matmul(**a)

    vm = lib.virtual_cube_matmul
    A = mat(rows=16, cols=8)                                                         # [m, k]
    B = mat(rows=8, cols=16, row_axis=c3.AXIS_Z, col_axis=c3.AXIS_Y, split=c3.SPLIT_COLS)   # [k, n]
    C = mat(rows=16, cols=16, row_axis=c3.AXIS_X, col_axis=c3.AXIS_Y)                # [m, n]
    ok = lambda f_, a_, b_, c_, pa=FAKE, pb=FAKE, pc_=FAKE, sa=1.0, sb=1.0: vm(
        f_, ctypes.byref(a_) if a_ is not None else None, ctypes.byref(b_), ctypes.byref(c_), sa, sb, pa, pb, pc_, None)
    assert ok(3, A, B, C) == c3.EINVAL
    assert ok(c3.FORM_AB, None, B, C) == c3.EINVAL
    assert ok(c3.FORM_AB, A, B, mat(rows=16, cols=32)) == c3.ESHAPE               # result size disagrees
    assert ok(c3.FORM_ABT, A, B, C) == c3.ESHAPE                                   # contraction lengths disagree
    assert ok(c3.FORM_AB, A, mat(rows=8, cols=16, q=1), C) == c3.EINVAL           # different cubes
    assert ok(c3.FORM_AB, A, mat(rows=8, cols=16, dtype=c3.BF16, split=c3.SPLIT_COLS), C) == c3.EDTYPE
    assert ok(c3.FORM_AB, A, B, mat(rows=16, cols=16, dtype=c3.FP8_E4M3)) == c3.EDTYPE
    assert ok(c3.FORM_AB, A, B, C, pa=None) == c3.EINVAL
    assert ok(c3.FORM_AB, A, B, C, pc_=ODD) == c3.EINVAL
    f8a, f8b = mat(rows=16, cols=8, dtype=c3.FP8_E4M3), mat(rows=8, cols=16, dtype=c3.FP8_E4M3, row_axis=c3.AXIS_Z,
                                                            col_axis=c3.AXIS_Y, split=c3.SPLIT_COLS)
    assert ok(c3.FORM_AB, f8a, f8b, C, sa=-1.0) == c3.EINVAL

    f = lib.cube3d_matmul_blocks
    assert f(None, FAKE, FAKE, FAKE, None, 0, None) == c3.EINVAL
    assert f(ctypes.byref(mm(form=3)), FAKE, FAKE, FAKE, None, 0, None) == c3.EINVAL
    assert f(ctypes.byref(mm(q=0)), FAKE, FAKE, FAKE, None, 0, None) == c3.EINVAL
    assert f(ctypes.byref(mm(k=0)), FAKE, FAKE, FAKE, None, 0, None) == c3.ESHAPE
    assert f(ctypes.byref(mm(in_dtype=5)), FAKE, FAKE, FAKE, None, 0, None) == c3.EDTYPE
    assert f(ctypes.byref(mm(out_dtype=c3.FP8_E4M3)), FAKE, FAKE, FAKE, None, 0, None) == c3.EDTYPE
    assert f(ctypes.byref(mm(in_dtype=c3.FP8_E4M3, scale_a=0.0)), FAKE, FAKE, FAKE, None, 0, None) == c3.EINVAL
    assert f(ctypes.byref(mm()), None, FAKE, FAKE, None, 0, None) == c3.EINVAL
    assert f(ctypes.byref(mm()), FAKE, FAKE, ODD, None, 0, None) == c3.EINVAL
    assert c3.cube3d_matmul_workspace_bytes(mm(form=7)) == 0
    # one 128 x 128 block per processor with a long contraction: split-K needs a workspace
    deep = mm(q=1, m=128, n=128, k=8192, in_dtype=c3.BF16, out_dtype=c3.BF16)
    need = c3.cube3d_matmul_workspace_bytes(deep)
    assert need > 0
    assert f(ctypes.byref(deep), FAKE, FAKE, FAKE, None, 0, None) == c3.EWORKSPACE
    assert f(ctypes.byref(deep), FAKE, FAKE, FAKE, FAKE, need - 1, None) == c3.EWORKSPACE


def test_activation_argument_errors(lib):
    f, b = lib.cube3d_activation_fwd, lib.cube3d_activation_bwd
    assert f(2, c3.F32, c3.F32, 64, FAKE, FAKE, None) == c3.EINVAL
    assert f(c3.ACT_GELU, c3.FP8_E4M3, c3.F32, 64, FAKE, FAKE, None) == c3.EDTYPE
    assert f(c3.ACT_GELU, c3.F32, 7, 64, FAKE, FAKE, None) == c3.EDTYPE
    assert f(c3.ACT_RELU, c3.F32, c3.F32, -1, FAKE, FAKE, None) == c3.ESHAPE
    assert f(c3.ACT_RELU, c3.F32, c3.F32, 64, None, FAKE, None) == c3.EINVAL
    assert f(c3.ACT_RELU, c3.F32, c3.F32, 64, FAKE, ODD, None) == c3.EINVAL
    assert f(c3.ACT_RELU, c3.F32, c3.BF16, 0, FAKE, FAKE, None) == c3.OK          # nothing to do, nothing launched
    assert b(-1, c3.F32, c3.F32, c3.F32, 64, FAKE, FAKE, FAKE, None) == c3.EINVAL
    assert b(c3.ACT_GELU, c3.F32, c3.FP8_E4M3, c3.F32, 64, FAKE, FAKE, FAKE, None) == c3.EDTYPE
    assert b(c3.ACT_GELU, c3.F32, c3.F32, c3.F32, 64, FAKE, None, FAKE, None) == c3.EINVAL
    assert b(c3.ACT_GELU, c3.F32, c3.F32, c3.F32, 64, FAKE, FAKE, ODD, None) == c3.EINVAL
    assert b(c3.ACT_GELU, c3.BF16, c3.BF16, c3.BF16, 0, FAKE, FAKE, FAKE, None) == c3.OK


def test_workspace_query_and_strings(lib):
    assert c3.cube3d_workspace_bytes(good(M=7), c3.OP_FWD, False) == 0
    assert c3.cube3d_workspace_bytes(good(), 42, False) == 0
    assert isinstance(c3.cube3d_workspace_bytes(good(), c3.OP_FWD, True), int)
    seen = set()
    for code in (c3.OK, c3.EINVAL, c3.ESHAPE, c3.EDTYPE, c3.EWORKSPACE, c3.ELAUNCH, c3.ENOTIMPL, c3.ESCRATCH, -99):
        s = c3.status_string(code)
        assert s and s not in seen
        seen.add(s)
    with pytest.raises(c3.binding.Cube3DError) as e:
        c3.binding._check(c3.ESHAPE, "where")
    assert e.value.status == c3.ESHAPE


def test_workspace_too_small_is_reported_before_any_launch(lib):
    # one 128x128 output tile with a long contraction: the plan splits K and needs fp32 partials
    d = c3.make_desc(1, 128, 8192, 128, in_dtype=c3.BF16, out_dtype=c3.BF16)
    need = c3.cube3d_workspace_bytes(d, c3.OP_FWD, False)
    assert need > 0 and need % (128 * 128 * 4) == 0
    assert fwd(lib, d, ws=None, ws_bytes=0) == c3.EWORKSPACE
    assert fwd(lib, d, ws=FAKE, ws_bytes=need - 1) == c3.EWORKSPACE
    assert fwd(lib, d, ws=ODD, ws_bytes=need) == c3.EINVAL
    # the same layer on a cube with many processors has enough tiles: no workspace
    big = c3.make_desc(4, 32768, 8192, 32768, in_dtype=c3.BF16, out_dtype=c3.BF16)
    for op in (c3.OP_FWD, c3.OP_BWD_DX, c3.OP_BWD_DW):
        assert c3.cube3d_workspace_bytes(big, op, False) == 0


def test_noalloc_entry_point_argument_errors(lib):
    def na(d, rank=(0, 0, 0), a=FAKE, b=FAKE, c=FAKE):
        dp = ctypes.byref(d) if d is not None else None
        return lib.cube3d_linear_bwd_dw_noalloc(dp, rank[0], rank[1], rank[2], a, b, c, None)
    assert na(None) == c3.EINVAL
    assert na(good(M=258)) == c3.ESHAPE
    assert na(good(in_dtype=9)) == c3.EDTYPE
    assert na(good(), rank=(2, 0, 0)) == c3.EINVAL
    assert na(good(), a=None) == c3.EINVAL
    assert na(good(), c=ODD) == c3.EINVAL
    # a plan with more split-K partial sums than the built-in scratch buffer holds is refused
    big = c3.make_desc(4, 4 * 65536, 4 * 768, 4 * 2048, in_dtype=c3.BF16, out_dtype=c3.BF16)
    assert c3.cube3d_workspace_bytes(big, c3.OP_BWD_DW, False) > c3.binding.NOALLOC_SCRATCH_BYTES
    assert na(big) == c3.ESCRATCH
    header = open(os.path.join(ROOT, "include", "cube3d.h")).read()
    assert "#define CUBE3D_NOALLOC_SCRATCH_BYTES (16u << 20)" in header and c3.binding.NOALLOC_SCRATCH_BYTES == 16 << 20


def test_binding_refuses_host_tensors():
    import torch
    d = good()
    t = torch.zeros(4)
    with pytest.raises(ValueError):
        c3.cube3d_linear_fwd(d, (0, 0, 0), t, t, t)
