// Driver for a build of libcube3d's HOST code under AddressSanitizer and
// UndefinedBehaviorSanitizer: every C entry point is called with arguments its validation must
// refuse (or with queries that enqueue nothing), so the whole argument-checking layer, the plan
// and the index-map construction run instrumented.  No call reaches a launch: no GPU is needed.
// Exit status 0 = every call returned the expected status and no sanitizer report was made.
#include <cstdint>
#include <cstdio>
#include <initializer_list>

#include "cube3d.h"

static int failures = 0;
#define EXPECT(call, want) do { const long long got_ = (long long)(call); if (got_ != (long long)(want)) { \
    std::fprintf(stderr, "line %d: %s = %lld, expected %lld\n", __LINE__, #call, got_, (long long)(want)); ++failures; } } while (0)

static cube3d_desc desc(int q, int64_t M, int64_t K, int64_t N, int in = CUBE3D_F32, int out = CUBE3D_F32, int shard = CUBE3D_F32,
                        int axis = CUBE3D_AXIS_Y)
{
    cube3d_desc d{};
    d.q = q; d.in_axis = axis; d.M = M; d.K = K; d.N = N;
    d.in_dtype = in; d.out_dtype = out; d.shard_dtype = shard;
    d.scale_x = d.scale_w = d.scale_dy = 1.f;
    return d;
}

int main()
{
    void *fake = reinterpret_cast<void *>(0x10000), *odd = reinterpret_cast<void *>(0x10008);
    cube3d_desc good = desc(2, 256, 128, 128);

    // products
    EXPECT(cube3d_linear_fwd(nullptr, 0, 0, 0, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EINVAL);
    for (cube3d_desc bad : {desc(0, 256, 128, 128), desc(-3, 256, 128, 128), desc(2, 256, 128, 128, 0, 0, 0, CUBE3D_AXIS_X)})
        EXPECT(cube3d_linear_fwd(&bad, 0, 0, 0, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EINVAL);
    for (cube3d_desc bad : {desc(2, 258, 128, 128), desc(2, 256, 127, 128), desc(2, 256, 128, 130), desc(2, 0, 128, 128),
                            desc(2, 256, -128, 128), desc(64, 4096, 64, 4096)})
        EXPECT(cube3d_linear_bwd_dx(&bad, 0, 0, 0, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_ESHAPE);
    for (cube3d_desc bad : {desc(2, 256, 128, 128, 9), desc(2, 256, 128, 128, 0, CUBE3D_FP8_E4M3), desc(2, 256, 128, 128, 0, 0, 5)})
        EXPECT(cube3d_linear_bwd_dw(&bad, 0, 0, 0, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EDTYPE);
    {
        cube3d_desc f8 = desc(2, 256, 128, 128, CUBE3D_FP8_E4M3);
        f8.scale_w = 0.f;
        EXPECT(cube3d_linear_fwd(&f8, 0, 0, 0, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EINVAL);
    }
    const int ranks[][3] = {{2, 0, 0}, {0, -2, 0}, {0, 0, 5}, {-1, 0, 0}, {-1, -1, 0}};
    for (auto &r : ranks) EXPECT(cube3d_linear_fwd(&good, r[0], r[1], r[2], fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EINVAL);
    EXPECT(cube3d_linear_fwd(&good, 0, 0, 0, nullptr, fake, fake, nullptr, 0, nullptr), CUBE3D_EINVAL);
    EXPECT(cube3d_linear_fwd(&good, 0, 0, 0, fake, odd, fake, nullptr, 0, nullptr), CUBE3D_EINVAL);
    EXPECT(cube3d_linear_fwd(&good, 0, 0, 0, fake, fake, fake, odd, 64, nullptr), CUBE3D_EINVAL);

    // workspace: the plan (pure host arithmetic) over a sweep of shapes, and the too-small path
    cube3d_desc deep = desc(1, 128, 8192, 128, CUBE3D_BF16, CUBE3D_BF16, CUBE3D_BF16);
    const size_t need = cube3d_workspace_bytes(&deep, CUBE3D_OP_FWD, 0);
    EXPECT(need > 0, 1);
    EXPECT(cube3d_linear_fwd(&deep, 0, 0, 0, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EWORKSPACE);
    EXPECT(cube3d_linear_fwd(&deep, 0, 0, 0, fake, fake, fake, fake, need - 1, nullptr), CUBE3D_EWORKSPACE);
    size_t total = 0;
    for (int q : {1, 2, 4, 8})
        for (int64_t m : {128, 1024, 8192, 65536})
            for (int64_t k : {64, 512, 2048})
                for (int64_t n : {128, 1536, 8192})
                    for (int dt : {(int)CUBE3D_F32, (int)CUBE3D_BF16, (int)CUBE3D_FP8_E4M3})
                        for (int op : {(int)CUBE3D_OP_FWD, (int)CUBE3D_OP_BWD_DX, (int)CUBE3D_OP_BWD_DW, (int)CUBE3D_OP_BIAS_BWD, 42})
                            for (int batched : {0, 1}) {
                                cube3d_desc d = desc(q, m * q, k * q, n * q, dt, CUBE3D_BF16, CUBE3D_BF16);
                                total += cube3d_workspace_bytes(&d, op, batched);
                            }
    EXPECT(total > 0, 1);
    cube3d_desc big = desc(4, 4 * 65536, 4 * 768, 4 * 2048, CUBE3D_BF16, CUBE3D_BF16, CUBE3D_BF16);
    EXPECT(cube3d_workspace_bytes(&big, CUBE3D_OP_BWD_DW, 0) > CUBE3D_NOALLOC_SCRATCH_BYTES, 1);
    EXPECT(cube3d_linear_bwd_dw_noalloc(&big, 0, 0, 0, fake, fake, fake, nullptr), CUBE3D_ESCRATCH);
    EXPECT(cube3d_linear_bwd_dw_noalloc(&good, 0, 0, 0, nullptr, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(cube3d_linear_bwd_dw_noalloc(nullptr, 0, 0, 0, fake, fake, fake, nullptr), CUBE3D_EINVAL);

    // virtual-cube movement
    EXPECT(virtual_cube_gather(&good, CUBE3D_OPERAND_X, CUBE3D_AXIS_Z, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_gather(&good, CUBE3D_OPERAND_W, CUBE3D_AXIS_Y, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_gather(&good, CUBE3D_OPERAND_Y, CUBE3D_AXIS_Y, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_gather(&good, CUBE3D_OPERAND_X, CUBE3D_AXIS_Y, nullptr, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_reduce_scatter(&good, CUBE3D_OPERAND_Y, CUBE3D_AXIS_Y, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_reduce_scatter(&good, CUBE3D_OPERAND_DW, CUBE3D_AXIS_X, fake, odd, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_reduce_scatter(&good, CUBE3D_OPERAND_X, CUBE3D_AXIS_X, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_scatter(&good, 17, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_assemble(&good, CUBE3D_OPERAND_BIAS, nullptr, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_bias_gather(&good, fake, odd, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_reduce_scatter_bias(&good, CUBE3D_AXIS_Y, fake, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_bias_bwd(&good, fake, fake, nullptr, 0, nullptr), CUBE3D_EWORKSPACE);
    EXPECT(virtual_cube_linear_fwd(&good, fake, nullptr, nullptr, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_linear_bwd_dx(&good, fake, fake, odd, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_linear_bwd_dw(nullptr, fake, fake, fake, nullptr), CUBE3D_EINVAL);

    // placements and the three product forms
    cube3d_matrix m{};
    m.q = 2; m.row_axis = CUBE3D_AXIS_X; m.col_axis = CUBE3D_AXIS_Z; m.split = CUBE3D_SPLIT_ROWS; m.rows = 256; m.cols = 128;
    m.dtype = CUBE3D_BF16;
    cube3d_matrix same_axis = m;
    same_axis.col_axis = CUBE3D_AXIS_X;
    EXPECT(virtual_cube_matrix_scatter(&same_axis, fake, fake, nullptr), CUBE3D_EINVAL);
    cube3d_matrix ragged = m;
    ragged.rows = 254;
    EXPECT(virtual_cube_matrix_gather(&ragged, fake, fake, nullptr), CUBE3D_ESHAPE);
    EXPECT(virtual_cube_matrix_assemble(&m, fake, nullptr, nullptr), CUBE3D_EINVAL);
    EXPECT(virtual_cube_matrix_reduce_scatter(&m, CUBE3D_FP8_E4M3, fake, fake, nullptr), CUBE3D_EDTYPE);
    cube3d_matrix b = m, c = m;
    b.rows = 64; b.cols = 128; b.row_axis = CUBE3D_AXIS_Z; b.col_axis = CUBE3D_AXIS_Y; b.split = CUBE3D_SPLIT_COLS;
    c.cols = 128; c.col_axis = CUBE3D_AXIS_Y;
    EXPECT(virtual_cube_matmul(CUBE3D_FORM_AB, &m, &b, &c, 1.f, 1.f, fake, fake, fake, nullptr), CUBE3D_ESHAPE);   // k differs
    EXPECT(virtual_cube_matmul(7, &m, &b, &c, 1.f, 1.f, fake, fake, fake, nullptr), CUBE3D_EINVAL);
    cube3d_matmul mm{};
    mm.q = 1; mm.form = CUBE3D_FORM_ABT; mm.m = 128; mm.n = 128; mm.k = 8192; mm.in_dtype = CUBE3D_BF16; mm.out_dtype = CUBE3D_BF16;
    mm.scale_a = mm.scale_b = 1.f;
    EXPECT(cube3d_matmul_workspace_bytes(&mm) > 0, 1);
    EXPECT(cube3d_matmul_blocks(&mm, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EWORKSPACE);
    mm.form = 9;
    EXPECT(cube3d_matmul_blocks(&mm, fake, fake, fake, nullptr, 0, nullptr), CUBE3D_EINVAL);

    // activation
    EXPECT(cube3d_activation_fwd(2, CUBE3D_F32, CUBE3D_F32, 64, fake, fake, nullptr), CUBE3D_EINVAL);
    EXPECT(cube3d_activation_fwd(CUBE3D_ACT_GELU, CUBE3D_FP8_E4M3, CUBE3D_F32, 64, fake, fake, nullptr), CUBE3D_EDTYPE);
    EXPECT(cube3d_activation_bwd(CUBE3D_ACT_RELU, CUBE3D_F32, CUBE3D_F32, CUBE3D_F32, -1, fake, fake, fake, nullptr), CUBE3D_ESHAPE);
    EXPECT(cube3d_activation_bwd(CUBE3D_ACT_GELU, CUBE3D_BF16, CUBE3D_BF16, CUBE3D_BF16, 0, fake, fake, fake, nullptr), CUBE3D_OK);

    for (int s : {0, -1, -2, -3, -4, -5, -6, -7, -99}) EXPECT(cube3d_status_string(s) != nullptr, 1);
    EXPECT(cube3d_version(), CUBE3D_VERSION);
    if (failures) { std::fprintf(stderr, "%d call(s) returned an unexpected status\n", failures); return 1; }
    std::printf("C ABI validation layer under sanitizers: ok\n");
    return 0;
}
