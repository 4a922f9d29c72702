// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "cube3d.h"

namespace cube3d {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// One (possibly batched) product  C[Mo,No] = alpha * opA * opB  with fp32 accumulation.
//   a_kmajor: A is stored [Mo, Kc] (contraction index contiguous), else [Kc, Mo]
//   b_kmajor: B is stored [No, Kc] (contraction index contiguous), else [Kc, No]
// The three products of the linear layer map onto it as
//   forward  X W      : a_kmajor = 1, b_kmajor = 0
//   dX = dY W^T       : a_kmajor = 1, b_kmajor = 1
//   dW = X^T dY       : a_kmajor = 0, b_kmajor = 0
struct GemmArgs {
    const void *A;
    const void *B;
    void *C;
    int64_t Mo, No, Kc;
    int64_t lda, ldb, ldc;              // leading dimensions in elements
    int64_t strideA, strideB, strideC;  // batch strides in elements
    int batch;
    float alpha;
    bool a_kmajor, b_kmajor;
    int in_dtype, out_dtype;
    void *workspace;
    size_t workspace_bytes;
    hipStream_t stream;
};

// Any shape, any supported dtype; bounds-checked.  Returns a cube3d_status.
int gemm_generic(const GemmArgs &g);

// Tuned bf16 / fp8 path; returns CUBE3D_ENOTIMPL when the shape does not fit its tiles.
int gemm_fast(const GemmArgs &g);
size_t gemm_fast_workspace(const GemmArgs &g);

// Geometry of the virtual cube and the data-movement kernels over it.
struct CubeGeom {
    int q;
    int in_axis_z;  // 0: input gathered along y, output reduced along z; 1: exchanged
    int64_t M, K, N, Mb, Kb, Nb, Ms, Ns;
};

enum MoveMode {
    MV_GATHER_X = 0,
    MV_GATHER_W,
    MV_GATHER_DY,
    MV_SCATTER_X,   // full matrix -> shards
    MV_SCATTER_W,
    MV_SCATTER_Y,
    MV_ASSEMBLE_X,  // shards -> full matrix
    MV_ASSEMBLE_W,
    MV_ASSEMBLE_Y,
    MV_REDUCE_Y,
    MV_REDUCE_DX,
    MV_REDUCE_DW,
    MV_SCATTER_BIAS,   // full vector -> diagonal storage
    MV_ASSEMBLE_BIAS,  // diagonal storage -> full vector
    MV_GATHER_BIAS     // diagonal storage -> one [Nb] block per processor
};

int cube_move(const CubeGeom &g, int mode, int es, const void *src, void *dst, hipStream_t stream);
// bias: optional [q^3][Nb] fp32 blocks added to the sum (MV_REDUCE_Y only), or nullptr
int cube_reduce(const CubeGeom &g, int mode, int partial_dtype, int shard_dtype, const void *partials, void *shards,
                const float *bias, hipStream_t stream);
int cube_bias_move(const CubeGeom &g, int mode, const float *src, float *dst, hipStream_t stream);
// fp32 partial column sums of the two-stage bias gradient (bytes); depends on the shape only
size_t cube_bias_bwd_workspace(const CubeGeom &g, int dy_dtype);
int cube_bias_bwd(const CubeGeom &g, int dy_dtype, float scale_dy, const void *dy_shards, float *dbias_diag,
                  void *workspace, size_t workspace_bytes, hipStream_t stream);

inline int launch_status()
{
    return hipGetLastError() == hipSuccess ? CUBE3D_OK : CUBE3D_ELAUNCH;
}

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short b)
{
    return __uint_as_float(((unsigned)b) << 16);
}

// fp32 -> bf16, round to nearest even (finite inputs; NaN stays NaN).
__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f)
{
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

}  // namespace cube3d
