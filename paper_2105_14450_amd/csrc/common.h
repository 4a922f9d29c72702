// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "cube3d.h"

namespace cube3d {

// ---- per-device facts and one-time set-up (device.hip) --------------------------------------------------
constexpr int MAX_DEVICES = 64;     // device ordinals the per-device tables cover
constexpr int DEFAULT_CUS = 256;    // MI355X; used only where no device can be queried (host-only checks)
// Ordinal of the calling thread's current device, or -1 when there is none.
int current_device();
// Compute units of the current device (cached per device).
int num_compute_units();
// A kernel instantiation's one-time set-up on the current device (raises its dynamic LDS limit);
// idempotent and thread-safe, returns a cube3d_status.  Every instantiation of the tuned product
// kernel registers one, so that cube3d_init() can do all of them ahead of the first launch.
typedef int (*KernelSetup)();
std::vector<KernelSetup> &kernel_setups();
int setup_all_kernels();

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

// Piecewise-linear placement of one matrix index in memory, two panel levels deep:
//   offset(x) = (x / P1) * s1 + ((x % P1) / P2) * s2 + (x % P2) * u        (elements)
// with P2 dividing P1.  It describes how a row or column index of a full matrix lands in a
// cube buffer of shards (Section 3.1.1): P1 = block size, P2 = shard size, s1 / s2 = distances
// between the processors that hold consecutive blocks / shards, u = distance inside a shard.
// An index that is split once uses P2 = P1, s2 = 0.
struct AxisMap {
    int32_t P1, P2;
    int64_t s1, s2, u;
    // Filled by prepare_axis_map(): constants for dividing an index below 2^31 by P1 / P2 exactly
    // without a divide instruction,  x / P = (x * M) >> N  with N = 31 + ceil(log2 P) and
    // M = ceil(2^N / P) (at most 34 bits, so x * M stays below 2^64).
    uint64_t M1, M2;
    int32_t N1, N2;
};

inline void prepare_axis_map(AxisMap &m)
{
    auto magic = [](int32_t P, uint64_t *M, int32_t *N) {
        int L = 0;
        while ((1ll << L) < P) ++L;
        *N = 31 + L;
        *M = (uint64_t)(((((unsigned __int128)1) << *N) + (unsigned)P - 1) / (unsigned)P);
    };
    magic(m.P1, &m.M1, &m.N1);
    magic(m.P2, &m.M2, &m.N2);
}

__host__ __device__ __forceinline__ int64_t axis_offset(const AxisMap &m, int64_t x)
{
    const uint32_t xx = (uint32_t)x;
    const uint32_t hi = xx / (uint32_t)m.P1, r1 = xx - hi * (uint32_t)m.P1;
    const uint32_t mid = r1 / (uint32_t)m.P2, lo = r1 - mid * (uint32_t)m.P2;
    return (int64_t)hi * m.s1 + (int64_t)mid * m.s2 + (int64_t)lo * m.u;
}

// The same value for a prepared map and 0 <= x < 2^31, with multiplications in place of the divisions
// (a division by a run-time divisor is some forty instructions on the vector ALU).
__device__ __forceinline__ int64_t axis_offset_fast(const AxisMap &m, int64_t x)
{
    const uint32_t xx = (uint32_t)x;
    const uint32_t hi = (uint32_t)(((uint64_t)xx * m.M1) >> m.N1), r1 = xx - hi * (uint32_t)m.P1;
    const uint32_t mid = (uint32_t)(((uint64_t)r1 * m.M2) >> m.N2), lo = r1 - mid * (uint32_t)m.P2;
    return (int64_t)hi * m.s1 + (int64_t)mid * m.s2 + (int64_t)lo * m.u;
}

// Element (mn, k) of operand A sits at A[a_mn(mn) + a_k(k)], of B at B[b_mn(mn) + b_k(k)];
// output element (m, n) at C[c_m(m) + c_n(n)].  bias (optional, fp32) is indexed by bias_n(n)
// and added to the scaled accumulator before the store (the tuned kernels carry it in the forward
// product's layout only; a bias with another layout runs on the bounds-checked kernel).
struct GemmMaps {
    AxisMap a_mn, a_k, b_mn, b_k, c_m, c_n, bias_n;
    const float *bias;
};

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
    // nullptr: plain row-major operands (lda / ldb / ldc).  Otherwise the operands and the output
    // are addressed through these maps (batch must be 1; leading dimensions and strides unused).
    const GemmMaps *maps;
};

// Any shape, any supported dtype; bounds-checked.  Returns a cube3d_status.
int gemm_generic(const GemmArgs &g);

// Tuned bf16 / fp8 path; returns CUBE3D_ENOTIMPL when the shape does not fit its tiles.
int gemm_fast(const GemmArgs &g);
size_t gemm_fast_workspace(const GemmArgs &g);
// Launch of the tuned kernel's map-addressed instantiations (tile = 256 or 128, chosen by gemm_fast).
int gemm_fast_mapped(const GemmArgs &g, int tile);

// Geometry of the virtual cube and the data-movement kernels over it.
struct CubeGeom {
    int q;
    int in_axis_z;  // 0: input gathered along y, output reduced along z; 1: exchanged
    int64_t M, K, N, Mb, Kb, Nb, Ms, Ns;
    // MV_PLACE_* modes only: placement of one [pR, pC] matrix (Section 3.1.1 generalised to the
    // operands of Algorithms 3-6).  Cube directions 0 / 1 / 2 = x / y / z: the index along p_ra picks
    // the block row, along p_ca the block column; along p_sa a [pRb, pCb] block is cut once more into
    // q pieces [pRs, pCs], by rows (p_split_rows) or by columns.
    int p_ra, p_ca, p_sa, p_split_rows;
    int64_t pR, pC, pRb, pCb, pRs, pCs;
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
    MV_GATHER_BIAS,    // diagonal storage -> one [Nb] block per processor
    MV_PLACE_GATHER,   // any placement: shards -> one whole block per processor (all-gather along p_sa)
    MV_PLACE_SCATTER,  // full matrix -> shards
    MV_PLACE_ASSEMBLE, // shards -> full matrix
    MV_PLACE_REDUCE    // partial blocks -> shards (reduce-scatter along p_sa)
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

// Element-wise activation over n elements (dtypes F32 or BF16 already checked by the caller).
int activation_fwd(int kind, int z_dtype, int h_dtype, int64_t n, const void *z, void *h, hipStream_t stream);
int activation_bwd(int kind, int z_dtype, int g_dtype, int dz_dtype, int64_t n, const void *z, const void *dh, void *dz,
                   hipStream_t stream);

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

// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

}  // namespace cube3d
