// Shape-agnostic MFMA product kernel: every dtype, every operand layout, any
// size (bounds-checked loads and stores, zero-filled tails).  It is the path
// for the fp32 configuration, for ragged shapes and for anything the tuned
// kernels decline.  One workgroup (4 wavefronts) makes a 64x64 output tile; each
// wavefront owns one 32x32 MFMA accumulator.
//
// Implements the local products of Algorithm 1 step 3 and Algorithm 2 lines 1-2.
#include "common.h"

namespace cube3d {
namespace {

constexpr int TM = 64, TN = 64, TK = 32;

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int PAD = 1;
    static constexpr int KSTEP = 2;
};
template <> struct Elem<unsigned short> {   // bf16 bit patterns
    static constexpr int PAD = 8;
    static constexpr int KSTEP = 16;
};
template <> struct Elem<unsigned char> {    // fp8 e4m3 codes
    static constexpr int PAD = 8;
    static constexpr int KSTEP = 16;
};

template <typename T>
__device__ __forceinline__ f32x16 mfma_step(const T *arow, const T *brow, int kk, int khalf, f32x16 acc);

template <>
__device__ __forceinline__ f32x16 mfma_step<float>(const float *arow, const float *brow, int kk, int khalf, f32x16 acc)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(arow[kk + khalf], brow[kk + khalf], acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x16 mfma_step<unsigned short>(const unsigned short *arow, const unsigned short *brow,
                                                             int kk, int khalf, f32x16 acc)
{
    bf16x8 a = *reinterpret_cast<const bf16x8 *>(arow + kk + 8 * khalf);
    bf16x8 b = *reinterpret_cast<const bf16x8 *>(brow + kk + 8 * khalf);
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x16 mfma_step<unsigned char>(const unsigned char *arow, const unsigned char *brow,
                                                            int kk, int khalf, f32x16 acc)
{
    long a = *reinterpret_cast<const long *>(arow + kk + 8 * khalf);
    long b = *reinterpret_cast<const long *>(brow + kk + 8 * khalf);
    return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a, b, acc, 0, 0, 0);
}

template <typename TOut> __device__ __forceinline__ void store_out(TOut *p, float v);
template <> __device__ __forceinline__ void store_out<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_out<unsigned short>(unsigned short *p, float v)
{
    *p = f32_to_bf16_bits(v);
}

// MAPPED: every element address goes through the index maps (operands and output are cubes of
// shards, Section 3.1.1) and the optional bias is added; the leading dimensions are unused.
template <typename TIn, typename TOut, bool AK, bool BK, bool MAPPED>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const TIn *__restrict__ A, const TIn *__restrict__ B,
                                                           TOut *__restrict__ C, int64_t Mo, int64_t No, int64_t Kc,
                                                           int64_t lda, int64_t ldb, int64_t ldc, int64_t sA,
                                                           int64_t sB, int64_t sC, float alpha, GemmMaps maps)
{
    // address of operand element (mn, k): plain leading dimension, or the two index maps
    auto a_at = [&](int64_t gm, int64_t gk) -> int64_t {
        if (MAPPED) return axis_offset(maps.a_mn, gm) + axis_offset(maps.a_k, gk);
        return AK ? gm * lda + gk : gk * lda + gm;
    };
    auto b_at = [&](int64_t gn, int64_t gk) -> int64_t {
        if (MAPPED) return axis_offset(maps.b_mn, gn) + axis_offset(maps.b_k, gk);
        return BK ? gn * ldb + gk : gk * ldb + gn;
    };
    constexpr int LD = TK + Elem<TIn>::PAD;
    __shared__ __attribute__((aligned(16))) TIn As[TM * LD];
    __shared__ __attribute__((aligned(16))) TIn Bs[TN * LD];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int64_t m0 = (int64_t)blockIdx.y * TM;
    const int64_t n0 = (int64_t)blockIdx.x * TN;
    A += (int64_t)blockIdx.z * sA;
    B += (int64_t)blockIdx.z * sB;
    C += (int64_t)blockIdx.z * sC;

    f32x16 acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
    const TIn *arow = As + (wm + (lane & 31)) * LD;
    const TIn *brow = Bs + (wn + (lane & 31)) * LD;
    const int khalf = lane >> 5;

    for (int64_t k0 = 0; k0 < Kc; k0 += TK) {
        // stage both tiles as [row][k]; out-of-range elements are zero
        if (AK) {
            const int k = tid & 31;
            for (int r = tid >> 5; r < TM; r += 8) {
                const int64_t gm = m0 + r, gk = k0 + k;
                As[r * LD + k] = (gm < Mo && gk < Kc) ? A[a_at(gm, gk)] : TIn(0);
            }
        } else {
            const int r = tid & 63;
            for (int k = tid >> 6; k < TK; k += 4) {
                const int64_t gm = m0 + r, gk = k0 + k;
                As[r * LD + k] = (gm < Mo && gk < Kc) ? A[a_at(gm, gk)] : TIn(0);
            }
        }
        if (BK) {
            const int k = tid & 31;
            for (int r = tid >> 5; r < TN; r += 8) {
                const int64_t gn = n0 + r, gk = k0 + k;
                Bs[r * LD + k] = (gn < No && gk < Kc) ? B[b_at(gn, gk)] : TIn(0);
            }
        } else {
            const int r = tid & 63;
            for (int k = tid >> 6; k < TK; k += 4) {
                const int64_t gn = n0 + r, gk = k0 + k;
                Bs[r * LD + k] = (gn < No && gk < Kc) ? B[b_at(gn, gk)] : TIn(0);
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; kk += Elem<TIn>::KSTEP) acc = mfma_step<TIn>(arow, brow, kk, khalf, acc);
        __syncthreads();
    }

    // 32x32 accumulator: register v of lane holds row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
    const int64_t col = n0 + wn + (lane & 31);
    if (col < No) {
        const float bias = (MAPPED && maps.bias) ? maps.bias[axis_offset(maps.bias_n, col)] : 0.f;
        const int64_t col_off = MAPPED ? axis_offset(maps.c_n, col) : col;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = m0 + wm + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (row < Mo) {
                const int64_t row_off = MAPPED ? axis_offset(maps.c_m, row) : row * ldc;
                store_out<TOut>(C + row_off + col_off, MAPPED ? acc[v] * alpha + bias : acc[v] * alpha);
            }
        }
    }
}

template <typename TIn, typename TOut>
int launch_layout(const GemmArgs &g)
{
    dim3 grid((unsigned)((g.No + TN - 1) / TN), (unsigned)((g.Mo + TM - 1) / TM), (unsigned)g.batch);
    dim3 block(256);
    const TIn *A = static_cast<const TIn *>(g.A);
    const TIn *B = static_cast<const TIn *>(g.B);
    TOut *C = static_cast<TOut *>(g.C);
    const GemmMaps maps = g.maps ? *g.maps : GemmMaps{};
#define CUBE3D_LAUNCH(AKV, BKV, MP)                                                                               \
    hipLaunchKernelGGL((gemm_generic_kernel<TIn, TOut, AKV, BKV, MP>), grid, block, 0, g.stream, A, B, C, g.Mo, \
                       g.No, g.Kc, g.lda, g.ldb, g.ldc, g.strideA, g.strideB, g.strideC, g.alpha, maps)
    if (g.maps) {
        if (g.batch != 1) return CUBE3D_EINVAL;
        if (g.a_kmajor && g.b_kmajor) CUBE3D_LAUNCH(true, true, true);
        else if (g.a_kmajor && !g.b_kmajor) CUBE3D_LAUNCH(true, false, true);
        else if (!g.a_kmajor && !g.b_kmajor) CUBE3D_LAUNCH(false, false, true);
        else return CUBE3D_ENOTIMPL;
    } else if (g.a_kmajor && g.b_kmajor) CUBE3D_LAUNCH(true, true, false);
    else if (g.a_kmajor && !g.b_kmajor) CUBE3D_LAUNCH(true, false, false);
    else if (!g.a_kmajor && !g.b_kmajor) CUBE3D_LAUNCH(false, false, false);
    else CUBE3D_LAUNCH(false, true, false);
#undef CUBE3D_LAUNCH
    return launch_status();
}

template <typename TIn>
int launch_out(const GemmArgs &g)
{
    if (g.out_dtype == CUBE3D_F32) return launch_layout<TIn, float>(g);
    if (g.out_dtype == CUBE3D_BF16) return launch_layout<TIn, unsigned short>(g);
    return CUBE3D_EDTYPE;
}

}  // namespace

int gemm_generic(const GemmArgs &g)
{
    if (g.Mo <= 0 || g.No <= 0 || g.batch <= 0) return CUBE3D_OK;
    if ((g.Mo + TM - 1) / TM > 65535 || g.batch > 65535) return CUBE3D_ESHAPE;
    switch (g.in_dtype) {
    case CUBE3D_F32: return launch_out<float>(g);
    case CUBE3D_BF16: return launch_out<unsigned short>(g);
    case CUBE3D_FP8_E4M3: return launch_out<unsigned char>(g);
    default: return CUBE3D_EDTYPE;
    }
}

}  // namespace cube3d
