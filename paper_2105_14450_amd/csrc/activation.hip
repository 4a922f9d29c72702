// Element-wise activation between the two linear layers of the MLP block (Section 3.2), forward
// and backward, over a whole cube buffer: the activation acts on every processor's shard
// independently, so on one GPU it is a single streaming pass.  HBM-bandwidth work.
//   forward   h = act(z)
//   backward  dz = dh * act'(z)
// act = rectifier max(z, 0) (slope 0 at 0) or the Gaussian error linear unit z * Phi(z) in its exact
// (erf) form, evaluated in fp32.  Eight elements per lane per step, 16-byte accesses.
#include "common.h"

namespace cube3d {

namespace {

constexpr int VEC = 8;

template <typename T> struct __attribute__((aligned(sizeof(T) * VEC))) Pack8 {
    T v[VEC];
};

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<unsigned short>(unsigned short x) { return bf16_bits_to_f32(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ unsigned short from_f32<unsigned short>(float x) { return f32_to_bf16_bits(x); }

template <int KIND> __device__ __forceinline__ float act_value(float z)
{
    if (KIND == CUBE3D_ACT_RELU) return z > 0.f ? z : 0.f;
    return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
}

template <int KIND> __device__ __forceinline__ float act_slope(float z)
{
    if (KIND == CUBE3D_ACT_RELU) return z > 0.f ? 1.f : 0.f;
    const float cdf = 0.5f * (1.f + erff(z * 0.70710678118654752f));
    const float pdf = 0.39894228040143268f * __expf(-0.5f * z * z);
    return cdf + z * pdf;
}

template <int KIND, typename TZ, typename TH>
__global__ __launch_bounds__(256) void act_fwd_kernel(const TZ *__restrict__ z, TH *__restrict__ h, int64_t n)
{
    const int64_t nvec = n / VEC;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
        const Pack8<TZ> a = reinterpret_cast<const Pack8<TZ> *>(z)[i];
        Pack8<TH> o;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o.v[e] = from_f32<TH>(act_value<KIND>(to_f32<TZ>(a.v[e])));
        reinterpret_cast<Pack8<TH> *>(h)[i] = o;
    }
    if (blockIdx.x == 0)
        for (int64_t i = nvec * VEC + threadIdx.x; i < n; i += 256) h[i] = from_f32<TH>(act_value<KIND>(to_f32<TZ>(z[i])));
}

template <int KIND, typename TZ, typename TG, typename TD>
__global__ __launch_bounds__(256) void act_bwd_kernel(const TZ *__restrict__ z, const TG *__restrict__ dh,
                                                      TD *__restrict__ dz, int64_t n)
{
    const int64_t nvec = n / VEC;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
        const Pack8<TZ> a = reinterpret_cast<const Pack8<TZ> *>(z)[i];
        const Pack8<TG> g = reinterpret_cast<const Pack8<TG> *>(dh)[i];
        Pack8<TD> o;
#pragma unroll
        for (int e = 0; e < VEC; ++e) o.v[e] = from_f32<TD>(to_f32<TG>(g.v[e]) * act_slope<KIND>(to_f32<TZ>(a.v[e])));
        reinterpret_cast<Pack8<TD> *>(dz)[i] = o;
    }
    if (blockIdx.x == 0)
        for (int64_t i = nvec * VEC + threadIdx.x; i < n; i += 256)
            dz[i] = from_f32<TD>(to_f32<TG>(dh[i]) * act_slope<KIND>(to_f32<TZ>(z[i])));
}

unsigned grid_for(int64_t n)
{
    const int64_t want = (n / VEC + 255) / 256;
    const int64_t cap = 256 * 8;   // eight blocks per CU
    return (unsigned)(want < 1 ? 1 : want > cap ? cap : want);
}

template <int KIND, typename TZ> int fwd_out(int h_dtype, int64_t n, const void *z, void *h, hipStream_t s)
{
    const TZ *zp = static_cast<const TZ *>(z);
    if (h_dtype == CUBE3D_F32)
        hipLaunchKernelGGL((act_fwd_kernel<KIND, TZ, float>), dim3(grid_for(n)), dim3(256), 0, s, zp, static_cast<float *>(h), n);
    else
        hipLaunchKernelGGL((act_fwd_kernel<KIND, TZ, unsigned short>), dim3(grid_for(n)), dim3(256), 0, s, zp,
                           static_cast<unsigned short *>(h), n);
    return launch_status();
}

template <int KIND, typename TZ, typename TG>
int bwd_out(int dz_dtype, int64_t n, const void *z, const void *dh, void *dz, hipStream_t s)
{
    const TZ *zp = static_cast<const TZ *>(z);
    const TG *gp = static_cast<const TG *>(dh);
    if (dz_dtype == CUBE3D_F32)
        hipLaunchKernelGGL((act_bwd_kernel<KIND, TZ, TG, float>), dim3(grid_for(n)), dim3(256), 0, s, zp, gp,
                           static_cast<float *>(dz), n);
    else
        hipLaunchKernelGGL((act_bwd_kernel<KIND, TZ, TG, unsigned short>), dim3(grid_for(n)), dim3(256), 0, s, zp, gp,
                           static_cast<unsigned short *>(dz), n);
    return launch_status();
}

template <int KIND, typename TZ>
int bwd_g(int g_dtype, int dz_dtype, int64_t n, const void *z, const void *dh, void *dz, hipStream_t s)
{
    return g_dtype == CUBE3D_F32 ? bwd_out<KIND, TZ, float>(dz_dtype, n, z, dh, dz, s)
                                 : bwd_out<KIND, TZ, unsigned short>(dz_dtype, n, z, dh, dz, s);
}

}  // namespace

int activation_fwd(int kind, int z_dtype, int h_dtype, int64_t n, const void *z, void *h, hipStream_t s)
{
    if (kind == CUBE3D_ACT_RELU)
        return z_dtype == CUBE3D_F32 ? fwd_out<CUBE3D_ACT_RELU, float>(h_dtype, n, z, h, s)
                                     : fwd_out<CUBE3D_ACT_RELU, unsigned short>(h_dtype, n, z, h, s);
    return z_dtype == CUBE3D_F32 ? fwd_out<CUBE3D_ACT_GELU, float>(h_dtype, n, z, h, s)
                                 : fwd_out<CUBE3D_ACT_GELU, unsigned short>(h_dtype, n, z, h, s);
}

int activation_bwd(int kind, int z_dtype, int g_dtype, int dz_dtype, int64_t n, const void *z, const void *dh, void *dz,
                   hipStream_t s)
{
    if (kind == CUBE3D_ACT_RELU)
        return z_dtype == CUBE3D_F32 ? bwd_g<CUBE3D_ACT_RELU, float>(g_dtype, dz_dtype, n, z, dh, dz, s)
                                     : bwd_g<CUBE3D_ACT_RELU, unsigned short>(g_dtype, dz_dtype, n, z, dh, dz, s);
    return z_dtype == CUBE3D_F32 ? bwd_g<CUBE3D_ACT_GELU, float>(g_dtype, dz_dtype, n, z, dh, dz, s)
                                 : bwd_g<CUBE3D_ACT_GELU, unsigned short>(g_dtype, dz_dtype, n, z, dh, dz, s);
}

}  // namespace cube3d
