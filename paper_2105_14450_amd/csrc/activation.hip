// Element-wise activation between the two linear layers of the MLP block (Section 3.2), forward
// and backward, over a whole cube buffer: the activation acts on every processor's shard
// independently, so on one GPU it is a single streaming pass.  HBM-bandwidth work.
//   forward   h = act(z)
//   backward  dz = dh * act'(z)
// act = rectifier max(z, 0) (slope 0 at 0) or the Gaussian error linear unit in its exact form
// z * Phi(z) (no tanh or logistic stand-in), Phi evaluated in fp32.  Eight elements per lane per step,
// 16-byte accesses.
#include "common.h"

namespace cube3d {

namespace {

constexpr int VEC = 8;
constexpr int UNROLL = 2;

template <typename T> struct __attribute__((aligned(sizeof(T) * VEC))) Pack8 {
    T v[VEC];
};

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<unsigned short>(unsigned short x) { return bf16_bits_to_f32(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ unsigned short from_f32<unsigned short>(float x) { return f32_to_bf16_bits(x); }

// eight results to the stored type (bf16: four packed conversions, round to nearest even)
template <typename T> __device__ __forceinline__ Pack8<T> pack_out(const float (&v)[VEC]);
template <> __device__ __forceinline__ Pack8<float> pack_out<float>(const float (&v)[VEC])
{
    Pack8<float> o;
#pragma unroll
    for (int e = 0; e < VEC; ++e) o.v[e] = v[e];
    return o;
}
template <> __device__ __forceinline__ Pack8<unsigned short> pack_out<unsigned short>(const float (&v)[VEC])
{
    uint4 w;
    w.x = pack_bf16x2(v[0], v[1]);
    w.y = pack_bf16x2(v[2], v[3]);
    w.z = pack_bf16x2(v[4], v[5]);
    w.w = pack_bf16x2(v[6], v[7]);
    return __builtin_bit_cast(Pack8<unsigned short>, w);
}

// Phi(z), the standard normal distribution function, and phi(z), its density, in fp32 without
// branches.  For t = |z| < 6 the lower tail is Phi(-t) = 2^(-r(t)) / 2 with r(t) = -log2(2 Phi(-t)),
// a smooth function (r(0) = 0, r ~ t^2 log2(e) / 2 for large t) taken as t times a degree-9 polynomial
// (least-squares fit at 4000 Chebyshev nodes of [0, 6]: 1.2e-6 relative to the tail); beyond 6, where
// the tail is below 1e-9, the Gaussian bound 2^(-t^2 log2(e) / 2) / 2 stands in, which goes to zero
// as t grows.  The upper side is 1 - Phi(-t).  The tail keeps its relative accuracy (4e-6 after fp32
// rounding of r) however small it is, which 1 + erf(z / sqrt 2) does not; z Phi(z) is within 4e-7 of
// the exact value for |z| < 12.  One v_exp_f32 per function instead of the library erf's two ranges.
struct NormalFn {
    float cdf, pdf;
};

__device__ __forceinline__ NormalFn normal_fn(float z)
{
    const float t = fabsf(z);
    const float tq = t * t * 0.72134752f;               // t^2 / 2 in units of log2
    float r = 1.945418582e-08f;
    r = fmaf(r, t, -6.227335234e-07f);
    r = fmaf(r, t, 8.505122423e-06f);
    r = fmaf(r, t, -6.270727317e-05f);
    r = fmaf(r, t, 2.353099990e-04f);
    r = fmaf(r, t, 8.306837117e-05f);
    r = fmaf(r, t, -7.032936905e-03f);
    r = fmaf(r, t, 5.248502642e-02f);
    r = fmaf(r, t, 4.592124820e-01f);
    r = fmaf(r, t, 1.151104450e+00f);
    r = t < 6.f ? r * t : tq;
    const float tail = 0.5f * __builtin_amdgcn_exp2f(-r);
    NormalFn f;
    f.cdf = z < 0.f ? tail : 1.f - tail;
    f.pdf = 0.39894228040143268f * __builtin_amdgcn_exp2f(-tq);
    return f;
}

template <int KIND> __device__ __forceinline__ float act_value(float z)
{
    if (KIND == CUBE3D_ACT_RELU) return z > 0.f ? z : 0.f;
    return z * normal_fn(z).cdf;
}

template <int KIND> __device__ __forceinline__ float act_slope(float z)
{
    if (KIND == CUBE3D_ACT_RELU) return z > 0.f ? 1.f : 0.f;
    const NormalFn f = normal_fn(z);
    return f.cdf + z * f.pdf;
}

template <int KIND, typename TZ, typename TH>
__global__ __launch_bounds__(256) void act_fwd_kernel(const TZ *__restrict__ z, TH *__restrict__ h, int64_t n)
{
    const int64_t nvec = n / VEC, stride = (int64_t)gridDim.x * 256;
    const Pack8<TZ> *zv = reinterpret_cast<const Pack8<TZ> *>(z);
    Pack8<TH> *hv = reinterpret_cast<Pack8<TH> *>(h);
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + (UNROLL - 1) * stride < nvec; i += UNROLL * stride) {   // UNROLL loads in flight per lane
        Pack8<TZ> a[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) a[u] = zv[i + u * stride];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float o[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = act_value<KIND>(to_f32<TZ>(a[u].v[e]));
            hv[i + u * stride] = pack_out<TH>(o);
        }
    }
    for (; i < nvec; i += stride) {
        const Pack8<TZ> a = zv[i];
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = act_value<KIND>(to_f32<TZ>(a.v[e]));
        hv[i] = pack_out<TH>(o);
    }
    if (blockIdx.x == 0)
        for (int64_t i = nvec * VEC + threadIdx.x; i < n; i += 256) h[i] = from_f32<TH>(act_value<KIND>(to_f32<TZ>(z[i])));
}

template <int KIND, typename TZ, typename TG, typename TD>
__global__ __launch_bounds__(256) void act_bwd_kernel(const TZ *__restrict__ z, const TG *__restrict__ dh,
                                                      TD *__restrict__ dz, int64_t n)
{
    const int64_t nvec = n / VEC, stride = (int64_t)gridDim.x * 256;
    const Pack8<TZ> *zv = reinterpret_cast<const Pack8<TZ> *>(z);
    const Pack8<TG> *gv = reinterpret_cast<const Pack8<TG> *>(dh);
    Pack8<TD> *dv = reinterpret_cast<Pack8<TD> *>(dz);
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + (UNROLL - 1) * stride < nvec; i += UNROLL * stride) {
        Pack8<TZ> a[UNROLL];
        Pack8<TG> g[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            a[u] = zv[i + u * stride];
            g[u] = gv[i + u * stride];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float o[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = to_f32<TG>(g[u].v[e]) * act_slope<KIND>(to_f32<TZ>(a[u].v[e]));
            dv[i + u * stride] = pack_out<TD>(o);
        }
    }
    for (; i < nvec; i += stride) {
        const Pack8<TZ> a = zv[i];
        const Pack8<TG> g = gv[i];
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = to_f32<TG>(g.v[e]) * act_slope<KIND>(to_f32<TZ>(a.v[e]));
        dv[i] = pack_out<TD>(o);
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
