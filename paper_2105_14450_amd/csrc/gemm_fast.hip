// Dispatch of the tuned MFMA product kernel (gemm_mfma_kernel.h): tile configuration per
// shape and dtype, deterministic split-K for shapes with very few output tiles, and the
// fixed-order reduction of the split partials.
#include "gemm_mfma_kernel.h"

namespace cube3d {
using namespace mfk;

namespace {

struct Plan {
    int tile;     // 256 or 128 (square output tile); 0 = shape not supported by the tuned kernel
    int splits;
};

// What the map-addressed instantiations assume of an index placement.
//   walked (the contraction index): shards are whole passes over the LDS stages long (`granule` indices),
//     so that a K-tile never straddles a shard and boundaries fall on pass boundaries
//   contiguous: the index that is contiguous in memory moves in 16-byte pieces of `piece` elements
//   rows: a run of `run` consecutive indices (a load chunk, an output strip) lies in one shard
bool map_ok(const AxisMap &m, int64_t extent, int64_t stride_align, bool contiguous, int64_t granule)
{
    if (m.P1 <= 0 || m.P2 <= 0 || m.P1 % m.P2 || extent % m.P1) return false;
    if (m.P2 % granule) return false;
    if (contiguous ? m.u != 1 : m.u % stride_align != 0) return false;
    return m.s1 % stride_align == 0 && m.s2 % stride_align == 0;
}

// Pure function of the shape, so that cube3d_workspace_bytes() and the launch agree.
Plan make_plan(const GemmArgs &g)
{
    Plan p{0, 1};
    const int NUM_CU = num_compute_units();
    const bool fp8 = g.in_dtype == CUBE3D_FP8_E4M3;
    if (g.in_dtype != CUBE3D_BF16 && !fp8) return p;
    const int es = fp8 ? 1 : 2;
    const int64_t align = 16 / es;              // operands are moved in 16-byte pieces
    if (g.maps) {
        // a cube of shards read in place: one product over the whole cube, no split-K
        if (g.batch != 1 || g.Mo >= (1ll << 31) || g.No >= (1ll << 31) || g.Kc >= (1ll << 31)) return p;
        if (g.out_dtype != CUBE3D_F32 && g.out_dtype != CUBE3D_BF16) return p;
        const GemmMaps &m = *g.maps;
        // contraction indices per pass over the LDS stages (four 64-byte K-tiles, or two of 128 bytes): shards
        // and blocks of a walked index must be whole passes long
        const int64_t kpt = 256 / es;
        const int64_t oalign = g.out_dtype == CUBE3D_F32 ? 4 : 8;
        if (!map_ok(m.a_k, g.Kc, align, g.a_kmajor, kpt) || !map_ok(m.b_k, g.Kc, align, g.b_kmajor, kpt)) return p;
        if (!map_ok(m.a_mn, g.Mo, align, !g.a_kmajor, 16) || !map_ok(m.b_mn, g.No, align, !g.b_kmajor, 16)) return p;
        if (!map_ok(m.c_m, g.Mo, oalign, false, 32) || !map_ok(m.c_n, g.No, oalign, true, oalign)) return p;
        // the bias is the forward product's (the tuned kernels of the other layouts carry none)
        if (m.bias && (!g.a_kmajor || g.b_kmajor || !map_ok(m.bias_n, g.No, 1, true, 4))) return p;
        if (g.Kc % kpt) return p;                // the K loop takes the four LDS stages per pass
        // the kernel addresses an operand as buffer start + 32-bit byte offset
        if ((axis_offset(m.a_mn, g.Mo - 1) + axis_offset(m.a_k, g.Kc - 1) + 1) * es >= (1ll << 32)) return p;
        if ((axis_offset(m.b_mn, g.No - 1) + axis_offset(m.b_k, g.Kc - 1) + 1) * es >= (1ll << 32)) return p;
        const bool f256 = g.Mo % 256 == 0 && g.No % 256 == 0, f128 = !fp8 && g.Mo % 128 == 0 && g.No % 128 == 0;
        if (!f256 && !f128) return p;
        p.tile = (f256 && ((g.Mo / 256) * (g.No / 256) >= (3 * NUM_CU) / 4 || !f128)) ? 256 : 128;
        return p;
    }
    if (g.lda % align || g.ldb % align || g.strideA % align || g.strideB % align) return p;
    // a tile's rows are addressed as tile start + 32-bit byte offset
    if (g.lda * es * 256 >= (1ll << 32) || g.ldb * es * 256 >= (1ll << 32)) return p;
    if (g.ldc % 8 || g.strideC % 8) return p;
    if (g.batch > 16384) return p;
    if (g.out_dtype != CUBE3D_F32 && g.out_dtype != CUBE3D_BF16) return p;
    const int64_t ktile = 64 / es;              // K elements per 64-byte K-tile
    if (g.Kc % (4 * ktile)) return p;           // the K loop takes the four LDS stages per pass
    const int64_t nk = g.Kc / ktile;
    const bool fits256 = g.Mo % 256 == 0 && g.No % 256 == 0;
    const bool fits128 = g.Mo % 128 == 0 && g.No % 128 == 0;
    if (!fits256 && !fits128) return p;
    const int64_t tiles256 = fits256 ? (g.Mo / 256) * (g.No / 256) * g.batch : 0;
    // large tiles when they occupy at least 3/4 of the CUs (fp8: half; measured on 144 tiles of a 1536 x 6144
    // output: 23.2 us against 24.3 us with 576 small tiles), else small ones
    const int64_t enough = fp8 ? NUM_CU / 2 : (3 * NUM_CU) / 4;
    if (fits256 && (tiles256 >= enough || !fits128)) p.tile = 256;
    else p.tile = 128;
    // Split-K when it shortens the launch: a split WG walks nk / splits K-tiles, but the fp32 partials
    // cost splits * Mo * No * 4 bytes each way and a second (reduction) launch.  Estimated per split
    // count from measured figures (microseconds: K-tile time per workgroup, fixed cost of a workgroup,
    // fixed cost and bandwidth of the reduction), smallest estimate wins.
    const int64_t tiles = (g.Mo / p.tile) * (g.No / p.tile) * g.batch;
    // The figures are those of one MI355X under this kernel (shader clock 1.5-2.3 GHz depending on the
    // data): a 64-byte K-tile takes a workgroup 1024 MFMA cycles at 256 x 256 and 256 at 128 x 128; start-up,
    // first loads and epilogue of a workgroup 4 us; the reduction launch 3 us plus its traffic at
    // 2.5 TB/s (short launches do not reach more).  They only rank split counts; a device twice as fast
    // in everything picks the same plan.
    constexpr double T_KTILE_256_US = 0.44, T_KTILE_128_US = 0.14, T_WORKGROUP_US = 4.0, T_REDUCE_LAUNCH_US = 3.0,
                     REDUCE_BYTES_PER_US = 2.5e6;
    const double t_ktile = p.tile == 128 ? T_KTILE_128_US : T_KTILE_256_US, t_wg = T_WORKGROUP_US, t_reduce = T_REDUCE_LAUNCH_US,
                 bytes_per_us = REDUCE_BYTES_PER_US;
    const double out_bytes = (double)g.Mo * g.No * g.batch;
    int splits = 1;
    double best = 0;
    for (int s = 1; s <= 16; s *= 2) {
        if (nk % (s * 8) != 0 && s > 1) break;            // every split takes whole passes over the LDS stages
        if (s > 1 && (double)s * out_bytes * 4 > (double)(64ll << 20)) break;
        const double rounds = (double)((tiles * s + NUM_CU - 1) / NUM_CU);
        double t = rounds * ((double)nk / s * t_ktile + t_wg);
        if (s > 1) t += t_reduce + ((double)s * 4 + 2) * out_bytes / bytes_per_us;
        if (s == 1 || t < best) {
            best = t;
            splits = s;
        }
    }
    if ((int64_t)g.batch * splits > 65535) splits = 1;
    p.splits = splits;
    return p;
}

// out[b][m][n] = sum over s (ascending) of ws[b][s][m][n], rounded once to the output type.
template <typename TOut>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ ws, TOut *__restrict__ out,
                                                           int splits, int64_t mn, int64_t ldc, int64_t No,
                                                           int64_t sC)
{
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= mn) return;
    const int b = blockIdx.y;
    const float *src = ws + (int64_t)b * splits * mn + e;
    f32x4 acc = *reinterpret_cast<const f32x4 *>(src);
    for (int s = 1; s < splits; ++s) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(src + s * mn);
        acc += v;
    }
    const int64_t row = e / No, col = e - row * No;
    TOut *dst = out + b * sC + row * ldc + col;
    if (sizeof(TOut) == 4) {
        *reinterpret_cast<f32x4 *>(dst) = acc;
    } else {
        uint2 v;
        v.x = (unsigned)f32_to_bf16_bits(acc[0]) | ((unsigned)f32_to_bf16_bits(acc[1]) << 16);
        v.y = (unsigned)f32_to_bf16_bits(acc[2]) | ((unsigned)f32_to_bf16_bits(acc[3]) << 16);
        *reinterpret_cast<uint2 *>(dst) = v;
    }
}

// K-tile depth per operand layout (measured on config-4 shapes).  A K-major operand with 64-byte
// K-tiles asks for every 128-byte cache line twice, one K-tile apart, and by then the line has left
// the CU's vector L1: with both operands K-major (dX) that doubles the L2 -> L1 fill traffic and the
// loads hold up the MFMA stream.  So dX takes 128-byte K-tiles, two stages; the layouts with a
// transposed operand take 64-byte K-tiles, four stages (shorter prologue, more slack for the loads).
template <typename E, int T, typename TOut>
int launch_for_layout(const GemmArgs &g, int splits, void *out, int64_t ld, int64_t bs, int64_t ss)
{
    if (g.a_kmajor && g.b_kmajor && T == 256 && (g.Kc * E::ELT / splits) % 256 == 0)
        return launch_cfg<E, T, T, 128, 2, true, true, TOut>(g, splits, out, ld, bs, ss, g.alpha);
    if constexpr (T == 128) {
        // small tiles of the dX layout: 128-byte K-tiles four stages deep, the whole LDS for one workgroup
        // per CU: whole cache lines per row, half as many barriers and twice the time for a load to
        // arrive (337 against 522 cycles per 64 bytes of K, also where two shallower workgroups would fit)
        if (g.a_kmajor && g.b_kmajor && (g.Kc * E::ELT / splits) % 512 == 0)
            return launch_cfg<E, T, T, 128, 4, true, true, TOut>(g, splits, out, ld, bs, ss, g.alpha);
    }
    return launch_layout<E, T, T, 64, 4, TOut>(g, splits, out, ld, bs, ss, g.alpha);
}

template <typename E, int T, typename TOut> int run_tile(const GemmArgs &g, const Plan &pl)
{
    if (pl.splits == 1) return launch_for_layout<E, T, TOut>(g, 1, g.C, g.ldc, g.strideC, 0);
    // the scale is applied once, to the partials, before the fixed-order sum
    const int64_t mn = g.Mo * g.No;
    int rc = launch_for_layout<E, T, float>(g, pl.splits, g.workspace, g.No, (int64_t)pl.splits * mn, mn);
    if (rc != CUBE3D_OK) return rc;
    dim3 grid((unsigned)((mn / 4 + 255) / 256), (unsigned)g.batch, 1);
    hipLaunchKernelGGL((splitk_reduce_kernel<TOut>), grid, dim3(256), 0, g.stream,
                       static_cast<const float *>(g.workspace), static_cast<TOut *>(g.C), pl.splits, mn, g.ldc, g.No,
                       g.strideC);
    return launch_status();
}

}  // namespace

size_t gemm_fast_workspace(const GemmArgs &g)
{
    const Plan pl = make_plan(g);
    if (pl.tile == 0 || pl.splits == 1) return 0;
    return (size_t)g.batch * pl.splits * g.Mo * g.No * sizeof(float);
}

int gemm_fast(const GemmArgs &g)
{
    const Plan pl = make_plan(g);
    if (pl.tile == 0) return CUBE3D_ENOTIMPL;
    if (g.maps) return gemm_fast_mapped(g, pl.tile);
    const bool f32 = g.out_dtype == CUBE3D_F32;
    if (g.in_dtype == CUBE3D_FP8_E4M3) {
        if (pl.tile == 256) return f32 ? run_tile<Fp8, 256, float>(g, pl) : run_tile<Fp8, 256, unsigned short>(g, pl);
        return f32 ? run_tile<Fp8, 128, float>(g, pl) : run_tile<Fp8, 128, unsigned short>(g, pl);
    }
    if (pl.tile == 256) return f32 ? run_tile<Bf16, 256, float>(g, pl) : run_tile<Bf16, 256, unsigned short>(g, pl);
    return f32 ? run_tile<Bf16, 128, float>(g, pl) : run_tile<Bf16, 128, unsigned short>(g, pl);
}

}  // namespace cube3d
