// Map-addressed instantiations of the tuned MFMA product kernel: the operands are cubes of
// shards in the load-balanced storage of Section 3.1.1, read in place, and the output goes
// straight into the shards of the result.  One product over the whole cube then does the work
// of Algorithm 1 (or of one line of Algorithm 2) for all q^3 processors: the all-gathers become
// address arithmetic, and the sum that the reduce-scatter takes over the q partial products is
// the continuation of the K loop across the shards of the contraction index.
#include "gemm_mfma_kernel.h"

namespace cube3d {
using namespace mfk;

namespace {

template <typename E, int T, typename TOut> int launch_mapped(const GemmArgs &g)
{
    if (g.a_kmajor && !g.b_kmajor)
        return launch_cfg<E, T, T, 64, 4, true, false, TOut, true>(g, 1, g.C, 0, 0, 0, g.alpha);
    if (g.a_kmajor && g.b_kmajor) {
        // 128-byte K-tiles (whole cache lines per row), two stages: a pass is 256 bytes as with four 64-byte tiles
        if (T == 256 && g.Kc * E::ELT % 256 == 0 && g.maps->a_k.P2 * E::ELT % 256 == 0 && g.maps->b_k.P2 * E::ELT % 256 == 0)
            return launch_cfg<E, T, T, 128, 2, true, true, TOut, true>(g, 1, g.C, 0, 0, 0, g.alpha);
        return launch_cfg<E, T, T, 64, 4, true, true, TOut, true>(g, 1, g.C, 0, 0, 0, g.alpha);
    }
    if (!g.a_kmajor && !g.b_kmajor)
        return launch_cfg<E, T, T, 64, 4, false, false, TOut, true>(g, 1, g.C, 0, 0, 0, g.alpha);
    return CUBE3D_ENOTIMPL;
}

}  // namespace

int gemm_fast_mapped(const GemmArgs &g, int tile)
{
    if (!g.maps) return CUBE3D_EINVAL;
    const bool f32 = g.out_dtype == CUBE3D_F32;
    if (g.in_dtype == CUBE3D_FP8_E4M3) {
        if (tile != 256) return CUBE3D_ENOTIMPL;
        return f32 ? launch_mapped<Fp8, 256, float>(g) : launch_mapped<Fp8, 256, unsigned short>(g);
    }
    if (g.in_dtype != CUBE3D_BF16) return CUBE3D_ENOTIMPL;
    if (tile == 256) return f32 ? launch_mapped<Bf16, 256, float>(g) : launch_mapped<Bf16, 256, unsigned short>(g);
    if (tile == 128) return f32 ? launch_mapped<Bf16, 128, float>(g) : launch_mapped<Bf16, 128, unsigned short>(g);
    return CUBE3D_ENOTIMPL;
}

}  // namespace cube3d
