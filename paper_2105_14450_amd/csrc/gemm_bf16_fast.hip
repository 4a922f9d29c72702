// Dispatch of the tuned bf16 product kernel (see gemm_bf16_kernel.h).
#include "gemm_bf16_kernel.h"

namespace cube3d {
using namespace bf16k;

size_t gemm_bf16_fast_workspace(const GemmArgs &) { return 0; }

int gemm_bf16_fast(const GemmArgs &g)
{
    constexpr int BM = 256, BN = 256, BK = 32, NSTAGE = 4;
    if (g.Mo % BM || g.No % BN || g.Kc % BK || g.Kc < BK) return CUBE3D_ENOTIMPL;
    if (g.lda % 8 || g.ldb % 8 || g.ldc % 8) return CUBE3D_ENOTIMPL;
    if (g.strideA % 8 || g.strideB % 8 || g.strideC % 8) return CUBE3D_ENOTIMPL;
    if (g.batch > 65535 || (g.Mo / BM) * (g.No / BN) > 0x7fffffff) return CUBE3D_ENOTIMPL;
    if (g.alpha != 1.f) return CUBE3D_ENOTIMPL;
    if (g.out_dtype == CUBE3D_F32) return launch_layout<BM, BN, BK, NSTAGE, float>(g);
    if (g.out_dtype == CUBE3D_BF16) return launch_layout<BM, BN, BK, NSTAGE, unsigned short>(g);
    return CUBE3D_ENOTIMPL;
}

}  // namespace cube3d
