#include "common.h"
namespace cube3d {
size_t gemm_bf16_fast_workspace(const GemmArgs &) { return 0; }
int gemm_bf16_fast(const GemmArgs &) { return CUBE3D_ENOTIMPL; }
}
