#include "common.h"
namespace cube3d {
int gemm_fp8_fast(const GemmArgs &) { return CUBE3D_ENOTIMPL; }
}
