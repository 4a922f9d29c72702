// C-ABI entry points: argument validation on the host, then dispatch to the
// kernels.  Nothing here touches the device before every check has passed.
#include <mutex>

#include "common.h"

using namespace cube3d;

namespace {

int elem_size(int dtype)
{
    switch (dtype) {
    case CUBE3D_F32: return 4;
    case CUBE3D_BF16: return 2;
    case CUBE3D_FP8_E4M3: return 1;
    default: return 0;
    }
}

int check_desc(const cube3d_desc *d, CubeGeom *g)
{
    if (!d) return CUBE3D_EINVAL;
    if (d->q < 1) return CUBE3D_EINVAL;
    if (d->in_axis != CUBE3D_AXIS_Y && d->in_axis != CUBE3D_AXIS_Z) return CUBE3D_EINVAL;
    if (d->q > 40) return CUBE3D_ESHAPE;  // q^3 processors must fit a grid dimension
    if (d->M < 1 || d->K < 1 || d->N < 1) return CUBE3D_ESHAPE;
    const int64_t q = d->q, q2 = q * q;
    if (d->M % q2 || d->N % q2 || d->K % q) return CUBE3D_ESHAPE;
    if (elem_size(d->in_dtype) == 0) return CUBE3D_EDTYPE;
    if (d->out_dtype != CUBE3D_F32 && d->out_dtype != CUBE3D_BF16) return CUBE3D_EDTYPE;
    if (d->shard_dtype != CUBE3D_F32 && d->shard_dtype != CUBE3D_BF16) return CUBE3D_EDTYPE;
    if (d->in_dtype == CUBE3D_FP8_E4M3) {
        const float s[3] = {d->scale_x, d->scale_w, d->scale_dy};
        for (float v : s)
            if (!(v > 0.f) || v > 3.0e38f) return CUBE3D_EINVAL;
    }
    if (g) {
        g->q = d->q;
        g->in_axis_z = d->in_axis == CUBE3D_AXIS_Z;
        g->M = d->M; g->K = d->K; g->N = d->N;
        g->Mb = d->M / q; g->Kb = d->K / q; g->Nb = d->N / q;
        g->Ms = d->M / q2; g->Ns = d->N / q2;
    }
    return CUBE3D_OK;
}

// 1 = one processor, q^3 = all of them; negative = error
int check_coords(const cube3d_desc *d, int i, int j, int l)
{
    if (i == -1 && j == -1 && l == -1) return d->q * d->q * d->q;
    if (i < 0 || j < 0 || l < 0 || i >= d->q || j >= d->q || l >= d->q) return CUBE3D_EINVAL;
    return 1;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int build_gemm(const cube3d_desc *d, int op, int batch, const void *A, const void *B, void *C, void *ws,
               size_t ws_bytes, void *stream, GemmArgs *out)
{
    CubeGeom g;
    int rc = check_desc(d, &g);
    if (rc != CUBE3D_OK) return rc;
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C;
    a.batch = batch;
    a.in_dtype = d->in_dtype;
    a.out_dtype = d->out_dtype;
    a.workspace = ws;
    a.workspace_bytes = ws_bytes;
    a.stream = static_cast<hipStream_t>(stream);
    const bool fp8 = d->in_dtype == CUBE3D_FP8_E4M3;
    switch (op) {
    case CUBE3D_OP_FWD:      // P[Mb,Nb] = X[Mb,Kb] W[Kb,Nb]
        a.Mo = g.Mb; a.No = g.Nb; a.Kc = g.Kb;
        a.a_kmajor = true; a.b_kmajor = false;
        a.lda = g.Kb; a.ldb = g.Nb; a.ldc = g.Nb;
        a.alpha = fp8 ? d->scale_x * d->scale_w : 1.f;
        break;
    case CUBE3D_OP_BWD_DX:   // Q[Mb,Kb] = dY[Mb,Nb] W[Kb,Nb]^T
        a.Mo = g.Mb; a.No = g.Kb; a.Kc = g.Nb;
        a.a_kmajor = true; a.b_kmajor = true;
        a.lda = g.Nb; a.ldb = g.Nb; a.ldc = g.Kb;
        a.alpha = fp8 ? d->scale_dy * d->scale_w : 1.f;
        break;
    case CUBE3D_OP_BWD_DW:   // R[Kb,Nb] = X[Mb,Kb]^T dY[Mb,Nb]
        a.Mo = g.Kb; a.No = g.Nb; a.Kc = g.Mb;
        a.a_kmajor = false; a.b_kmajor = false;
        a.lda = g.Kb; a.ldb = g.Nb; a.ldc = g.Nb;
        a.alpha = fp8 ? d->scale_x * d->scale_dy : 1.f;
        break;
    default: return CUBE3D_EINVAL;
    }
    // batch strides: one packed block per processor
    a.strideA = (a.a_kmajor ? a.Mo : a.Kc) * a.lda;
    a.strideB = (a.b_kmajor ? a.No : a.Kc) * a.ldb;
    a.strideC = a.Mo * a.ldc;
    *out = a;
    return CUBE3D_OK;
}

size_t workspace_for(const GemmArgs &a)
{
    return gemm_fast_workspace(a);
}

int run_product(const cube3d_desc *d, int op, int i, int j, int l, const void *A, const void *B, void *C, void *ws,
                size_t ws_bytes, void *stream)
{
    int rc = check_desc(d, nullptr);
    if (rc != CUBE3D_OK) return rc;
    const int batch = check_coords(d, i, j, l);
    if (batch < 0) return batch;
    if (!A || !B || !C) return CUBE3D_EINVAL;
    if (misaligned(A) || misaligned(B) || misaligned(C) || misaligned(ws)) return CUBE3D_EINVAL;
    GemmArgs a;
    rc = build_gemm(d, op, batch, A, B, C, ws, ws_bytes, stream, &a);
    if (rc != CUBE3D_OK) return rc;
    const size_t need = workspace_for(a);
    if (need > 0 && (!ws || ws_bytes < need)) return CUBE3D_EWORKSPACE;
    rc = gemm_fast(a);
    if (rc != CUBE3D_ENOTIMPL) return rc;
    return gemm_generic(a);
}

// Where the indices of the full matrices land in the cube buffers of shards (Section 3.1.1):
//   X shard of (i, a, b) = X[i*Mb + a*Ms : +Ms, b*Kb : +Kb]               stored [Ms, Kb]
//   W shard of (i, a, b) = W[b*Kb : +Kb, a*Nb + i*Ns : +Ns]               stored [Kb, Ns]
//   Y shard of (i, a, b) = Y[i*Mb + b*Ms : +Ms, a*Nb : +Nb]               stored [Ms, Nb]
//   bias on (i, a, a)    = b[a*Nb + i*Ns : +Ns]
// with (a, b) the processor's indices along the input / output direction.
struct ShardMaps {
    AxisMap xm, xk, wk, wn, ym, yn, bn;
};

ShardMaps shard_maps(const CubeGeom &g)
{
    const int64_t Ri = (int64_t)g.q * g.q, Ra = g.in_axis_z ? 1 : g.q, Rb = g.in_axis_z ? g.q : 1;
    const int64_t xs = g.Ms * g.Kb, ws = g.Kb * g.Ns, ys = g.Ms * g.Nb;
    ShardMaps m;
    m.xm = AxisMap{(int32_t)g.Mb, (int32_t)g.Ms, Ri * xs, Ra * xs, g.Kb};
    m.xk = AxisMap{(int32_t)g.Kb, (int32_t)g.Kb, Rb * xs, 0, 1};
    m.wk = AxisMap{(int32_t)g.Kb, (int32_t)g.Kb, Rb * ws, 0, g.Ns};
    m.wn = AxisMap{(int32_t)g.Nb, (int32_t)g.Ns, Ra * ws, Ri * ws, 1};
    m.ym = AxisMap{(int32_t)g.Mb, (int32_t)g.Ms, Ri * ys, Rb * ys, g.Nb};
    m.yn = AxisMap{(int32_t)g.Nb, (int32_t)g.Nb, Ra * ys, 0, 1};
    m.bn = AxisMap{(int32_t)g.Nb, (int32_t)g.Ns, (Ra + Rb) * g.Ns, Ri * g.Ns, 1};
    return m;
}

// One product over the whole cube with the shards read and written in place.
int run_cube_product(const cube3d_desc *d, int op, const void *A, const void *B, const void *bias, void *C, void *stream)
{
    CubeGeom g;
    int rc = check_desc(d, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!A || !B || !C || misaligned(A) || misaligned(B) || misaligned(C) || misaligned(bias)) return CUBE3D_EINVAL;
    if (g.M >= (1ll << 31) || g.K >= (1ll << 31) || g.N >= (1ll << 31)) return CUBE3D_ESHAPE;
    const ShardMaps sm = shard_maps(g);
    const bool fp8 = d->in_dtype == CUBE3D_FP8_E4M3;
    GemmMaps mp{};
    GemmArgs a{};
    a.A = A; a.B = B; a.C = C;
    a.batch = 1;
    a.in_dtype = d->in_dtype;
    a.out_dtype = d->shard_dtype;
    a.stream = static_cast<hipStream_t>(stream);
    switch (op) {
    case CUBE3D_OP_FWD:      // Y[M,N] = X[M,K] W[K,N] (+ b)
        a.Mo = g.M; a.No = g.N; a.Kc = g.K;
        a.a_kmajor = true; a.b_kmajor = false;
        mp.a_mn = sm.xm; mp.a_k = sm.xk; mp.b_mn = sm.wn; mp.b_k = sm.wk; mp.c_m = sm.ym; mp.c_n = sm.yn;
        mp.bias = static_cast<const float *>(bias);
        mp.bias_n = sm.bn;
        a.alpha = fp8 ? d->scale_x * d->scale_w : 1.f;
        break;
    case CUBE3D_OP_BWD_DX:   // dX[M,K] = dY[M,N] W[K,N]^T
        a.Mo = g.M; a.No = g.K; a.Kc = g.N;
        a.a_kmajor = true; a.b_kmajor = true;
        mp.a_mn = sm.ym; mp.a_k = sm.yn; mp.b_mn = sm.wk; mp.b_k = sm.wn; mp.c_m = sm.xm; mp.c_n = sm.xk;
        a.alpha = fp8 ? d->scale_dy * d->scale_w : 1.f;
        break;
    case CUBE3D_OP_BWD_DW:   // dW[K,N] = X[M,K]^T dY[M,N]
        a.Mo = g.K; a.No = g.N; a.Kc = g.M;
        a.a_kmajor = false; a.b_kmajor = false;
        mp.a_mn = sm.xk; mp.a_k = sm.xm; mp.b_mn = sm.yn; mp.b_k = sm.ym; mp.c_m = sm.wk; mp.c_n = sm.wn;
        a.alpha = fp8 ? d->scale_x * d->scale_dy : 1.f;
        break;
    default: return CUBE3D_EINVAL;
    }
    if (mp.bias == nullptr) mp.bias_n = sm.bn;
    a.maps = &mp;
    rc = gemm_fast(a);
    if (rc != CUBE3D_ENOTIMPL) return rc;
    return gemm_generic(a);
}

// ---- built-in scratch of the entry point that may not allocate --------------------------------------------
// Device memory that is part of the loaded code object: every GPU the library runs on holds its own
// copy, at its own address, until the process ends.  In host code the array's name only stands for
// the symbol; the device address comes from hipGetSymbolAddress, once per device, and only that
// address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[CUBE3D_NOALLOC_SCRATCH_BYTES];

int scratch_address(void **out)
{
    static std::mutex mu;
    static void *address[MAX_DEVICES] = {};
    const int dev = current_device();
    if (dev < 0 || dev >= MAX_DEVICES) return CUBE3D_ELAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (address[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            (void)hipGetLastError();
            return CUBE3D_ELAUNCH;
        }
        address[dev] = ptr;
    }
    *out = address[dev];
    return CUBE3D_OK;
}

}  // namespace

extern "C" {

int cube3d_linear_fwd(const cube3d_desc *desc, int i, int j, int l, const void *X_block, const void *W_block, void *P,
                      void *workspace, size_t workspace_bytes, void *stream)
{
    return run_product(desc, CUBE3D_OP_FWD, i, j, l, X_block, W_block, P, workspace, workspace_bytes, stream);
}

int cube3d_linear_bwd_dx(const cube3d_desc *desc, int i, int j, int l, const void *dY_block, const void *W_block,
                         void *Q, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_product(desc, CUBE3D_OP_BWD_DX, i, j, l, dY_block, W_block, Q, workspace, workspace_bytes, stream);
}

int cube3d_linear_bwd_dw(const cube3d_desc *desc, int i, int j, int l, const void *X_block, const void *dY_block,
                         void *R, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_product(desc, CUBE3D_OP_BWD_DW, i, j, l, X_block, dY_block, R, workspace, workspace_bytes, stream);
}

size_t cube3d_workspace_bytes(const cube3d_desc *desc, int op, int batched)
{
    CubeGeom g;
    if (check_desc(desc, &g) != CUBE3D_OK) return 0;
    if (op == CUBE3D_OP_BIAS_BWD) return cube_bias_bwd_workspace(g, desc->in_dtype);
    GemmArgs a;
    const int batch = batched ? desc->q * desc->q * desc->q : 1;
    if (build_gemm(desc, op, batch, nullptr, nullptr, nullptr, nullptr, 0, nullptr, &a) != CUBE3D_OK) return 0;
    return workspace_for(a);
}

int virtual_cube_gather(const cube3d_desc *desc, int which, int axis, const void *shards, void *gathered, void *stream)
{
    CubeGeom g;
    int rc = check_desc(desc, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!shards || !gathered || misaligned(shards) || misaligned(gathered)) return CUBE3D_EINVAL;
    const int out_axis = desc->in_axis == CUBE3D_AXIS_Y ? CUBE3D_AXIS_Z : CUBE3D_AXIS_Y;
    int mode;
    switch (which) {
    case CUBE3D_OPERAND_X: if (axis != desc->in_axis) return CUBE3D_EINVAL; mode = MV_GATHER_X; break;
    case CUBE3D_OPERAND_W: if (axis != CUBE3D_AXIS_X) return CUBE3D_EINVAL; mode = MV_GATHER_W; break;
    case CUBE3D_OPERAND_DY: if (axis != out_axis) return CUBE3D_EINVAL; mode = MV_GATHER_DY; break;
    default: return CUBE3D_EINVAL;
    }
    return cube_move(g, mode, elem_size(desc->in_dtype), shards, gathered, static_cast<hipStream_t>(stream));
}

int virtual_cube_reduce_scatter(const cube3d_desc *desc, int which, int axis, const void *partials, void *shards,
                                void *stream)
{
    CubeGeom g;
    int rc = check_desc(desc, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!partials || !shards || misaligned(partials) || misaligned(shards)) return CUBE3D_EINVAL;
    const int out_axis = desc->in_axis == CUBE3D_AXIS_Y ? CUBE3D_AXIS_Z : CUBE3D_AXIS_Y;
    int mode;
    switch (which) {
    case CUBE3D_OPERAND_Y: if (axis != out_axis) return CUBE3D_EINVAL; mode = MV_REDUCE_Y; break;
    case CUBE3D_OPERAND_DX: if (axis != desc->in_axis) return CUBE3D_EINVAL; mode = MV_REDUCE_DX; break;
    case CUBE3D_OPERAND_DW: if (axis != CUBE3D_AXIS_X) return CUBE3D_EINVAL; mode = MV_REDUCE_DW; break;
    default: return CUBE3D_EINVAL;
    }
    return cube_reduce(g, mode, desc->out_dtype, desc->shard_dtype, partials, shards, nullptr,
                       static_cast<hipStream_t>(stream));
}

int virtual_cube_reduce_scatter_bias(const cube3d_desc *desc, int axis, const void *partials, const void *bias_blocks,
                                     void *shards, void *stream)
{
    CubeGeom g;
    int rc = check_desc(desc, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!partials || !shards || !bias_blocks || misaligned(partials) || misaligned(shards) || misaligned(bias_blocks))
        return CUBE3D_EINVAL;
    const int out_axis = desc->in_axis == CUBE3D_AXIS_Y ? CUBE3D_AXIS_Z : CUBE3D_AXIS_Y;
    if (axis != out_axis) return CUBE3D_EINVAL;
    return cube_reduce(g, MV_REDUCE_Y, desc->out_dtype, desc->shard_dtype, partials, shards,
                       static_cast<const float *>(bias_blocks), static_cast<hipStream_t>(stream));
}

int virtual_cube_bias_gather(const cube3d_desc *desc, const void *bias_diag, void *bias_blocks, void *stream)
{
    CubeGeom g;
    int rc = check_desc(desc, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!bias_diag || !bias_blocks || misaligned(bias_diag) || misaligned(bias_blocks)) return CUBE3D_EINVAL;
    return cube_bias_move(g, MV_GATHER_BIAS, static_cast<const float *>(bias_diag), static_cast<float *>(bias_blocks),
                          static_cast<hipStream_t>(stream));
}

int virtual_cube_bias_bwd(const cube3d_desc *desc, const void *dY_shards, void *dbias_diag, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    CubeGeom g;
    int rc = check_desc(desc, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!dY_shards || !dbias_diag || misaligned(dY_shards) || misaligned(dbias_diag) || misaligned(workspace))
        return CUBE3D_EINVAL;
    return cube_bias_bwd(g, desc->in_dtype, desc->scale_dy, dY_shards, static_cast<float *>(dbias_diag), workspace,
                         workspace_bytes, static_cast<hipStream_t>(stream));
}

int virtual_cube_linear_fwd(const cube3d_desc *desc, const void *X_shards, const void *W_shards, const void *bias_diag,
                            void *Y_shards, void *stream)
{
    return run_cube_product(desc, CUBE3D_OP_FWD, X_shards, W_shards, bias_diag, Y_shards, stream);
}

int virtual_cube_linear_bwd_dx(const cube3d_desc *desc, const void *dY_shards, const void *W_shards, void *dX_shards,
                               void *stream)
{
    return run_cube_product(desc, CUBE3D_OP_BWD_DX, dY_shards, W_shards, nullptr, dX_shards, stream);
}

int virtual_cube_linear_bwd_dw(const cube3d_desc *desc, const void *X_shards, const void *dY_shards, void *dW_shards,
                               void *stream)
{
    return run_cube_product(desc, CUBE3D_OP_BWD_DW, X_shards, dY_shards, nullptr, dW_shards, stream);
}

static int storage_move(const cube3d_desc *desc, int which, bool scatter, const void *src, void *dst, void *stream)
{
    CubeGeom g;
    int rc = check_desc(desc, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!src || !dst || misaligned(src) || misaligned(dst)) return CUBE3D_EINVAL;
    if (which == CUBE3D_OPERAND_BIAS)
        return cube_bias_move(g, scatter ? MV_SCATTER_BIAS : MV_ASSEMBLE_BIAS, static_cast<const float *>(src),
                              static_cast<float *>(dst), static_cast<hipStream_t>(stream));
    int mode, es;
    switch (which) {
    case CUBE3D_OPERAND_X: mode = scatter ? MV_SCATTER_X : MV_ASSEMBLE_X; es = elem_size(desc->in_dtype); break;
    case CUBE3D_OPERAND_W: mode = scatter ? MV_SCATTER_W : MV_ASSEMBLE_W; es = elem_size(desc->in_dtype); break;
    case CUBE3D_OPERAND_DY: mode = scatter ? MV_SCATTER_Y : MV_ASSEMBLE_Y; es = elem_size(desc->in_dtype); break;
    case CUBE3D_OPERAND_Y: mode = scatter ? MV_SCATTER_Y : MV_ASSEMBLE_Y; es = elem_size(desc->shard_dtype); break;
    case CUBE3D_OPERAND_DX: mode = scatter ? MV_SCATTER_X : MV_ASSEMBLE_X; es = elem_size(desc->shard_dtype); break;
    case CUBE3D_OPERAND_DW: mode = scatter ? MV_SCATTER_W : MV_ASSEMBLE_W; es = elem_size(desc->shard_dtype); break;
    default: return CUBE3D_EINVAL;
    }
    return cube_move(g, mode, es, src, dst, static_cast<hipStream_t>(stream));
}

int virtual_cube_scatter(const cube3d_desc *desc, int which, const void *full, void *shards, void *stream)
{
    return storage_move(desc, which, true, full, shards, stream);
}

int virtual_cube_assemble(const cube3d_desc *desc, int which, const void *shards, void *full, void *stream)
{
    return storage_move(desc, which, false, shards, full, stream);
}

}  // extern "C"

// ---- matrices placed anywhere on the cube; the three product forms (Algorithms 1-6) ----------------------
namespace {

int check_matrix(const cube3d_matrix *m, CubeGeom *g)
{
    if (!m) return CUBE3D_EINVAL;
    if (m->q < 1) return CUBE3D_EINVAL;
    if (m->row_axis < 0 || m->row_axis > 2 || m->col_axis < 0 || m->col_axis > 2 || m->row_axis == m->col_axis)
        return CUBE3D_EINVAL;
    if (m->split != CUBE3D_SPLIT_ROWS && m->split != CUBE3D_SPLIT_COLS) return CUBE3D_EINVAL;
    if (m->q > 40) return CUBE3D_ESHAPE;
    if (m->rows < 1 || m->cols < 1) return CUBE3D_ESHAPE;
    const int64_t q = m->q, q2 = q * q;
    const bool by_rows = m->split == CUBE3D_SPLIT_ROWS;
    if (m->rows % (by_rows ? q2 : q) || m->cols % (by_rows ? q : q2)) return CUBE3D_ESHAPE;
    if (elem_size(m->dtype) == 0) return CUBE3D_EDTYPE;
    CubeGeom z{};
    z.q = m->q;
    z.p_ra = m->row_axis;
    z.p_ca = m->col_axis;
    z.p_sa = 3 - m->row_axis - m->col_axis;
    z.p_split_rows = by_rows;
    z.pR = m->rows; z.pC = m->cols;
    z.pRb = m->rows / q; z.pCb = m->cols / q;
    z.pRs = by_rows ? z.pRb / q : z.pRb;
    z.pCs = by_rows ? z.pCb : z.pCb / q;
    *g = z;
    return CUBE3D_OK;
}

// Where a row / column index of the full matrix lands in the cube buffer of pieces (processor
// number r = (i*q + j)*q + l, pieces [pRs, pCs] packed back to back): block index along the row /
// column direction, piece index along the remaining direction when that direction cuts this index.
int64_t axis_rank_stride(const CubeGeom &g, int axis) { return axis == 0 ? (int64_t)g.q * g.q : axis == 1 ? g.q : 1; }

AxisMap place_row_map(const CubeGeom &g)
{
    const int64_t piece = g.pRs * g.pCs;
    if (g.p_split_rows)
        return AxisMap{(int32_t)g.pRb, (int32_t)g.pRs, axis_rank_stride(g, g.p_ra) * piece, axis_rank_stride(g, g.p_sa) * piece,
                       g.pCs};
    return AxisMap{(int32_t)g.pRb, (int32_t)g.pRb, axis_rank_stride(g, g.p_ra) * piece, 0, g.pCs};
}

AxisMap place_col_map(const CubeGeom &g)
{
    const int64_t piece = g.pRs * g.pCs;
    if (!g.p_split_rows)
        return AxisMap{(int32_t)g.pCb, (int32_t)g.pCs, axis_rank_stride(g, g.p_ca) * piece, axis_rank_stride(g, g.p_sa) * piece, 1};
    return AxisMap{(int32_t)g.pCb, (int32_t)g.pCb, axis_rank_stride(g, g.p_ca) * piece, 0, 1};
}

int matrix_move(const cube3d_matrix *m, int mode, const void *src, void *dst, void *stream)
{
    CubeGeom g;
    int rc = check_matrix(m, &g);
    if (rc != CUBE3D_OK) return rc;
    if (!src || !dst || misaligned(src) || misaligned(dst)) return CUBE3D_EINVAL;
    return cube_move(g, mode, elem_size(m->dtype), src, dst, static_cast<hipStream_t>(stream));
}

int build_matmul(const cube3d_matmul *mm, GemmArgs *out)
{
    if (!mm) return CUBE3D_EINVAL;
    if (mm->q < 1) return CUBE3D_EINVAL;
    if (mm->form != CUBE3D_FORM_AB && mm->form != CUBE3D_FORM_ABT && mm->form != CUBE3D_FORM_ATB) return CUBE3D_EINVAL;
    if (mm->q > 40) return CUBE3D_ESHAPE;
    if (mm->m < 1 || mm->n < 1 || mm->k < 1) return CUBE3D_ESHAPE;
    if (elem_size(mm->in_dtype) == 0) return CUBE3D_EDTYPE;
    if (mm->out_dtype != CUBE3D_F32 && mm->out_dtype != CUBE3D_BF16) return CUBE3D_EDTYPE;
    const bool fp8 = mm->in_dtype == CUBE3D_FP8_E4M3;
    if (fp8)
        for (float v : {mm->scale_a, mm->scale_b})
            if (!(v > 0.f) || v > 3.0e38f) return CUBE3D_EINVAL;
    GemmArgs a{};
    a.batch = mm->q * mm->q * mm->q;
    a.in_dtype = mm->in_dtype;
    a.out_dtype = mm->out_dtype;
    a.Mo = mm->m; a.No = mm->n; a.Kc = mm->k;
    a.a_kmajor = mm->form != CUBE3D_FORM_ATB;     // A stored [m, k] unless the form transposes it
    a.b_kmajor = mm->form == CUBE3D_FORM_ABT;     // B stored [n, k] only for A B^T
    a.lda = a.a_kmajor ? mm->k : mm->m;
    a.ldb = a.b_kmajor ? mm->k : mm->n;
    a.ldc = mm->n;
    a.alpha = fp8 ? mm->scale_a * mm->scale_b : 1.f;
    a.strideA = mm->m * mm->k;
    a.strideB = mm->n * mm->k;
    a.strideC = mm->m * mm->n;
    *out = a;
    return CUBE3D_OK;
}

}  // namespace

extern "C" {

int virtual_cube_matrix_scatter(const cube3d_matrix *m, const void *full, void *pieces, void *stream)
{
    return matrix_move(m, MV_PLACE_SCATTER, full, pieces, stream);
}

int virtual_cube_matrix_assemble(const cube3d_matrix *m, const void *pieces, void *full, void *stream)
{
    return matrix_move(m, MV_PLACE_ASSEMBLE, pieces, full, stream);
}

int virtual_cube_matrix_gather(const cube3d_matrix *m, const void *pieces, void *blocks, void *stream)
{
    return matrix_move(m, MV_PLACE_GATHER, pieces, blocks, stream);
}

int virtual_cube_matrix_reduce_scatter(const cube3d_matrix *m, int partial_dtype, const void *partials, void *pieces,
                                       void *stream)
{
    CubeGeom g;
    int rc = check_matrix(m, &g);
    if (rc != CUBE3D_OK) return rc;
    if (partial_dtype != CUBE3D_F32 && partial_dtype != CUBE3D_BF16) return CUBE3D_EDTYPE;
    if (m->dtype != CUBE3D_F32 && m->dtype != CUBE3D_BF16) return CUBE3D_EDTYPE;
    if (!partials || !pieces || misaligned(partials) || misaligned(pieces)) return CUBE3D_EINVAL;
    return cube_reduce(g, MV_PLACE_REDUCE, partial_dtype, m->dtype, partials, pieces, nullptr,
                       static_cast<hipStream_t>(stream));
}

int virtual_cube_matmul(int form, const cube3d_matrix *A, const cube3d_matrix *B, const cube3d_matrix *C,
                        float scale_a, float scale_b, const void *A_pieces, const void *B_pieces, void *C_pieces,
                        void *stream)
{
    if (form != CUBE3D_FORM_AB && form != CUBE3D_FORM_ABT && form != CUBE3D_FORM_ATB) return CUBE3D_EINVAL;
    CubeGeom ga, gb, gc;
    int rc = check_matrix(A, &ga);
    if (rc == CUBE3D_OK) rc = check_matrix(B, &gb);
    if (rc == CUBE3D_OK) rc = check_matrix(C, &gc);
    if (rc != CUBE3D_OK) return rc;
    if (A->q != B->q || A->q != C->q) return CUBE3D_EINVAL;
    if (A->dtype != B->dtype) return CUBE3D_EDTYPE;
    if (C->dtype != CUBE3D_F32 && C->dtype != CUBE3D_BF16) return CUBE3D_EDTYPE;
    const bool fp8 = A->dtype == CUBE3D_FP8_E4M3;
    if (fp8)
        for (float v : {scale_a, scale_b})
            if (!(v > 0.f) || v > 3.0e38f) return CUBE3D_EINVAL;
    // global sizes: result [m, n], contraction k
    const int64_t m = form == CUBE3D_FORM_ATB ? A->cols : A->rows, ka = form == CUBE3D_FORM_ATB ? A->rows : A->cols;
    const int64_t n = form == CUBE3D_FORM_ABT ? B->rows : B->cols, kb = form == CUBE3D_FORM_ABT ? B->cols : B->rows;
    if (ka != kb || C->rows != m || C->cols != n) return CUBE3D_ESHAPE;
    if (m >= (1ll << 31) || n >= (1ll << 31) || ka >= (1ll << 31)) return CUBE3D_ESHAPE;
    if (!A_pieces || !B_pieces || !C_pieces || misaligned(A_pieces) || misaligned(B_pieces) || misaligned(C_pieces))
        return CUBE3D_EINVAL;
    GemmMaps mp{};
    const bool a_t = form == CUBE3D_FORM_ATB, b_t = form == CUBE3D_FORM_ABT;
    mp.a_mn = a_t ? place_col_map(ga) : place_row_map(ga);
    mp.a_k = a_t ? place_row_map(ga) : place_col_map(ga);
    mp.b_mn = b_t ? place_row_map(gb) : place_col_map(gb);
    mp.b_k = b_t ? place_col_map(gb) : place_row_map(gb);
    mp.c_m = place_row_map(gc);
    mp.c_n = place_col_map(gc);
    mp.bias = nullptr;
    mp.bias_n = mp.c_n;
    GemmArgs a{};
    a.A = A_pieces; a.B = B_pieces; a.C = C_pieces;
    a.batch = 1;
    a.Mo = m; a.No = n; a.Kc = ka;
    a.a_kmajor = !a_t;
    a.b_kmajor = b_t;
    a.in_dtype = A->dtype;
    a.out_dtype = C->dtype;
    a.alpha = fp8 ? scale_a * scale_b : 1.f;
    a.stream = static_cast<hipStream_t>(stream);
    a.maps = &mp;
    rc = gemm_fast(a);
    if (rc != CUBE3D_ENOTIMPL) return rc;
    return gemm_generic(a);
}

size_t cube3d_matmul_workspace_bytes(const cube3d_matmul *mm)
{
    GemmArgs a;
    if (build_matmul(mm, &a) != CUBE3D_OK) return 0;
    return workspace_for(a);
}

int cube3d_matmul_blocks(const cube3d_matmul *mm, const void *A_blocks, const void *B_blocks, void *C_blocks,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    GemmArgs a;
    int rc = build_matmul(mm, &a);
    if (rc != CUBE3D_OK) return rc;
    if (!A_blocks || !B_blocks || !C_blocks) return CUBE3D_EINVAL;
    if (misaligned(A_blocks) || misaligned(B_blocks) || misaligned(C_blocks) || misaligned(workspace)) return CUBE3D_EINVAL;
    a.A = A_blocks; a.B = B_blocks; a.C = C_blocks;
    a.workspace = workspace;
    a.workspace_bytes = workspace_bytes;
    a.stream = static_cast<hipStream_t>(stream);
    const size_t need = workspace_for(a);
    if (need > 0 && (!workspace || workspace_bytes < need)) return CUBE3D_EWORKSPACE;
    rc = gemm_fast(a);
    if (rc != CUBE3D_ENOTIMPL) return rc;
    return gemm_generic(a);
}

}  // extern "C"

extern "C" {

int cube3d_activation_fwd(int kind, int z_dtype, int h_dtype, int64_t n, const void *z, void *h, void *stream)
{
    if (kind != CUBE3D_ACT_RELU && kind != CUBE3D_ACT_GELU) return CUBE3D_EINVAL;
    if (n < 0) return CUBE3D_ESHAPE;
    for (int t : {z_dtype, h_dtype})
        if (t != CUBE3D_F32 && t != CUBE3D_BF16) return CUBE3D_EDTYPE;
    if (!z || !h || misaligned(z) || misaligned(h)) return CUBE3D_EINVAL;
    if (n == 0) return CUBE3D_OK;
    return activation_fwd(kind, z_dtype, h_dtype, n, z, h, static_cast<hipStream_t>(stream));
}

int cube3d_activation_bwd(int kind, int z_dtype, int dh_dtype, int dz_dtype, int64_t n, const void *z, const void *dh,
                          void *dz, void *stream)
{
    if (kind != CUBE3D_ACT_RELU && kind != CUBE3D_ACT_GELU) return CUBE3D_EINVAL;
    if (n < 0) return CUBE3D_ESHAPE;
    for (int t : {z_dtype, dh_dtype, dz_dtype})
        if (t != CUBE3D_F32 && t != CUBE3D_BF16) return CUBE3D_EDTYPE;
    if (!z || !dh || !dz || misaligned(z) || misaligned(dh) || misaligned(dz)) return CUBE3D_EINVAL;
    if (n == 0) return CUBE3D_OK;
    return activation_bwd(kind, z_dtype, dh_dtype, dz_dtype, n, z, dh, dz, static_cast<hipStream_t>(stream));
}

int cube3d_init(void)
{
    if (current_device() < 0) return CUBE3D_ELAUNCH;
    (void)num_compute_units();
    void *ws;
    const int rc = scratch_address(&ws);
    if (rc != CUBE3D_OK) return rc;
    return setup_all_kernels();
}

int cube3d_linear_bwd_dw_noalloc(const cube3d_desc *desc, int i, int j, int l, const void *X_block, const void *dY_block,
                                 void *R, void *stream)
{
    int rc = check_desc(desc, nullptr);
    if (rc != CUBE3D_OK) return rc;
    const int batch = check_coords(desc, i, j, l);
    if (batch < 0) return batch;
    GemmArgs a;
    rc = build_gemm(desc, CUBE3D_OP_BWD_DW, batch, X_block, dY_block, R, nullptr, 0, stream, &a);
    if (rc != CUBE3D_OK) return rc;
    const size_t need = workspace_for(a);
    if (need > CUBE3D_NOALLOC_SCRATCH_BYTES) return CUBE3D_ESCRATCH;
    void *ws = nullptr;
    if (need > 0) {
        rc = scratch_address(&ws);
        if (rc != CUBE3D_OK) return rc;
    }
    return run_product(desc, CUBE3D_OP_BWD_DW, i, j, l, X_block, dY_block, R, ws, need, stream);
}

const char *cube3d_status_string(int status)
{
    switch (status) {
    case CUBE3D_OK: return "ok";
    case CUBE3D_EINVAL: return "invalid argument (null or misaligned pointer, bad enum, bad rank coordinates or scale)";
    case CUBE3D_ESHAPE: return "bad shape (q^2 must divide M and N, q must divide K, sizes positive)";
    case CUBE3D_EDTYPE: return "unsupported dtype combination";
    case CUBE3D_EWORKSPACE: return "workspace too small";
    case CUBE3D_ELAUNCH: return "HIP launch failed";
    case CUBE3D_ENOTIMPL: return "not implemented";
    case CUBE3D_ESCRATCH: return "the call needs more scratch memory than the library's built-in buffer holds";
    default: return "unknown status";
    }
}

int cube3d_version(void) { return CUBE3D_VERSION; }

}  // extern "C"
