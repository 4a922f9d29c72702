/*
 * cube3d — per-rank hot path of the 3-D model-parallel linear layer
 * (Bian, Xu, Wang, You: "Maximizing Parallelism in Distributed Training for
 * Huge Neural Networks"), for AMD MI355X (gfx950).
 *
 * The layer computes Y = X W on a q x q x q processor cube.  Processor
 * (i, j, l) multiplies one [M/q, K/q] block of X by one [K/q, N/q] block of W
 * (Section 2.3; Algorithm 1), and in the backward pass forms dX = dY W^T and
 * dW = X^T dY block products (Section 3.1.2, first differentiation formula;
 * Algorithm 2).  Before the products the blocks are all-gathered along one
 * cube direction from evenly spread shards, after them the partial results are
 * reduce-scattered along another (Section 3.1.1).  On one GPU the cube is
 * "virtual": the buffers of all q^3 processors live in one device's memory and
 * the collectives are copy / reduction kernels.
 *
 * Notation (repository <-> paper): X [M,K] = A (M,N); W [K,N] = B (N,K);
 * Y [M,N] = C (M,K); q = p.  Sizes derived by the library:
 *     Mb = M/q, Kb = K/q, Nb = N/q   (block sizes)
 *     Ms = M/q^2, Ns = N/q^2         (shard sizes)
 * All matrices are row-major and densely packed (leading dimension = number of
 * columns).
 *
 * Directions.  Processor (i, j, l) has index i along x, j along y, l along z.
 * Weights always move along x.  `in_axis` names the direction in which the
 * input X is gathered; the output is reduce-scattered along the other one of
 * {y, z}.  in_axis = CUBE3D_AXIS_Y is the layout printed in Section 3.1.1;
 * in_axis = CUBE3D_AXIS_Z is the exchanged assignment used by a layer that
 * consumes the previous layer's output in place (Section 3.1.1, last
 * paragraph; Section 3.2).  With a = index along the input direction and
 * b = index along the output direction ((a,b) = (j,l) or (l,j)):
 *     X shard  = X[i*Mb + a*Ms : +Ms, b*Kb : +Kb]          [Ms, Kb]
 *     W shard  = W[b*Kb : +Kb,       a*Nb + i*Ns : +Ns]    [Kb, Ns]
 *     Y shard  = Y[i*Mb + b*Ms : +Ms, a*Nb : +Nb]          [Ms, Nb]
 *     X block  = X[i*Mb : +Mb, b*Kb : +Kb]                 [Mb, Kb]
 *     W block  = W[b*Kb : +Kb, a*Nb : +Nb]                 [Kb, Nb]
 *     Y block  = Y[i*Mb : +Mb, a*Nb : +Nb]                 [Mb, Nb]
 * dY is stored like Y, dX like X, dW like W.
 *
 * Virtual-cube buffers.  A cube buffer holds one packed row-major block per
 * processor, q^3 blocks back to back, processor (i, j, l) at block index
 * r = (i*q + j)*q + l.  (The paper fixes no linear order; this is ours.)
 *
 * Ownership and execution.  Every data pointer is DEVICE memory owned by the
 * caller; `desc` is HOST memory read during the call only.  The library
 * allocates nothing, never synchronises the device and enqueues work only on
 * the caller's stream (`stream` is a hipStream_t passed as void*; NULL = the
 * default stream).  Outputs are fully overwritten.  Inputs and outputs must
 * not overlap.  Data pointers must be 16-byte aligned.
 *
 * State.  No result depends on an earlier call.  What the library keeps per
 * device, guarded by locks (calls may come from several threads): the number
 * of compute units, read once from the device, and one flag per kernel
 * variant saying that its one-time set-up (raising the kernel's dynamic LDS
 * limit with hipFuncSetAttribute) has been done on that device; and the
 * device address of the built-in scratch buffer of
 * cube3d_linear_bwd_dw_noalloc.  A variant is
 * set up on its first use, or all at once by cube3d_init(); call cube3d_init()
 * on each device before capturing calls into a HIP graph, so that no set-up
 * falls into the capture.
 *
 * Errors.  Every call returns a cube3d_status; 0 is success.  All argument
 * checks happen on the host before anything is enqueued, so a failed call has
 * no effect on the device.
 */
#ifndef CUBE3D_H
#define CUBE3D_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CUBE3D_VERSION 100

typedef enum cube3d_status {
    CUBE3D_OK = 0,
    CUBE3D_EINVAL = -1,     /* null pointer, q < 1, bad enum, bad rank coordinates */
    CUBE3D_ESHAPE = -2,     /* q^2 must divide M and N, q must divide K; sizes must be positive */
    CUBE3D_EDTYPE = -3,     /* unsupported in/out dtype combination */
    CUBE3D_EWORKSPACE = -4, /* workspace smaller than cube3d_workspace_bytes() */
    CUBE3D_ELAUNCH = -5,    /* the HIP runtime refused a launch */
    CUBE3D_ENOTIMPL = -6,
    CUBE3D_ESCRATCH = -7    /* cube3d_linear_bwd_dw_noalloc: the call needs more than the built-in scratch */
} cube3d_status;

typedef enum cube3d_dtype {
    CUBE3D_F32 = 0,
    CUBE3D_BF16 = 1,
    CUBE3D_FP8_E4M3 = 2     /* OCP e4m3 "fn": bias 7, no infinities, max finite 448 */
} cube3d_dtype;

typedef enum cube3d_axis {
    CUBE3D_AXIS_X = 0,      /* over i */
    CUBE3D_AXIS_Y = 1,      /* over j */
    CUBE3D_AXIS_Z = 2       /* over l */
} cube3d_axis;

typedef enum cube3d_operand {
    CUBE3D_OPERAND_X = 0,
    CUBE3D_OPERAND_W = 1,
    CUBE3D_OPERAND_DY = 2,
    CUBE3D_OPERAND_Y = 3,
    CUBE3D_OPERAND_DX = 4,
    CUBE3D_OPERAND_DW = 5,
    CUBE3D_OPERAND_BIAS = 6 /* vector parameter of length N (scatter / assemble only) */
} cube3d_operand;

typedef enum cube3d_op {
    CUBE3D_OP_FWD = 0,
    CUBE3D_OP_BWD_DX = 1,
    CUBE3D_OP_BWD_DW = 2,
    CUBE3D_OP_BIAS_BWD = 3  /* virtual_cube_bias_bwd (workspace query only) */
} cube3d_op;

/*
 * Problem descriptor (host memory).  M, K, N are the GLOBAL sizes of the layer.
 *   in_dtype     storage type of X, W and dY (shards and gathered blocks)
 *   out_dtype    storage type of the per-processor partial products written by
 *                the three product calls and read by the reduce-scatter:
 *                CUBE3D_F32 or CUBE3D_BF16.  Products always accumulate in fp32.
 *   shard_dtype  storage type of reduce-scatter results (Y, dX, dW shards):
 *                CUBE3D_F32 or CUBE3D_BF16
 *   scale_x/w/dy per-tensor dequantisation scales (real value = code * scale),
 *                used when in_dtype is CUBE3D_FP8_E4M3 and ignored otherwise;
 *                a product multiplies its fp32 accumulator by the two scales
 *                of its operands before the store.
 * The paper states no precision; these follow the benchmark configurations.
 */
typedef struct cube3d_desc {
    int32_t q;
    int32_t in_axis;        /* CUBE3D_AXIS_Y or CUBE3D_AXIS_Z */
    int64_t M, K, N;
    int32_t in_dtype;
    int32_t out_dtype;
    int32_t shard_dtype;
    float scale_x, scale_w, scale_dy;
} cube3d_desc;

/*
 * Rank coordinates for the three product calls: either a processor of the
 * cube, 0 <= i, j, l < q, in which case the data pointers address that one
 * processor's packed blocks; or i = j = l = -1, meaning ALL q^3 processors in
 * one batched launch, in which case every data pointer addresses a cube
 * buffer (block r of each buffer belongs to processor r).  The coordinates do
 * not change the arithmetic of a single-processor call.
 *
 * `workspace` is device scratch of at least cube3d_workspace_bytes() bytes
 * (may be NULL when that is 0).  Its contents are undefined afterwards.
 */

/* Algorithm 1, step 3:  P = X_block * W_block.
 *   X_block [Mb, Kb] in_dtype, W_block [Kb, Nb] in_dtype  ->  P [Mb, Nb] out_dtype */
int cube3d_linear_fwd(const cube3d_desc *desc, int i, int j, int l,
                      const void *X_block, const void *W_block, void *P,
                      void *workspace, size_t workspace_bytes, void *stream);

/* Algorithm 2, line 1 (the local product of Algorithm 3):  Q = dY_block * W_block^T.
 *   dY_block [Mb, Nb], W_block [Kb, Nb]  ->  Q [Mb, Kb] out_dtype */
int cube3d_linear_bwd_dx(const cube3d_desc *desc, int i, int j, int l,
                         const void *dY_block, const void *W_block, void *Q,
                         void *workspace, size_t workspace_bytes, void *stream);

/* Algorithm 2, line 2 (the local product of Algorithm 5):  R = X_block^T * dY_block.
 *   X_block [Mb, Kb], dY_block [Mb, Nb]  ->  R [Kb, Nb] out_dtype */
int cube3d_linear_bwd_dw(const cube3d_desc *desc, int i, int j, int l,
                         const void *X_block, const void *dY_block, void *R,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * cube3d_linear_bwd_dw for callers that cannot allocate or pass device scratch: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without
 * the workspace, same kernels, same result bits.  Where cube3d_linear_bwd_dw would need a
 * workspace (split-K partial sums, see cube3d_workspace_bytes), this call uses a buffer of
 * CUBE3D_NOALLOC_SCRATCH_BYTES that is built into the library's device code: each GPU the library
 * runs on holds one such buffer from the first use of the library on it until the process ends.
 * The call allocates nothing and frees nothing.  A shape whose plan needs more scratch than that
 * is refused with CUBE3D_ESCRATCH before anything is enqueued (use cube3d_linear_bwd_dw with a
 * workspace for it).  All calls on one GPU share the one buffer: calls that may run at the same
 * time on one GPU (different streams, or several threads) race on it and must be serialised by
 * the caller.  Nothing in the buffer has to start at zero (every partial sum is written before it
 * is read), so it is never cleared and keeps the last call's contents.  The buffer's address is
 * looked up on the call's first use on a device, or by cube3d_init().
 */
#define CUBE3D_NOALLOC_SCRATCH_BYTES (16u << 20)
int cube3d_linear_bwd_dw_noalloc(const cube3d_desc *desc, int i, int j, int l,
                                 const void *X_block, const void *dY_block, void *R, void *stream);

/* Scratch needed by a product call or by virtual_cube_bias_bwd.  op is a cube3d_op;
 * batched != 0 asks for the all-processors launch (ignored for CUBE3D_OP_BIAS_BWD, which
 * always covers the whole cube).  Returns 0 for an invalid descriptor. */
size_t cube3d_workspace_bytes(const cube3d_desc *desc, int op, int batched);

/*
 * All-gather over the whole virtual cube (Section 3.1.1; Algorithm 1 steps 1-2;
 * for dY, the first step of the products Algorithm 2 invokes).
 *   which = X  : axis must be desc->in_axis.  shards: cube buffer of [Ms, Kb];
 *                gathered: cube buffer of [Mb, Kb], row panel a' taken from the
 *                processor with input index a'.
 *   which = W  : axis must be CUBE3D_AXIS_X.  shards [Kb, Ns] -> gathered
 *                [Kb, Nb], column panel i' taken from the processor with x index i'.
 *   which = DY : axis must be the output direction.  shards [Ms, Nb] ->
 *                gathered [Mb, Nb], row panel b' from the processor with output index b'.
 * Elements are in_dtype and are copied bit for bit.
 */
int virtual_cube_gather(const cube3d_desc *desc, int which, int axis,
                        const void *shards, void *gathered, void *stream);

/*
 * Reduce-scatter over the whole virtual cube (Section 3.1.1; Algorithm 1 step 4;
 * third directions of Algorithm 2).  Partials are out_dtype, sums are formed in
 * fp32 in ascending order of the index along `axis`, and rounded once to
 * shard_dtype (nearest even).
 *   which = Y  : axis = output direction.  partials [Mb, Nb] -> shards [Ms, Nb];
 *                the processor with output index b keeps row panel b.
 *   which = DX : axis = desc->in_axis.  partials [Mb, Kb] -> shards [Ms, Kb];
 *                the processor with input index a keeps row panel a.
 *   which = DW : axis = CUBE3D_AXIS_X.  partials [Kb, Nb] -> shards [Kb, Ns];
 *                processor i keeps column panel i.
 */
int virtual_cube_reduce_scatter(const cube3d_desc *desc, int which, int axis,
                                const void *partials, void *shards, void *stream);

/*
 * The load-balanced storage itself (Section 3.1.1): spread a full row-major
 * matrix over the cube, or collect it back.
 *   which = X / DX : full [M, K] <-> cube buffer of [Ms, Kb]
 *   which = W / DW : full [K, N] <-> cube buffer of [Kb, Ns]
 *   which = Y / DY : full [M, N] <-> cube buffer of [Ms, Nb]
 *   which = BIAS   : full [N] fp32 <-> diagonal storage (see the vector-parameter calls below)
 * X, W, DY are in_dtype; Y, DX, DW are shard_dtype.  Bit-for-bit copies.
 */
int virtual_cube_scatter(const cube3d_desc *desc, int which,
                         const void *full, void *shards, void *stream);
int virtual_cube_assemble(const cube3d_desc *desc, int which,
                          const void *shards, void *full, void *stream);

/*
 * Vector parameters: the bias b of Y = X W + b (Section 3.1.1, paragraph on vectors;
 * Algorithms 7 and 8).  b has length N and is fp32 here, and so is its gradient.
 *
 * Diagonal storage: a cube buffer of [Ns] fp32 per processor in which only the processors
 * whose y and z indices coincide hold data, processor (i, j, j) holding b[j*Nb + i*Ns : +Ns].
 * Entries of the other processors are ignored on input and written as zero on output.
 * virtual_cube_scatter / virtual_cube_assemble with which = CUBE3D_OPERAND_BIAS convert
 * between the full vector [N] and this storage.
 *
 * virtual_cube_bias_gather: Algorithm 7 steps 1-2 for the output-side add: broadcast along the
 *   output direction, all-gather along x.  bias_blocks: cube buffer of [Nb] fp32; every
 *   processor receives the Nb entries of its output block.
 * virtual_cube_reduce_scatter_bias: Algorithm 1 step 4 followed by Algorithm 7 step 3 in one
 *   pass: Y shard = (sum of the q partials along `axis`, fp32, ascending) + bias block, rounded
 *   once to shard_dtype.  `axis` must be the output direction.
 * virtual_cube_bias_bwd: Algorithm 8: db = column sums of dY.  dY_shards: cube buffer of
 *   [Ms, Nb] in_dtype (fp8 codes are multiplied by scale_dy); dbias_diag: diagonal storage.
 *   The sums run over the rows in a fixed order in fp32 (run-to-run identical), in two stages:
 *   partial sums over groups of rows go to `workspace` (device memory, 16-byte aligned, at least
 *   cube3d_workspace_bytes(desc, CUBE3D_OP_BIAS_BWD, 1) bytes, else CUBE3D_EWORKSPACE; contents
 *   undefined afterwards), then the partials are added in ascending order.  The printed
 *   algorithm reduces along x only; the reduce along the output direction onto the diagonal
 *   (the adjoint of Algorithm 7's broadcast) is included, otherwise rows would be lost.
 */
int virtual_cube_bias_gather(const cube3d_desc *desc, const void *bias_diag, void *bias_blocks, void *stream);
int virtual_cube_reduce_scatter_bias(const cube3d_desc *desc, int axis, const void *partials, const void *bias_blocks,
                                     void *shards, void *stream);
int virtual_cube_bias_bwd(const cube3d_desc *desc, const void *dY_shards, void *dbias_diag, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * The whole virtual cube in one product, shards read and written in place.  On one GPU all
 * q^3 processors' shards share one memory, so the collectives of Algorithms 1 and 2 need not
 * move data: the all-gathers (Algorithm 1 steps 1-2, and of dY in Algorithm 2) become address
 * arithmetic on the shards (Section 3.1.1 fixes where every index lives), and the reduce-scatter's
 * sum over the q partial products is the K loop running on across the shards of the contraction
 * index, so each output element is accumulated in fp32 over the full contraction and rounded
 * once to shard_dtype (desc->out_dtype is not used).  Results equal those of gather -> product
 * -> reduce-scatter up to fp32 summation order (bit for bit on small-integer data).
 *   fwd:     X_shards cube of [Ms, Kb], W_shards cube of [Kb, Ns] (in_dtype) -> Y_shards cube of
 *            [Ms, Nb] (shard_dtype); bias_diag: NULL, or the diagonal storage of b (fp32), then
 *            Y = X W + b (Algorithm 7 folded into the store).
 *   bwd_dx:  dY_shards [Ms, Nb], W_shards [Kb, Ns] -> dX_shards [Ms, Kb]   (Algorithm 2 line 1)
 *   bwd_dw:  X_shards [Ms, Kb], dY_shards [Ms, Nb] -> dW_shards [Kb, Ns]   (Algorithm 2 line 2)
 * fp8 inputs are scaled by the product of the two operand scales.  Needs no workspace.
 * Any valid descriptor is accepted; shapes that fit the tuned kernel's tiles (bf16 or fp8 inputs,
 * M, K, N multiples of 128, the contraction length a multiple of four 64-byte K-tiles, shard
 * sizes multiples of 32, cube buffers shorter than 4 GB) run on it, the rest on the
 * bounds-checked kernel.
 */
int virtual_cube_linear_fwd(const cube3d_desc *desc, const void *X_shards, const void *W_shards, const void *bias_diag,
                            void *Y_shards, void *stream);
int virtual_cube_linear_bwd_dx(const cube3d_desc *desc, const void *dY_shards, const void *W_shards, void *dX_shards,
                               void *stream);
int virtual_cube_linear_bwd_dw(const cube3d_desc *desc, const void *X_shards, const void *dY_shards, void *dW_shards,
                               void *stream);

/*
 * The three matrix-product forms of Section 3.1.2 on the cube: C = A B, C = A B^T, C = A^T B
 * (Algorithms 1, 3, 5) and their backward passes (Algorithms 2, 4, 6), for matrices placed
 * anywhere on the cube.  Every algorithm is the same four steps: all-gather the first
 * operand, all-gather the second, multiply locally, reduce-scatter the result; a backward
 * algorithm is two such products with the directions permuted (the three differentiation
 * formulas of Section 3.1.2).  The calls below are those steps; the caller strings them
 * together with the placements of its matrices.
 *
 * Placement of a [rows, cols] matrix (Section 3.1.1, generalised from the three cases printed
 * there): the matrix is cut into q x q blocks; the processor's index along `row_axis` picks
 * the block row, its index along `col_axis` the block column, and along the remaining
 * direction each block is cut once more into q pieces, by rows (CUBE3D_SPLIT_ROWS: pieces
 * [rows/q^2, cols/q]) or by columns (CUBE3D_SPLIT_COLS: pieces [rows/q, cols/q^2]).  The paper's
 * A_ijl is (x, z, rows), B_lji is (z, y, cols), C_ilj is (x, y, rows).  The all-gather of a
 * matrix and the reduce-scatter of a result run along the remaining direction.  Requires
 * row_axis != col_axis, q^2 | rows and q | cols (rows split) or q | rows and q^2 | cols.
 *
 * virtual_cube_matrix_scatter / _assemble: full row-major matrix <-> cube buffer of pieces.
 * virtual_cube_matrix_gather: cube buffer of pieces -> cube buffer of whole blocks
 *   [rows/q, cols/q], pieces in index order.  Bit-for-bit copies of `dtype` elements.
 * virtual_cube_matrix_reduce_scatter: cube buffer of partial blocks [rows/q, cols/q] of
 *   `partial_dtype` (F32 or BF16) -> cube buffer of pieces of m->dtype (F32 or BF16): sum over
 *   the q processors of the remaining direction in fp32, ascending index, one rounding; the
 *   processor with index s keeps piece s.
 */
typedef enum cube3d_split {
    CUBE3D_SPLIT_ROWS = 0,
    CUBE3D_SPLIT_COLS = 1
} cube3d_split;

typedef struct cube3d_matrix {
    int32_t q;
    int32_t row_axis;       /* cube3d_axis */
    int32_t col_axis;       /* cube3d_axis */
    int32_t split;          /* cube3d_split */
    int64_t rows, cols;     /* global sizes */
    int32_t dtype;          /* storage type of the pieces (and of the blocks of a gather) */
} cube3d_matrix;

int virtual_cube_matrix_scatter(const cube3d_matrix *m, const void *full, void *pieces, void *stream);
int virtual_cube_matrix_assemble(const cube3d_matrix *m, const void *pieces, void *full, void *stream);
int virtual_cube_matrix_gather(const cube3d_matrix *m, const void *pieces, void *blocks, void *stream);
int virtual_cube_matrix_reduce_scatter(const cube3d_matrix *m, int partial_dtype, const void *partials, void *pieces,
                                       void *stream);

/*
 * Step 3 of Algorithms 1, 3, 5 (and of each line of Algorithms 2, 4, 6) for all q^3 processors
 * in one batched launch: C_r = op(A_r, B_r) on the gathered blocks of processor r.
 *   form = CUBE3D_FORM_AB  : A blocks [m, k], B blocks [k, n]
 *   form = CUBE3D_FORM_ABT : A blocks [m, k], B blocks [n, k]
 *   form = CUBE3D_FORM_ATB : A blocks [k, m], B blocks [k, n]
 * -> C blocks [m, n] of out_dtype (F32 or BF16), fp32 accumulation, multiplied by
 * scale_a * scale_b when in_dtype is CUBE3D_FP8_E4M3 (scales ignored otherwise).  m, n, k are
 * the BLOCK sizes.  All buffers are cube buffers (block r belongs to processor r).
 * `workspace`: at least cube3d_matmul_workspace_bytes() bytes of device scratch (may be NULL when
 * that is 0), else CUBE3D_EWORKSPACE.
 */
typedef enum cube3d_form {
    CUBE3D_FORM_AB = 0,
    CUBE3D_FORM_ABT = 1,
    CUBE3D_FORM_ATB = 2
} cube3d_form;

typedef struct cube3d_matmul {
    int32_t q;
    int32_t form;           /* cube3d_form */
    int64_t m, n, k;        /* block sizes: result block [m, n], contraction length k */
    int32_t in_dtype;
    int32_t out_dtype;
    float scale_a, scale_b;
} cube3d_matmul;

size_t cube3d_matmul_workspace_bytes(const cube3d_matmul *mm);

/*
 * One of the three products over the whole virtual cube with the pieces read and written in
 * place: what all-gather, all-gather, cube3d_matmul_blocks and reduce-scatter compute together
 * (Algorithms 1, 3, 5, and each line of Algorithms 2, 4, 6), without gathered copies and without
 * partial products.  Every index of the full matrices has one fixed place in the cube buffers
 * (Section 3.1.1), so the gathers are address arithmetic and the reduce-scatter's sum is the
 * contraction loop running on across the pieces: each result element is accumulated in fp32 over
 * the whole contraction and rounded once to C->dtype.
 *   form = AB  : A [m, k], B [k, n];  ABT : A [m, k], B [n, k];  ATB : A [k, m], B [k, n]
 *   -> C [m, n]  (global sizes, taken from the three descriptors, which must agree)
 * A and B have the same dtype (F32, BF16 or FP8_E4M3; fp8 results are multiplied by
 * scale_a * scale_b, scales ignored otherwise); C->dtype is F32 or BF16; all three the same q.
 * Any placements are accepted (the result is the plain product of the full matrices wherever the
 * pieces live); with the directions of the paper's algorithms this is their result.  Needs no
 * workspace.  Results equal those of the four-step path up to fp32 summation order (bit for bit on
 * small-integer data).
 */
int virtual_cube_matmul(int form, const cube3d_matrix *A, const cube3d_matrix *B, const cube3d_matrix *C,
                        float scale_a, float scale_b, const void *A_pieces, const void *B_pieces, void *C_pieces,
                        void *stream);
int cube3d_matmul_blocks(const cube3d_matmul *mm, const void *A_blocks, const void *B_blocks, void *C_blocks,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * The activation between the two 3-D linear layers of the MLP block (Section 3.2): it acts
 * element by element, so every processor applies it to its own shard and no data moves; here
 * one call covers any array of n elements (a whole cube buffer).  The output of a layer that
 * gathers its input in y is, as stored, the input of a layer that gathers in z (Section 3.1.1,
 * last paragraph), so the chain is: linear (in_axis = y) -> activation -> linear (in_axis = z).
 *   cube3d_activation_fwd:  h = act(z)
 *   cube3d_activation_bwd:  dz = dh * act'(z)
 * kind: CUBE3D_ACT_RELU = max(z, 0), slope 0 at 0; CUBE3D_ACT_GELU = z * Phi(z), Phi the standard
 * normal distribution function (erf form), evaluated in fp32.  (The paper does not name the
 * activation.)  Every dtype is CUBE3D_F32 or CUBE3D_BF16, results rounded once to nearest even;
 * n >= 0; pointers 16-byte aligned; z / dh and the output may not overlap partially (in place,
 * with equal dtypes, is allowed).
 */
typedef enum cube3d_activation {
    CUBE3D_ACT_RELU = 0,
    CUBE3D_ACT_GELU = 1
} cube3d_activation;

int cube3d_activation_fwd(int kind, int z_dtype, int h_dtype, int64_t n, const void *z, void *h, void *stream);
int cube3d_activation_bwd(int kind, int z_dtype, int dh_dtype, int dz_dtype, int64_t n, const void *z, const void *dh,
                          void *dz, void *stream);

/* One-time set-up of every kernel variant on the calling thread's current device (optional:
 * a variant is otherwise set up on its first use).  Enqueues nothing.  CUBE3D_ELAUNCH when
 * there is no device or the runtime refuses. */
int cube3d_init(void);

const char *cube3d_status_string(int status);
int cube3d_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CUBE3D_H */
