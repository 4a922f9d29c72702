// Tuned bf16 product kernel for gfx950: the local products of Algorithm 1 step 3
// and Algorithm 2 lines 1-2 at tile-aligned shapes.
//
// One workgroup of four wavefronts (one per SIMD) makes a BM x BN output tile;
// each wavefront owns a (BM/2) x (BN/2) sub-tile held in 32x32 MFMA accumulators.
// Operand tiles travel HBM -> LDS with direct-to-LDS 16-byte loads (no register
// staging), NSTAGE tiles deep.  An LDS tile is a byte-for-byte image of the global
// tile with the 16-byte slots of each row permuted (XOR swizzle) so that fragment
// reads are bank-conflict free; the permutation is applied by choosing which
// global address each lane loads, because a direct-to-LDS load always writes
// lane s to slot s of its 1 KB chunk.
//   * operand with the contraction index contiguous ("K-major"): fragments are
//     read with 16-byte LDS reads (8 consecutive k per lane);
//   * operand with the output index contiguous ("MN-major", i.e. the operand the
//     product needs transposed): fragments are read with the transposing LDS read
//     (ds_read_b64_tr_b16), which hands lane n the 4 consecutive k of column n
//     out of a 4(k) x 16(n) block; two of them make one 8-k fragment.
// The MFMA is issued with the operands exchanged (B fragment first), so a lane's
// accumulator registers hold 4 consecutive output columns of one output row and
// the epilogue can move packed rows through LDS into 16-byte coalesced stores.
#pragma once
#include <type_traits>

#include "common.h"

namespace cube3d {
namespace bf16k {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int WAVES = 4;

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

// Wait until at most N of this wavefront's direct-to-LDS loads are outstanding and all of
// its LDS reads have returned, then meet the other wavefronts.  After it, every tile whose
// loads were waited for is visible to all wavefronts, and no wavefront still reads the stage
// that is overwritten next.  The "memory" clobber keeps the compiler from moving LDS
// accesses across it.
template <int N> __device__ __forceinline__ void tile_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" : : "n"(N) : "memory");
}

// Direct-to-LDS 16-byte load: lane s of the wavefront writes LDS bytes [lds_base + 16 s, +16).
// Issued as inline assembly so that its completion is tracked by the explicit
// s_waitcnt vmcnt(..) + barrier of the pipeline below and by nothing else (the
// compiler would otherwise drain every outstanding load before each LDS read).
__device__ __forceinline__ void async_load16(const void *gptr, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_base)
                 : "m0");
}

// ---- LDS image of a K-major operand tile: ROWS x BK, k contiguous -------------------------------
template <int ROWS, int BK> struct KMajorTile {
    static constexpr int SPR = BK / 8;           // 16-byte slots per row
    static constexpr int RPC = 64 / SPR;         // rows per 1 KB chunk
    static constexpr int BYTES = ROWS * BK * 2;
    static constexpr int CPW = BYTES / 1024 / WAVES;  // chunks per wavefront
    static_assert(BYTES % (1024 * WAVES) == 0, "tile must split into whole chunks per wavefront");
    __device__ static __forceinline__ int swz(int row) { return (row / (16 / SPR)) % SPR; }
    // element offset from the tile origin (row 0, k 0) of what lane loads for this wave's first chunk
    __device__ static __forceinline__ int64_t lane_src(int wave, int lane, int64_t ld)
    {
        const int row = wave * RPC + lane / SPR;
        const int c = (lane % SPR) ^ swz(row);
        return (int64_t)row * ld + c * 8;
    }
    static constexpr int CHUNK_ROWS = WAVES * RPC;  // rows between a wave's consecutive chunks
    __device__ static __forceinline__ int64_t chunk_step(int64_t ld) { return (int64_t)CHUNK_ROWS * ld; }
    __device__ static __forceinline__ int64_t ktile_step(int64_t) { return BK; }
    // byte address inside the tile of the fragment piece (row r, 16-byte slot c)
    __device__ static __forceinline__ int frag_addr(int r, int c) { return (r * SPR + (c ^ swz(r))) * 16; }
};

// ---- LDS image of an MN-major operand tile: BK rows (k) x COLS, output index contiguous ---------
template <int COLS, int BK> struct MNMajorTile {
    static constexpr int RB = COLS * 2;          // bytes per k-row
    static constexpr int SPR = RB / 16;
    static constexpr int RPC = 1024 / RB;        // k-rows per 1 KB chunk
    static constexpr int BYTES = BK * RB;
    static constexpr int CPW = BYTES / 1024 / WAVES;
    static_assert(BYTES % (1024 * WAVES) == 0, "tile must split into whole chunks per wavefront");
    static_assert(SPR >= 16, "swizzle flips slot bits 2-3");
    __device__ static __forceinline__ int64_t lane_src(int wave, int lane, int64_t ld)
    {
        const int k = wave * RPC + lane / SPR;
        const int slot = (lane % SPR) ^ (4 * (k % 4));
        return (int64_t)k * ld + slot * 8;
    }
    static constexpr int CHUNK_ROWS = WAVES * RPC;
    static_assert(CHUNK_ROWS % 4 == 0, "k mod 4 must not change between a wave's chunks");
    __device__ static __forceinline__ int64_t chunk_step(int64_t ld) { return (int64_t)CHUNK_ROWS * ld; }
    __device__ static __forceinline__ int64_t ktile_step(int64_t ld) { return (int64_t)BK * ld; }
    // per-lane byte address (inside the tile) of the transposing read for column block `cb`
    // (32 columns), k-step 0, first half; add (ks*16 + 4*half) * RB for the others.
    __device__ static __forceinline__ int tr_addr(int lane, int cb)
    {
        const int g = lane / 16, s = lane % 16;
        const int k = 8 * (g / 2) + s / 4;
        const int slot = cb * 4 + 2 * (g % 2) + (s % 4) / 2;
        return k * RB + ((slot ^ (4 * (k % 4))) * 16) + (s % 2) * 8;
    }
};

template <typename TOut> struct OutTraits;
template <> struct OutTraits<float> {
    static constexpr int ESZ = 4;
};
template <> struct OutTraits<unsigned short> {
    static constexpr int ESZ = 2;
};

__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi)
{
    return (unsigned)f32_to_bf16_bits(lo) | ((unsigned)f32_to_bf16_bits(hi) << 16);
}

struct FastParams {
    const unsigned short *A;
    const unsigned short *B;
    void *C;
    int64_t lda, ldb, ldc;
    int64_t sA, sB, sC;
    int tiles_m, tiles_n, nk;   // nk = K-tiles per workgroup
    int group_m;
};

template <int BM, int BN, int BK, int NSTAGE, bool AK, bool BKM, typename TOut>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(const FastParams p)
{
    using ATile = typename std::conditional<AK, KMajorTile<BM, BK>, MNMajorTile<BM, BK>>::type;
    using BTile = typename std::conditional<BKM, KMajorTile<BN, BK>, MNMajorTile<BN, BK>>::type;
    constexpr int A_BYTES = ATile::BYTES, B_BYTES = BTile::BYTES, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32, KS = BK / 16;
    constexpr int LPT = ATile::CPW + BTile::CPW;   // async loads per K-tile per wavefront
    constexpr int ESZ = OutTraits<TOut>::ESZ;
    constexpr int EPI_STRIDE = WN * ESZ + 16;
    constexpr int EPI_BYTES = 32 * EPI_STRIDE;
    static_assert(NSTAGE * STAGE_BYTES <= 160 * 1024, "LDS budget");
    static_assert(WAVES * EPI_BYTES <= NSTAGE * STAGE_BYTES, "epilogue staging must fit");
    constexpr int LPS = LPT / KS;                  // async loads issued per k-step
    constexpr int LOAD_FIRST = 1, LOAD_EVERY = 2;  // behind which MFMAs of a k-step they go
    static_assert(KS % 2 == 0 && LPT % KS == 0, "loads must split evenly over the k-steps");
    static_assert(LOAD_FIRST + (LPS - 1) * LOAD_EVERY < TM * TN, "not enough MFMAs to hang the loads on");
    static_assert(NSTAGE >= 3, "a tile's loads are spread over a whole iteration");
    static_assert((NSTAGE - 2) * LPT <= 63, "vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // ---- which output tile: spread consecutive tiles of a group over one XCD's L2 ----------------
    int tile = blockIdx.x;
    {
        const int total = p.tiles_m * p.tiles_n;
        if (total % 8 == 0) tile = (tile % 8) * (total / 8) + tile / 8;   // workgroup id mod 8 = XCD
        const int per_group = p.group_m * p.tiles_n;
        const int gid = tile / per_group;
        const int first_m = gid * p.group_m;
        const int gsz = min(p.tiles_m - first_m, p.group_m);
        const int in_group = tile - gid * per_group;
        const int tm_ = first_m + in_group % gsz;
        const int tn_ = in_group / gsz;
        tile = tm_ * p.tiles_n + tn_;
    }
    const int tile_m = tile / p.tiles_n, tile_n = tile % p.tiles_n;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int batch = blockIdx.y;

    // ---- global source pointers of this lane's async loads ---------------------------------------
    const unsigned short *a_src = p.A + batch * p.sA + (AK ? m0 * p.lda : m0) + ATile::lane_src(wave, lane, p.lda);
    const unsigned short *b_src = p.B + batch * p.sB + (BKM ? n0 * p.ldb : n0) + BTile::lane_src(wave, lane, p.ldb);
    const int64_t a_chunk = ATile::chunk_step(p.lda), b_chunk = BTile::chunk_step(p.ldb);
    const int64_t a_ktile = ATile::ktile_step(p.lda), b_ktile = BTile::ktile_step(p.ldb);

    // async load number idx (compile-time) of the tile the source pointers stand on
    auto issue_load = [&](int idx, int stage) {
        const unsigned a_lds = lds0 + stage * STAGE_BYTES + wave * 1024;
        if (idx < ATile::CPW) async_load16(a_src + idx * a_chunk, a_lds + idx * (WAVES * 1024));
        else async_load16(b_src + (idx - ATile::CPW) * b_chunk, a_lds + A_BYTES + (idx - ATile::CPW) * (WAVES * 1024));
    };
    auto next_tile = [&]() {
        a_src += a_ktile;
        b_src += b_ktile;
    };

    // ---- per-lane fragment addresses (relative to the stage base) ---------------------------------
    unsigned a_addr[AK ? KS : TM], b_addr[BKM ? KS : TN];
    if (AK) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            a_addr[ks] = KMajorTile<BM, BK>::frag_addr(wm * WM + (lane & 31), ks * 2 + (lane >> 5));
    } else {
#pragma unroll
        for (int t = 0; t < TM; ++t) a_addr[t] = MNMajorTile<BM, BK>::tr_addr(lane, wm * TM + t);
    }
    if (BKM) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            b_addr[ks] = A_BYTES + KMajorTile<BN, BK>::frag_addr(wn * WN + (lane & 31), ks * 2 + (lane >> 5));
    } else {
#pragma unroll
        for (int t = 0; t < TN; ++t) b_addr[t] = A_BYTES + MNMajorTile<BN, BK>::tr_addr(lane, wn * TN + t);
    }

    // one fragment (32 rows or columns x 16 k) of k-step ks from the stage at stage_base
    auto read_a = [&](unsigned stage_base, int ks, int t) -> bf16x8 {
        if (AK) {
            const unsigned ad = stage_base + a_addr[ks] + t * (32 * KMajorTile<BM, BK>::SPR * 16);
            return *(const __attribute__((address_space(3))) bf16x8 *)(uintptr_t)ad;
        } else {
            constexpr int RB = MNMajorTile<BM, BK>::RB;
            const unsigned ad = stage_base + a_addr[t] + ks * 16 * RB;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(uintptr_t)ad);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4 *)(uintptr_t)(ad + 4 * RB));
            s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    };
    auto read_b = [&](unsigned stage_base, int ks, int t) -> bf16x8 {
        if (BKM) {
            const unsigned ad = stage_base + b_addr[ks] + t * (32 * KMajorTile<BN, BK>::SPR * 16);
            return *(const __attribute__((address_space(3))) bf16x8 *)(uintptr_t)ad;
        } else {
            constexpr int RB = MNMajorTile<BN, BK>::RB;
            const unsigned ad = stage_base + b_addr[t] + ks * 16 * RB;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(uintptr_t)ad);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4 *)(uintptr_t)(ad + 4 * RB));
            s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, v);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // ---- pipeline prologue: tiles 0 .. NSTAGE-2 in flight, tile 0 landed --------------------------
    const int nk = p.nk;
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) {
        if (s < nk) {
#pragma unroll
            for (int idx = 0; idx < LPT; ++idx) issue_load(idx, s);
            next_tile();
        }
    }
    if (nk >= NSTAGE - 1) tile_barrier<(NSTAGE - 2) * LPT>();
    else tile_barrier<0>();

    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t) fa[0][t] = read_a(lds0, 0, t);
#pragma unroll
    for (int t = 0; t < TN; ++t) fb[0][t] = read_b(lds0, 0, t);

    // ---- main loop ------------------------------------------------------------------------------
    // Each k-step issues its TM*TN MFMAs in a fixed order with, behind the first ones, the fragment
    // reads of the following k-step (one per MFMA) and this step's share of the async loads of tile
    // kt+NSTAGE-1.  The order is pinned with scheduling barriers: with one wavefront per SIMD nothing
    // else hides a latency, so reads must be in flight a whole k-step before their first use.
    // The body is instantiated three times (steady state, drain, last tile) so that the hot loop
    // carries no branches.
    int stage = 0;
    auto k_tile = [&](auto more_c, auto has_next_c) {
        constexpr bool more = decltype(more_c)::value;          // tile kt+NSTAGE-1 exists: load it
        constexpr bool has_next = decltype(has_next_c)::value;  // tile kt+1 exists
        const unsigned stage_base = lds0 + stage * STAGE_BYTES;
        int pre = stage + NSTAGE - 1;
        if (pre >= NSTAGE) pre -= NSTAGE;
        int next = stage + 1;
        if (next == NSTAGE) next = 0;
        const unsigned next_base = lds0 + next * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = ks & 1;
            const bool last = ks == KS - 1;
            if (last && has_next) {
                // fragments of this tile are all in registers; tile kt+1 must be visible, and
                // nobody may still read the stage that the next iteration's loads overwrite
                if (more) tile_barrier<(NSTAGE - 3) * LPT + (KS - 1) * LPS>();
                else tile_barrier<0>();
            }
            const unsigned rbase = last ? next_base : stage_base;
            const int rks = last ? 0 : ks + 1;
            const bool do_read = !last || has_next;
#pragma unroll
            for (int m = 0; m < TM * TN; ++m) {
                const int i = m / TN, j = m % TN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (do_read && m < TM + TN) {
                    if (m < TM) fa[cur ^ 1][m] = read_a(rbase, rks, m);
                    else fb[cur ^ 1][m - TM] = read_b(rbase, rks, m - TM);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (more && m >= LOAD_FIRST && (m - LOAD_FIRST) % LOAD_EVERY == 0 && (m - LOAD_FIRST) / LOAD_EVERY < LPS) {
                    issue_load(ks * LPS + (m - LOAD_FIRST) / LOAD_EVERY, pre);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        if (more) next_tile();
        stage = next;
    };
    {
        int kt = 0;
        for (; kt + NSTAGE - 1 < nk; ++kt) k_tile(std::true_type{}, std::true_type{});
        for (; kt + 1 < nk; ++kt) k_tile(std::false_type{}, std::true_type{});
        k_tile(std::false_type{}, std::false_type{});
    }

    // ---- epilogue: 32 rows at a time through a wave-private LDS strip -------------------------------
    __syncthreads();   // all fragment reads of the stage buffers are done
    char *epi = smem + wave * EPI_BYTES;
    TOut *C = static_cast<TOut *>(p.C) + batch * p.sC + (m0 + wm * WM) * p.ldc + n0 + wn * WN;
    constexpr int LPR = WN * ESZ / 16;   // lanes per output row
    constexpr int RPP = 64 / LPR;        // rows per pass
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // registers 4g..4g+3 of lane: row lane%32, columns j*32 + 8g + 4*(lane/32) + 0..3
                char *dst = epi + (lane & 31) * EPI_STRIDE + (j * 32 + 8 * g + 4 * (lane >> 5)) * ESZ;
                if (ESZ == 4) {
                    f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                    *reinterpret_cast<f32x4 *>(dst) = v;
                } else {
                    uint2 v;
                    v.x = pack_bf16x2(acc[i][j][4 * g], acc[i][j][4 * g + 1]);
                    v.y = pack_bf16x2(acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
                    *reinterpret_cast<uint2 *>(dst) = v;
                }
            }
        }
#pragma unroll
        for (int pass = 0; pass < 32 / RPP; ++pass) {
            const int row = pass * RPP + lane / LPR;
            const i32x4 v = *reinterpret_cast<const i32x4 *>(epi + row * EPI_STRIDE + (lane % LPR) * 16);
            char *gp = reinterpret_cast<char *>(C + (int64_t)(i * 32 + row) * p.ldc) + (lane % LPR) * 16;
            *reinterpret_cast<i32x4 *>(gp) = v;
        }
    }
}

template <int BM, int BN, int BK, int NSTAGE, bool AK, bool BKM, typename TOut>
int launch_cfg(const GemmArgs &g)
{
    using ATile = typename std::conditional<AK, KMajorTile<BM, BK>, MNMajorTile<BM, BK>>::type;
    using BTile = typename std::conditional<BKM, KMajorTile<BN, BK>, MNMajorTile<BN, BK>>::type;
    constexpr int LDS = NSTAGE * (ATile::BYTES + BTile::BYTES);
    auto kern = gemm_bf16_kernel<BM, BN, BK, NSTAGE, AK, BKM, TOut>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS) !=
            hipSuccess)
            return CUBE3D_ELAUNCH;
        configured = true;
    }
    FastParams p;
    p.A = static_cast<const unsigned short *>(g.A);
    p.B = static_cast<const unsigned short *>(g.B);
    p.C = g.C;
    p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.sA = g.strideA; p.sB = g.strideB; p.sC = g.strideC;
    p.tiles_m = (int)(g.Mo / BM);
    p.tiles_n = (int)(g.No / BN);
    p.nk = (int)(g.Kc / BK);
    p.group_m = 8;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)g.batch, 1);
    hipLaunchKernelGGL(kern, grid, dim3(256), LDS, g.stream, p);
    return launch_status();
}

template <int BM, int BN, int BK, int NSTAGE, typename TOut>
int launch_layout(const GemmArgs &g)
{
    if (g.a_kmajor && !g.b_kmajor) return launch_cfg<BM, BN, BK, NSTAGE, true, false, TOut>(g);
    if (g.a_kmajor && g.b_kmajor) return launch_cfg<BM, BN, BK, NSTAGE, true, true, TOut>(g);
    if (!g.a_kmajor && !g.b_kmajor) return launch_cfg<BM, BN, BK, NSTAGE, false, false, TOut>(g);
    return CUBE3D_ENOTIMPL;
}

}  // namespace bf16k
}  // namespace cube3d
