// Tuned MFMA product kernel for gfx950 (bf16 and fp8-e4m3 inputs, fp32 accumulation): the
// local products of Algorithm 1 step 3 and Algorithm 2 lines 1-2 at tile-aligned shapes.
//
// One workgroup of four wavefronts (2 x 2, one per SIMD) makes a BM x BN output tile; each
// wavefront owns a (BM/2) x (BN/2) sub-tile held in 32x32 MFMA accumulators.
// Operand tiles travel HBM -> LDS with direct-to-LDS 16-byte loads (no register staging),
// NSTAGE tiles deep.  An LDS tile is a byte-for-byte image of the global tile with the
// 16-byte slots of each row permuted (XOR swizzle) so that fragment reads are free of bank
// conflicts; the permutation is applied by choosing which global address each lane loads,
// because a direct-to-LDS load always writes lane s to slot s of its 1 KB chunk.
//   * operand with the contraction index contiguous ("K-major"): fragments are read with
//     16-byte LDS reads;
//   * operand with the output index contiguous ("MN-major", the operand the product needs
//     transposed): fragments are read with the transposing LDS reads of gfx950
//     (ds_read_b64_tr_b16 turns a 4(k) x 16(n) block of 16-bit elements into "lane n holds its
//     4 k"; ds_read_b64_tr_b8 does the same for an 8(k) x 16(n) block of bytes).
// The k index inside one MFMA may be permuted freely as long as both operands agree; both
// kinds of read give lane-half h the k range [h*K/2, (h+1)*K/2) of the k-step in ascending order.
// The MFMA is issued with the operands exchanged (B fragment first), so a lane's accumulator
// registers hold 4 consecutive output columns of one output row and the epilogue can move
// packed rows through LDS into 16-byte coalesced stores.
#pragma once
#include <type_traits>

#include "common.h"

namespace cube3d {
namespace mfk {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef int i32x2 __attribute__((ext_vector_type(2)));

constexpr int WAVES = 4;

#define CUBE3D_LDS(T) const __attribute__((address_space(3))) T *

// Wait until at most N of this wavefront's direct-to-LDS loads are outstanding and all of
// its LDS reads have returned, then meet the other wavefronts.  After it, every tile whose
// loads were waited for is visible to all wavefronts, and no wavefront still reads the stage
// that is overwritten next.  The wait is the s_waitcnt builtin, not assembly text, so that the
// compiler's own counter bookkeeping knows that no LDS read is outstanding behind it (otherwise
// it protects reads that are long complete with waits that also cover the reads issued just
// before, and every such wait stalls the MFMA stream).  The empty asm statements keep the
// compiler from moving LDS accesses across the barrier.
template <int N> __device__ __forceinline__ void tile_barrier()
{
    // gfx9 encoding: vmcnt = bits 3:0 and 15:14, expcnt = bits 6:4 (7: no wait), lgkmcnt = bits 11:8
    constexpr int imm = (N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(imm);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Direct-to-LDS 16-byte load: lane s of the wavefront writes LDS bytes [lds_base + 16 s, +16).
// Issued as inline assembly so that its completion is tracked by the explicit
// s_waitcnt vmcnt(..) + barrier of the pipeline and by nothing else (the compiler would
// otherwise drain every outstanding load before each LDS read).
__device__ __forceinline__ void async_load16(const void *gptr, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_base) : "m0");
}

// ---- element traits --------------------------------------------------------------------------------
struct Bf16 {
    typedef unsigned short Elem;
    typedef bf16x8 Frag;                        // 8 bf16 = 16 bytes per lane
    static constexpr int ELT = 2;
    static constexpr int KSTEP = 16;            // k per MFMA
    static constexpr int TR_ROWS = 4;           // k-rows covered by one transposing read
    __device__ static __forceinline__ int mn_swz(int k) { return 4 * (k & 3); }
    __device__ static __forceinline__ f32x16 mfma(Frag first, Frag second, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(first, second, c, 0, 0, 0);
    }
    // K-major fragment: 16 bytes at `ad`
    __device__ static __forceinline__ Frag read_k(unsigned ad0, unsigned) { return *(CUBE3D_LDS(Frag))(uintptr_t)ad0; }
    // MN-major fragment: two transposing reads, k-rows +0..3 and +4..7
    __device__ static __forceinline__ Frag read_tr(unsigned ad, int row_bytes)
    {
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(uintptr_t)ad);
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(uintptr_t)(ad + 4 * row_bytes));
        s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(Frag, v);
    }
};

struct Fp8 {
    typedef unsigned char Elem;
    typedef i32x8 Frag;                         // 32 fp8 = 32 bytes per lane
    static constexpr int ELT = 1;
    static constexpr int KSTEP = 64;
    static constexpr int TR_ROWS = 8;
    __device__ static __forceinline__ int mn_swz(int k) { return 2 * (k & 7); }
    __device__ static __forceinline__ f32x16 mfma(Frag first, Frag second, f32x16 c)
    {
        // both operands e4m3 (format code 0), block scales 2^0
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(first, second, c, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    }
    __device__ static __forceinline__ Frag read_k(unsigned ad0, unsigned ad1)
    {
        const i32x4 lo = *(CUBE3D_LDS(i32x4))(uintptr_t)ad0;
        const i32x4 hi = *(CUBE3D_LDS(i32x4))(uintptr_t)ad1;
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    __device__ static __forceinline__ Frag read_tr(unsigned ad, int row_bytes)
    {
        i32x2 r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            r[j] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                (__attribute__((address_space(3))) i32x2 *)(uintptr_t)(ad + 8 * j * row_bytes));
        Frag f = {r[0][0], r[0][1], r[1][0], r[1][1], r[2][0], r[2][1], r[3][0], r[3][1]};
        return f;
    }
};

// ---- LDS image of a K-major operand tile: ROWS rows of BKB bytes, k contiguous ------------------------
template <typename E, int ROWS, int BKB> struct KMajorTile {
    static constexpr int SPR = BKB / 16;         // 16-byte slots per row
    static_assert(SPR == 4 || SPR == 8, "rows of 64 or 128 bytes");
    static constexpr int RPC = 64 / SPR;         // rows per 1 KB chunk
    static constexpr int BYTES = ROWS * BKB;
    static constexpr int CPW = BYTES / 1024 / WAVES;  // chunks per wavefront
    static_assert(BYTES % (1024 * WAVES) == 0, "tile must split into whole chunks per wavefront");
    static constexpr int FSLOTS = (E::KSTEP * E::ELT / 2) / 16;   // 16-byte reads per fragment (1 or 2)
    // 16 consecutive rows must hit 16 different slots modulo 256 bytes
    __device__ static __forceinline__ int swz(int row) { return (row / (16 / SPR)) % SPR; }
    // element offset from the tile origin (row 0, k 0) of what `lane` loads for this wave's first chunk
    __device__ static __forceinline__ int64_t lane_src(int wave, int lane, int64_t ld)
    {
        const int row = wave * RPC + lane / SPR;
        const int c = (lane % SPR) ^ swz(row);
        return (int64_t)row * ld + c * (16 / E::ELT);
    }
    static constexpr int CHUNK_ROWS = WAVES * RPC;  // rows between a wave's consecutive chunks
    __device__ static __forceinline__ int64_t chunk_step(int64_t ld) { return (int64_t)CHUNK_ROWS * ld; }
    __device__ static __forceinline__ int64_t ktile_step(int64_t) { return BKB / E::ELT; }
    // byte address inside the tile of (row r, 16-byte slot c)
    __device__ static __forceinline__ int slot_addr(int r, int c) { return (r * SPR + (c ^ swz(r))) * 16; }
    static constexpr int BLOCK_STEP = 32 * SPR * 16;   // bytes between consecutive 32-row blocks
};

// ---- LDS image of an MN-major operand tile: BKB/ELT rows (k) of COLS elements ---------------------------
template <typename E, int COLS, int BKB> struct MNMajorTile {
    static constexpr int KROWS = BKB / E::ELT;
    static constexpr int RB = COLS * E::ELT;     // bytes per k-row
    static constexpr int SPR = RB / 16;
    static constexpr int RPC = 1024 / RB;        // k-rows per 1 KB chunk
    static constexpr int BYTES = KROWS * RB;
    static constexpr int CPW = BYTES / 1024 / WAVES;
    static_assert(BYTES % (1024 * WAVES) == 0, "tile must split into whole chunks per wavefront");
    static_assert(SPR >= 16 && RB <= 1024, "the swizzle permutes slots inside aligned groups of 16");
    __device__ static __forceinline__ int64_t lane_src(int wave, int lane, int64_t ld)
    {
        const int k = wave * RPC + lane / SPR;
        const int slot = (lane % SPR) ^ E::mn_swz(k);
        return (int64_t)k * ld + slot * (16 / E::ELT);
    }
    static constexpr int CHUNK_ROWS = WAVES * RPC;
    static_assert(CHUNK_ROWS % E::TR_ROWS == 0, "the swizzle phase of a lane must not change between its chunks");
    __device__ static __forceinline__ int64_t chunk_step(int64_t ld) { return (int64_t)CHUNK_ROWS * ld; }
    __device__ static __forceinline__ int64_t ktile_step(int64_t ld) { return (int64_t)KROWS * ld; }
    // per-lane byte address (inside the tile) of the first transposing read of k-step 0 for the
    // 32-column block `cb`; k-step ks adds ks * KSTEP * RB, the further reads of a fragment add
    // TR_ROWS * RB each.  A group of 16 lanes reads TR_ROWS k-rows x 16 columns.
    __device__ static __forceinline__ int tr_addr(int lane, int cb)
    {
        constexpr int LR = 16 / E::TR_ROWS;       // lanes per k-row
        constexpr int EPL = 8 / E::ELT;           // elements per lane per read
        const int g = lane / 16, s = lane % 16;
        const int k = (E::KSTEP / 2) * (g / 2) + s / LR;
        const int byte = (cb * 32 + 16 * (g % 2) + EPL * (s % LR)) * E::ELT;
        return k * RB + (((byte / 16) ^ E::mn_swz(k)) * 16) + byte % 16;
    }
};

__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi)
{
    return (unsigned)f32_to_bf16_bits(lo) | ((unsigned)f32_to_bf16_bits(hi) << 16);
}

// Advance of a map-addressed operand from one K-tile to the next (all values in elements): the
// plain step inside a shard, and the corrections when the tile walks off a shard (jump2) or off
// a block (jump1) of the contraction index.
struct KWalk {
    int64_t step, jump1, jump2;
    int32_t P1, P2;
};

inline KWalk make_kwalk(const AxisMap &m, int k_per_tile)
{
    KWalk w;
    w.step = (int64_t)k_per_tile * m.u;
    w.jump2 = m.s2 - (int64_t)m.P2 * m.u;
    w.jump1 = m.s1 - (int64_t)m.P2 * m.u - (int64_t)(m.P1 / m.P2 - 1) * m.s2;
    w.P1 = m.P1;
    w.P2 = m.P2;
    return w;
}

struct Params {
    const void *A;
    const void *B;
    void *C;
    int64_t lda, ldb, ldc;
    int64_t sA, sB, sC;
    int tiles_m, tiles_n, nk;   // nk = K-tiles per workgroup
    int group_m;
    int splits;                 // split-K: blockIdx.y = batch * splits + split; split s takes K-tiles [s*nk, (s+1)*nk)
    int64_t sSplit;             // output distance between the partial results of consecutive splits (elements)
    float alpha;
    // MAPPED instantiations only (then lda / ldb / ldc, the strides and the splits are unused)
    GemmMaps maps;
    KWalk ka, kb;
};

// TOut: float or unsigned short (bf16 bits).  MAPPED: operands, output and the optional bias are
// addressed through p.maps (a cube of shards read in place) instead of leading dimensions.
template <typename E, int BM, int BN, int BKB, int NSTAGE, bool AK, bool BKM, typename TOut, bool MAPPED = false>
__global__ __launch_bounds__(256, (BM * BN <= 128 * 128) ? 2 : 1) void gemm_mfma_kernel(const Params p)
{
    typedef typename E::Elem Elem;
    typedef typename E::Frag Frag;
    using ATile = typename std::conditional<AK, KMajorTile<E, BM, BKB>, MNMajorTile<E, BM, BKB>>::type;
    using BTile = typename std::conditional<BKM, KMajorTile<E, BN, BKB>, MNMajorTile<E, BN, BKB>>::type;
    constexpr int A_BYTES = ATile::BYTES, B_BYTES = BTile::BYTES, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int KS = BKB / (E::KSTEP * E::ELT);      // k-steps (MFMAs deep) per K-tile
    constexpr int NM = TM * TN;                        // MFMAs per k-step
    constexpr int NR = TM + TN;                        // fragments per k-step
    constexpr int LPT = ATile::CPW + BTile::CPW;       // async loads per K-tile per wavefront
    constexpr int TOT = KS * NM;                       // MFMAs per K-tile
    constexpr int UNROLL = (KS % 2) ? 2 : 1;           // K-tiles per loop body (fragment buffers alternate per k-step)
    constexpr int ESZ = sizeof(TOut);
    constexpr int EPI_STRIDE = WN * ESZ + 16;
    constexpr int EPI_BYTES = 32 * EPI_STRIDE;
    constexpr int FS = (E::KSTEP * E::ELT / 2) / 16;   // 16-byte reads per K-major fragment
    static_assert(KS >= 1 && BKB % (E::KSTEP * E::ELT) == 0, "K-tile must hold whole k-steps");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wavefront tile is made of 32x32 MFMA tiles");
    // NSTAGE >= 3: the loads of tile kt+NSTAGE-1 are spread over the whole of iteration kt.
    // NSTAGE == 2: the loads of tile kt+2 go into the stage of tile kt as soon as the barrier
    // before its last k-step has shown that nobody reads it any more (all behind that k-step's MFMAs).
    constexpr bool TWO_STAGE = NSTAGE == 2;
    constexpr int PRE = TWO_STAGE ? 2 : NSTAGE - 1;    // tiles in flight after the prologue
    static_assert(NSTAGE >= 2, "at least double buffering");
    static_assert(!TWO_STAGE || KS % 2 == 0, "the two-stage schedule is written for an even number of k-steps");
    static_assert(NSTAGE * STAGE_BYTES <= 160 * 1024, "LDS budget");
    static_assert(WAVES * EPI_BYTES + BN * 4 <= NSTAGE * STAGE_BYTES, "epilogue staging (and the bias strip) must fit");
    static_assert((NSTAGE - 2) * LPT <= 63, "vmcnt range");
    // loads of this iteration already issued when the tile barrier (before the last k-step) is reached
    constexpr int LOADS_BEFORE_BARRIER = ((KS - 1) * NM * LPT) / TOT;
    // loads that may still be in flight behind the steady-state barrier: those of the tiles after kt+1
    constexpr int STEADY_VMCNT = (NSTAGE == 2) ? 0 : (NSTAGE - 3) * LPT + LOADS_BEFORE_BARRIER;

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // ---- which output tile: consecutive ids go to different XCDs (id mod 8), so regroup them so
    //      that the tiles one XCD runs together form a compact patch of the tile grid (shared L2)
    int tile = blockIdx.x;
    {
        const int total = p.tiles_m * p.tiles_n;
        if (total % 8 == 0) tile = (tile % 8) * (total / 8) + tile / 8;
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
    const int batch = blockIdx.y / p.splits;
    const int split = blockIdx.y - batch * p.splits;

    // ---- global source pointers of this lane's async loads -------------------------------------------
    const int64_t a_chunk = ATile::chunk_step(p.lda), b_chunk = BTile::chunk_step(p.ldb);
    const int64_t a_ktile = ATile::ktile_step(p.lda), b_ktile = BTile::ktile_step(p.ldb);
    const int64_t kt0 = (int64_t)split * p.nk;   // first K-tile of this split
    const Elem *a_src, *b_src;
    // MAPPED: distance from a wavefront's first chunk to its chunk idx (wave-uniform: a chunk's rows
    // lie in one shard), and the position of the K walk inside the current shard / block
    int64_t a_coff[ATile::CPW], b_coff[BTile::CPW];
    int a_c1 = 0, a_c2 = 0, b_c1 = 0, b_c2 = 0;
    if constexpr (!MAPPED) {
        a_src = static_cast<const Elem *>(p.A) + batch * p.sA + (AK ? m0 * p.lda : m0) + kt0 * a_ktile +
                ATile::lane_src(wave, lane, p.lda);
        b_src = static_cast<const Elem *>(p.B) + batch * p.sB + (BKM ? n0 * p.ldb : n0) + kt0 * b_ktile +
                BTile::lane_src(wave, lane, p.ldb);
    } else {
        constexpr int EPS = 16 / E::ELT;   // elements per 16-byte slot
        {
            const int first = wave * ATile::RPC + lane / ATile::SPR;   // tile row (K-major) or k-row (MN-major)
            if constexpr (AK) {
                const int c = (lane % ATile::SPR) ^ KMajorTile<E, BM, BKB>::swz(first);
                a_src = static_cast<const Elem *>(p.A) + axis_offset(p.maps.a_mn, m0 + first) + c * EPS;
                const int64_t base = axis_offset(p.maps.a_mn, m0 + wave * ATile::RPC);
#pragma unroll
                for (int idx = 0; idx < ATile::CPW; ++idx)
                    a_coff[idx] = axis_offset(p.maps.a_mn, m0 + wave * ATile::RPC + idx * ATile::CHUNK_ROWS) - base;
            } else {
                const int slot = (lane % ATile::SPR) ^ E::mn_swz(first);
                a_src = static_cast<const Elem *>(p.A) + axis_offset(p.maps.a_mn, m0 + slot * EPS) + first * p.maps.a_k.u;
#pragma unroll
                for (int idx = 0; idx < ATile::CPW; ++idx) a_coff[idx] = (int64_t)idx * ATile::CHUNK_ROWS * p.maps.a_k.u;
            }
        }
        {
            const int first = wave * BTile::RPC + lane / BTile::SPR;
            if constexpr (BKM) {
                const int c = (lane % BTile::SPR) ^ KMajorTile<E, BN, BKB>::swz(first);
                b_src = static_cast<const Elem *>(p.B) + axis_offset(p.maps.b_mn, n0 + first) + c * EPS;
                const int64_t base = axis_offset(p.maps.b_mn, n0 + wave * BTile::RPC);
#pragma unroll
                for (int idx = 0; idx < BTile::CPW; ++idx)
                    b_coff[idx] = axis_offset(p.maps.b_mn, n0 + wave * BTile::RPC + idx * BTile::CHUNK_ROWS) - base;
            } else {
                const int slot = (lane % BTile::SPR) ^ E::mn_swz(first);
                b_src = static_cast<const Elem *>(p.B) + axis_offset(p.maps.b_mn, n0 + slot * EPS) + first * p.maps.b_k.u;
#pragma unroll
                for (int idx = 0; idx < BTile::CPW; ++idx) b_coff[idx] = (int64_t)idx * BTile::CHUNK_ROWS * p.maps.b_k.u;
            }
        }
    }

    // async load number idx (compile-time) of the tile the source pointers stand on
    auto issue_load = [&](int idx, int stage) {
        const unsigned a_lds = lds0 + stage * STAGE_BYTES + wave * 1024;
        if constexpr (!MAPPED) {
            if (idx < ATile::CPW) async_load16(a_src + idx * a_chunk, a_lds + idx * (WAVES * 1024));
            else async_load16(b_src + (idx - ATile::CPW) * b_chunk, a_lds + A_BYTES + (idx - ATile::CPW) * (WAVES * 1024));
        } else {
            if (idx < ATile::CPW) async_load16(a_src + a_coff[idx], a_lds + idx * (WAVES * 1024));
            else async_load16(b_src + b_coff[idx - ATile::CPW], a_lds + A_BYTES + (idx - ATile::CPW) * (WAVES * 1024));
        }
    };
    auto next_tile = [&]() {
        if constexpr (!MAPPED) {
            a_src += a_ktile;
            b_src += b_ktile;
        } else {
            constexpr int KPT = BKB / E::ELT;   // contraction indices per K-tile
            int64_t da = p.ka.step, db = p.kb.step;
            a_c1 += KPT; a_c2 += KPT;
            if (a_c1 == p.ka.P1) { a_c1 = 0; a_c2 = 0; da += p.ka.jump1; }
            else if (a_c2 == p.ka.P2) { a_c2 = 0; da += p.ka.jump2; }
            b_c1 += KPT; b_c2 += KPT;
            if (b_c1 == p.kb.P1) { b_c1 = 0; b_c2 = 0; db += p.kb.jump1; }
            else if (b_c2 == p.kb.P2) { b_c2 = 0; db += p.kb.jump2; }
            a_src += da;
            b_src += db;
        }
    };

    // ---- per-lane fragment addresses (relative to the stage base) -------------------------------------
    unsigned a_addr[AK ? KS * FS : TM], b_addr[BKM ? KS * FS : TN];
    if (AK) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int f = 0; f < FS; ++f)
                a_addr[ks * FS + f] =
                    KMajorTile<E, BM, BKB>::slot_addr(wm * WM + (lane & 31), ks * 2 * FS + (lane >> 5) * FS + f);
    } else {
#pragma unroll
        for (int t = 0; t < TM; ++t) a_addr[t] = MNMajorTile<E, BM, BKB>::tr_addr(lane, wm * TM + t);
    }
    if (BKM) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int f = 0; f < FS; ++f)
                b_addr[ks * FS + f] = A_BYTES + KMajorTile<E, BN, BKB>::slot_addr(wn * WN + (lane & 31),
                                                                                 ks * 2 * FS + (lane >> 5) * FS + f);
    } else {
#pragma unroll
        for (int t = 0; t < TN; ++t) b_addr[t] = A_BYTES + MNMajorTile<E, BN, BKB>::tr_addr(lane, wn * TN + t);
    }

    // one fragment (32 rows or columns x one k-step) from the stage at stage_base
    auto read_a = [&](unsigned stage_base, int ks, int t) -> Frag {
        if (AK) {
            const unsigned off = stage_base + t * KMajorTile<E, BM, BKB>::BLOCK_STEP;
            return E::read_k(off + a_addr[ks * FS], off + a_addr[ks * FS + FS - 1]);
        } else {
            constexpr int RB = MNMajorTile<E, BM, BKB>::RB;
            return E::read_tr(stage_base + a_addr[t] + ks * E::KSTEP * RB, RB);
        }
    };
    auto read_b = [&](unsigned stage_base, int ks, int t) -> Frag {
        if (BKM) {
            const unsigned off = stage_base + t * KMajorTile<E, BN, BKB>::BLOCK_STEP;
            return E::read_k(off + b_addr[ks * FS], off + b_addr[ks * FS + FS - 1]);
        } else {
            constexpr int RB = MNMajorTile<E, BN, BKB>::RB;
            return E::read_tr(stage_base + b_addr[t] + ks * E::KSTEP * RB, RB);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // ---- pipeline prologue: tiles 0 .. NSTAGE-2 in flight, tile 0 landed ------------------------------
    const int nk = p.nk;
#pragma unroll
    for (int s = 0; s < PRE; ++s) {
        if (s < nk) {
#pragma unroll
            for (int idx = 0; idx < LPT; ++idx) issue_load(idx, s);
            next_tile();
        }
    }
    if (nk >= PRE) tile_barrier<(PRE - 1) * LPT>();
    else tile_barrier<0>();

    Frag fa[2][TM], fb[2][TN];
#pragma unroll
    for (int t = 0; t < TM; ++t) fa[0][t] = read_a(lds0, 0, t);
#pragma unroll
    for (int t = 0; t < TN; ++t) fb[0][t] = read_b(lds0, 0, t);

    // ---- main loop ----------------------------------------------------------------------------------
    // Each k-step issues its MFMAs in a fixed order with, spread between them, the fragment reads of
    // the following k-step and this step's share of the async loads of tile kt+NSTAGE-1.  The order
    // is pinned with scheduling barriers: with one wavefront per SIMD nothing else hides a latency,
    // so reads must be in flight well before their first use.  The body is instantiated for the
    // steady state, the drain and the last tile so that the hot loop carries no branches.
    int stage = 0;
    auto k_tile = [&](auto more_c, auto has_next_c, auto parity_c) {
        constexpr bool more = decltype(more_c)::value;          // tile kt+PRE exists: load it
        constexpr bool has_next = decltype(has_next_c)::value;  // tile kt+1 exists
        constexpr int parity = decltype(parity_c)::value;       // fragment buffer holding this tile's k-step 0
        const unsigned stage_base = lds0 + stage * STAGE_BYTES;
        int pre = TWO_STAGE ? stage : stage + NSTAGE - 1;   // stage the loads of this iteration go to
        if (pre >= NSTAGE) pre -= NSTAGE;
        int next = stage + 1;
        if (next == NSTAGE) next = 0;
        const unsigned next_base = lds0 + next * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = (parity + ks) & 1;
            const bool last = ks == KS - 1;
            if (last && has_next) {
                // fragments of this tile are all in registers (or being read from an older barrier's
                // tile); tile kt+1 must be visible, and nobody may still read the stage that the
                // next iteration's loads overwrite
                if (more) tile_barrier<STEADY_VMCNT>();
                else tile_barrier<0>();
            }
            const unsigned rbase = last ? next_base : stage_base;
            const int rks = last ? 0 : ks + 1;
            const bool do_read = !last || has_next;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int i = m / TN, j = m % TN;
                acc[i][j] = E::mfma(fb[cur][j], fa[cur][i], acc[i][j]);
                __builtin_amdgcn_sched_barrier(0);
                if (do_read) {
#pragma unroll
                    for (int u = 0; u < NR; ++u) {
                        // fragments in the order the next k-step first needs them: a0 b0 a1 b1 ..., then
                        // the rest of the longer side; unit u goes behind MFMA (u * NM) / NR
                        if (u < (m * NR) / NM || u >= ((m + 1) * NR) / NM) continue;
                        constexpr int TMIN = TM < TN ? TM : TN;
                        if (u < 2 * TMIN) {
                            if (u % 2 == 0) fa[cur ^ 1][u / 2] = read_a(rbase, rks, u / 2);
                            else fb[cur ^ 1][u / 2] = read_b(rbase, rks, u / 2);
                        } else {
                            const int r = u - TMIN;
                            if (TM > TN) fa[cur ^ 1][r] = read_a(rbase, rks, r);
                            else fb[cur ^ 1][r] = read_b(rbase, rks, r);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (more && !TWO_STAGE) {
                    const int f = ks * NM + m;
#pragma unroll
                    for (int idx = 0; idx < LPT; ++idx) {
                        if (idx < (f * LPT) / TOT || idx >= ((f + 1) * LPT) / TOT) continue;
                        issue_load(idx, pre);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (more && TWO_STAGE && last) {
#pragma unroll
                    for (int idx = 0; idx < LPT; ++idx) {
                        if (idx < (m * LPT) / NM || idx >= ((m + 1) * LPT) / NM) continue;
                        issue_load(idx, pre);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
        if (more) next_tile();
        stage = next;
    };
    {
        using T = std::true_type;
        using F = std::false_type;
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, (KS & 1)>;   // parity of the second tile of a pair
        // Straight-line phases only: selecting an instantiation at run time inside a loop makes the
        // register allocator spill the accumulators.
        int kt = 0;
        if (UNROLL == 2) {
            // odd KS: the fragment buffers alternate per K-tile, so tiles go in pairs (nk is even)
            static_assert(UNROLL == 1 || NSTAGE == 4, "the pair schedule below is written for four stages");
            for (; kt + NSTAGE < nk; kt += 2) {
                k_tile(T{}, T{}, P0{});
                k_tile(T{}, T{}, P1{});
            }
            if (nk - kt == 4) {
                k_tile(T{}, T{}, P0{});
                k_tile(F{}, T{}, P1{});
            }
            k_tile(F{}, T{}, P0{});
            k_tile(F{}, F{}, P1{});
        } else {
            for (; kt + PRE < nk; ++kt) k_tile(T{}, T{}, P0{});
            for (; kt + 1 < nk; ++kt) k_tile(F{}, T{}, P0{});
            k_tile(F{}, F{}, P0{});
        }
    }

    // ---- epilogue: 32 rows at a time through a wave-private LDS strip -----------------------------------
    __syncthreads();   // all fragment reads of the stage buffers are done
    char *epi = smem + wave * EPI_BYTES;
    constexpr int LPR = WN * ESZ / 16;   // lanes per output row
    constexpr int RPP = 64 / LPR;        // rows per pass
    TOut *C;
    const float *bias_lds = nullptr;     // MAPPED with a bias: the bias of this wavefront's first column
    if constexpr (!MAPPED) {
        C = static_cast<TOut *>(p.C) + batch * p.sC + split * p.sSplit + (m0 + wm * WM) * p.ldc + n0 + wn * WN;
    } else {
        C = static_cast<TOut *>(p.C) + axis_offset(p.maps.c_n, n0 + wn * WN + (lane % LPR) * (16 / ESZ));
        if (p.maps.bias) {
            float *strip = reinterpret_cast<float *>(smem + WAVES * EPI_BYTES);
            for (int x = tid; x < BN; x += 256) strip[x] = p.maps.bias[axis_offset(p.maps.bias_n, n0 + x)];
            __syncthreads();
            bias_lds = strip + wn * WN + 4 * (lane >> 5);
        }
    }
    const float alpha = p.alpha;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // registers 4g..4g+3 of lane: row lane%32, columns j*32 + 8g + 4*(lane/32) + 0..3
                char *dst = epi + (lane & 31) * EPI_STRIDE + (j * 32 + 8 * g + 4 * (lane >> 5)) * ESZ;
                float v0 = acc[i][j][4 * g] * alpha, v1 = acc[i][j][4 * g + 1] * alpha;
                float v2 = acc[i][j][4 * g + 2] * alpha, v3 = acc[i][j][4 * g + 3] * alpha;
                if constexpr (MAPPED) {
                    if (bias_lds) {
                        const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias_lds + j * 32 + 8 * g);
                        v0 += bv[0]; v1 += bv[1]; v2 += bv[2]; v3 += bv[3];
                    }
                }
                if (ESZ == 4) {
                    f32x4 v = {v0, v1, v2, v3};
                    *reinterpret_cast<f32x4 *>(dst) = v;
                } else {
                    uint2 v;
                    v.x = pack_bf16x2(v0, v1);
                    v.y = pack_bf16x2(v2, v3);
                    *reinterpret_cast<uint2 *>(dst) = v;
                }
            }
        }
        int64_t strip = 0;   // MAPPED: where this 32-row strip (inside one shard) starts
        if constexpr (MAPPED) strip = axis_offset(p.maps.c_m, m0 + wm * WM + i * 32);
#pragma unroll
        for (int pass = 0; pass < 32 / RPP; ++pass) {
            const int row = pass * RPP + lane / LPR;
            const i32x4 v = *reinterpret_cast<const i32x4 *>(epi + row * EPI_STRIDE + (lane % LPR) * 16);
            char *gp;
            if constexpr (!MAPPED) gp = reinterpret_cast<char *>(C + (int64_t)(i * 32 + row) * p.ldc) + (lane % LPR) * 16;
            else gp = reinterpret_cast<char *>(C + strip + (int64_t)row * p.maps.c_m.u);
            *reinterpret_cast<i32x4 *>(gp) = v;
        }
    }
}

// Launch one configuration.  splits > 1: every split writes its own fp32 partial result
// [batch][split][Mo][No] to `out` (then out_ld = No); splits == 1: `out` is the final C.
template <typename E, int BM, int BN, int BKB, int NSTAGE, bool AK, bool BKM, typename TOut, bool MAPPED = false>
int launch_cfg(const GemmArgs &g, int splits, void *out, int64_t out_ld, int64_t out_batch_stride, int64_t out_split_stride,
               float alpha)
{
    using ATile = typename std::conditional<AK, KMajorTile<E, BM, BKB>, MNMajorTile<E, BM, BKB>>::type;
    using BTile = typename std::conditional<BKM, KMajorTile<E, BN, BKB>, MNMajorTile<E, BN, BKB>>::type;
    constexpr int LDS = NSTAGE * (ATile::BYTES + BTile::BYTES);
    auto kern = gemm_mfma_kernel<E, BM, BN, BKB, NSTAGE, AK, BKM, TOut, MAPPED>;
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS) !=
            hipSuccess)
            return CUBE3D_ELAUNCH;
        configured = true;
    }
    Params p;
    p.A = g.A;
    p.B = g.B;
    p.C = out;
    p.lda = g.lda; p.ldb = g.ldb; p.ldc = out_ld;
    p.sA = g.strideA; p.sB = g.strideB; p.sC = out_batch_stride;
    p.tiles_m = (int)(g.Mo / BM);
    p.tiles_n = (int)(g.No / BN);
    p.nk = (int)(g.Kc * E::ELT / BKB / splits);
    p.group_m = 8;
    p.splits = splits;
    p.sSplit = out_split_stride;
    p.alpha = alpha;
    if (MAPPED) {
        p.maps = *g.maps;
        p.ka = make_kwalk(g.maps->a_k, BKB / E::ELT);
        p.kb = make_kwalk(g.maps->b_k, BKB / E::ELT);
    }
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)(g.batch * splits), 1);
    hipLaunchKernelGGL(kern, grid, dim3(256), LDS, g.stream, p);
    return launch_status();
}

template <typename E, int BM, int BN, int BKB, int NSTAGE, typename TOut>
int launch_layout(const GemmArgs &g, int splits, void *out, int64_t out_ld, int64_t out_batch_stride,
                  int64_t out_split_stride, float alpha)
{
    if (g.a_kmajor && !g.b_kmajor)
        return launch_cfg<E, BM, BN, BKB, NSTAGE, true, false, TOut>(g, splits, out, out_ld, out_batch_stride,
                                                                    out_split_stride, alpha);
    if (g.a_kmajor && g.b_kmajor)
        return launch_cfg<E, BM, BN, BKB, NSTAGE, true, true, TOut>(g, splits, out, out_ld, out_batch_stride,
                                                                   out_split_stride, alpha);
    if (!g.a_kmajor && !g.b_kmajor)
        return launch_cfg<E, BM, BN, BKB, NSTAGE, false, false, TOut>(g, splits, out, out_ld, out_batch_stride,
                                                                     out_split_stride, alpha);
    return CUBE3D_ENOTIMPL;
}

}  // namespace mfk
}  // namespace cube3d
