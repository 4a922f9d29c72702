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
//
// Issue schedule.  With one wavefront per SIMD the matrix pipe stays full only if the wavefront
// is back at the next MFMA when the previous one retires (32 cycles): everything else has to fit
// into those gaps, a few instructions per gap.  Measured on gfx950: an LDS read with an
// immediate offset or a direct-to-LDS load addressed as scalar base + 32-bit lane offset costs
// no MFMA time when it sits alone in a gap; address arithmetic on the vector ALU, loads with
// 64-bit lane addresses, bursts of scalar instructions and, most of all, branches do.  So the
// K loop is unrolled over the NSTAGE stages (every LDS address is a lane-constant register plus
// an immediate, every M0 value a scalar add of a constant), the global addresses are one scalar
// pointer per operand advanced once per K-tile plus lane-constant offsets, and the reads and
// loads of a k-step are dealt out one per gap.
#pragma once
#include <atomic>
#include <cstdlib>
#include <mutex>
#include <type_traits>

#include "common.h"

namespace cube3d {
namespace mfk {

typedef short s16x4 __attribute__((ext_vector_type(4)));
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

// Direct-to-LDS 16-byte load: lane s of the wavefront writes LDS bytes [lds_base + 16 s, +16)
// with the 16 bytes at base + offset (scalar 64-bit base, 32-bit unsigned lane offset).
// Issued as inline assembly so that its completion is tracked by the explicit
// s_waitcnt vmcnt(..) + barrier of the pipeline and by nothing else (the compiler would
// otherwise drain every outstanding load before each LDS read).
__device__ __forceinline__ void async_load16(const char *base, unsigned offset, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(offset), "s"(base), "s"(lds_base) : "m0");
}

// -1 if the two wavefront-uniform values are equal, else 0; opaque to the compiler, which would
// otherwise turn arithmetic on the result back into a branch.
__device__ __forceinline__ int eq_mask(int a, int b)
{
    int m;
    asm volatile("s_cmp_eq_u32 %1, %2\n\ts_cselect_b32 %0, -1, 0" : "=s"(m) : "s"(a), "s"(b) : "scc");
    return m;
}

// ---- element traits --------------------------------------------------------------------------------
// A fragment (one operand of one MFMA: 32 rows or columns x one k-step) is FI 32-bit registers
// per lane, read from LDS in pieces: PK 16-byte reads when the operand is K-major, PT
// transposing 8-byte reads (TR_ROWS k-rows apart) when it is MN-major.
struct Bf16 {
    typedef unsigned short Elem;
    typedef i32x4 FragI;                        // 8 bf16 = 16 bytes per lane
    static constexpr int ELT = 2;
    static constexpr int KSTEP = 16;            // k per MFMA
    static constexpr int TR_ROWS = 4;           // k-rows covered by one transposing read
    static constexpr int FI = 4, PK = 1, PT = 2;
    // slot permutation of an MN-major row (spr = 16-byte slots per row, at least 16): see MNMajorTile
    __device__ static __forceinline__ int mn_swz(int k, int) { return 4 * (k & 3); }
    __device__ static __forceinline__ f32x16 mfma(FragI first, FragI second, f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, first), __builtin_bit_cast(bf16x8, second),
                                                       c, 0, 0, 0);
    }
    __device__ static __forceinline__ i32x2 read_tr(unsigned ad)
    {
        return __builtin_bit_cast(
            i32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(uintptr_t)ad));
    }
};

struct Fp8 {
    typedef unsigned char Elem;
    typedef i32x8 FragI;                        // 32 fp8 = 32 bytes per lane
    static constexpr int ELT = 1;
    static constexpr int KSTEP = 64;
    static constexpr int TR_ROWS = 8;
    static constexpr int FI = 8, PK = 2, PT = 4;
    // rows of 16 slots or more: the 8 k-rows of a transposing read go to 8 different slot pairs; rows of 8
    // slots (128-byte rows): k-rows of equal parity lie 256 bytes apart, so the pair index is permuted by k / 2
    __device__ static __forceinline__ int mn_swz(int k, int spr) { return spr >= 16 ? 2 * (k & 7) : 2 * ((k >> 1) & 3); }
    __device__ static __forceinline__ f32x16 mfma(FragI first, FragI second, f32x16 c)
    {
        // both operands e4m3 (format code 0), block scales 2^0
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(first, second, c, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    }
    __device__ static __forceinline__ i32x2 read_tr(unsigned ad)
    {
        return __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) i32x2 *)(uintptr_t)ad);
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
    static_assert((SPR >= 16 || (E::ELT == 1 && SPR == 8)) && RB <= 1024,
                  "the swizzle permutes slots inside aligned groups of 16 (fp8 rows of 128 bytes: of 8)");
    __device__ static __forceinline__ int64_t lane_src(int wave, int lane, int64_t ld)
    {
        const int k = wave * RPC + lane / SPR;
        const int slot = (lane % SPR) ^ E::mn_swz(k, SPR);
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
        return k * RB + (((byte / 16) ^ E::mn_swz(k, SPR)) * 16) + byte % 16;
    }
};

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
    int splits;                 // split-K: y = batch * splits + split; split s takes K-tiles [s*nk, (s+1)*nk)
    int y_items;                // batch * splits: an item is (y, output tile), item number = y * tiles + tile
    int64_t sSplit;             // output distance between the partial results of consecutive splits (elements)
    float alpha;
    int stagger;                // start delay of the last workgroup in units of 10 ns (0: none); workgroup w waits w / grid of it
    // MAPPED instantiations only (then lda / ldb / ldc, the strides and the splits are unused)
    GemmMaps maps;
    KWalk ka, kb;
#ifdef CUBE3D_PROFILE
    unsigned long long *prof;   // 64 stamps per workgroup: (shader clock, 100 MHz clock) pairs
#endif
};

// TOut: float or unsigned short (bf16 bits).  MAPPED: operands, output and the optional bias are
// addressed through p.maps (a cube of shards read in place) instead of leading dimensions.
// The number of K-tiles per workgroup (p.nk) must be a positive multiple of NSTAGE.
template <typename E, int BM, int BN, int BKB, int NSTAGE, bool AK, bool BKM, typename TOut, bool MAPPED = false>
__global__ __launch_bounds__(256, (BM * BN <= 128 * 128) ? 2 : 1) void gemm_mfma_kernel(const Params p)
{
    typedef typename E::Elem Elem;
    typedef typename E::FragI FragI;
    using ATile = typename std::conditional<AK, KMajorTile<E, BM, BKB>, MNMajorTile<E, BM, BKB>>::type;
    using BTile = typename std::conditional<BKM, KMajorTile<E, BN, BKB>, MNMajorTile<E, BN, BKB>>::type;
    constexpr int A_BYTES = ATile::BYTES, B_BYTES = BTile::BYTES, STAGE_BYTES = A_BYTES + B_BYTES;
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int KS = BKB / (E::KSTEP * E::ELT);      // k-steps (MFMAs deep) per K-tile
    constexpr int NM = TM * TN;                        // MFMAs per k-step = gaps per k-step
    constexpr int LPT = ATile::CPW + BTile::CPW;       // async loads per K-tile per wavefront
    constexpr int LPK = LPT / KS;                      // ... per k-step
    constexpr int PA = AK ? E::PK : E::PT, PB = BKM ? E::PK : E::PT;   // LDS reads per fragment
    constexpr int NRD = TM * PA + TN * PB;             // LDS reads per k-step
    constexpr int RG = NM > 4 ? NM - 2 : NM;           // gaps of a k-step that take the reads of the next one
    constexpr int NBA = AK ? KS * E::PK : TM;          // lane-constant LDS address registers per operand
    constexpr int NBB = BKM ? KS * E::PK : TN;
    constexpr int PRE = NSTAGE - 1;                    // tiles in flight after the prologue
    constexpr int ESZ = sizeof(TOut);
    // Epilogue staging: a wave-private strip of 32 rows x JH 32-column blocks.  The large tiles keep it
    // behind the stage buffers (the CU's LDS is theirs alone), so that the loads of the next item can
    // already fill the stages while this item is written out; the small tiles (two workgroups per CU)
    // reuse the stage memory.
    constexpr bool EPI_SEPARATE = BM * BN > 128 * 128;
    constexpr int JH = EPI_SEPARATE ? (TN * 32 * ESZ > 128 ? 128 / (32 * ESZ) : TN) : TN;
    // A strip row is ROWB bytes, unpadded; its 16-byte slots are permuted by the row number so that both
    // the lanes' writes (32 rows at one column) and the row-wise 16-byte reads spread over all banks.
    // Two strips per wavefront where there is room: the next strip is converted and written while the
    // reads of the previous one are in flight.
    constexpr int ROWB = JH * 32 * ESZ;
    constexpr int NBUF = MAPPED ? 1 : 2;
    // The optional bias belongs to the forward product (Algorithm 7 follows Algorithm 1): only the
    // map-addressed kernel of that layout stages and adds it; the launcher sends a bias with any other
    // layout to the bounds-checked kernel.
    constexpr bool BIAS = MAPPED && AK && !BKM;
    constexpr int STRIP_BYTES = 32 * ROWB;
    constexpr int EPI_BYTES = NBUF * STRIP_BYTES;
    static_assert(ROWB == 128 || ROWB == 256, "strip rows of 8 or 16 slots");
    constexpr int EPI_BASE = EPI_SEPARATE ? NSTAGE * STAGE_BYTES : 0;
    static_assert(TN % JH == 0, "whole strips");
    static_assert(KS >= 1 && BKB % (E::KSTEP * E::ELT) == 0, "K-tile must hold whole k-steps");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wavefront tile is made of 32x32 MFMA tiles");
    static_assert((NSTAGE == 2 || NSTAGE == 4) && (NSTAGE * KS) % 2 == 0, "the fragment buffers alternate per k-step and must line up per pass over the stages");
    static_assert(NSTAGE != 2 || KS >= 2, "the two-stage schedule loads in the first and in the last k-step of a tile");
    static_assert(LPT % KS == 0, "the loads of a K-tile are dealt out evenly over its k-steps");
    static_assert(NSTAGE * STAGE_BYTES <= 160 * 1024, "LDS budget");
    static_assert(NSTAGE * STAGE_BYTES <= 2 * 65536, "an LDS address is one of two lane registers plus a 16-bit immediate");
    static_assert(EPI_BASE + WAVES * EPI_BYTES + (BIAS ? BN * 4 : 0) <= (EPI_SEPARATE ? 160 * 1024 : NSTAGE * STAGE_BYTES),
                  "epilogue staging (and the bias strip) must fit");
    static_assert((NSTAGE - 2) * LPT <= 63, "vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63, lane_id = lane;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
#ifdef CUBE3D_PROFILE
    int prof_n = 0;
    auto stamp = [&]() {
        // (wave-uniform condition: all lanes of the first wavefront store the same two values)
        if (p.prof && wave == 0 && prof_n < 32) {
            p.prof[(blockIdx.x * 32 + prof_n) * 2] = __builtin_readcyclecounter();
            p.prof[(blockIdx.x * 32 + prof_n) * 2 + 1] = __builtin_amdgcn_s_memrealtime();
        }
        ++prof_n;
    };
#define CUBE3D_STAMP() stamp()
// inside the K loop only for plain operands: the map-addressed K loop has no scalar registers to spare
#define CUBE3D_STAMP_LOOP() do { if constexpr (!MAPPED) stamp(); } while (0)
#else
#define CUBE3D_STAMP()
#define CUBE3D_STAMP_LOOP()
#endif

    // ---- work items ------------------------------------------------------------------------------------
    // The workgroups are persistent: workgroup w takes the items w, w + gridDim.x, ...  An item is one
    // output tile of one (batch, split).  Consecutive workgroup ids go to different XCDs (id mod 8), and
    // gridDim.x is a multiple of 8 whenever a workgroup gets more than one item, so an item's number mod 8
    // names its XCD too: the numbers are regrouped so that the tiles one XCD runs together form a compact
    // patch of the tile grid, or belong to the same problem of a batch (shared L2).
    const int tiles_total = p.tiles_m * p.tiles_n;
    const int items = tiles_total * p.y_items;
    int64_t m0, n0;            // origin of the item whose operands are being loaded
    int batch, split;
    auto decode_item = [&](int item) {
        int y, tile;
        if (p.y_items % 8 == 0) {
            // batched launch: every XCD takes whole (batch, split) problems, its CUs the tiles of one
            // problem after the other, so that a problem's operand panels are fetched into one L2 only
            const int v = item / 8;
            y = (v / tiles_total) * 8 + item % 8;
            tile = v - (v / tiles_total) * tiles_total;
        } else {
            y = item / tiles_total;
            tile = item - y * tiles_total;
            if (tiles_total % 8 == 0) tile = (tile % 8) * (tiles_total / 8) + tile / 8;
        }
        const int per_group = p.group_m * p.tiles_n;
        const int gid = tile / per_group;
        const int first_m = gid * p.group_m;
        const int gsz = min(p.tiles_m - first_m, p.group_m);
        const int in_group = tile - gid * per_group;
        const int tm_ = first_m + in_group % gsz;
        const int tn_ = in_group / gsz;
        m0 = (int64_t)tm_ * BM;
        n0 = (int64_t)tn_ * BN;
        batch = y / p.splits;
        split = y - batch * p.splits;
    };

    // ---- global sources of this lane's async loads: one scalar pointer per operand, standing on the
    //      K-tile that is loaded next, plus one 32-bit byte offset per load that never changes
    const char *a_base, *b_base;
    unsigned a_voff[ATile::CPW], b_voff[BTile::CPW];
    int64_t a_step = 0, b_step = 0;              // bytes from one K-tile to the next (plain operands)
    // MAPPED: state of an operand's walk along the contraction index
    struct Walk {
        int c1, c2;            // position inside the current block / shard
        int m1, m2;            // masks of the pending step: walked off a block / off a shard
        int64_t delta;         // bytes to add
    };
    Walk wa{0, 0, 0, 0, 0}, wb{0, 0, 0, 0, 0};
    auto setup_sources = [&]() {
    if constexpr (!MAPPED) {
        const int64_t kt0 = (int64_t)split * p.nk;   // first K-tile of this split
        a_step = ATile::ktile_step(p.lda) * E::ELT;
        b_step = BTile::ktile_step(p.ldb) * E::ELT;
        a_base = static_cast<const char *>(p.A) + (batch * p.sA + (AK ? m0 * p.lda : m0)) * E::ELT + kt0 * a_step;
        b_base = static_cast<const char *>(p.B) + (batch * p.sB + (BKM ? n0 * p.ldb : n0)) * E::ELT + kt0 * b_step;
#pragma unroll
        for (int idx = 0; idx < ATile::CPW; ++idx)
            a_voff[idx] = (unsigned)((ATile::lane_src(wave, lane, p.lda) + idx * ATile::chunk_step(p.lda)) * E::ELT);
#pragma unroll
        for (int idx = 0; idx < BTile::CPW; ++idx)
            b_voff[idx] = (unsigned)((BTile::lane_src(wave, lane, p.ldb) + idx * BTile::chunk_step(p.ldb)) * E::ELT);
    } else {
        // offsets relative to the start of the operand's cube buffer (the launcher checks that the
        // buffer is shorter than 4 GB); a chunk's rows lie in one shard
        constexpr int EPS = 16 / E::ELT;   // elements per 16-byte slot
        a_base = static_cast<const char *>(p.A);
        b_base = static_cast<const char *>(p.B);
        a_step = p.ka.step * E::ELT;
        b_step = p.kb.step * E::ELT;
        wa.c1 = wa.c2 = wb.c1 = wb.c2 = 0;
        {
            const int first = wave * ATile::RPC + lane / ATile::SPR;   // tile row (K-major) or k-row (MN-major)
#pragma unroll
            for (int idx = 0; idx < ATile::CPW; ++idx) {
                int64_t off;
                if constexpr (AK) {
                    const int c = (lane % ATile::SPR) ^ KMajorTile<E, BM, BKB>::swz(first);
                    off = axis_offset_fast(p.maps.a_mn, m0 + first + idx * ATile::CHUNK_ROWS) + c * EPS;
                } else {
                    const int slot = (lane % ATile::SPR) ^ E::mn_swz(first, ATile::SPR);
                    off = axis_offset_fast(p.maps.a_mn, m0 + slot * EPS) + (int64_t)(first + idx * ATile::CHUNK_ROWS) * p.maps.a_k.u;
                }
                a_voff[idx] = (unsigned)(off * E::ELT);
            }
        }
        {
            const int first = wave * BTile::RPC + lane / BTile::SPR;
#pragma unroll
            for (int idx = 0; idx < BTile::CPW; ++idx) {
                int64_t off;
                if constexpr (BKM) {
                    const int c = (lane % BTile::SPR) ^ KMajorTile<E, BN, BKB>::swz(first);
                    off = axis_offset_fast(p.maps.b_mn, n0 + first + idx * BTile::CHUNK_ROWS) + c * EPS;
                } else {
                    const int slot = (lane % BTile::SPR) ^ E::mn_swz(first, BTile::SPR);
                    off = axis_offset_fast(p.maps.b_mn, n0 + slot * EPS) + (int64_t)(first + idx * BTile::CHUNK_ROWS) * p.maps.b_k.u;
                }
                b_voff[idx] = (unsigned)(off * E::ELT);
            }
        }
    }
    };

    // async load number idx of the K-tile the scalar pointers stand on, into LDS stage `stage`
    // (idx and stage are constants wherever this is called: the LDS address is wave base + constant)
    unsigned wave_lds = lds0 + wave * 1024;
    auto issue_load = [&](int idx, int stage) {
        if (idx < ATile::CPW) async_load16(a_base, a_voff[idx], wave_lds + stage * STAGE_BYTES + idx * (WAVES * 1024));
        else async_load16(b_base, b_voff[idx - ATile::CPW],
                          wave_lds + stage * STAGE_BYTES + A_BYTES + (idx - ATile::CPW) * (WAVES * 1024));
    };
    // Move an operand's scalar pointer to the next K-tile.  MAPPED: the walk along the contraction
    // index steps through shards and blocks.  Shards and blocks are whole passes over the LDS stages
    // long (the launcher checks it), so a pointer can only cross a boundary when it moves onto a
    // K-tile whose number is a multiple of NSTAGE: those moves ("checked") look at the position and
    // add the jump to the next shard or block, all others add the plain step like an ordinary
    // operand.  The corrections of a checked move are selected with masks, because a branch in the K
    // loop holds up the MFMA stream far longer than a dozen scalar instructions; even so its scalar
    // work is more than fits behind one MFMA, so inside the K loop it is dealt out in three parts
    // over three gaps (walk_part), and only the final add sits behind the operand's last load
    // (walk_apply).  The position counts the contraction indices since the last boundary, one pass
    // at a time.
    auto walk_part = [&](Walk &w, const KWalk &k, int part) {
        if constexpr (MAPPED) {
            constexpr int PASS = NSTAGE * (BKB / E::ELT);   // contraction indices per pass over the stages
            if (part == 0) {
                w.c1 += PASS;
                w.c2 += PASS;
                w.m1 = eq_mask(w.c1, k.P1);
                w.m2 = eq_mask(w.c2, k.P2) & ~w.m1;
            } else if (part == 1) {
                w.delta = (k.step + (k.jump1 & (int64_t)w.m1) + (k.jump2 & (int64_t)w.m2)) * E::ELT;
            } else {
                w.c1 &= ~w.m1;
                w.c2 &= ~(w.m1 | w.m2);
            }
        }
    };
    auto walk_apply = [&](const char *&base, int64_t plain_step, const Walk &w, bool checked) {
        if (MAPPED && checked) base += w.delta;
        else base += plain_step;
    };
    // whole moves at once (prologue): plain, or checked
    auto advance_a = [&](bool checked = false) {
        if (checked) { walk_part(wa, p.ka, 0); walk_part(wa, p.ka, 1); walk_part(wa, p.ka, 2); }
        walk_apply(a_base, a_step, wa, checked);
    };
    auto advance_b = [&](bool checked = false) {
        if (checked) { walk_part(wb, p.kb, 0); walk_part(wb, p.kb, 1); walk_part(wb, p.kb, 2); }
        walk_apply(b_base, b_step, wb, checked);
    };

    // ---- lane-constant LDS addresses of the fragment reads; every read adds an immediate -------------
    // K-major operand: one register per 16-byte piece of a k-step; MN-major operand: one per 32-wide
    // block of the wavefront's sub-tile.  Each exists twice, 64 KB apart, so that the immediate
    // (stage, operand, block, k-step, piece) always fits the 16-bit offset field of the read.
    // (fp8 fragments are twice as large: there the registers are needed for the fragments, and the
    // reads of the upper stages form their address with one add instead.)
    // (so do the map-addressed two-stage kernels, which need a few registers for their K walk)
    constexpr bool HI_REGS = E::FI <= 4 && !(MAPPED && NSTAGE == 2);
    unsigned a_lo[NBA], a_hi[NBA], b_lo[NBB], b_hi[NBB];
#pragma unroll
    for (int x = 0; x < NBA; ++x) {
        if constexpr (AK)
            a_lo[x] = lds0 + KMajorTile<E, BM, BKB>::slot_addr(wm * WM + (lane & 31),
                                                               (x / E::PK) * 2 * E::PK + (lane >> 5) * E::PK + x % E::PK);
        else a_lo[x] = lds0 + MNMajorTile<E, BM, BKB>::tr_addr(lane, wm * TM + x);
        a_hi[x] = a_lo[x] + 65536;
        if constexpr (HI_REGS) asm volatile("" : "+v"(a_hi[x]));   // keep it in a register of its own
    }
#pragma unroll
    for (int x = 0; x < NBB; ++x) {
        if constexpr (BKM)
            b_lo[x] = lds0 + KMajorTile<E, BN, BKB>::slot_addr(wn * WN + (lane & 31),
                                                               (x / E::PK) * 2 * E::PK + (lane >> 5) * E::PK + x % E::PK);
        else b_lo[x] = lds0 + MNMajorTile<E, BN, BKB>::tr_addr(lane, wn * TN + x);
        b_hi[x] = b_lo[x] + 65536;
        if constexpr (HI_REGS) asm volatile("" : "+v"(b_hi[x]));
    }

    // A fragment is kept as the pieces it was read in (whole registers each, so that no read
    // rewrites part of a live value) and put together where the MFMA takes it.
    using APiece = typename std::conditional<AK, i32x4, i32x2>::type;
    using BPiece = typename std::conditional<BKM, i32x4, i32x2>::type;
    APiece fa[2][TM][PA];
    BPiece fb[2][TN][PB];
    // piece `pc` of the fragment of block t, k-step ks, in LDS stage `stage`, into fragment buffer `buf`
    auto read_a = [&](int buf, int stage, int ks, int t, int pc) {
        if constexpr (AK) {
            const int c = stage * STAGE_BYTES + t * KMajorTile<E, BM, BKB>::BLOCK_STEP;
            const int x = ks * E::PK + pc;
            const unsigned ad = c < 65536 ? a_lo[x] + c : a_hi[x] + (c - 65536);
            fa[buf][t][pc] = *(CUBE3D_LDS(i32x4))(uintptr_t)ad;
        } else {
            constexpr int RB = MNMajorTile<E, BM, BKB>::RB;
            const int c = stage * STAGE_BYTES + (ks * E::KSTEP + pc * E::TR_ROWS) * RB;
            fa[buf][t][pc] = E::read_tr(c < 65536 ? a_lo[t] + c : a_hi[t] + (c - 65536));
        }
    };
    auto read_b = [&](int buf, int stage, int ks, int t, int pc) {
        if constexpr (BKM) {
            const int c = stage * STAGE_BYTES + A_BYTES + t * KMajorTile<E, BN, BKB>::BLOCK_STEP;
            const int x = ks * E::PK + pc;
            const unsigned ad = c < 65536 ? b_lo[x] + c : b_hi[x] + (c - 65536);
            fb[buf][t][pc] = *(CUBE3D_LDS(i32x4))(uintptr_t)ad;
        } else {
            constexpr int RB = MNMajorTile<E, BN, BKB>::RB;
            const int c = stage * STAGE_BYTES + A_BYTES + (ks * E::KSTEP + pc * E::TR_ROWS) * RB;
            fb[buf][t][pc] = E::read_tr(c < 65536 ? b_lo[t] + c : b_hi[t] + (c - 65536));
        }
    };
    auto frag_a = [&](int buf, int t) -> FragI {
        FragI f;
        constexpr int W = AK ? 4 : 2;
#pragma unroll
        for (int pc = 0; pc < PA; ++pc)
#pragma unroll
            for (int e = 0; e < W; ++e) f[pc * W + e] = fa[buf][t][pc][e];
        return f;
    };
    auto frag_b = [&](int buf, int t) -> FragI {
        FragI f;
        constexpr int W = BKM ? 4 : 2;
#pragma unroll
        for (int pc = 0; pc < PB; ++pc)
#pragma unroll
            for (int e = 0; e < W; ++e) f[pc * W + e] = fb[buf][t][pc][e];
        return f;
    };
    // LDS read number r of a k-step, in the order the MFMAs (block row i outer, block column j
    // inner) first need the fragments: A0, B0 .. B(TN-1), A1 .. A(TM-1)
    auto read_piece = [&](int r, int buf, int stage, int ks) {
        if (r < PA) read_a(buf, stage, ks, 0, r);
        else if (r < PA + TN * PB) read_b(buf, stage, ks, (r - PA) / PB, (r - PA) % PB);
        else read_a(buf, stage, ks, 1 + (r - PA - TN * PB) / PA, (r - PA - TN * PB) % PA);
    };

    f32x16 acc[TM][TN];

    // ---- pipeline prologue of an item, in two parts -----------------------------------------------------
    // early: the loads that go to stages which nobody reads any more once this wavefront has left the K
    // loop of the previous item (all stages but the one of its last K-tile); late: the rest, behind a
    // workgroup barrier.  Four stages: tiles 0..2 are all early.  Two stages: tile 0 early, operand A of
    // tile 1 late (operand B of tile 1 follows in the first k-step, see the schedule below).
    auto early_loads = [&]() {
        if constexpr (NSTAGE == 2) {
#pragma unroll
            for (int idx = 0; idx < LPT; ++idx) issue_load(idx, 0);
            advance_a();
            advance_b();
        } else {
#pragma unroll
            for (int s = 0; s < PRE; ++s) {
#pragma unroll
                for (int idx = 0; idx < LPT; ++idx) issue_load(idx, s);
                advance_a();
                advance_b();
            }
        }
    };
    // `stores`: global stores of the previous item's epilogue issued behind the early loads; they stay in
    // flight (memory operations of a wavefront complete in the order they were issued)
    auto finish_prologue = [&](auto stores_c) {
        constexpr int stores = decltype(stores_c)::value;
        if constexpr (NSTAGE == 2) {
            __builtin_amdgcn_s_barrier();   // everyone has left the last K-tile of the previous item
#pragma unroll
            for (int idx = 0; idx < ATile::CPW; ++idx) issue_load(idx, 1);
            advance_a(true);   // onto K-tile 2: a multiple of the two stages
            tile_barrier<(ATile::CPW + stores <= 63 ? ATile::CPW + stores : 63)>();
        } else {
            tile_barrier<((PRE - 1) * LPT + stores <= 63 ? (PRE - 1) * LPT + stores : 63)>();
        }
#pragma unroll
        for (int r = 0; r < NRD; ++r) read_piece(r, 0, 0, 0);
    };

    // ---- main loop ----------------------------------------------------------------------------------
    // K-tile number kt lives in stage kt mod NSTAGE; one pass of the loop body takes NSTAGE tiles, so
    // stage, fragment buffer and every address constant are fixed per copy of the tile body.  Per
    // k-step: NM MFMAs; behind MFMA g come the LDS reads of the following k-step that fall into gap g
    // (all of them inside the first RG gaps, so that they have landed when the tile barrier or the next
    // k-step asks for them) and this k-step's share of the async loads.  The order is pinned with
    // scheduling barriers.  ALLOW = loads that may stay in flight across the tile barrier.
    //   four stages: tile kt+3 is loaded during tile kt, its loads dealt out over all k-steps;
    //   two stages (deeper K-tiles: whole cache lines per row of a K-major operand, half as many
    //   barriers): the stage of tile kt is free behind the tile barrier, so operand A of tile kt+2 is
    //   loaded in the last k-step of tile kt and operand B in the first k-step of tile kt+1, which
    //   leaves them the k-steps in between to land.
    auto k_tile = [&](auto stage_c, auto more_c, auto has_next_c, auto allow_c, auto first_c) {
        constexpr int stage = decltype(stage_c)::value;
        constexpr bool first = decltype(first_c)::value;        // first K-tile of the item: its first k-step starts the sums
        constexpr bool more = decltype(more_c)::value;          // tile kt+NSTAGE-1 (two stages: kt+2) exists: load it
        constexpr bool has_next = decltype(has_next_c)::value;  // tile kt+1 exists
        constexpr int ALLOW = decltype(allow_c)::value;
        constexpr int pre = (stage + NSTAGE - 1) % NSTAGE;      // stage the loads of this tile body go to
        constexpr int next = (stage + 1) % NSTAGE;
        constexpr int parity = (stage * KS) & 1;                // fragment buffer holding this tile's k-step 0
        // MAPPED: the moves of this tile body that land on a K-tile number that is a multiple of NSTAGE.
        // Four stages: tile body kt loads tile kt+3 and moves both pointers onto kt+4: checked where
        // kt is a multiple of 4.  Two stages: body kt moves B (the first to move) onto kt+2, checked
        // for even kt, and A onto kt+3, checked for odd kt.
        constexpr bool chk_first = stage == 0;
        constexpr bool chk_second = NSTAGE == 2 ? stage == 1 : stage == 0;
        constexpr bool chk_a = NSTAGE == 2 ? chk_second : chk_first, chk_b = NSTAGE == 2 ? chk_first : chk_second;
        // the LDS targets of this tile body's loads are formed here, one scalar add each, not kept
        // in registers across the whole loop
        asm volatile("" : "+s"(wave_lds));
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = (parity + ks) & 1;
            const bool last = ks == KS - 1;
            // before the reads of tile kt+1 start: its loads have landed everywhere, and nobody still reads
            // the stage that the next tile body's loads overwrite
            if (last && has_next) tile_barrier<ALLOW>();
            const int rstage = last ? next : stage;
            const int rks = last ? 0 : ks + 1;
            const bool do_read = !last || has_next;
#pragma unroll
            for (int g = 0; g < NM; ++g) {
                // serpentine over the sub-tile's blocks: from one MFMA to the next only one operand changes,
                // also at the end of a block row (fewer operand-bus toggles: the chip is power-limited)
                const int i = g / TN, j = (i & 1) ? TN - 1 - g % TN : g % TN;
                if (first && ks == 0) {
                    f32x16 zero;
#pragma unroll
                    for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                    acc[i][j] = E::mfma(frag_b(cur, j), frag_a(cur, i), zero);
                } else {
                    acc[i][j] = E::mfma(frag_b(cur, j), frag_a(cur, i), acc[i][j]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (MAPPED) {
                    // scalar work of the checked moves of this tile body: the operand whose pointer moves
                    // first (A with four stages, B with two) in the first twelfth-steps, the other from the middle
                    const int f = ks * NM + g;
                    constexpr int TOTG = KS * NM;
#pragma unroll
                    for (int part = 0; part < 3; ++part) {
                        const bool first_moves = (NSTAGE == 2 ? has_next : more) && chk_first;    // its loads are issued at all
                        const bool second_moves = more && chk_second;
                        if (f == (part * TOTG) / 12 && first_moves) {
                            if (NSTAGE == 2) walk_part(wb, p.kb, part);
                            else walk_part(wa, p.ka, part);
                        }
                        if (f == TOTG / 2 + (part * TOTG) / 12 && second_moves) {
                            if (NSTAGE == 2) walk_part(wa, p.ka, part);
                            else walk_part(wb, p.kb, part);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (do_read) {
#pragma unroll
                    for (int r = 0; r < NRD; ++r) {
                        if ((r * RG) / NRD != g) continue;
                        read_piece(r, cur ^ 1, rstage, rks);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (NSTAGE > 2 && more) {
#pragma unroll
                    for (int l = 0; l < LPK; ++l) {
                        if (((2 * l + 1) * NM) / (2 * LPK) != g) continue;
                        issue_load(ks * LPK + l, pre);
                        // behind an operand's last load of the tile: its pointer moves on
                        if (ks * LPK + l == ATile::CPW - 1) walk_apply(a_base, a_step, wa, chk_a);
                        if (ks * LPK + l == LPT - 1) walk_apply(b_base, b_step, wb, chk_b);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (NSTAGE == 2 && ks == 0 && has_next) {
#pragma unroll
                    for (int l = 0; l < BTile::CPW; ++l) {
                        if (((2 * l + 1) * NM) / (2 * BTile::CPW) != g) continue;
                        issue_load(ATile::CPW + l, next);
                        if (l == BTile::CPW - 1) walk_apply(b_base, b_step, wb, chk_b);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if (NSTAGE == 2 && last && more) {
#pragma unroll
                    for (int l = 0; l < ATile::CPW; ++l) {
                        if (((2 * l + 1) * NM) / (2 * ATile::CPW) != g) continue;
                        issue_load(l, stage);
                        if (l == ATile::CPW - 1) walk_apply(a_base, a_step, wa, chk_a);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        }
    };
    // The accumulators are not cleared: the first k-step of an item's first K-tile starts the sums from
    // a zero operand.  That tile body exists in several copies (more K-tiles than one pass or not; first
    // item of the workgroup or not).  `after_stores`: the epilogue of the previous item has issued `stores`
    // global stores behind this item's first loads; they may stay in flight across the first two tile
    // barriers (four stages), so the K loop does not wait for the previous item's output to reach memory.
    auto k_loop = [&](bool after_stores, auto stores_c) {
        using T = std::true_type;
        using F = std::false_type;
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        using Z = std::integral_constant<int, 0>;
        constexpr int stores = decltype(stores_c)::value;
        const int passes = p.nk / NSTAGE;
        if constexpr (NSTAGE == 2) {
            // nothing is issued between the last load of tile kt+1 and the barrier that waits for it
            if (passes > 1) {
                k_tile(S0{}, T{}, T{}, Z{}, T{});
                k_tile(S1{}, T{}, T{}, Z{}, F{});
                for (int ps = 2; ps < passes; ++ps) {
                    k_tile(S0{}, T{}, T{}, Z{}, F{});
                    k_tile(S1{}, T{}, T{}, Z{}, F{});
                }
                k_tile(S0{}, F{}, T{}, Z{}, F{});
            } else {
                k_tile(S0{}, F{}, T{}, Z{}, T{});
            }
            k_tile(S1{}, F{}, F{}, Z{}, F{});
        } else {
            using S2 = std::integral_constant<int, 2>;
            using S3 = std::integral_constant<int, 3>;
            // in flight across the barrier: tile kt+2, and what this tile body has issued of tile kt+3
            constexpr int steady = LPT + (KS - 1) * LPK;
            using STEADY = std::integral_constant<int, steady>;
            using STEADY_ST = std::integral_constant<int, (steady + stores <= 63 ? steady + stores : 63)>;
            using DRAIN_ST = std::integral_constant<int, (LPT + stores <= 63 ? LPT + stores : 63)>;
            if (passes > 1) {
                if (after_stores) {
                    k_tile(S0{}, T{}, T{}, STEADY_ST{}, T{});
                    k_tile(S1{}, T{}, T{}, STEADY_ST{}, F{});
                } else {
                    k_tile(S0{}, T{}, T{}, STEADY{}, T{});
                    k_tile(S1{}, T{}, T{}, STEADY{}, F{});
                }
                CUBE3D_STAMP_LOOP();   // two K-tiles in (stores may still be in flight)
                k_tile(S2{}, T{}, T{}, STEADY{}, F{});
                CUBE3D_STAMP_LOOP();   // third K-tile done: its barrier waited for the previous item's stores
                k_tile(S3{}, T{}, T{}, STEADY{}, F{});
                for (int ps = 2; ps < passes; ++ps) {
                    k_tile(S0{}, T{}, T{}, STEADY{}, F{});
                    k_tile(S1{}, T{}, T{}, STEADY{}, F{});
                    k_tile(S2{}, T{}, T{}, STEADY{}, F{});
                    k_tile(S3{}, T{}, T{}, STEADY{}, F{});
                }
                k_tile(S0{}, T{}, T{}, STEADY{}, F{});
                k_tile(S1{}, F{}, T{}, std::integral_constant<int, LPT>{}, F{});
            } else if (after_stores) {
                k_tile(S0{}, T{}, T{}, STEADY_ST{}, T{});
                k_tile(S1{}, F{}, T{}, DRAIN_ST{}, F{});
            } else {
                k_tile(S0{}, T{}, T{}, STEADY{}, T{});
                k_tile(S1{}, F{}, T{}, std::integral_constant<int, LPT>{}, F{});
            }
            // rest of the last pass: the pipeline drains (and so have the stores, issued before these loads)
            k_tile(S2{}, F{}, T{}, Z{}, F{});
            k_tile(S3{}, F{}, F{}, Z{}, F{});
        }
    };

    // ---- epilogue: 32 rows x JH column blocks at a time through wave-private LDS strips --------------------
    constexpr int LPR = ROWB / 16;            // lanes per strip row = 16-byte slots per row
    constexpr int RPP = 64 / LPR;             // rows per pass
    constexpr int NPASS = 32 / RPP;           // passes (16-byte loads and global stores) per strip
    constexpr int NSTRIP = TM * (TN / JH);    // strips per wavefront
    constexpr int STORES = NSTRIP * NPASS;    // global stores per wavefront
    constexpr int RP256 = 256 / ROWB;         // strip rows per 256 bytes of LDS (all banks once)
    auto epilogue_impl = [&](auto scaled_c, int64_t em0, int64_t en0, int ebatch, int esplit) {
        constexpr bool scaled = decltype(scaled_c)::value;   // alpha != 1: one more multiply per element
        // The lane number and the row stride are made opaque here, so that the strip and row addresses
        // below are formed inside the epilogue: hoisted out of the item loop they would occupy
        // registers (and spill) through the whole K loop.
        int lane = lane_id;
        asm volatile("" : "+v"(lane));
        char *epi = smem + EPI_BASE + wave * EPI_BYTES;
        TOut *C;
        const float *bias_lds = nullptr;     // BIAS: the bias of this wavefront's first column (zeros without a bias)
        if constexpr (!MAPPED) {
            C = static_cast<TOut *>(p.C) + ebatch * p.sC + esplit * p.sSplit + (em0 + wm * WM) * p.ldc + en0 + wn * WN;
        } else {
            C = static_cast<TOut *>(p.C);
        }
        if constexpr (BIAS) {
            // one add per output element whether or not there is a bias: no branch inside the unrolled loops
            float *strip = reinterpret_cast<float *>(smem + EPI_BASE + WAVES * EPI_BYTES);
            __syncthreads();   // the previous item's strip has been read
            for (int x = tid; x < BN; x += 256) strip[x] = p.maps.bias ? p.maps.bias[axis_offset_fast(p.maps.bias_n, en0 + x)] : 0.f;
            __syncthreads();
            bias_lds = strip + wn * WN + 4 * (lane >> 5);
        }
        const float alpha = p.alpha;
        int64_t row_stride = MAPPED ? p.maps.c_m.u : p.ldc;
        asm volatile("" : "+s"(row_stride));
        // write side: this lane's row of the strip, the byte inside a slot, and its rows' slot permutation
        const int wr_row = lane & 31;
        const unsigned wr_base = (unsigned)(wr_row * ROWB + (ESZ == 2 ? 8 * (lane >> 5) : 0));
        const unsigned wr_perm = (unsigned)(((wr_row / RP256) & (LPR - 1)) << 4);
        // read side: row (lane / LPR) of a pass, slot (lane % LPR); the permutation of pass `ps` differs from
        // that of pass 0 by a constant (RPP is a multiple of RP256)
        const int rd_row = lane / LPR;
        const unsigned rd_base = (unsigned)(rd_row * ROWB);
        const unsigned rd_slot = (unsigned)(((lane % LPR) ^ ((rd_row / RP256) & (LPR - 1))) << 4);

        auto write_strip = [&](int sidx, char *buf) {
            const int i = sidx / (TN / JH), jh = sidx % (TN / JH);
#pragma unroll
            for (int jj = 0; jj < JH; ++jj) {
                const int j = jh * JH + jj;
                // BIAS: the bias values of a 32-column block are read from LDS in one go, ahead of the
                // conversions (read where they are used, every group of four columns waits a whole LDS
                // latency for its own read)
                f32x4 bv[4];
                if constexpr (BIAS) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) bv[g] = *reinterpret_cast<const f32x4 *>(bias_lds + j * 32 + 8 * g);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    // registers 4g..4g+3 of lane: row lane%32, columns j*32 + 8g + 4*(lane/32) + 0..3
                    const unsigned cb = (unsigned)((jj * 32 + 8 * g) * ESZ);     // byte of column 8g in the strip row
                    const unsigned slot16 = ESZ == 2 ? (cb & ~15u) : cb;          // fp32: the lane half picks the next slot
                    unsigned ad = wr_base + ((slot16 + (ESZ == 4 ? 16u * (unsigned)(lane >> 5) : 0u)) ^ wr_perm);
                    char *dst = buf + ad;
                    float v0 = acc[i][j][4 * g], v1 = acc[i][j][4 * g + 1];
                    float v2 = acc[i][j][4 * g + 2], v3 = acc[i][j][4 * g + 3];
                    if (scaled) { v0 *= alpha; v1 *= alpha; v2 *= alpha; v3 *= alpha; }
                    if constexpr (BIAS) {
                        v0 += bv[g][0]; v1 += bv[g][1]; v2 += bv[g][2]; v3 += bv[g][3];
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
        };
        auto read_strip = [&](const char *buf, i32x4 (&v)[NPASS]) {
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps) {
                const unsigned perm_ps = (unsigned)((((ps * RPP) / RP256) & (LPR - 1)) << 4);
                v[ps] = *reinterpret_cast<const i32x4 *>(buf + rd_base + ps * RPP * ROWB + (rd_slot ^ perm_ps));
            }
        };
        auto store_strip = [&](int sidx, const i32x4 (&v)[NPASS]) {
            const int i = sidx / (TN / JH), jh = sidx % (TN / JH);
            int64_t strip_m = 0, col = 0;   // MAPPED: where this 32-row strip (inside one shard) starts, and this lane's 16 bytes
            if constexpr (MAPPED) {
                strip_m = axis_offset_fast(p.maps.c_m, em0 + wm * WM + i * 32);
                col = axis_offset_fast(p.maps.c_n, en0 + wn * WN + jh * JH * 32 + (lane % LPR) * (16 / ESZ));
            }
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps) {
                const int row = ps * RPP + rd_row;
                char *gp;
                if constexpr (!MAPPED)
                    gp = reinterpret_cast<char *>(C + (int64_t)(i * 32 + row) * row_stride + jh * JH * 32) + (lane % LPR) * 16;
                else gp = reinterpret_cast<char *>(C + col + strip_m + (int64_t)row * row_stride);
                // streaming store: the product is not read again by this kernel, and kept out of the
                // caches it leaves them to the operand panels that other XCDs still fetch (measured
                // on the large bf16 shapes, three products back to back: +1.4 %, dX +3.8 %)
                __builtin_nontemporal_store(v[ps], reinterpret_cast<i32x4 *>(gp));
            }
        };

        if constexpr (NBUF == 2) {
            // strip s is written while the reads of strip s-1 are in flight; its stores follow those reads
            i32x4 held[2][NPASS];
#pragma unroll
            for (int sidx = 0; sidx < NSTRIP; ++sidx) {
                write_strip(sidx, epi + (sidx & 1) * STRIP_BYTES);
                __builtin_amdgcn_sched_barrier(0);
                if (sidx > 0) store_strip(sidx - 1, held[(sidx - 1) & 1]);
                read_strip(epi + (sidx & 1) * STRIP_BYTES, held[sidx & 1]);
                // one strip at a time: without this the scheduler pulls all accumulator reads to the
                // front and needs a register for every output element at once
                __builtin_amdgcn_sched_barrier(0);
            }
            store_strip(NSTRIP - 1, held[(NSTRIP - 1) & 1]);
        } else {
#pragma unroll
            for (int sidx = 0; sidx < NSTRIP; ++sidx) {
                i32x4 held[NPASS];
                write_strip(sidx, epi);
                read_strip(epi, held);
                store_strip(sidx, held);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    auto epilogue = [&](int64_t em0, int64_t en0, int ebatch, int esplit) {
        if (p.alpha == 1.f) epilogue_impl(std::false_type{}, em0, en0, ebatch, esplit);
        else epilogue_impl(std::true_type{}, em0, en0, ebatch, esplit);
    };

    // ---- the items of this workgroup ----------------------------------------------------------------------
    CUBE3D_STAMP();
    int item = blockIdx.x;
    decode_item(item);
    setup_sources();
    early_loads();
    if (p.stagger > 0) {
        // Staggered start (launches in which a workgroup takes several items): the workgroups reach
        // their epilogues at different times, so that the output of one round of items is not written
        // by all CUs at once (the fabric takes 4.5 TB/s of writes; a burst of 128 KB per CU from every CU
        // holds each of them up for microseconds, four times per launch).  The first loads are in flight
        // meanwhile.  The wait ends on a free-running clock, whatever else happens.
        const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
        const unsigned long long wait = (unsigned long long)p.stagger * blockIdx.x / gridDim.x;
        while (__builtin_amdgcn_s_memrealtime() - t0 < wait) __builtin_amdgcn_s_sleep(16);
    }
    finish_prologue(std::integral_constant<int, 0>{});
    bool after_stores = false;
    while (true) {
        k_loop(after_stores, std::integral_constant<int, STORES>{});
        CUBE3D_STAMP();   // K loop done
        after_stores = EPI_SEPARATE;   // only there are the stores younger than the next item's first loads
        const int64_t em0 = m0, en0 = n0;
        const int ebatch = batch, esplit = split;
        item += gridDim.x;
        const bool again = item < items;
        if constexpr (EPI_SEPARATE) {
            // the operands of the next item start to arrive while this one is written out
            if (again) {
                decode_item(item);
                setup_sources();
                early_loads();
            }
            CUBE3D_STAMP();   // next item's first loads issued
            epilogue(em0, en0, ebatch, esplit);
            CUBE3D_STAMP();   // epilogue issued
            if (!again) break;
            finish_prologue(std::integral_constant<int, STORES>{});
            CUBE3D_STAMP();   // first fragments read
        } else {
            __syncthreads();   // all fragment reads of the stage buffers are done
            epilogue(em0, en0, ebatch, esplit);
            if (!again) break;
            __syncthreads();   // ... and all reads of the staging strips
            decode_item(item);
            setup_sources();
            early_loads();
            finish_prologue(std::integral_constant<int, 0>{});   // the stores are older than these loads
        }
    }
}

// LDS bytes of one configuration: the stage buffers; the large tiles add the epilogue staging (and
// the bias strip) behind them.
template <typename E, int BM, int BN, int BKB, int NSTAGE, bool AK, bool BKM> constexpr int cfg_lds_bytes()
{
    using ATile = typename std::conditional<AK, KMajorTile<E, BM, BKB>, MNMajorTile<E, BM, BKB>>::type;
    using BTile = typename std::conditional<BKM, KMajorTile<E, BN, BKB>, MNMajorTile<E, BN, BKB>>::type;
    return NSTAGE * (ATile::BYTES + BTile::BYTES) + (BM * BN > 128 * 128 ? 32 * 1024 : 0);
}

// One-time set-up of a configuration on the current device: the kernel needs more dynamic LDS than
// the default limit.  Done once per device, under a lock (the flags are the only state the product
// kernels keep); registered with kernel_setups() so that cube3d_init() can run it before the first
// launch (a first launch from inside a stream capture would otherwise do it there).
template <typename E, int BM, int BN, int BKB, int NSTAGE, bool AK, bool BKM, typename TOut, bool MAPPED> struct CfgSetup {
    static int run()
    {
        static std::mutex mu;
        static std::atomic<uint64_t> done{0};
        const int dev = current_device();
        if (dev < 0 || dev >= MAX_DEVICES) return CUBE3D_ELAUNCH;
        const uint64_t bit = 1ull << dev;
        if (done.load(std::memory_order_acquire) & bit) return CUBE3D_OK;
        std::lock_guard<std::mutex> lock(mu);
        if (done.load(std::memory_order_relaxed) & bit) return CUBE3D_OK;
        auto kern = gemm_mfma_kernel<E, BM, BN, BKB, NSTAGE, AK, BKM, TOut, MAPPED>;
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                cfg_lds_bytes<E, BM, BN, BKB, NSTAGE, AK, BKM>()) != hipSuccess) {
            (void)hipGetLastError();
            return CUBE3D_ELAUNCH;
        }
        done.fetch_or(bit, std::memory_order_release);
        return CUBE3D_OK;
    }
    struct Registrar {
        Registrar() { kernel_setups().push_back(&run); }
    };
    static inline Registrar registrar;
};

// Launch one configuration.  splits > 1: every split writes its own fp32 partial result
// [batch][split][Mo][No] to `out` (then out_ld = No); splits == 1: `out` is the final C.
template <typename E, int BM, int BN, int BKB, int NSTAGE, bool AK, bool BKM, typename TOut, bool MAPPED = false>
int launch_cfg(const GemmArgs &g, int splits, void *out, int64_t out_ld, int64_t out_batch_stride, int64_t out_split_stride,
               float alpha)
{
    constexpr int LDS = cfg_lds_bytes<E, BM, BN, BKB, NSTAGE, AK, BKM>();
    using Setup = CfgSetup<E, BM, BN, BKB, NSTAGE, AK, BKM, TOut, MAPPED>;
    (void)&Setup::registrar;   // instantiates the registration
    auto kern = gemm_mfma_kernel<E, BM, BN, BKB, NSTAGE, AK, BKM, TOut, MAPPED>;
    if (const int rc = Setup::run(); rc != CUBE3D_OK) return rc;
    Params p;
    p.A = g.A;
    p.B = g.B;
    p.C = out;
    p.lda = g.lda; p.ldb = g.ldb; p.ldc = out_ld;
    p.sA = g.strideA; p.sB = g.strideB; p.sC = out_batch_stride;
    p.tiles_m = (int)(g.Mo / BM);
    p.tiles_n = (int)(g.No / BN);
    p.nk = (int)(g.Kc * E::ELT / BKB / splits);
    if (p.nk < NSTAGE || p.nk % NSTAGE != 0 || (int64_t)p.nk * splits * BKB != g.Kc * E::ELT) return CUBE3D_ENOTIMPL;
    p.group_m = 8;
    p.splits = splits;
    p.sSplit = out_split_stride;
    p.alpha = alpha;
    p.stagger = 0;
    if (MAPPED) {
        p.maps = *g.maps;
        for (AxisMap *m : {&p.maps.a_mn, &p.maps.a_k, &p.maps.b_mn, &p.maps.b_k, &p.maps.c_m, &p.maps.c_n, &p.maps.bias_n})
            prepare_axis_map(*m);
        p.ka = make_kwalk(g.maps->a_k, BKB / E::ELT);
        p.kb = make_kwalk(g.maps->b_k, BKB / E::ELT);
    }
    p.y_items = g.batch * splits;
#ifdef CUBE3D_PROFILE
    p.prof = getenv("CUBE3D_PROF_PTR") ? reinterpret_cast<unsigned long long *>(strtoull(getenv("CUBE3D_PROF_PTR"), nullptr, 0)) : nullptr;
#endif
    // persistent workgroups: as many as the chip holds at once, or one per item.  The item -> XCD
    // regrouping in the kernel needs a grid that is a multiple of 8 whenever a workgroup takes more
    // than one item.
    const int64_t items = (int64_t)p.tiles_m * p.tiles_n * p.y_items;
    const int64_t per_cu = LDS > 80 * 1024 ? 1 : 2;   // workgroups the 160 KB of a CU's LDS hold
    const int64_t resident = (int64_t)num_compute_units() * per_cu / 8 * 8;
    if (items >= (1ll << 31) || resident < 8) return CUBE3D_ENOTIMPL;
    dim3 grid((unsigned)(items < resident ? items : resident), 1, 1);
    // Several items per workgroup: spread the workgroups' starts over about the time the fabric needs
    // to take one round's output (all resident tiles, at 4.5 TB/s of writes; 10 ns units), see the kernel.
    if (items > resident) p.stagger = (int)((int64_t)grid.x * BM * BN * (int64_t)sizeof(TOut) / 56000);
#ifdef CUBE3D_STAGGER_ENV
    if (items > resident && getenv("CUBE3D_STAGGER")) p.stagger = atoi(getenv("CUBE3D_STAGGER"));
#endif
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
