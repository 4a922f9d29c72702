// Virtual-cube data movement: the load-balanced storage of Section 3.1.1
// (scatter / assemble), the all-gathers of Algorithm 1 steps 1-2 (and of dY for
// Algorithm 2), and the reduce-scatters of Algorithm 1 step 4 and Algorithm 2.
// All q^3 processors' buffers live in this GPU's memory, so every "collective"
// is a streaming copy or a streaming sum: HBM-bandwidth work, no matrix cores.
//
// Work decomposition.  Scatter / assemble and the reduce-scatters: blockIdx.z =
// destination processor r, blockIdx.x = a group of destination rows; each
// wavefront takes whole rows, its lanes stride over 16-byte pieces of the row; all
// index decoding is wave-uniform.  All-gathers: blockIdx.z = SOURCE processor, whose
// shard is read once and written to the q members of its group (cube_gather_kernel).
#include "common.h"

namespace cube3d {

namespace {

constexpr int ROWS_PER_BLOCK = 16;

struct Coords {
    int i, a, b;
};

__device__ __forceinline__ Coords decode_rank(const CubeGeom &g, int r)
{
    const int l = r % g.q;
    const int j = (r / g.q) % g.q;
    Coords c;
    c.i = r / (g.q * g.q);
    c.a = g.in_axis_z ? l : j;
    c.b = g.in_axis_z ? j : l;
    return c;
}

__device__ __forceinline__ int64_t rank_index(const CubeGeom &g, int i, int a, int b)
{
    return g.in_axis_z ? ((int64_t)(i * g.q + b) * g.q + a) : ((int64_t)(i * g.q + a) * g.q + b);
}

// For destination row `row` of processor r: element offsets of the row in the
// destination and of its first source segment; `seg` = elements per contiguous
// source segment, `seg_stride` = source distance between consecutive segments
// of the same destination row (only the W gather has more than one).
struct RowMap {
    int64_t dst, src, seg, seg_stride;
};

// A processor's indices along the three cube directions of a placement: block row, block column,
// piece; and the distance in processor numbers between neighbours along the piece direction.
struct PlaceCoords {
    int rb, cb, s;
    int64_t rstride;
};

__device__ __forceinline__ PlaceCoords decode_place(const CubeGeom &g, int r)
{
    const int idx[3] = {r / (g.q * g.q), (r / g.q) % g.q, r % g.q};
    PlaceCoords c;
    c.rb = g.p_ra == 0 ? idx[0] : g.p_ra == 1 ? idx[1] : idx[2];
    c.cb = g.p_ca == 0 ? idx[0] : g.p_ca == 1 ? idx[1] : idx[2];
    c.s = g.p_sa == 0 ? idx[0] : g.p_sa == 1 ? idx[1] : idx[2];
    c.rstride = g.p_sa == 0 ? (int64_t)g.q * g.q : g.p_sa == 1 ? g.q : 1;
    return c;
}

__device__ __forceinline__ RowMap map_copy_row(const CubeGeom &g, int mode, int r, int64_t row)
{
    RowMap m;
    m.seg_stride = 0;
    if (mode >= MV_PLACE_GATHER) {
        const PlaceCoords pc = decode_place(g, r);
        if (mode == MV_PLACE_GATHER) {
            m.dst = ((int64_t)r * g.pRb + row) * g.pCb;
            if (g.p_split_rows) {   // row piece s' comes from the processor with piece index s'
                const int64_t s2 = row / g.pRs, rr = row - s2 * g.pRs;
                m.seg = g.pCb;
                m.src = ((r + (s2 - pc.s) * pc.rstride) * g.pRs + rr) * g.pCb;
            } else {                // every row is q column pieces, one per processor of the group
                m.seg = g.pCs;
                m.src = ((r - pc.s * pc.rstride) * g.pRb + row) * g.pCs;
                m.seg_stride = pc.rstride * g.pRb * g.pCs;
            }
        } else {
            m.seg = g.pCs;
            const int64_t sh = ((int64_t)r * g.pRs + row) * g.pCs;
            const int64_t fu = ((int64_t)pc.rb * g.pRb + (g.p_split_rows ? (int64_t)pc.s * g.pRs : 0) + row) * g.pC +
                               (int64_t)pc.cb * g.pCb + (g.p_split_rows ? 0 : (int64_t)pc.s * g.pCs);
            m.dst = mode == MV_PLACE_SCATTER ? sh : fu;
            m.src = mode == MV_PLACE_SCATTER ? fu : sh;
        }
        return m;
    }
    const Coords c = decode_rank(g, r);
    switch (mode) {
    case MV_GATHER_X: {  // dst [Mb,Kb]; row panel a' comes from processor (i, a', b)
        const int64_t a2 = row / g.Ms, rr = row - a2 * g.Ms;
        m.seg = g.Kb;
        m.dst = ((int64_t)r * g.Mb + row) * g.Kb;
        m.src = (rank_index(g, c.i, (int)a2, c.b) * g.Ms + rr) * g.Kb;
        break;
    }
    case MV_GATHER_DY: {  // dst [Mb,Nb]; row panel b' comes from processor (i, a, b')
        const int64_t b2 = row / g.Ms, rr = row - b2 * g.Ms;
        m.seg = g.Nb;
        m.dst = ((int64_t)r * g.Mb + row) * g.Nb;
        m.src = (rank_index(g, c.i, c.a, (int)b2) * g.Ms + rr) * g.Nb;
        break;
    }
    case MV_GATHER_W: {  // dst [Kb,Nb]; column panel i' comes from processor (i', a, b)
        m.seg = g.Ns;
        m.dst = ((int64_t)r * g.Kb + row) * g.Nb;
        m.src = (rank_index(g, 0, c.a, c.b) * g.Kb + row) * g.Ns;
        m.seg_stride = (rank_index(g, 1 % g.q, c.a, c.b) - rank_index(g, 0, c.a, c.b)) * g.Kb * g.Ns;
        break;
    }
    case MV_SCATTER_X:
    case MV_ASSEMBLE_X: {
        m.seg = g.Kb;
        const int64_t sh = ((int64_t)r * g.Ms + row) * g.Kb;
        const int64_t fu = ((int64_t)c.i * g.Mb + (int64_t)c.a * g.Ms + row) * g.K + (int64_t)c.b * g.Kb;
        m.dst = mode == MV_SCATTER_X ? sh : fu;
        m.src = mode == MV_SCATTER_X ? fu : sh;
        break;
    }
    case MV_SCATTER_W:
    case MV_ASSEMBLE_W: {
        m.seg = g.Ns;
        const int64_t sh = ((int64_t)r * g.Kb + row) * g.Ns;
        const int64_t fu = ((int64_t)c.b * g.Kb + row) * g.N + (int64_t)c.a * g.Nb + (int64_t)c.i * g.Ns;
        m.dst = mode == MV_SCATTER_W ? sh : fu;
        m.src = mode == MV_SCATTER_W ? fu : sh;
        break;
    }
    default: {  // MV_SCATTER_Y / MV_ASSEMBLE_Y
        m.seg = g.Nb;
        const int64_t sh = ((int64_t)r * g.Ms + row) * g.Nb;
        const int64_t fu = ((int64_t)c.i * g.Mb + (int64_t)c.b * g.Ms + row) * g.N + (int64_t)c.a * g.Nb;
        m.dst = mode == MV_SCATTER_Y ? sh : fu;
        m.src = mode == MV_SCATTER_Y ? fu : sh;
        break;
    }
    }
    return m;
}

// VecT = what one lane moves per step; es = element size in bytes.  A wavefront works on the
// four rows it owns in its block at the same time, four pieces per row in flight, so that every
// lane has up to sixteen independent loads outstanding before the first store (the rows are
// short: one row alone leaves the memory system idle).
template <typename VecT>
__global__ __launch_bounds__(256) void cube_copy_kernel(CubeGeom g, int mode, int64_t rows, int nseg, int es,
                                                        const char *__restrict__ src, char *__restrict__ dst)
{
    constexpr int RPW = ROWS_PER_BLOCK / 4;   // rows per wavefront
    constexpr int U = 4;                      // pieces per row per step
    const int r = blockIdx.z;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int64_t row0 = (int64_t)blockIdx.x * ROWS_PER_BLOCK + wave;

    const VecT *s[RPW];
    VecT *d[RPW];
    int64_t seg_vecs = 1, stride_vecs = 0;
#pragma unroll
    for (int w = 0; w < RPW; ++w) {
        const int64_t row = row0 + 4 * w;
        const RowMap m = map_copy_row(g, mode, r, row < rows ? row : rows - 1);
        seg_vecs = m.seg * es / (int64_t)sizeof(VecT);
        stride_vecs = m.seg_stride * es / (int64_t)sizeof(VecT);
        s[w] = reinterpret_cast<const VecT *>(src + m.src * es);
        d[w] = reinterpret_cast<VecT *>(dst + m.dst * es);
    }
    const int64_t total = seg_vecs * nseg;
    for (int64_t c0 = lane; c0 < total; c0 += 64 * U) {
        VecT v[RPW][U];
#pragma unroll
        for (int w = 0; w < RPW; ++w)
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t c = c0 + 64 * u;
                if (c < total && row0 + 4 * w < rows) {
                    const int64_t p = nseg == 1 ? 0 : c / seg_vecs;
                    v[w][u] = s[w][p * stride_vecs + (c - p * seg_vecs)];
                }
            }
#pragma unroll
        for (int w = 0; w < RPW; ++w)
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t c = c0 + 64 * u;
                if (c < total && row0 + 4 * w < rows) d[w][c] = v[w][u];
            }
    }
}

// All-gather, source-major: blockIdx.z = the SOURCE processor, whose shard (one contiguous array of
// rows x seg elements) is read exactly once and written to the q processors of its group, each row
// into its place in their gathered blocks.  (Destination-major, every shard would be fetched q times,
// by workgroups on different XCDs.)  A lane has U 16-byte loads in flight before its U * q stores; the
// stores are streaming stores (the gathered copies are not read again by this kernel).
//   destination of (member d, shard row, vector c) = first + d * step + row * ld + c      (in VecT units)
struct GatherMap {
    int64_t rows, seg;            // shard rows, elements per shard row
    int64_t first, step, ld;      // elements: offset for member 0, distance between members, destination row length
};

__device__ __forceinline__ GatherMap map_gather(const CubeGeom &g, int mode, int r)
{
    GatherMap m;
    if (mode == MV_PLACE_GATHER) {
        const PlaceCoords pc = decode_place(g, r);
        const int64_t blk = g.pRb * g.pCb;
        m.rows = g.pRs; m.seg = g.pCs;
        m.first = (r - pc.s * pc.rstride) * blk + (g.p_split_rows ? (int64_t)pc.s * g.pRs * g.pCb : (int64_t)pc.s * g.pCs);
        m.step = pc.rstride * blk;
        m.ld = g.pCb;
        return m;
    }
    const Coords c = decode_rank(g, r);
    if (mode == MV_GATHER_X) {          // shard of (i, a', b): row panel a' of the blocks of (i, ., b)
        m.rows = g.Ms; m.seg = g.Kb; m.ld = g.Kb;
        m.first = rank_index(g, c.i, 0, c.b) * g.Mb * g.Kb + (int64_t)c.a * g.Ms * g.Kb;
        m.step = (rank_index(g, c.i, 1 % g.q, c.b) - rank_index(g, c.i, 0, c.b)) * g.Mb * g.Kb;
    } else if (mode == MV_GATHER_DY) {  // shard of (i, a, b'): row panel b' of the blocks of (i, a, .)
        m.rows = g.Ms; m.seg = g.Nb; m.ld = g.Nb;
        m.first = rank_index(g, c.i, c.a, 0) * g.Mb * g.Nb + (int64_t)c.b * g.Ms * g.Nb;
        m.step = (rank_index(g, c.i, c.a, 1 % g.q) - rank_index(g, c.i, c.a, 0)) * g.Mb * g.Nb;
    } else {                            // MV_GATHER_W: shard of (i', a, b): column panel i' of the blocks of (., a, b)
        m.rows = g.Kb; m.seg = g.Ns; m.ld = g.Nb;
        m.first = rank_index(g, 0, c.a, c.b) * g.Kb * g.Nb + (int64_t)c.i * g.Ns;
        m.step = (rank_index(g, 1 % g.q, c.a, c.b) - rank_index(g, 0, c.a, c.b)) * g.Kb * g.Nb;
    }
    return m;
}

template <typename VecT, int U>
__global__ __launch_bounds__(256) void cube_gather_kernel(CubeGeom g, int mode, int es, const char *__restrict__ src,
                                                          char *__restrict__ dst)
{
    const int r = blockIdx.z;
    const GatherMap m = map_gather(g, mode, r);
    const int64_t vpr = m.seg * es / (int64_t)sizeof(VecT);          // vectors per shard row
    const int64_t total = m.rows * vpr;                              // vectors in the shard
    const int64_t ld = m.ld * es / (int64_t)sizeof(VecT), step = m.step * es / (int64_t)sizeof(VecT);
    const VecT *s = reinterpret_cast<const VecT *>(src) + (int64_t)r * total;
    VecT *d = reinterpret_cast<VecT *>(dst) + m.first * es / (int64_t)sizeof(VecT);
    const int q = g.q;
    const int64_t f0 = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
    VecT v[U];
    int64_t off[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t f = f0 + 256 * u;
        if (f < total) {
            v[u] = s[f];
            const int64_t row = (uint64_t)(f | vpr) < (1ull << 32) ? (int64_t)((uint32_t)f / (uint32_t)vpr) : f / vpr;
            off[u] = row * ld + (f - row * vpr);
        }
    }
    for (int member = 0; member < q; ++member) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (f0 + 256 * u < total) __builtin_nontemporal_store(v[u], d + member * step + off[u]);
    }
}

template <typename T> __device__ __forceinline__ float load_f32(const T *p);
template <> __device__ __forceinline__ float load_f32<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_f32<unsigned short>(const unsigned short *p)
{
    return bf16_bits_to_f32(*p);
}
template <typename T> __device__ __forceinline__ void store_f32(T *p, float v);
template <> __device__ __forceinline__ void store_f32<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_f32<unsigned short>(unsigned short *p, float v)
{
    *p = f32_to_bf16_bits(v);
}

template <typename T, int V> struct __attribute__((aligned(sizeof(T) * V))) Pack {
    T v[V];
};

// Streaming (non-temporal) access to a pack: data that is touched once should not displace what
// other kernels left in the caches.  The builtins take scalars or vectors, so a pack travels as the
// integer vector of its size.
template <int BYTES> struct RawVec;
template <> struct RawVec<16> { typedef i32x4 type; };
template <> struct RawVec<8> { typedef int type __attribute__((ext_vector_type(2))); };
template <> struct RawVec<4> { typedef int type; };
template <> struct RawVec<2> { typedef short type; };

template <typename P> __device__ __forceinline__ P stream_load_pack(const P *p)
{
    typedef typename RawVec<sizeof(P)>::type R;
    return __builtin_bit_cast(P, __builtin_nontemporal_load(reinterpret_cast<const R *>(p)));
}

template <typename P> __device__ __forceinline__ void stream_store_pack(P *p, const P &v)
{
    typedef typename RawVec<sizeof(P)>::type R;
    __builtin_nontemporal_store(__builtin_bit_cast(R, v), reinterpret_cast<R *>(p));
}

// Sum over the q partials of a reduce direction, fp32, ascending index, one rounding at the
// store.  V elements per lane per step; the loads of up to four partials are in flight together.
// STREAM: streaming loads and stores, for partials that cannot stay in the caches anyway.
template <typename TIn, typename TOut, int V, bool STREAM>
__global__ __launch_bounds__(256) void cube_reduce_kernel(CubeGeom g, int mode, int64_t rows,
                                                          const TIn *__restrict__ partials, TOut *__restrict__ shards,
                                                          const float *__restrict__ bias)
{
    constexpr int RPW = ROWS_PER_BLOCK / 4;
    constexpr int QU = 4;                     // partials loaded together
    const int r = blockIdx.z;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const Coords c = decode_rank(g, r);
    const int64_t row0 = (int64_t)blockIdx.x * ROWS_PER_BLOCK + wave;

    int64_t seg, src0, src_step, src_ld, dst_ld, src_row0, src_col0;
    if (mode == MV_REDUCE_Y) {  // keep row panel b of the sum over b'
        seg = g.Nb; dst_ld = g.Nb; src_ld = g.Nb; src_row0 = (int64_t)c.b * g.Ms; src_col0 = 0;
        src0 = rank_index(g, c.i, c.a, 0) * g.Mb * g.Nb;
        src_step = (rank_index(g, c.i, c.a, 1 % g.q) - rank_index(g, c.i, c.a, 0)) * g.Mb * g.Nb;
    } else if (mode == MV_REDUCE_DX) {  // keep row panel a of the sum over a'
        seg = g.Kb; dst_ld = g.Kb; src_ld = g.Kb; src_row0 = (int64_t)c.a * g.Ms; src_col0 = 0;
        src0 = rank_index(g, c.i, 0, c.b) * g.Mb * g.Kb;
        src_step = (rank_index(g, c.i, 1 % g.q, c.b) - rank_index(g, c.i, 0, c.b)) * g.Mb * g.Kb;
    } else if (mode == MV_REDUCE_DW) {  // keep column panel i of the sum over i'
        seg = g.Ns; dst_ld = g.Ns; src_ld = g.Nb; src_row0 = 0; src_col0 = (int64_t)c.i * g.Ns;
        src0 = rank_index(g, 0, c.a, c.b) * g.Kb * g.Nb;
        src_step = (rank_index(g, 1 % g.q, c.a, c.b) - rank_index(g, 0, c.a, c.b)) * g.Kb * g.Nb;
    } else {  // MV_PLACE_REDUCE: keep piece s of the sum over the processors of the piece direction
        const PlaceCoords pc = decode_place(g, r);
        seg = g.pCs; dst_ld = g.pCs; src_ld = g.pCb;
        src_row0 = g.p_split_rows ? (int64_t)pc.s * g.pRs : 0;
        src_col0 = g.p_split_rows ? 0 : (int64_t)pc.s * g.pCs;
        src0 = (r - pc.s * pc.rstride) * g.pRb * g.pCb;
        src_step = pc.rstride * g.pRb * g.pCb;
    }
    const int64_t dst_rows = mode == MV_PLACE_REDUCE ? g.pRs : mode == MV_REDUCE_DW ? g.Kb : g.Ms;
    const int q = g.q;

    for (int w = 0; w < RPW; ++w) {
        const int64_t row = row0 + 4 * w;
        if (row >= rows) break;
        const TIn *s = partials + src0 + (src_row0 + row) * src_ld + src_col0;
        TOut *d = shards + ((int64_t)r * dst_rows + row) * dst_ld;
        for (int64_t e = (int64_t)lane * V; e < seg; e += 64 * V) {
            float acc[V];
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] = 0.f;
            for (int k0 = 0; k0 < q; k0 += QU) {
                Pack<TIn, V> p[QU];
#pragma unroll
                for (int u = 0; u < QU; ++u)
                    if (k0 + u < q) {
                        const Pack<TIn, V> *src = reinterpret_cast<const Pack<TIn, V> *>(s + (k0 + u) * src_step + e);
                        p[u] = STREAM ? stream_load_pack(src) : *src;
                    }
#pragma unroll
                for (int u = 0; u < QU; ++u)          // ascending index along the reduce direction
                    if (k0 + u < q) {
#pragma unroll
                        for (int v = 0; v < V; ++v) acc[v] += load_f32<TIn>(&p[u].v[v]);
                    }
            }
            if (bias) {   // Algorithm 7 step 3: the output block's bias, added to the finished sum
                const Pack<float, V> b = *reinterpret_cast<const Pack<float, V> *>(bias + (int64_t)r * g.Nb + e);
#pragma unroll
                for (int v = 0; v < V; ++v) acc[v] += b.v[v];
            }
            Pack<TOut, V> o;
#pragma unroll
            for (int v = 0; v < V; ++v) store_f32<TOut>(&o.v[v], acc[v]);
            if (STREAM) stream_store_pack(reinterpret_cast<Pack<TOut, V> *>(d + e), o);
            else *reinterpret_cast<Pack<TOut, V> *>(d + e) = o;
        }
    }
}

template <typename TIn, typename TOut>
int launch_reduce(const CubeGeom &g, int mode, int64_t rows, int64_t seg, const void *partials, void *shards,
                  const float *bias, hipStream_t stream)
{
    dim3 grid((unsigned)((rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), 1, (unsigned)(g.q * g.q * g.q));
    const TIn *p = static_cast<const TIn *>(partials);
    TOut *s = static_cast<TOut *>(shards);
    // Partials larger than the 256 MB Infinity Cache are read once from HBM whatever the caches do:
    // streaming accesses then keep them from displacing everything else (measured on 1 GB of fp32
    // partials: 4.8 -> 5.1-5.4 TB/s); smaller ones may still be cache-resident from the producing kernel.
    const int64_t n = (int64_t)g.q * g.q * g.q;
    const bool streaming = n * g.q * rows * seg * (int64_t)sizeof(TIn) > (256ll << 20);
    if (seg % 4 == 0 && streaming)
        hipLaunchKernelGGL((cube_reduce_kernel<TIn, TOut, 4, true>), grid, dim3(256), 0, stream, g, mode, rows, p, s, bias);
    else if (seg % 4 == 0)
        hipLaunchKernelGGL((cube_reduce_kernel<TIn, TOut, 4, false>), grid, dim3(256), 0, stream, g, mode, rows, p, s, bias);
    else
        hipLaunchKernelGGL((cube_reduce_kernel<TIn, TOut, 1, false>), grid, dim3(256), 0, stream, g, mode, rows, p, s, bias);
    return launch_status();
}

}  // namespace

// rows: destination rows per processor; nseg: source segments per destination row
int cube_move(const CubeGeom &g, int mode, int es, const void *src, void *dst, hipStream_t stream)
{
    int64_t rows, seg;
    int nseg = 1;
    switch (mode) {
    case MV_GATHER_X: rows = g.Mb; seg = g.Kb; break;
    case MV_GATHER_DY: rows = g.Mb; seg = g.Nb; break;
    case MV_GATHER_W: rows = g.Kb; seg = g.Ns; nseg = g.q; break;
    case MV_SCATTER_X: case MV_ASSEMBLE_X: rows = g.Ms; seg = g.Kb; break;
    case MV_SCATTER_W: case MV_ASSEMBLE_W: rows = g.Kb; seg = g.Ns; break;
    case MV_SCATTER_Y: case MV_ASSEMBLE_Y: rows = g.Ms; seg = g.Nb; break;
    case MV_PLACE_GATHER:
        rows = g.pRb; seg = g.p_split_rows ? g.pCb : g.pCs; nseg = g.p_split_rows ? 1 : g.q; break;
    case MV_PLACE_SCATTER: case MV_PLACE_ASSEMBLE: rows = g.pRs; seg = g.pCs; break;
    default: return CUBE3D_EINVAL;
    }
    const char *s = static_cast<const char *>(src);
    char *d = static_cast<char *>(dst);
    const int64_t seg_bytes = seg * es;
    if (g.q * g.q * g.q > 65535) return CUBE3D_ESHAPE;
    if (mode == MV_GATHER_X || mode == MV_GATHER_DY || mode == MV_GATHER_W || mode == MV_PLACE_GATHER) {
        // source-major: one shard per grid plane
        const int64_t shard_rows = mode == MV_GATHER_W ? g.Kb : mode == MV_PLACE_GATHER ? g.pRs : g.Ms;
        const int64_t shard_seg = mode == MV_GATHER_W ? g.Ns : mode == MV_PLACE_GATHER ? g.pCs : seg;
        // every row start in source and destination is a multiple of the shard row length, so its
        // alignment decides the widest safe vector
        const int64_t row_bytes = shard_seg * es;
        const int vec = row_bytes % 16 == 0 ? 16 : row_bytes % 4 == 0 ? 4 : row_bytes % 2 == 0 ? 2 : 1;
        constexpr int U = 8;
        const int64_t nb = (shard_rows * row_bytes / vec + 256 * U - 1) / (256 * U);
        if (nb > 0x7fffffff) return CUBE3D_ESHAPE;
        dim3 ggrid((unsigned)nb, 1, (unsigned)(g.q * g.q * g.q));
        if (vec == 16) hipLaunchKernelGGL((cube_gather_kernel<i32x4, U>), ggrid, dim3(256), 0, stream, g, mode, es, s, d);
        else if (vec == 4) hipLaunchKernelGGL((cube_gather_kernel<int, U>), ggrid, dim3(256), 0, stream, g, mode, es, s, d);
        else if (vec == 2) hipLaunchKernelGGL((cube_gather_kernel<short, U>), ggrid, dim3(256), 0, stream, g, mode, es, s, d);
        else hipLaunchKernelGGL((cube_gather_kernel<char, U>), ggrid, dim3(256), 0, stream, g, mode, es, s, d);
        return launch_status();
    }
    const int64_t nblk = (rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    if (nblk > 0x7fffffff) return CUBE3D_ESHAPE;
    dim3 grid((unsigned)nblk, 1, (unsigned)(g.q * g.q * g.q));
    // every segment start is a multiple of the segment length, so alignment of the
    // segment length decides the widest safe vector
    if (seg_bytes % 16 == 0)
        hipLaunchKernelGGL((cube_copy_kernel<i32x4>), grid, dim3(256), 0, stream, g, mode, rows, nseg, es, s, d);
    else if (seg_bytes % 4 == 0)
        hipLaunchKernelGGL((cube_copy_kernel<int>), grid, dim3(256), 0, stream, g, mode, rows, nseg, es, s, d);
    else if (seg_bytes % 2 == 0)
        hipLaunchKernelGGL((cube_copy_kernel<short>), grid, dim3(256), 0, stream, g, mode, rows, nseg, es, s, d);
    else
        hipLaunchKernelGGL((cube_copy_kernel<char>), grid, dim3(256), 0, stream, g, mode, rows, nseg, es, s, d);
    return launch_status();
}

int cube_reduce(const CubeGeom &g, int mode, int partial_dtype, int shard_dtype, const void *partials, void *shards,
                const float *bias, hipStream_t stream)
{
    if (bias && mode != MV_REDUCE_Y) return CUBE3D_EINVAL;
    int64_t rows, seg;
    switch (mode) {
    case MV_REDUCE_Y: rows = g.Ms; seg = g.Nb; break;
    case MV_REDUCE_DX: rows = g.Ms; seg = g.Kb; break;
    case MV_REDUCE_DW: rows = g.Kb; seg = g.Ns; break;
    case MV_PLACE_REDUCE: rows = g.pRs; seg = g.pCs; break;
    default: return CUBE3D_EINVAL;
    }
    if (g.q * g.q * g.q > 65535) return CUBE3D_ESHAPE;
    if (partial_dtype == CUBE3D_F32 && shard_dtype == CUBE3D_F32)
        return launch_reduce<float, float>(g, mode, rows, seg, partials, shards, bias, stream);
    if (partial_dtype == CUBE3D_F32 && shard_dtype == CUBE3D_BF16)
        return launch_reduce<float, unsigned short>(g, mode, rows, seg, partials, shards, bias, stream);
    if (partial_dtype == CUBE3D_BF16 && shard_dtype == CUBE3D_F32)
        return launch_reduce<unsigned short, float>(g, mode, rows, seg, partials, shards, bias, stream);
    if (partial_dtype == CUBE3D_BF16 && shard_dtype == CUBE3D_BF16)
        return launch_reduce<unsigned short, unsigned short>(g, mode, rows, seg, partials, shards, bias, stream);
    return CUBE3D_EDTYPE;
}

// ---- vector parameters (Section 3.1.1; Algorithms 7 and 8) ---------------------------------------------
namespace {

// One block per destination processor (scatter, gather) or per source processor (assemble).
__global__ __launch_bounds__(256) void cube_bias_move_kernel(CubeGeom g, int mode, const float *__restrict__ src,
                                                             float *__restrict__ dst)
{
    const int r = blockIdx.x;
    const int l = r % g.q, j = (r / g.q) % g.q, i = r / (g.q * g.q);
    if (mode == MV_SCATTER_BIAS) {
        for (int64_t e = threadIdx.x; e < g.Ns; e += 256)
            dst[(int64_t)r * g.Ns + e] = (j == l) ? src[(int64_t)j * g.Nb + (int64_t)i * g.Ns + e] : 0.f;
    } else if (mode == MV_ASSEMBLE_BIAS) {
        if (j != l) return;
        for (int64_t e = threadIdx.x; e < g.Ns; e += 256)
            dst[(int64_t)j * g.Nb + (int64_t)i * g.Ns + e] = src[(int64_t)r * g.Ns + e];
    } else {  // MV_GATHER_BIAS: piece i' of block a comes from the diagonal processor (i', a, a)
        const int a = g.in_axis_z ? l : j;
        for (int64_t c = threadIdx.x; c < g.Nb; c += 256) {
            const int64_t i2 = c / g.Ns, e = c - i2 * g.Ns;
            dst[(int64_t)r * g.Nb + c] = src[((i2 * g.q + a) * g.q + a) * g.Ns + e];
        }
    }
}

template <typename T> __device__ __forceinline__ float dy_value(T raw);
template <> __device__ __forceinline__ float dy_value<float>(float raw) { return raw; }
template <> __device__ __forceinline__ float dy_value<unsigned short>(unsigned short raw) { return bf16_bits_to_f32(raw); }
// fp8 e4m3 "fn": 1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent 0 is subnormal
template <> __device__ __forceinline__ float dy_value<unsigned char>(unsigned char raw)
{
    const int e = (raw >> 3) & 15, m = raw & 7;
    const float mag = e == 0 ? (float)m * 0.001953125f                                      // m/8 * 2^-6
                             : __uint_as_float((unsigned)(e + 120) << 23 | (unsigned)m << 20);  // (1+m/8) * 2^(e-7)
    return (raw & 0x80) ? -mag : mag;
}

// Column sums of dY in two fixed-order stages (no atomics: every run adds in the same order).
//
// Stage 1: one block per (processor r, group of RG of its Ms rows, chunk of 64*V of its Nb columns).
// A lane owns V consecutive columns (one 16-byte load per row when V > 1); the four wavefronts
// take the rows 4u + wave of the group, eight rows in flight per wavefront, and add them in
// ascending order; the four sums are then added in wavefront order and written to
// part[(r * NRG + group) * Nb + column].
template <typename T, int V>
__global__ __launch_bounds__(256) void cube_bias_bwd_rows_kernel(CubeGeom g, int RG, int NRG,
                                                                 const T *__restrict__ dy, float *__restrict__ part)
{
    __shared__ float lds[4][64 * V];
    constexpr int U = 8;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int r = blockIdx.z, rg = blockIdx.y;
    const int64_t c0 = ((int64_t)blockIdx.x * 64 + lane) * V;
    const bool live = c0 < g.Nb;                       // Nb % V == 0: a lane is all in or all out
    const int64_t row_lo = (int64_t)rg * RG, row_hi = row_lo + RG < g.Ms ? row_lo + RG : g.Ms;
    const T *base = dy + ((int64_t)r * g.Ms) * g.Nb + c0;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    for (int64_t t0 = row_lo + wave; t0 < row_hi; t0 += 4 * U) {
        Pack<T, V> v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t t = t0 + 4 * u;
            if (live && t < row_hi) v[u] = *reinterpret_cast<const Pack<T, V> *>(base + t * g.Nb);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (live && t0 + 4 * u < row_hi) {
#pragma unroll
                for (int e = 0; e < V; ++e) acc[e] += dy_value<T>(v[u].v[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < V; ++e) lds[wave][e * 64 + lane] = acc[e];
    __syncthreads();
    float *out = part + ((int64_t)r * NRG + rg) * g.Nb + (int64_t)blockIdx.x * 64 * V;
    for (int x = threadIdx.x; x < 64 * V; x += 256) {
        const int ln = x / V, e = x % V;               // column x of the chunk sits at [e][ln]
        if ((int64_t)blockIdx.x * 64 * V + x < g.Nb)
            out[x] = ((lds[0][e * 64 + ln] + lds[1][e * 64 + ln]) + lds[2][e * 64 + ln]) + lds[3][e * 64 + ln];
    }
}

// Stage 2: one block of sixteen wavefronts per (processor r, chunk of 64 of its Ns columns).
// Processors off the diagonal get zeros.  On the diagonal processor (i, a, a), lane = column; the
// terms t = (i'*q + b')*NRG + group over every processor (i', a, b') of the output block's column
// of the cube are split into sixteen contiguous runs, one per wavefront, added in ascending order,
// and the sixteen sums are added in wavefront order: Algorithm 8's reduce along x plus the reduce
// along the output direction.
constexpr int FIN_WAVES = 16;
__global__ __launch_bounds__(64 * FIN_WAVES) void cube_bias_bwd_finish_kernel(CubeGeom g, int NRG, float scale,
                                                                              const float *__restrict__ part,
                                                                              float *__restrict__ db)
{
    __shared__ float lds[FIN_WAVES][64];
    constexpr int U = 32;   // a wavefront's run is at most 32 terms on the 64-processor cube: all of them in flight at once
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int r = blockIdx.x;
    const int l = r % g.q, j = (r / g.q) % g.q, i = r / (g.q * g.q);
    const int64_t c = (int64_t)blockIdx.y * 64 + lane;
    const bool live = c < g.Ns;
    if (j != l) {
        if (wave == 0 && live) db[(int64_t)r * g.Ns + c] = 0.f;
        return;
    }
    const int a = j;
    const int total = g.q * g.q * NRG, per = (total + FIN_WAVES - 1) / FIN_WAVES;
    const int t_lo = wave * per < total ? wave * per : total, t_hi = t_lo + per < total ? t_lo + per : total;
    // term t = (source processor (i', a, b'), its row group): walked with counters, one division per wavefront
    int src = t_lo / NRG, rg = t_lo - src * NRG;
    int si = src / g.q, sb = src - si * g.q;
    const float *col = part + (int64_t)i * g.Ns + c;
    float acc = 0.f;
    for (int t0 = t_lo; t0 < t_hi; t0 += U) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            v[u] = 0.f;
            if (t0 + u < t_hi) {
                if (live) v[u] = col[(rank_index(g, si, a, sb) * NRG + rg) * g.Nb];
                if (++rg == NRG) {
                    rg = 0;
                    if (++sb == g.q) { sb = 0; ++si; }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u];
    }
    lds[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && live) {
        float sum = lds[0][lane];
#pragma unroll
        for (int w = 1; w < FIN_WAVES; ++w) sum += lds[w][lane];
        db[(int64_t)r * g.Ns + c] = sum * scale;
    }
}

template <typename T>
void launch_bias_bwd_rows(const CubeGeom &g, int RG, int NRG, const void *dy, float *part, hipStream_t stream)
{
    constexpr int V = 16 / (int)sizeof(T);
    const unsigned nz = (unsigned)(g.q * g.q * g.q);
    if (g.Nb % V == 0) {
        dim3 grid((unsigned)((g.Nb + 64 * V - 1) / (64 * V)), (unsigned)NRG, nz);
        hipLaunchKernelGGL((cube_bias_bwd_rows_kernel<T, V>), grid, dim3(256), 0, stream, g, RG, NRG,
                           static_cast<const T *>(dy), part);
    } else {
        dim3 grid((unsigned)((g.Nb + 63) / 64), (unsigned)NRG, nz);
        hipLaunchKernelGGL((cube_bias_bwd_rows_kernel<T, 1>), grid, dim3(256), 0, stream, g, RG, NRG,
                           static_cast<const T *>(dy), part);
    }
}

// Rows per stage-1 block: as many as keep at least ~2048 blocks in flight (8 per compute unit),
// between 16 and 256, a power of two; depends on the shape only.
int bias_bwd_row_group(const CubeGeom &g, int es)
{
    const int V = g.Nb % (16 / es) == 0 ? 16 / es : 1;
    const int64_t chunks = (g.Nb + 64 * V - 1) / (64 * V) * (int64_t)g.q * g.q * g.q;
    int RG = 256;
    while (RG > 16 && chunks * ((g.Ms + RG - 1) / RG) < 2048) RG /= 2;
    return RG;
}

}  // namespace

int cube_bias_move(const CubeGeom &g, int mode, const float *src, float *dst, hipStream_t stream)
{
    if (mode != MV_SCATTER_BIAS && mode != MV_ASSEMBLE_BIAS && mode != MV_GATHER_BIAS) return CUBE3D_EINVAL;
    hipLaunchKernelGGL(cube_bias_move_kernel, dim3((unsigned)(g.q * g.q * g.q)), dim3(256), 0, stream, g, mode, src, dst);
    return launch_status();
}

size_t cube_bias_bwd_workspace(const CubeGeom &g, int dy_dtype)
{
    const int es = dy_dtype == CUBE3D_F32 ? 4 : dy_dtype == CUBE3D_BF16 ? 2 : 1;
    const int RG = bias_bwd_row_group(g, es);
    const int64_t NRG = (g.Ms + RG - 1) / RG;
    return (size_t)((int64_t)g.q * g.q * g.q * NRG * g.Nb) * sizeof(float);
}

int cube_bias_bwd(const CubeGeom &g, int dy_dtype, float scale_dy, const void *dy_shards, float *dbias_diag,
                  void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (dy_dtype != CUBE3D_F32 && dy_dtype != CUBE3D_BF16 && dy_dtype != CUBE3D_FP8_E4M3) return CUBE3D_EDTYPE;
    const int es = dy_dtype == CUBE3D_F32 ? 4 : dy_dtype == CUBE3D_BF16 ? 2 : 1;
    const int RG = bias_bwd_row_group(g, es);
    const int NRG = (int)((g.Ms + RG - 1) / RG);
    if (NRG > 65535 || (g.Ns + 63) / 64 > 65535 || (int64_t)g.q * g.q * g.q > 65535) return CUBE3D_ESHAPE;
    if (!workspace || workspace_bytes < cube_bias_bwd_workspace(g, dy_dtype)) return CUBE3D_EWORKSPACE;
    float *part = static_cast<float *>(workspace);
    switch (dy_dtype) {
    case CUBE3D_F32: launch_bias_bwd_rows<float>(g, RG, NRG, dy_shards, part, stream); break;
    case CUBE3D_BF16: launch_bias_bwd_rows<unsigned short>(g, RG, NRG, dy_shards, part, stream); break;
    default: launch_bias_bwd_rows<unsigned char>(g, RG, NRG, dy_shards, part, stream); break;
    }
    dim3 grid2((unsigned)(g.q * g.q * g.q), (unsigned)((g.Ns + 63) / 64), 1);
    hipLaunchKernelGGL(cube_bias_bwd_finish_kernel, grid2, dim3(64 * FIN_WAVES), 0, stream, g, NRG,
                       dy_dtype == CUBE3D_FP8_E4M3 ? scale_dy : 1.f, part, dbias_diag);
    return launch_status();
}

}  // namespace cube3d
