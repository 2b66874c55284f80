// Launch-shape and addressing study for the streaming kernels of the DaSGD parameter pipeline
// (gfx950).  A stand-alone program, not part of the library: it times variants of the local step
// (paper Eq. 2, first branch: three streams in, two out) and of the local step with the merge folded
// in (Eq. 2, both branches: plus one read of the average) on parameter sets of the benchmark's
// shapes, with three ways of finding the data:
//
//   flat     x, v, g are one W x ld matrix each: pure arithmetic on the block index
//   rows     one allocation per replica: the row's base pointers come from the kernel arguments,
//            selected by blockIdx.y (no value has to be loaded before the pointer can be)
//   records  one allocation per tensor: one record {x, v, g, position in the average, length} per
//            replica and piece of a tensor, looked up by block index; 2^CH blocks share a record
//
// and, for reference, the kernels the library used before this study decided its shapes (chunk table with
// 256 x 4 workgroups; flat matrix with a computed block order).  The figures decide which shapes the
// library uses; `profiles/` keeps the output.
//
//   shape_study resnet|bert [W]
#include "kernels.hpp"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

using namespace dasgd;

// ---- the kernels this library used before the study (chunk table; flat matrix with computed block order) ----
namespace legacy {
constexpr int kUnroll = 4;
constexpr int kChunk = kThreads * 4 * kUnroll;
// One unit of work: `len` consecutive elements of tensor `tensor`, starting at element `off` of the
// tensor and at element `foff` of a library-owned row (snapshot / average).
struct Chunk {
    int64_t off;
    int64_t foff;
    int32_t tensor;
    int32_t len;
};

// ------------------------------------------------------------------------------------------------
// Local step on every replica through the chunk table: grid = (chunks, W).
// 20 bytes per element (24 when both x and the snapshot are stored).
// MERGE: this step's merge is folded in -- the value stored to x is y + om (A - y), the snapshot
// (if any) still receives y (paper Eq. 2, both branches in one pass).  With xcd_order the grid is
// one-dimensional and ordered so that the W replicas of a chunk run back to back on one XCD: the
// chunk's piece of A comes from HBM once and from that XCD's L2 for the other W-1 replicas.
template <int MODE, bool MERGE>
__global__ void __launch_bounds__(kThreads)
k_local_step(const Chunk *__restrict__ chunks, float *const *__restrict__ xp, float *const *__restrict__ vp,
             const float *const *__restrict__ gp, float *__restrict__ S, int64_t P_pad, int n_tensors,
             float lr, float momentum, float wd, const float *__restrict__ A, float om, int W, int n_chunks, int xcd_order)
{
    constexpr bool WX = (MODE != kStoreS), WS = (MODE != kStoreX);
    static_assert(!(MERGE && MODE == kStoreS), "a folded merge always stores x");
    unsigned chunk_id = blockIdx.x;
    int j = blockIdx.y;
    if (MERGE && xcd_order) {
        const unsigned xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
        j = (int)(slot % (unsigned)W);
        chunk_id = (slot / (unsigned)W) * 8u + xcd;
        if (chunk_id >= (unsigned)n_chunks) return;
    }
    const Chunk c = chunks[chunk_id];
    const int64_t row = (int64_t)j * n_tensors + c.tensor;
    float *__restrict__ x = xp[row] + c.off;
    float *__restrict__ v = vp[row] + c.off;
    const float *__restrict__ g = gp[row] + c.off;
    float *__restrict__ s = WS ? S + (int64_t)j * P_pad + c.foff : nullptr;
    const float *__restrict__ a = MERGE ? A + c.foff : nullptr;
    const int tid = threadIdx.x;
    const int len = c.len;

    const bool aligned = ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(v) |
                           reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(s) |
                           reinterpret_cast<uintptr_t>(a)) & 15u) == 0;
    if (aligned) {
        v4f *x4 = reinterpret_cast<v4f *>(x);
        v4f *v4 = reinterpret_cast<v4f *>(v);
        const v4f *g4 = reinterpret_cast<const v4f *>(g);
        v4f *s4 = reinterpret_cast<v4f *>(s);
        const v4f *a4 = reinterpret_cast<const v4f *>(a);
        if (len == kChunk) {
            v4f xr[kUnroll], vr[kUnroll], gr[kUnroll], ar[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int i = tid + u * kThreads;
                xr[u] = ld4<true>(x4 + i);
                vr[u] = ld4<true>(v4 + i);
                gr[u] = ld4<true>(g4 + i);
                if (MERGE) ar[u] = ld4<false>(a4 + i);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int i = tid + u * kThreads;
                sgd4(xr[u], vr[u], gr[u], lr, momentum, wd);
                st4<true>(v4 + i, vr[u]);
                if (WS) st4<true>(s4 + i, xr[u]);
                if (WX) st4<true>(x4 + i, MERGE ? merge4(xr[u], ar[u], om) : xr[u]);
            }
        } else {
            const int n4 = len >> 2;
            for (int i = tid; i < n4; i += kThreads) {
                v4f xr = x4[i], vr = v4[i];
                const v4f gr = g4[i];
                sgd4(xr, vr, gr, lr, momentum, wd);
                v4[i] = vr;
                if (WS) s4[i] = xr;
                if (WX) x4[i] = MERGE ? merge4(xr, a4[i], om) : xr;
            }
            const int e = (n4 << 2) + tid;         // at most 3 leftover elements
            if (e < len) {
                float xs = x[e], vs = v[e];
                sgd1(xs, vs, g[e], lr, momentum, wd);
                v[e] = vs;
                if (WS) s[e] = xs;
                if (WX) x[e] = MERGE ? fmaf(om, a[e] - xs, xs) : xs;
            }
        }
    } else {
        for (int e = tid; e < len; e += kThreads) {
            float xs = x[e], vs = v[e];
            sgd1(xs, vs, g[e], lr, momentum, wd);
            v[e] = vs;
            if (WS) s[e] = xs;
            if (WX) x[e] = MERGE ? fmaf(om, a[e] - xs, xs) : xs;
        }
    }
}

// Work decomposition of the matrix-layout kernels that need the column of an element (to read the
// average A): the flat index space [0, W*row4) of 128-bit elements is cut into aligned blocks of 64
// (one wavefront, one whole kilobyte per array whatever the row length -- misaligned kilobytes cost
// 15 % of the bandwidth on MI355X).  A block that holds the boundary between rows j and j+1 belongs
// to row j and serves both.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2;
// the blocks of an XCD are issued in bands: B = 2^log_band column windows of row 0, the same windows
// of row 1, ... of row W-1, then the next band.  The band's piece of A (B KiB per XCD) is fetched from
// HBM once and re-read from that L2 by the other W-1 rows.  B = 1 issues the W replicas of one
// window back to back; which B is fastest depends on the row length (the host measures it).
// Returns false if this workgroup/lane has nothing to do; else the flat index i and the column c.
// The part of it that does not depend on the lane (also callable on the host, where the tests check
// that every block of every row is owned exactly once): block index, and the flat range of its row.
__host__ __device__ __forceinline__ bool decode_owner(unsigned b, unsigned W, unsigned row4, unsigned log_band,
                                                      unsigned &blk, unsigned &lo, unsigned &hi)
{
    const unsigned xcd = b & 7u, slot = b >> 3;
    const unsigned w = slot & ((1u << log_band) - 1u), t = slot >> log_band;
    const unsigned j = t % W, band = t / W;
    const unsigned q = (((band << log_band) + w) << 3) + xcd;    // column window
    lo = j * row4; hi = lo + row4;                           // flat range of row j
    const unsigned first = (lo + 63u) >> 6;                  // first block owned by row j
    const unsigned last = (hi - 1u) >> 6;                    // last one (it may reach into row j+1)
    blk = first + q;
    return blk <= last;
}
__device__ __forceinline__ bool decode_block(unsigned b, unsigned W, unsigned row4, unsigned n4, unsigned log_band,
                                             unsigned &i, unsigned &c)
{
    unsigned blk, lo, hi;
    if (!decode_owner(b, W, row4, log_band, blk, lo, hi)) return false;
    i = blk * kWave + threadIdx.x;
    if (i >= n4) return false;
    c = (i >= hi) ? i - hi : i - lo;
    return true;
}
// Largest useful log_band for a row length, and the number of workgroups decode_block needs.
static inline unsigned decode_windows_per_xcd(unsigned row4)
{
    return ((row4 >> 6) + 2u + 7u) / 8u;                     // blocks one row can own (upper bound), per XCD
}
static inline unsigned decode_clamp_log_band(unsigned row4, unsigned log_band)
{
    while (log_band > 0 && (1u << log_band) > decode_windows_per_xcd(row4)) --log_band;
    return log_band;
}
static inline uint64_t decode_grid(unsigned W, unsigned row4, unsigned log_band)
{
    const uint64_t per_xcd = decode_windows_per_xcd(row4), B = 1ull << log_band;
    return (per_xcd + B - 1) / B * B * 8ull * W;
}

// Matrix layout, local step with this step's merge folded in (paper Eq. 2, both branches in one
// pass): y = local update of x;  x <- y + (1 - xi)(A - y);  optionally snapshot <- y.
// Reads x, v, g once and the average A once (re-reads come from L2); writes x, v [, snapshot]:
// 20 + 4/W bytes per replica-element (24 + 4/W with the snapshot) instead of the 28 + 4/W (32 + 4/W)
// of separate local-step and merge kernels.  Needs n4 = W*P/4 < 2^31.
template <bool SNAP, int WT>   // WT > 0: W known at compile time; 0: any W
__global__ void __launch_bounds__(kWave)
k_step_merge_flat(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, v4f *__restrict__ s,
                  const v4f *__restrict__ A, unsigned n4, unsigned row4, int W, unsigned log_band,
                  float lr, float momentum, float wd, float om)
{
    unsigned i, c;
    if (!decode_block(blockIdx.x, WT > 0 ? (unsigned)WT : (unsigned)W, row4, n4, log_band, i, c)) return;
    v4f xr = ld4<true>(x + i);
    v4f vr = ld4<true>(v + i);
    const v4f gr = ld4<true>(g + i);
    const v4f a = ld4<false>(A + c);
    sgd4(xr, vr, gr, lr, momentum, wd);
    st4<true>(v + i, vr);
    if (SNAP) st4<true>(s + i, xr);
    st4<true>(x + i, merge4(xr, a, om));
}

// The same mean with the rows split over the NW wavefronts of a workgroup and the partial sums
// staged through LDS: wavefront w sums rows [w*R, (w+1)*R) of a 64-column window (R = W / NW loads
// in flight per lane), writes its partial to LDS, and after the barrier wavefront 0 adds the NW
// partials and stores the average.  With few rows per wave many more waves are in flight, which on
// MI355X is worth 2-6 % over the lane-owns-a-column form for W = 4, 8, 16 (measured: W=4 90 % vs 85 %
// of peak, W=8 82 % vs 80 %, W=16 80 % vs 76 %).  Tree order over rows is unchanged (identical bits).
template <int WT, int NW, bool RUNS>
__global__ void __launch_bounds__(kWave * NW)
k_mean_lds(const v4f *__restrict__ S, v4f *__restrict__ A, int64_t n4, int64_t row4, float inv_w)
{
    constexpr int R = WT / NW;
    static_assert(R * NW == WT && R >= 1, "rows must split evenly over the wavefronts");
    __shared__ v4f part[NW][kWave];
    __builtin_amdgcn_s_setprio(3);
    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int64_t blk = RUNS ? ((int64_t)(blockIdx.x >> 6) * 8 + (blockIdx.x & 7)) * 8 + ((blockIdx.x >> 3) & 7)
                             : (int64_t)blockIdx.x;
    const int64_t i = blk * kWave + l;
    if (i < n4) {
        v4f r[R];
#pragma unroll
        for (int j = 0; j < R; ++j) r[j] = ld4<true>(S + (int64_t)(w * R + j) * row4 + i);
        part[w][l] = tree_sum<0, R>(r);
    }
    __syncthreads();
    if (w == 0 && i < n4) {
        v4f p[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) p[k] = part[k][l];
        st4<false>(A + i, tree_sum<0, NW>(p) * inv_w);
    }
}

}  // namespace legacy
using namespace legacy;

#define CK(x)                                                                                     \
    do {                                                                                          \
        hipError_t e_ = (x);                                                                      \
        if (e_ != hipSuccess) {                                                                   \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);                 \
            exit(1);                                                                              \
        }                                                                                         \
    } while (0)

constexpr int kMaxW = 16;
struct RowPtrs {
    v4f *x[kMaxW];
    v4f *v[kMaxW];
    const v4f *g[kMaxW];
};
struct SRec {           // one piece (at most 2^CH blocks of 64 128-bit elements) of one tensor of one replica
    v4f *x;
    v4f *v;
    const v4f *g;
    unsigned a4;        // position of the piece in the average, in 128-bit elements
    unsigned len4;      // 128-bit elements in the piece
};

// ---- local step, flat ---------------------------------------------------------------------------
template <int THREADS, int UNROLL, bool NT>
__global__ void __launch_bounds__(THREADS) ls_flat(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, int64_t n4,
                                                   float lr, float mo, float wd)
{
    const int64_t base = (int64_t)blockIdx.x * (THREADS * UNROLL) + threadIdx.x;
    v4f xr[UNROLL], vr[UNROLL], gr[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t i = base + u * THREADS;
        if (i < n4) { xr[u] = ld4<NT>(x + i); vr[u] = ld4<NT>(v + i); gr[u] = ld4<NT>(g + i); }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const int64_t i = base + u * THREADS;
        if (i < n4) { sgd4(xr[u], vr[u], gr[u], lr, mo, wd); st4<NT>(x + i, xr[u]); st4<NT>(v + i, vr[u]); }
    }
}
// persistent grid-stride form
__global__ void __launch_bounds__(256) ls_flat_persistent(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, int64_t n4,
                                                          float lr, float mo, float wd)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        v4f xr = ld4<true>(x + i), vr = ld4<true>(v + i);
        const v4f gr = ld4<true>(g + i);
        sgd4(xr, vr, gr, lr, mo, wd);
        st4<true>(x + i, xr); st4<true>(v + i, vr);
    }
}
// ---- local step, rows: pointers from the kernel arguments ------------------------------------------
template <bool BY_Y>
__global__ void __launch_bounds__(64) ls_rows(const RowPtrs p, unsigned row4, unsigned blocks_per_row, float lr, float mo, float wd)
{
    unsigned j, q;
    if (BY_Y) { j = blockIdx.y; q = blockIdx.x; }
    else      { j = blockIdx.x / blocks_per_row; q = blockIdx.x - j * blocks_per_row; }
    const unsigned c = q * 64 + threadIdx.x;
    if (c >= row4) return;
    v4f *x = p.x[j], *v = p.v[j];
    const v4f *g = p.g[j];
    v4f xr = ld4<true>(x + c), vr = ld4<true>(v + c);
    const v4f gr = ld4<true>(g + c);
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<true>(x + c, xr); st4<true>(v + c, vr);
}
// ---- local step, records -------------------------------------------------------------------------
template <int CH>
__global__ void __launch_bounds__(64) ls_rec(const SRec *__restrict__ recs, unsigned recs_per_row, float lr, float mo, float wd)
{
    const SRec r = recs[(size_t)blockIdx.y * recs_per_row + (blockIdx.x >> CH)];
    const unsigned c = (blockIdx.x & ((1u << CH) - 1u)) * 64 + threadIdx.x;
    if (c >= r.len4) return;
    v4f xr = ld4<true>(r.x + c), vr = ld4<true>(r.v + c);
    const v4f gr = ld4<true>(r.g + c);
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<true>(r.x + c, xr); st4<true>(r.v + c, vr);
}
// ---- folded step, rows / records, band order through a three-dimensional grid ---------------------
// grid = (8 << LB, W, bands): workgroups are dispatched x fastest, then y, then z, and dealt round-robin
// to the 8 L2 partitions, so a partition sees 2^LB windows of replica 0, the same windows of replica 1,
// ... and the windows' piece of the average stays in its L2.  No division, no dependent load.
__global__ void __launch_bounds__(64) fm_rows(const RowPtrs p, const v4f *__restrict__ A, unsigned row4, float lr, float mo, float wd, float om)
{
    const unsigned q = blockIdx.z * gridDim.x + blockIdx.x, j = blockIdx.y;
    const unsigned c = q * 64 + threadIdx.x;
    if (c >= row4) return;
    v4f *x = p.x[j], *v = p.v[j];
    const v4f *g = p.g[j];
    v4f xr = ld4<true>(x + c), vr = ld4<true>(v + c);
    const v4f gr = ld4<true>(g + c);
    const v4f a = ld4<false>(A + c);
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<true>(v + c, vr);
    st4<true>(x + c, merge4(xr, a, om));
}
template <int CH>
__global__ void __launch_bounds__(64) fm_rec(const SRec *__restrict__ recs, unsigned recs_per_row, unsigned slots, const v4f *__restrict__ A,
                                             float lr, float mo, float wd, float om)
{
    const unsigned q = blockIdx.z * gridDim.x + blockIdx.x;
    if (q >= slots) return;
    const SRec r = recs[(size_t)blockIdx.y * recs_per_row + (q >> CH)];
    const unsigned c = (q & ((1u << CH) - 1u)) * 64 + threadIdx.x;
    if (c >= r.len4) return;
    v4f xr = ld4<true>(r.x + c), vr = ld4<true>(r.v + c);
    const v4f gr = ld4<true>(r.g + c);
    const v4f a = ld4<false>(A + r.a4 + c);
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<true>(r.v + c, vr);
    st4<true>(r.x + c, merge4(xr, a, om));
}
// ---- W-way mean with the rows found through the kernel arguments -----------------------------------
template <int WT, int NW>
__global__ void __launch_bounds__(64 * NW) mean_rows(const RowPtrs p, v4f *__restrict__ A, unsigned row4, float inv_w)
{
    constexpr int R = WT / NW;
    __shared__ v4f part[NW][64];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
    const unsigned c = blockIdx.x * 64 + l;
    if (c < row4) {
        v4f r[R];
#pragma unroll
        for (int j = 0; j < R; ++j) r[j] = ld4<true>(p.x[w * R + j] + c);
        part[w][l] = tree_sum<0, R>(r);
    }
    __syncthreads();
    if (w == 0 && c < row4) {
        v4f q[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) q[k] = part[k][l];
        st4<false>(A + c, tree_sum<0, NW>(q) * inv_w);
    }
}

// ---- the same with every load issued before the first wait ------------------------------------------
// The compiler likes to sink a load below arithmetic on the others (fewer live registers), which puts two
// or three memory latencies in a row; an empty asm that consumes all loaded values keeps them together.
__device__ __forceinline__ void issued(v4f &a, v4f &b, v4f &c, v4f &d) { asm volatile("" : "+v"(a), "+v"(b), "+v"(c), "+v"(d)); }
__device__ __forceinline__ v4f gld(cgv4f *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void gst(gv4f *p, v4f a) { __builtin_nontemporal_store(a, p); }

template <int WT>
__global__ void __launch_bounds__(64) fm_flat_issued(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, const v4f *__restrict__ A,
                                                     unsigned n4, unsigned row4, unsigned log_band, float lr, float mo, float wd, float om)
{
    unsigned i, c;
    if (!decode_block(blockIdx.x, (unsigned)WT, row4, n4, log_band, i, c)) return;
    v4f a = ld4<false>(A + c);
    v4f xr = ld4<true>(x + i), vr = ld4<true>(v + i), gr = ld4<true>(g + i);
    issued(a, xr, vr, gr);
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<true>(v + i, vr);
    st4<true>(x + i, merge4(xr, a, om));
}
__global__ void __launch_bounds__(64) fm_rows_issued(const RowPtrs p, const v4f *__restrict__ A, unsigned row4, float lr, float mo, float wd, float om)
{
    const unsigned q = blockIdx.z * gridDim.x + blockIdx.x, j = blockIdx.y;
    const unsigned c = q * 64 + threadIdx.x;
    if (c >= row4) return;
    gv4f *x = (gv4f *)p.x[j], *v = (gv4f *)p.v[j];
    cgv4f *g = (cgv4f *)p.g[j];
    v4f a = ld4<false>(A + c);
    v4f xr = gld(x + c), vr = gld(v + c), gr = gld(g + c);
    issued(a, xr, vr, gr);
    sgd4(xr, vr, gr, lr, mo, wd);
    gst(v + c, vr);
    gst(x + c, merge4(xr, a, om));
}
template <int CH>
__global__ void __launch_bounds__(64) fm_rec_issued(const SRec *__restrict__ recs, unsigned recs_per_row, unsigned slots, const v4f *__restrict__ A,
                                                    float lr, float mo, float wd, float om)
{
    const unsigned q = blockIdx.z * gridDim.x + blockIdx.x;
    if (q >= slots) return;
    const SRec r = recs[(size_t)blockIdx.y * recs_per_row + (q >> CH)];
    const unsigned c = (q & ((1u << CH) - 1u)) * 64 + threadIdx.x;
    if (c >= r.len4) return;
    gv4f *x = (gv4f *)r.x, *v = (gv4f *)r.v;
    cgv4f *g = (cgv4f *)r.g;
    v4f a = ld4<false>(A + r.a4 + c);
    v4f xr = gld(x + c), vr = gld(v + c), gr = gld(g + c);
    issued(a, xr, vr, gr);
    sgd4(xr, vr, gr, lr, mo, wd);
    gst(v + c, vr);
    gst(x + c, merge4(xr, a, om));
}
template <int CH>
__global__ void __launch_bounds__(64) ls_rec_global(const SRec *__restrict__ recs, unsigned recs_per_row, float lr, float mo, float wd)
{
    const SRec r = recs[(size_t)blockIdx.y * recs_per_row + (blockIdx.x >> CH)];
    const unsigned c = (blockIdx.x & ((1u << CH) - 1u)) * 64 + threadIdx.x;
    if (c >= r.len4) return;
    gv4f *x = (gv4f *)r.x, *v = (gv4f *)r.v;
    cgv4f *g = (cgv4f *)r.g;
    v4f xr = gld(x + c), vr = gld(v + c), gr = gld(g + c);
    sgd4(xr, vr, gr, lr, mo, wd);
    gst(x + c, xr); gst(v + c, vr);
}

// ---- issue order of the loads of one wave -----------------------------------------------------------
__device__ __forceinline__ void arrived(v4f &a, v4f &b) { asm volatile("" : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void arrived(v4f &a, v4f &b, v4f &c) { asm volatile("" : "+v"(a), "+v"(b), "+v"(c)); }
// ORDER 0: x, v, g together;  1: x, then v, then g, each after the previous has arrived;  2: x and v, then g
template <int ORDER>
__global__ void __launch_bounds__(64) ls_flat_order(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, int64_t n4,
                                                    float lr, float mo, float wd)
{
    const int64_t i = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= n4) return;
    v4f xr, vr, gr;
    if (ORDER == 0) { xr = ld4<true>(x + i); vr = ld4<true>(v + i); gr = ld4<true>(g + i); arrived(xr, vr, gr); }
    if (ORDER == 1) { xr = ld4<true>(x + i); arrived(xr); vr = ld4<true>(v + i); arrived(vr); gr = ld4<true>(g + i); arrived(gr); }
    if (ORDER == 2) { xr = ld4<true>(x + i); vr = ld4<true>(v + i); arrived(xr, vr); gr = ld4<true>(g + i); arrived(gr); }
    if (ORDER == 3) { gr = ld4<true>(g + i); arrived(gr); vr = ld4<true>(v + i); arrived(vr); xr = ld4<true>(x + i); arrived(xr); }
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<true>(x + i, xr); st4<true>(v + i, vr);
}
// loads one after the other; which of loads and stores are non-temporal
template <bool LD_NT, bool ST_NT>
__global__ void __launch_bounds__(64) ls_flat_hints(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, int64_t n4,
                                                    float lr, float mo, float wd)
{
    const int64_t i = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (i >= n4) return;
    v4f xr = ld4<LD_NT>(x + i); arrived(xr);
    v4f vr = ld4<LD_NT>(v + i); arrived(vr);
    v4f gr = ld4<LD_NT>(g + i); arrived(gr);
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<ST_NT>(x + i, xr); st4<ST_NT>(v + i, vr);
}
// the same through raw buffer loads and stores (one descriptor per row), whose cache-policy operand can be set
// freely: bit 0 = sc0, bit 1 = nt, bit 4 = sc1 (the non-temporal builtins give nt alone)
typedef unsigned v4u __attribute__((ext_vector_type(4)));
template <int AUX_LD, int AUX_ST>
__global__ void __launch_bounds__(64) ls_buf(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, unsigned ld4,
                                             float lr, float mo, float wd)
{
    const unsigned c = blockIdx.x * 64 + threadIdx.x;
    if (c >= ld4) return;
    const size_t row = (size_t)blockIdx.y * ld4;
    const int bytes = (int)(ld4 * 16u);
    __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)(x + row), 0, bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)(v + row), 0, bytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc((void *)(g + row), 0, bytes, 0x00020000);
    const int off = (int)(c * 16u);
    v4u xu = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, AUX_LD);
    v4f xr = __builtin_bit_cast(v4f, xu); arrived(xr);
    v4u vu = __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, AUX_LD);
    v4f vr = __builtin_bit_cast(v4f, vu); arrived(vr);
    v4u gu = __builtin_amdgcn_raw_buffer_load_b128(rg, off, 0, AUX_LD);
    v4f gr = __builtin_bit_cast(v4f, gu); arrived(gr);
    sgd4(xr, vr, gr, lr, mo, wd);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, xr), rx, off, 0, AUX_ST);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, vr), rv, off, 0, AUX_ST);
}
// two kilobytes per array and wave, the arrays one after the other
template <int THREADS>
__global__ void __launch_bounds__(THREADS) ls_flat_pairs(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, int64_t n4,
                                                         float lr, float mo, float wd)
{
    const int64_t i = (int64_t)blockIdx.x * (2 * THREADS) + threadIdx.x, k = i + THREADS;
    if (k >= n4) return;        // (the study's sizes are whole multiples)
    v4f x0 = ld4<true>(x + i), x1 = ld4<true>(x + k); arrived(x0, x1);
    v4f v0 = ld4<true>(v + i), v1 = ld4<true>(v + k); arrived(v0, v1);
    v4f g0 = ld4<true>(g + i), g1 = ld4<true>(g + k); arrived(g0, g1);
    sgd4(x0, v0, g0, lr, mo, wd); sgd4(x1, v1, g1, lr, mo, wd);
    st4<true>(x + i, x0); st4<true>(x + k, x1); st4<true>(v + i, v0); st4<true>(v + k, v1);
}
template <int THREADS>
__global__ void __launch_bounds__(THREADS) ls_flat_serial_wg(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, int64_t n4,
                                                             float lr, float mo, float wd)
{
    const int64_t i = (int64_t)blockIdx.x * THREADS + threadIdx.x;
    if (i >= n4) return;
    v4f xr = ld4<true>(x + i); arrived(xr);
    v4f vr = ld4<true>(v + i); arrived(vr);
    v4f gr = ld4<true>(g + i); arrived(gr);
    sgd4(xr, vr, gr, lr, mo, wd);
    st4<true>(x + i, xr); st4<true>(v + i, vr);
}
// ORDER 1: x, v, g together, then the average;  2: the average first, then x, v, g;  3: x and v, then g and the average
template <int ORDER>
__global__ void __launch_bounds__(64) fm_rows_order(const RowPtrs p, const v4f *__restrict__ A, unsigned row4, float lr, float mo, float wd, float om)
{
    const unsigned q = blockIdx.z * gridDim.x + blockIdx.x, j = blockIdx.y;
    const unsigned c = q * 64 + threadIdx.x;
    if (c >= row4) return;
    gv4f *x = (gv4f *)p.x[j], *v = (gv4f *)p.v[j];
    cgv4f *g = (cgv4f *)p.g[j];
    v4f a, xr, vr, gr;
    if (ORDER == 1) { xr = gld(x + c); vr = gld(v + c); gr = gld(g + c); arrived(xr, vr, gr); a = ld4<false>(A + c); arrived(a); }
    if (ORDER == 2) { a = ld4<false>(A + c); arrived(a); xr = gld(x + c); vr = gld(v + c); gr = gld(g + c); arrived(xr, vr, gr); }
    if (ORDER == 3) { xr = gld(x + c); vr = gld(v + c); arrived(xr, vr); gr = gld(g + c); a = ld4<false>(A + c); arrived(gr, a); }
    if (ORDER == 4) { xr = gld(x + c); arrived(xr); vr = gld(v + c); arrived(vr); gr = gld(g + c); arrived(gr); a = ld4<false>(A + c); arrived(a); }
    if (ORDER == 5) { a = ld4<false>(A + c); arrived(a); xr = gld(x + c); arrived(xr); vr = gld(v + c); arrived(vr); gr = gld(g + c); arrived(gr); }
    if (ORDER == 6) { xr = gld(x + c); arrived(xr); vr = gld(v + c); arrived(vr); gr = gld(g + c); a = ld4<false>(A + c); arrived(gr, a); }
    sgd4(xr, vr, gr, lr, mo, wd);
    gst(v + c, vr);
    gst(x + c, merge4(xr, a, om));
}

// W-way mean, rows over NW wavefronts, each wave's loads one after the other
template <int WT, int NW>
__global__ void __launch_bounds__(64 * NW) mean_rows_serial(const RowPtrs p, v4f *__restrict__ A, unsigned row4, float inv_w)
{
    constexpr int R = WT / NW;
    __shared__ v4f part[NW][64];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
    const unsigned c = blockIdx.x * 64 + l;
    if (c < row4) {
        v4f r[R];
#pragma unroll
        for (int j = 0; j < R; ++j) { r[j] = ld4<true>(p.x[w * R + j] + c); arrived(r[j]); }
        part[w][l] = tree_sum<0, R>(r);
    }
    __syncthreads();
    if (w == 0 && c < row4) {
        v4f q[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) q[k] = part[k][l];
        st4<false>(A + c, tree_sum<0, NW>(q) * inv_w);
    }
}
// the merged-in average undone on the mean: in double precision as the library does it, and in single
// precision on differences to the first row (mean x' = x'_0 + mean (x'_j - x'_0)), the merge undone with one fma
template <int WT, int NW, bool F64>
__global__ void __launch_bounds__(64 * NW) mean_undo(const RowPtrs p, const v4f *__restrict__ A_old, v4f *__restrict__ A_new, unsigned row4,
                                                     float inv_w, float om, float inv_xi)
{
    constexpr int R = WT / NW;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
    const unsigned c = blockIdx.x * 64 + l;
    if constexpr (F64) {
        typedef double v4d __attribute__((ext_vector_type(4)));
        __shared__ v4d part[NW][64];
        v4d acc = {0, 0, 0, 0};
        if (c < row4)
            for (int j = 0; j < R; ++j) acc += __builtin_convertvector(ld4<true>(p.x[w * R + j] + c), v4d);
        part[w][l] = acc;
        __syncthreads();
        if (w == 0 && c < row4) {
            v4d m = part[0][l];
#pragma unroll
            for (int k = 1; k < NW; ++k) m += part[k][l];
            const v4d a = __builtin_convertvector(ld4<false>(A_old + c), v4d);
            st4<false>(A_new + c, __builtin_convertvector((m * (double)inv_w - (double)om * a) * (double)inv_xi, v4f));
        }
    } else {
        __shared__ v4f first[NW][64], dsum[NW][64];
        if (c < row4) {
            const v4f r0 = ld4<true>(p.x[w * R] + c);
            v4f d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 1; j < R; ++j) d += ld4<true>(p.x[w * R + j] + c) - r0;
            first[w][l] = r0; dsum[w][l] = d;
        }
        __syncthreads();
        if (w == 0 && c < row4) {
            const v4f r0 = first[0][l];
            v4f d = dsum[0][l];
#pragma unroll
            for (int k = 1; k < NW; ++k) d += dsum[k][l] + (float)R * (first[k][l] - r0);
            const v4f a = ld4<false>(A_old + c);
            v4f t;
            t.x = fmaf(-om, a.x, r0.x); t.y = fmaf(-om, a.y, r0.y); t.z = fmaf(-om, a.z, r0.z); t.w = fmaf(-om, a.w, r0.w);
            st4<false>(A_new + c, (t + d * inv_w) * inv_xi);
        }
    }
}

// ---- local step, mean and merge in one pass (fusion level 3): who walks the W rows of a column window --------
// one wave walks all W rows of its 64-column window, row after row (TOGETHER: the three loads of a row at once)
template <int WT, bool TOGETHER>
__global__ void __launch_bounds__(64) all_walk(const RowPtrs p, const v4f *__restrict__ A_old, v4f *__restrict__ A_new, unsigned row4,
                                               float lr, float mo, float wd, float om, float inv_w)
{
    const unsigned c = blockIdx.x * 64 + threadIdx.x;
    if (c >= row4) return;
    v4f a = ld4<false>(A_old + c); arrived(a);
    v4f y[WT];
#pragma unroll
    for (int j = 0; j < WT; ++j) {
        v4f xr, vr, gr;
        if (TOGETHER) { xr = ld4<true>(p.x[j] + c); vr = ld4<true>(p.v[j] + c); gr = ld4<true>(p.g[j] + c); arrived(xr, vr, gr); }
        else { xr = ld4<true>(p.x[j] + c); arrived(xr); vr = ld4<true>(p.v[j] + c); arrived(vr); gr = ld4<true>(p.g[j] + c); arrived(gr); }
        sgd4(xr, vr, gr, lr, mo, wd);
        st4<true>(p.v[j] + c, vr);
        st4<true>(p.x[j] + c, merge4(xr, a, om));
        y[j] = xr;
    }
    st4<false>(A_new + c, tree_sum<0, WT>(y) * inv_w);
}
// NW waves per workgroup, each walks WT / NW rows; partial sums through LDS
template <int WT, int NW>
__global__ void __launch_bounds__(64 * NW) all_groups(const RowPtrs p, const v4f *__restrict__ A_old, v4f *__restrict__ A_new, unsigned row4,
                                                      float lr, float mo, float wd, float om, float inv_w)
{
    constexpr int R = WT / NW;
    __shared__ v4f part[NW][64];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
    const unsigned c = blockIdx.x * 64 + l;
    if (c < row4) {
        v4f a = ld4<false>(A_old + c); arrived(a);
        v4f y[R];
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int j = w * R + k;
            v4f xr = ld4<true>(p.x[j] + c); arrived(xr);
            v4f vr = ld4<true>(p.v[j] + c); arrived(vr);
            v4f gr = ld4<true>(p.g[j] + c); arrived(gr);
            sgd4(xr, vr, gr, lr, mo, wd);
            st4<true>(p.v[j] + c, vr);
            st4<true>(p.x[j] + c, merge4(xr, a, om));
            y[k] = xr;
        }
        part[w][l] = tree_sum<0, R>(y);
    }
    __syncthreads();
    if (w == 0 && c < row4) {
        v4f q[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) q[k] = part[k][l];
        st4<false>(A_new + c, tree_sum<0, NW>(q) * inv_w);
    }
}

// W waves per workgroup, one row each, y through LDS -- but no barrier behind the loads: every wave announces
// itself on an LDS counter and leaves; the last to arrive adds the W values and stores the average
template <int WT>
__global__ void __launch_bounds__(64 * WT) all_last_arriver(const RowPtrs p, const v4f *__restrict__ A_old, v4f *__restrict__ A_new, unsigned row4,
                                                           float lr, float mo, float wd, float om, float inv_w)
{
    __shared__ v4f part[WT][64];
    __shared__ unsigned count;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63;
    if (threadIdx.x == 0) count = 0;
    __syncthreads();                                   // before any memory latency: costs next to nothing
    const unsigned c = blockIdx.x * 64 + l;
    if (c < row4) {
        v4f a = ld4<false>(A_old + c); arrived(a);
        v4f xr = ld4<true>(p.x[w] + c); arrived(xr);
        v4f vr = ld4<true>(p.v[w] + c); arrived(vr);
        v4f gr = ld4<true>(p.g[w] + c); arrived(gr);
        sgd4(xr, vr, gr, lr, mo, wd);
        st4<true>(p.v[w] + c, vr);
        st4<true>(p.x[w] + c, merge4(xr, a, om));
        part[w][l] = xr;
    }
    __threadfence_block();
    unsigned before = 0;
    if (l == 0) before = atomicAdd(&count, 1u);
    before = __builtin_amdgcn_readfirstlane(before);
    if (before != WT - 1) return;
    __threadfence_block();
    if (c < row4) {
        v4f q[WT];
#pragma unroll
        for (int k = 0; k < WT; ++k) q[k] = part[k][l];
        st4<false>(A_new + c, tree_sum<0, WT>(q) * inv_w);
    }
}
// one wave, the W rows on W groups of 64/W lanes (a window is 64/W columns wide), sums by cross-lane exchange
template <int WT>
__global__ void __launch_bounds__(64) all_lanes(const RowPtrs p, const v4f *__restrict__ A_old, v4f *__restrict__ A_new, unsigned row4,
                                                float lr, float mo, float wd, float om, float inv_w)
{
    constexpr int G = 64 / WT;
    const int r = threadIdx.x / G;
    const unsigned c = blockIdx.x * G + threadIdx.x % G;
    const bool in = c < row4;
    v4f y = {0.f, 0.f, 0.f, 0.f};
    if (in) {
        v4f a = ld4<false>(A_old + c); arrived(a);
        v4f xr = ld4<true>(p.x[r] + c); arrived(xr);
        v4f vr = ld4<true>(p.v[r] + c); arrived(vr);
        v4f gr = ld4<true>(p.g[r] + c); arrived(gr);
        sgd4(xr, vr, gr, lr, mo, wd);
        st4<true>(p.v[r] + c, vr);
        st4<true>(p.x[r] + c, merge4(xr, a, om));
        y = xr;
    }
#pragma unroll
    for (int off = G; off < 64; off <<= 1) {
        v4f o;
        o.x = __shfl_xor(y.x, off); o.y = __shfl_xor(y.y, off); o.z = __shfl_xor(y.z, off); o.w = __shfl_xor(y.w, off);
        y = y + o;
    }
    if (in && r == 0) st4<false>(A_new + c, y * inv_w);
}

__global__ void k_fill(float *p, size_t n, unsigned seed, float scale)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    unsigned h = (unsigned)i * 2654435761u ^ seed;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
    p[i] = ((int)(h & 0xffffff) - 0x800000) * (scale / 8388608.0f);
}
static void fill(void *p, size_t n, unsigned seed, float scale)
{
    hipLaunchKernelGGL(k_fill, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, 0, (float *)p, n, seed, scale);
}

static std::vector<int64_t> resnet50_shapes()
{
    std::vector<int64_t> s;
    auto bn = [&](int64_t c) { s.push_back(c); s.push_back(c); };
    s.push_back(64 * 3 * 7 * 7); bn(64);
    int64_t in = 64;
    const int blocks[4] = {3, 4, 6, 3}, width[4] = {64, 128, 256, 512};
    for (int st = 0; st < 4; ++st)
        for (int b = 0; b < blocks[st]; ++b) {
            const int64_t w = width[st];
            s.push_back(w * in); bn(w);
            s.push_back(w * w * 9); bn(w);
            s.push_back(4 * w * w); bn(4 * w);
            if (b == 0) { s.push_back(4 * w * in); bn(4 * w); }
            in = 4 * w;
        }
    s.push_back(1000 * 2048); s.push_back(1000);
    return s;
}
static std::vector<int64_t> bert_large_shapes()
{
    std::vector<int64_t> s;
    const int64_t H = 1024, F = 4096;
    s.push_back(30522 * H); s.push_back(512 * H); s.push_back(2 * H); s.push_back(H); s.push_back(H);
    for (int l = 0; l < 24; ++l) {
        for (int k = 0; k < 4; ++k) { s.push_back(H * H); s.push_back(H); }
        s.push_back(H); s.push_back(H);
        s.push_back(F * H); s.push_back(F);
        s.push_back(H * F); s.push_back(H);
        s.push_back(H); s.push_back(H);
    }
    s.push_back(H * H); s.push_back(H);
    return s;
}

int main(int argc, char **argv)
{
    const std::string set = argc > 1 ? argv[1] : "resnet";
    const std::vector<int64_t> numel = set == "bert" ? bert_large_shapes() : resnet50_shapes();
    const int W = argc > 2 ? atoi(argv[2]) : (set == "bert" ? 4 : 8);
    if (W != 4 && W != 8 && W != 16) { printf("W must be 4, 8 or 16\n"); return 1; }
    int64_t P = 0;
    for (int64_t n : numel) { if (n % 4) { printf("sizes must be multiples of 4\n"); return 1; } P += n; }
    const int nt = (int)numel.size();
    const int64_t ld = (P + 255) / 256 * 256;
    const unsigned row4 = (unsigned)(ld / 4);
    const int64_t n4 = (int64_t)W * row4;
    printf("set %s: %d tensors, P = %lld, W = %d, row stride %lld floats; weight-like random data\n", set.c_str(), nt, (long long)P, W, (long long)ld);
    const float lr = 0.1f, mo = 0.9f, wd = 1e-4f, om = 0.75f;
    const double RP = (double)W * (double)P;

    // flat matrices
    v4f *fx, *fv, *fg, *A, *A2;
    CK(hipMalloc(&fx, n4 * 16)); CK(hipMalloc(&fv, n4 * 16)); CK(hipMalloc(&fg, n4 * 16));
    CK(hipMalloc(&A, ld * 4)); CK(hipMalloc(&A2, ld * 4));
    fill(fx, n4 * 4, 1u, 0.05f); fill(fv, n4 * 4, 2u, 0.01f); fill(fg, n4 * 4, 3u, 0.001f); fill(A, ld, 4u, 0.05f);
    // one allocation per replica
    RowPtrs rows;
    memset(&rows, 0, sizeof rows);
    for (int j = 0; j < W; ++j) {
        CK(hipMalloc(&rows.x[j], ld * 4)); CK(hipMalloc(&rows.v[j], ld * 4)); CK(hipMalloc((void **)&rows.g[j], ld * 4));
        fill(rows.x[j], ld, 10u + j, 0.05f); fill(rows.v[j], ld, 30u + j, 0.01f); fill((void *)rows.g[j], ld, 50u + j, 0.001f);
    }
    // one allocation per tensor, and the library's tables for them
    std::vector<float *> tx((size_t)W * nt), tv((size_t)W * nt), tg((size_t)W * nt);
    for (int j = 0; j < W; ++j)
        for (int t = 0; t < nt; ++t) {
            const size_t r = (size_t)j * nt + t;
            CK(hipMalloc(&tx[r], numel[t] * 4)); CK(hipMalloc(&tv[r], numel[t] * 4)); CK(hipMalloc(&tg[r], numel[t] * 4));
            fill(tx[r], numel[t], 100u + r, 0.05f); fill(tv[r], numel[t], 7000u + r, 0.01f); fill(tg[r], numel[t], 15000u + r, 0.001f);
        }
    CK(hipDeviceSynchronize());
    auto make_recs = [&](int CH, unsigned *recs_per_row, bool from_rows = false) {
        const int64_t piece = 256ll << CH;                  // floats per record
        std::vector<SRec> h;
        unsigned per_row = 0;
        for (int j = 0; j < W; ++j) {
            int64_t apos = 0;
            unsigned n = 0;
            for (int t = 0; t < nt; ++t) {
                for (int64_t off = 0; off < numel[t]; off += piece) {
                    const size_t r = (size_t)j * nt + t;
                    SRec rec;
                    if (from_rows) {
                        rec.x = rows.x[j] + (apos + off) / 4; rec.v = rows.v[j] + (apos + off) / 4; rec.g = rows.g[j] + (apos + off) / 4;
                    } else {
                        rec.x = reinterpret_cast<v4f *>(tx[r] + off); rec.v = reinterpret_cast<v4f *>(tv[r] + off);
                        rec.g = reinterpret_cast<const v4f *>(tg[r] + off);
                    }
                    rec.a4 = (unsigned)((apos + off) / 4);
                    rec.len4 = (unsigned)(((numel[t] - off) < piece ? (numel[t] - off) : piece) / 4);
                    h.push_back(rec);
                    ++n;
                }
                apos += numel[t];
            }
            per_row = n;
        }
        *recs_per_row = per_row;
        SRec *d;
        CK(hipMalloc(&d, h.size() * sizeof(SRec)));
        CK(hipMemcpy(d, h.data(), h.size() * sizeof(SRec), hipMemcpyHostToDevice));
        return d;
    };
    unsigned rpr4, rpr6, rpr8;
    SRec *rec4 = make_recs(4, &rpr4), *rec6 = make_recs(6, &rpr6), *rec8 = make_recs(8, &rpr8);
    unsigned rpr4r;
    SRec *rec4r = make_recs(4, &rpr4r, true);          // the same records over the per-replica arenas
    RowPtrs into_flat;                                 // row pointers into the flat matrices
    memset(&into_flat, 0, sizeof into_flat);
    for (int j = 0; j < W; ++j) { into_flat.x[j] = fx + (size_t)j * row4; into_flat.v[j] = fv + (size_t)j * row4; into_flat.g[j] = fg + (size_t)j * row4; }
    // the library's chunk and pointer tables
    std::vector<Chunk> chunks;
    {
        int64_t f = 0;
        for (int t = 0; t < nt; ++t) {
            for (int64_t off = 0; off < numel[t]; off += kChunk) {
                Chunk c; c.off = off; c.foff = f + off; c.tensor = t;
                c.len = (int32_t)((numel[t] - off) < kChunk ? (numel[t] - off) : kChunk);
                chunks.push_back(c);
            }
            f += numel[t];
        }
    }
    Chunk *d_chunks; float **d_xp, **d_vp; const float **d_gp;
    CK(hipMalloc(&d_chunks, chunks.size() * sizeof(Chunk))); CK(hipMemcpy(d_chunks, chunks.data(), chunks.size() * sizeof(Chunk), hipMemcpyHostToDevice));
    CK(hipMalloc(&d_xp, tx.size() * 8)); CK(hipMemcpy(d_xp, tx.data(), tx.size() * 8, hipMemcpyHostToDevice));
    CK(hipMalloc(&d_vp, tv.size() * 8)); CK(hipMemcpy(d_vp, tv.data(), tv.size() * 8, hipMemcpyHostToDevice));
    CK(hipMalloc(&d_gp, tg.size() * 8)); CK(hipMemcpy(d_gp, tg.data(), tg.size() * 8, hipMemcpyHostToDevice));
    const int n_chunks = (int)chunks.size();

    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    auto run = [&](const char *name, double bytes_per_rp, auto launch) {
        const int it = 10;
        float total = 0.f;
        for (int k = 0; k < it + 2; ++k) {
            CK(hipEventRecord(e0, 0));
            launch();
            CK(hipEventRecord(e1, 0));
            CK(hipEventSynchronize(e1));
            CK(hipGetLastError());
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            if (k >= 2) total += ms;
        }
        const double us = total / it * 1e3, tbs = bytes_per_rp * RP / (us * 1e-6) / 1e12;
        printf("%-66s %8.1f us  %5.2f TB/s  %.3f of 8 TB/s\n", name, us, tbs, tbs / 8.0);
        fflush(stdout);
    };
    const unsigned bpr = (row4 + 63) / 64;
    const double B_LS = 20.0, B_FM = 20.0 + 4.0 / W, B_MEAN = 4.0 + 4.0 / W;

    for (int rep = 0; rep < 2; ++rep) {
        printf("-- pass %d: local step (20 B per replica-parameter)\n", rep + 1);
        run("flat, 64 threads x 1, non-temporal", B_LS, [&] { hipLaunchKernelGGL((ls_flat<64, 1, true>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 threads x 1, plain loads and stores", B_LS, [&] { hipLaunchKernelGGL((ls_flat<64, 1, false>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 256 threads x 1, non-temporal", B_LS, [&] { hipLaunchKernelGGL((ls_flat<256, 1, true>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 256 threads x 4 unrolled, non-temporal", B_LS, [&] { hipLaunchKernelGGL((ls_flat<256, 4, true>), dim3((unsigned)((n4 + 1023) / 1024)), dim3(256), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 threads x 4 unrolled, non-temporal", B_LS, [&] { hipLaunchKernelGGL((ls_flat<64, 4, true>), dim3((unsigned)((n4 + 255) / 256)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, persistent grid-stride (2048 x 256), non-temporal", B_LS, [&] { hipLaunchKernelGGL(ls_flat_persistent, dim3(2048), dim3(256), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 x 1, loads: x v g together (forced)", B_LS, [&] { hipLaunchKernelGGL((ls_flat_order<0>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 x 1, loads: x, then v, then g", B_LS, [&] { hipLaunchKernelGGL((ls_flat_order<1>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 x 1, loads: x and v, then g", B_LS, [&] { hipLaunchKernelGGL((ls_flat_order<2>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 x 1, loads: g, then v, then x", B_LS, [&] { hipLaunchKernelGGL((ls_flat_order<3>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 x 1, loads one after the other, non-temporal loads, plain stores", B_LS, [&] { hipLaunchKernelGGL((ls_flat_hints<true, false>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 x 1, loads one after the other, plain loads, non-temporal stores", B_LS, [&] { hipLaunchKernelGGL((ls_flat_hints<false, true>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 64 x 1, loads one after the other, plain loads and stores", B_LS, [&] { hipLaunchKernelGGL((ls_flat_hints<false, false>), dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
#define LS_BUF(LD, ST, what) run("flat rows, raw buffer accesses, " what, B_LS, [&] { \
            hipLaunchKernelGGL((ls_buf<LD, ST>), dim3((unsigned)((ld / 4 + 63) / 64), (unsigned)W), dim3(64), 0, 0, fx, fv, fg, (unsigned)(ld / 4), lr, mo, wd); })
        LS_BUF(2, 2, "loads nt, stores nt");
        LS_BUF(2, 3, "loads nt, stores sc0 nt");
        LS_BUF(2, 18, "loads nt, stores sc1 nt");
        LS_BUF(2, 19, "loads nt, stores sc0 sc1 nt");
        LS_BUF(2, 17, "loads nt, stores sc0 sc1");
        LS_BUF(3, 2, "loads sc0 nt, stores nt");
        LS_BUF(18, 2, "loads sc1 nt, stores nt");
        LS_BUF(19, 2, "loads sc0 sc1 nt, stores nt");
        LS_BUF(19, 19, "loads sc0 sc1 nt, stores sc0 sc1 nt");
        LS_BUF(0, 0, "plain");
#undef LS_BUF
        run("flat, 64 x 2: x x, then v v, then g g", B_LS, [&] { hipLaunchKernelGGL((ls_flat_pairs<64>), dim3((unsigned)(n4 / 128)), dim3(64), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 128 x 1, loads: x, then v, then g", B_LS, [&] { hipLaunchKernelGGL((ls_flat_serial_wg<128>), dim3((unsigned)((n4 + 127) / 128)), dim3(128), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("flat, 256 x 1, loads: x, then v, then g", B_LS, [&] { hipLaunchKernelGGL((ls_flat_serial_wg<256>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, 0, fx, fv, fg, n4, lr, mo, wd); });
        run("rows, pointer by blockIdx.y", B_LS, [&] { hipLaunchKernelGGL((ls_rows<true>), dim3(bpr, W), dim3(64), 0, 0, rows, row4, bpr, lr, mo, wd); });
        run("rows, pointer by blockIdx.x / blocks_per_row", B_LS, [&] { hipLaunchKernelGGL((ls_rows<false>), dim3(bpr * W), dim3(64), 0, 0, rows, row4, bpr, lr, mo, wd); });
        run("records of 16 blocks (4096 floats)", B_LS, [&] { hipLaunchKernelGGL((ls_rec<4>), dim3(rpr4 << 4, W), dim3(64), 0, 0, rec4, rpr4, lr, mo, wd); });
        run("records of 64 blocks (16384 floats)", B_LS, [&] { hipLaunchKernelGGL((ls_rec<6>), dim3(rpr6 << 6, W), dim3(64), 0, 0, rec6, rpr6, lr, mo, wd); });
        run("records of 256 blocks (65536 floats)", B_LS, [&] { hipLaunchKernelGGL((ls_rec<8>), dim3(rpr8 << 8, W), dim3(64), 0, 0, rec8, rpr8, lr, mo, wd); });
        run("records of 16 blocks, global loads", B_LS, [&] { hipLaunchKernelGGL((ls_rec_global<4>), dim3(rpr4 << 4, W), dim3(64), 0, 0, rec4, rpr4, lr, mo, wd); });
        run("records of 16 blocks over the per-replica arenas, global loads", B_LS, [&] { hipLaunchKernelGGL((ls_rec_global<4>), dim3(rpr4r << 4, W), dim3(64), 0, 0, rec4r, rpr4r, lr, mo, wd); });
        run("rows into the flat matrices, pointer by blockIdx.y", B_LS, [&] { hipLaunchKernelGGL((ls_rows<true>), dim3(bpr, W), dim3(64), 0, 0, into_flat, row4, bpr, lr, mo, wd); });
        run("previous chunk table (256 x 4, chunk -> tensor -> pointer)", B_LS, [&] {
            hipLaunchKernelGGL((k_local_step<kStoreX, false>), dim3((unsigned)n_chunks, (unsigned)W), dim3(kThreads), 0, 0, d_chunks, d_xp, d_vp, d_gp,
                               (float *)nullptr, ld, nt, lr, mo, wd, (const float *)nullptr, om, W, n_chunks, 0); });

        printf("-- pass %d: local step with the merge folded in (20 + 4/W B per replica-parameter)\n", rep + 1);
        for (unsigned lb : {0u, 8u, 9u, 10u, 11u}) {
            const unsigned l = decode_clamp_log_band(row4, lb);
            char nm[96];
            snprintf(nm, sizeof nm, "flat, computed block order (previous kernel), band 2^%u", l);
            const unsigned grid = (unsigned)decode_grid((unsigned)W, row4, l);
            run(nm, B_FM, [&] {
                switch (W) {
                case 4:  hipLaunchKernelGGL((k_step_merge_flat<false, 4>), dim3(grid), dim3(64), 0, 0, fx, fv, fg, (v4f *)nullptr, A, (unsigned)n4, row4, W, l, lr, mo, wd, om); break;
                case 8:  hipLaunchKernelGGL((k_step_merge_flat<false, 8>), dim3(grid), dim3(64), 0, 0, fx, fv, fg, (v4f *)nullptr, A, (unsigned)n4, row4, W, l, lr, mo, wd, om); break;
                default: hipLaunchKernelGGL((k_step_merge_flat<false, 16>), dim3(grid), dim3(64), 0, 0, fx, fv, fg, (v4f *)nullptr, A, (unsigned)n4, row4, W, l, lr, mo, wd, om); break;
                } });
        }
        for (unsigned lb : {5u, 8u, 9u, 10u, 11u}) {
            const unsigned gx = 8u << lb, bands = (bpr + gx - 1) / gx;
            if (bands > 65535u) continue;
            char nm[96];
            snprintf(nm, sizeof nm, "rows, 3-d grid, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL(fm_rows, dim3(gx, W, bands), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
        }
        for (unsigned lb : {0u, 9u, 10u}) {
            const unsigned l = decode_clamp_log_band(row4, lb);
            char nm[96];
            snprintf(nm, sizeof nm, "flat, loads issued together, band 2^%u", l);
            const unsigned grid = (unsigned)decode_grid((unsigned)W, row4, l);
            run(nm, B_FM, [&] {
                switch (W) {
                case 4:  hipLaunchKernelGGL((fm_flat_issued<4>), dim3(grid), dim3(64), 0, 0, fx, fv, fg, A, (unsigned)n4, row4, l, lr, mo, wd, om); break;
                case 8:  hipLaunchKernelGGL((fm_flat_issued<8>), dim3(grid), dim3(64), 0, 0, fx, fv, fg, A, (unsigned)n4, row4, l, lr, mo, wd, om); break;
                default: hipLaunchKernelGGL((fm_flat_issued<16>), dim3(grid), dim3(64), 0, 0, fx, fv, fg, A, (unsigned)n4, row4, l, lr, mo, wd, om); break;
                } });
        }
        for (unsigned lb : {5u, 8u, 9u, 10u, 11u}) {
            const unsigned gx = 8u << lb, bands = (bpr + gx - 1) / gx;
            if (bands > 65535u) continue;
            char nm[96];
            snprintf(nm, sizeof nm, "rows, loads issued together, 3-d grid, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL(fm_rows_issued, dim3(gx, W, bands), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into the flat matrices, issued together, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL(fm_rows_issued, dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
        }
        for (unsigned lb : {9u, 10u}) {
            const unsigned gx = 8u << lb, bands = (bpr + gx - 1) / gx;
            if (bands > 65535u) continue;
            char nm[112];
            snprintf(nm, sizeof nm, "rows, x v g then the average, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<1>), dim3(gx, W, bands), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into flat, x v g then the average, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<1>), dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows, the average then x v g, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<2>), dim3(gx, W, bands), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into flat, the average then x v g, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<2>), dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows, x v then g and the average, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<3>), dim3(gx, W, bands), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into flat, x v then g and the average, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<3>), dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into flat, x, v, g, average one after the other, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<4>), dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows, x, v, g, average one after the other, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<4>), dim3(gx, W, bands), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into flat, average, x, v, g one after the other, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<5>), dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into flat, x, then v, then g with the average, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rows_order<6>), dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "rows into flat, compiler's order, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL(fm_rows, dim3(gx, W, bands), dim3(64), 0, 0, into_flat, A, row4, lr, mo, wd, om); });
        }
        run("rows, loads issued together, replica after replica", B_FM, [&] { hipLaunchKernelGGL(fm_rows_issued, dim3(bpr, W, 1), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
        for (unsigned lb : {8u, 9u, 10u, 11u}) {
            const unsigned gx = 8u << lb, slots = rpr4 << 4, bands = (slots + gx - 1) / gx;
            if (bands > 65535u) continue;
            char nm[96];
            snprintf(nm, sizeof nm, "records of 16 blocks, issued together, global, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rec_issued<4>), dim3(gx, W, bands), dim3(64), 0, 0, rec4, rpr4, slots, A, lr, mo, wd, om); });
            snprintf(nm, sizeof nm, "records over the per-replica arenas, issued together, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rec_issued<4>), dim3(gx, W, bands), dim3(64), 0, 0, rec4r, rpr4r, rpr4r << 4, A, lr, mo, wd, om); });
        }
        run("rows, replica after replica (grid x = blocks, y = W)", B_FM, [&] { hipLaunchKernelGGL(fm_rows, dim3(bpr, W, 1), dim3(64), 0, 0, rows, A, row4, lr, mo, wd, om); });
        for (unsigned lb : {8u, 9u, 10u, 11u}) {
            const unsigned gx = 8u << lb, slots = rpr4 << 4, bands = (slots + gx - 1) / gx;
            if (bands > 65535u) continue;
            char nm[96];
            snprintf(nm, sizeof nm, "records of 16 blocks, 3-d grid, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rec<4>), dim3(gx, W, bands), dim3(64), 0, 0, rec4, rpr4, slots, A, lr, mo, wd, om); });
        }
        for (unsigned lb : {9u, 10u}) {
            const unsigned gx = 8u << lb, slots = rpr6 << 6, bands = (slots + gx - 1) / gx;
            if (bands > 65535u) continue;
            char nm[96];
            snprintf(nm, sizeof nm, "records of 64 blocks, 3-d grid, band 2^%u", lb);
            run(nm, B_FM, [&] { hipLaunchKernelGGL((fm_rec<6>), dim3(gx, W, bands), dim3(64), 0, 0, rec6, rpr6, slots, A, lr, mo, wd, om); });
        }
        run("records of 16 blocks, replica after replica", B_FM, [&] { hipLaunchKernelGGL((fm_rec<4>), dim3(rpr4 << 4, W, 1), dim3(64), 0, 0, rec4, rpr4, rpr4 << 4, A, lr, mo, wd, om); });
        for (int xo : {0, 1}) {
            char nm[96];
            snprintf(nm, sizeof nm, "previous chunk table (256 x 4), %s", xo ? "replicas of a chunk on one L2 partition" : "replica after replica");
            const dim3 grid = xo ? dim3((unsigned)((n_chunks + 7) / 8 * 8 * W)) : dim3((unsigned)n_chunks, (unsigned)W);
            run(nm, B_FM, [&] {
                hipLaunchKernelGGL((k_local_step<kStoreX, true>), grid, dim3(kThreads), 0, 0, d_chunks, d_xp, d_vp, d_gp, (float *)nullptr, ld, nt,
                                   lr, mo, wd, (const float *)A, om, W, n_chunks, xo); });
        }


        printf("-- pass %d: local step, mean and merge in one pass (20 + 8/W B per replica-parameter), rows into flat\n", rep + 1);
        {
            const double B_ALL = 20.0 + 8.0 / W;
            RowSet ax = {}, av = {}; ConstRowSet ag = {};
            for (int j = 0; j < W; ++j) { ax.p[j] = (float *)into_flat.x[j]; av.p[j] = (float *)into_flat.v[j]; ag.p[j] = (const float *)into_flat.g[j]; }
#define ALL_VARIANTS(WT)                                                                                                                          \
            run("library kernel: W waves per workgroup, one row each, LDS", B_ALL, [&] { hipLaunchKernelGGL((k_step_all_rows<WT, true>), dim3(bpr), dim3(64 * WT), 0, 0, ax, av, ag, A, A2, row4, lr, mo, wd, om, 1.0f / W); }); \
            run("one wave walks the W rows, a row's loads one after the other", B_ALL, [&] { hipLaunchKernelGGL((all_walk<WT, false>), dim3(bpr), dim3(64), 0, 0, into_flat, A, A2, row4, lr, mo, wd, om, 1.0f / W); }); \
            run("one wave walks the W rows, a row's loads together", B_ALL, [&] { hipLaunchKernelGGL((all_walk<WT, true>), dim3(bpr), dim3(64), 0, 0, into_flat, A, A2, row4, lr, mo, wd, om, 1.0f / W); }); \
            run("2 waves per workgroup, W/2 rows each, LDS", B_ALL, [&] { hipLaunchKernelGGL((all_groups<WT, 2>), dim3(bpr), dim3(128), 0, 0, into_flat, A, A2, row4, lr, mo, wd, om, 1.0f / W); }); \
            run("4 waves per workgroup, W/4 rows each, LDS", B_ALL, [&] { hipLaunchKernelGGL((all_groups<WT, 4>), dim3(bpr), dim3(256), 0, 0, into_flat, A, A2, row4, lr, mo, wd, om, 1.0f / W); }); \
            run("W waves per workgroup, LDS, the last wave to arrive sums (no barrier behind the loads)", B_ALL, [&] { hipLaunchKernelGGL((all_last_arriver<WT>), dim3(bpr), dim3(64 * WT), 0, 0, into_flat, A, A2, row4, lr, mo, wd, om, 1.0f / W); }); \
            run("one wave, the W rows on W lane groups, cross-lane sums", B_ALL, [&] { hipLaunchKernelGGL((all_lanes<WT>), dim3((row4 + 64 / WT - 1) / (64 / WT)), dim3(64), 0, 0, into_flat, A, A2, row4, lr, mo, wd, om, 1.0f / W); });
            switch (W) { case 4: { ALL_VARIANTS(4) } break; case 8: { ALL_VARIANTS(8) } break; default: { ALL_VARIANTS(16) } break; }
#undef ALL_VARIANTS
        }
        printf("-- pass %d: W-way mean (4 + 4/W B per replica-parameter)\n", rep + 1);
        run("flat (rows over wavefronts, LDS)", B_MEAN, [&] {
            const unsigned grid = (bpr + 63) / 64 * 64;
            switch (W) {
            case 4:  hipLaunchKernelGGL((k_mean_lds<4, 4, false>), dim3(grid), dim3(256), 0, 0, fx, A2, (int64_t)row4, (int64_t)row4, 1.0f / W); break;
            case 8:  hipLaunchKernelGGL((k_mean_lds<8, 4, false>), dim3(grid), dim3(256), 0, 0, fx, A2, (int64_t)row4, (int64_t)row4, 1.0f / W); break;
            default: hipLaunchKernelGGL((k_mean_lds<16, 8, false>), dim3(grid), dim3(512), 0, 0, fx, A2, (int64_t)row4, (int64_t)row4, 1.0f / W); break;
            } });
        run("rows into flat, each wave's loads one after the other", B_MEAN, [&] {
            switch (W) {
            case 4:  hipLaunchKernelGGL((mean_rows_serial<4, 2>), dim3(bpr), dim3(128), 0, 0, into_flat, A2, row4, 1.0f / W); break;
            case 8:  hipLaunchKernelGGL((mean_rows_serial<8, 4>), dim3(bpr), dim3(256), 0, 0, into_flat, A2, row4, 1.0f / W); break;
            default: hipLaunchKernelGGL((mean_rows_serial<16, 8>), dim3(bpr), dim3(512), 0, 0, into_flat, A2, row4, 1.0f / W); break;
            } });
        run("rows into flat, merge undone in double precision", 4.0 + 8.0 / W, [&] {
            switch (W) {
            case 4:  hipLaunchKernelGGL((mean_undo<4, 4, true>), dim3(bpr), dim3(256), 0, 0, into_flat, A, A2, row4, 1.0f / W, om, 4.0f); break;
            case 8:  hipLaunchKernelGGL((mean_undo<8, 4, true>), dim3(bpr), dim3(256), 0, 0, into_flat, A, A2, row4, 1.0f / W, om, 4.0f); break;
            default: hipLaunchKernelGGL((mean_undo<16, 4, true>), dim3(bpr), dim3(256), 0, 0, into_flat, A, A2, row4, 1.0f / W, om, 4.0f); break;
            } });
        run("rows into flat, merge undone in single precision on differences", 4.0 + 8.0 / W, [&] {
            switch (W) {
            case 4:  hipLaunchKernelGGL((mean_undo<4, 4, false>), dim3(bpr), dim3(256), 0, 0, into_flat, A, A2, row4, 1.0f / W, om, 4.0f); break;
            case 8:  hipLaunchKernelGGL((mean_undo<8, 4, false>), dim3(bpr), dim3(256), 0, 0, into_flat, A, A2, row4, 1.0f / W, om, 4.0f); break;
            default: hipLaunchKernelGGL((mean_undo<16, 4, false>), dim3(bpr), dim3(256), 0, 0, into_flat, A, A2, row4, 1.0f / W, om, 4.0f); break;
            } });
        run("rows, pointers from the kernel arguments", B_MEAN, [&] {
            switch (W) {
            case 4:  hipLaunchKernelGGL((mean_rows<4, 4>), dim3(bpr), dim3(256), 0, 0, rows, A2, row4, 1.0f / W); break;
            case 8:  hipLaunchKernelGGL((mean_rows<8, 4>), dim3(bpr), dim3(256), 0, 0, rows, A2, row4, 1.0f / W); break;
            default: hipLaunchKernelGGL((mean_rows<16, 8>), dim3(bpr), dim3(512), 0, 0, rows, A2, row4, 1.0f / W); break;
            } });
        // how many wavefronts share the W rows of a window
#define MEAN_SPLIT(WT, NW) run("rows, " #NW " wavefronts per workgroup (" #WT "/" #NW " rows each)", B_MEAN, [&] { \
            hipLaunchKernelGGL((mean_rows<WT, NW>), dim3(bpr), dim3(64 * NW), 0, 0, rows, A2, row4, 1.0f / W); })
        switch (W) {
        case 4:  MEAN_SPLIT(4, 1); MEAN_SPLIT(4, 2); MEAN_SPLIT(4, 4); break;
        case 8:  MEAN_SPLIT(8, 1); MEAN_SPLIT(8, 2); MEAN_SPLIT(8, 4); MEAN_SPLIT(8, 8); break;
        default: MEAN_SPLIT(16, 1); MEAN_SPLIT(16, 2); MEAN_SPLIT(16, 4); MEAN_SPLIT(16, 8); MEAN_SPLIT(16, 16); break;
        }
#undef MEAN_SPLIT
    }
    return 0;
}
