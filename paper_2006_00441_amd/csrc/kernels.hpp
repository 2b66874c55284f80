// Device code of the DaSGD parameter pipeline for gfx950 (CDNA4, 64-wide wavefronts).
//
// All kernels are streaming passes bound by HBM bandwidth (<= 0.3 flop per byte), so the design is
// about memory traffic only: 128-bit accesses, every byte touched once, non-temporal hints on
// everything that streams, whole aligned kilobytes per wavefront, no MFMA (nothing is a contraction).
//
//   local step   x, v, g -> x, v [, snapshot]        (paper Eq. 2, first branch; Section 4.1)
//   mean         rows of y (or of merged x) -> A      ((X - eta G) J of the matrix form, appendix)
//   merge        y, A -> x                            (Eq. 2, second branch)
//   and the fused forms: local step + merge; local step + mean + merge.
//
// Two families.  The "matrix" kernels (k_*_flat, k_mean*) serve the layout the paper's matrix form
// suggests: X, V, G are W x P row-major matrices (one row per replica, one row stride).  They
// address by pure arithmetic and run one 64-lane wavefront per workgroup with one 128-bit access per
// lane per array: measured on MI355X this shape sustains the highest HBM throughput (short-lived
// single-wave workgroups keep the memory system evenly fed; anything that delays a wave's first
// load -- a descriptor fetch, a larger workgroup -- costs bandwidth).  The one exception is the mean,
// whose many loads per column are better split over the wavefronts of a workgroup and combined
// through LDS.  The "table" kernels (k_local_step, k_merge) serve arbitrary per-tensor pointers
// through a chunk table.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dasgd {

constexpr int kThreads = 256;                        // 4 wavefronts per workgroup
constexpr int kUnroll  = 4;                          // independent 128-bit accesses per lane per array
constexpr int kChunk   = kThreads * 4 * kUnroll;     // 4096 elements: the unit of work of one workgroup
constexpr int kPad     = 64;                         // tensors start on 256-byte boundaries in library-owned rows

// One unit of work: `len` consecutive elements of tensor `tensor`, starting at element `off` of the
// tensor and at element `foff` of a library-owned row (snapshot / average).
struct Chunk {
    int64_t off;
    int64_t foff;
    int32_t tensor;
    int32_t len;
};

typedef float v4f __attribute__((ext_vector_type(4)));

// What a local step stores besides the momentum buffer.
enum : int {
    kStoreX  = 0,   // x only                      (no average is launched after this step)
    kStoreXS = 1,   // x and the snapshot          (an average is launched, no merge follows this step)
    kStoreS  = 2    // the snapshot only           (a merge follows in the same step and reads the
                    //                              snapshot, so x need not hold the intermediate value)
};

template <bool NT> __device__ __forceinline__ v4f ld4(const v4f *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT> __device__ __forceinline__ void st4(v4f *p, v4f a) {
    if constexpr (NT) __builtin_nontemporal_store(a, p);
    else *p = a;
}

// Heavy-ball momentum with coupled weight decay, one element:
//   g' = g + wd x ;  v <- momentum v + g' ;  x <- x - lr v
__device__ __forceinline__ void sgd1(float &x, float &v, float g, float lr, float momentum, float wd) {
    const float gp = fmaf(wd, x, g);
    const float vn = fmaf(momentum, v, gp);
    v = vn;
    x = fmaf(-lr, vn, x);
}
__device__ __forceinline__ void sgd4(v4f &x, v4f &v, const v4f g, float lr, float momentum, float wd) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float xs = x[e], vs = v[e];
        sgd1(xs, vs, g[e], lr, momentum, wd);
        x[e] = xs;
        v[e] = vs;
    }
}

// Merge of one value: xi y + (1 - xi) a, computed as y + om (a - y) with om = 1 - xi  (Eq. 2, second branch).
__device__ __forceinline__ v4f merge4(v4f x, v4f a, float om) {
    v4f r;
    r.x = fmaf(om, a.x - x.x, x.x);
    r.y = fmaf(om, a.y - x.y, x.y);
    r.z = fmaf(om, a.z - x.z, x.z);
    r.w = fmaf(om, a.w - x.w, x.w);
    return r;
}

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

// Matrix layout: x, v, g (and the snapshot) are W*P contiguous floats each, 16-byte aligned, with
// n4 = W*P/4.  One wavefront per workgroup, one 128-bit access per lane per array.
constexpr int kWave = 64;

template <int MODE>
__global__ void __launch_bounds__(kWave)
k_local_step_flat(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g, v4f *__restrict__ s,
                  int64_t n4, float lr, float momentum, float wd)
{
    constexpr bool WX = (MODE != kStoreS), WS = (MODE != kStoreX);
    const int64_t i = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (i >= n4) return;
    v4f xr = ld4<true>(x + i);
    v4f vr = ld4<true>(v + i);
    const v4f gr = ld4<true>(g + i);
    sgd4(xr, vr, gr, lr, momentum, wd);
    if (WX) st4<true>(x + i, xr);
    st4<true>(v + i, vr);
    if (WS) st4<true>(s + i, xr);
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

// ------------------------------------------------------------------------------------------------
// Sum of r[LO..HI) in pairwise (tree) order.
template <int LO, int HI> __device__ __forceinline__ v4f tree_sum(const v4f *r) {
    if constexpr (HI - LO == 1) return r[LO];
    else {
        constexpr int MID = LO + (HI - LO + 1) / 2;
        return tree_sum<LO, MID>(r) + tree_sum<MID, HI>(r);
    }
}

// W-way replica mean over library-owned rows: A[i] = (1/W) sum_j S[j][i].  One lane owns one
// 128-bit column and reads it from all W rows (W independent loads in flight), so the reduction
// needs no cross-lane traffic.  (4 + 4/W) bytes per replica-element.  Single-wave workgroups.  WT > 0: W known at compile
// time, the whole column set is loaded before the tree sum; WT == 0: any W, four rows at a time.
template <int WT, int U, bool NT, bool RUNS>
__global__ void __launch_bounds__(kWave)
k_mean(const v4f *__restrict__ S, v4f *__restrict__ A, int64_t n4, int64_t row4, int W, float inv_w)
{
    // The mean runs beside whatever the caller has on the main stream (typically dense compute that
    // leaves wave slots free but keeps the issue ports busy): its few instructions go first.
    __builtin_amdgcn_s_setprio(3);
    // RUNS: eight consecutive 64-column windows go to the same XCD back to back.  When the rows are
    // not 128-byte aligned relative to each other, the cache line two neighbouring windows share is
    // then found in that XCD's L2 instead of being fetched from HBM twice.  Aligned rows share no
    // lines and keep the plain order, which is a little faster.
    const int64_t blk = RUNS ? ((int64_t)(blockIdx.x >> 6) * 8 + (blockIdx.x & 7)) * 8 + ((blockIdx.x >> 3) & 7)
                             : (int64_t)blockIdx.x;
    const int64_t base = blk * (kWave * U) + threadIdx.x;
    if constexpr (WT > 0) {
        v4f r[U][WT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * kWave;
            if (i < n4) {
#pragma unroll
                for (int j = 0; j < WT; ++j) r[u][j] = ld4<NT>(S + (int64_t)j * row4 + i);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * kWave;
            if (i < n4) st4<false>(A + i, tree_sum<0, WT>(r[u]) * inv_w);
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * kWave;
            if (i >= n4) continue;
            v4f acc = {0.f, 0.f, 0.f, 0.f};
            int j = 0;
            for (; j + 4 <= W; j += 4) {
                const v4f a = ld4<NT>(S + (int64_t)(j + 0) * row4 + i);
                const v4f b = ld4<NT>(S + (int64_t)(j + 1) * row4 + i);
                const v4f c = ld4<NT>(S + (int64_t)(j + 2) * row4 + i);
                const v4f d = ld4<NT>(S + (int64_t)(j + 3) * row4 + i);
                acc += (a + b) + (c + d);
            }
            for (; j < W; ++j) acc += ld4<NT>(S + (int64_t)j * row4 + i);
            st4<false>(A + i, acc * inv_w);
        }
    }
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

// Zero-copy snapshot with reconstruction.  When a step both launches an average and merges an older
// one, the folded kernel leaves only the merged weights x' = y + om (A_old - y) = xi y + om A_old in
// memory.  The average of the y is still recoverable from them, because the merge is affine and the
// same for every replica:   mean_j y_j = (mean_j x'_j - om A_old) / xi .
// So the mean kernel reads the live weights (no snapshot was stored) and undoes the merge on the
// mean.  The subtraction cancels (operands ~|x|, result ~xi |x|), hence fp64 inside: what remains is
// the fp32 rounding of the x'_j themselves, averaged over W and amplified by 1/xi.  Rows are split
// over the NW wavefronts as in k_mean_lds (wave w takes rows w, w+NW, ...: any W).
typedef double v4d __attribute__((ext_vector_type(4)));

template <int NW, bool RUNS>
__global__ void __launch_bounds__(kWave * NW)
k_mean_reconstruct(const v4f *__restrict__ X, const v4f *__restrict__ A_old, v4f *__restrict__ A_new,
                   int64_t n4, int64_t row4, int W, double inv_w, double om, double inv_xi)
{
    __shared__ v4d part[NW][kWave];
    __builtin_amdgcn_s_setprio(3);
    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int64_t blk = RUNS ? ((int64_t)(blockIdx.x >> 6) * 8 + (blockIdx.x & 7)) * 8 + ((blockIdx.x >> 3) & 7)
                             : (int64_t)blockIdx.x;
    const int64_t i = blk * kWave + l;
    v4d acc = {0.0, 0.0, 0.0, 0.0};
    if (i < n4) {
        for (int j = w; j < W; j += NW) {
            const v4f r = ld4<true>(X + (int64_t)j * row4 + i);
            acc += __builtin_convertvector(r, v4d);
        }
    }
    part[w][l] = acc;
    __syncthreads();
    if (w == 0 && i < n4) {
        v4d m = part[0][l];
#pragma unroll
        for (int k = 1; k < NW; ++k) m += part[k][l];
        const v4d a = __builtin_convertvector(ld4<false>(A_old + i), v4d);
        const v4d y = (m * inv_w - om * a) * inv_xi;
        st4<false>(A_new + i, __builtin_convertvector(y, v4f));
    }
}

// Matrix layout, everything of one iteration in ONE pass: a wavefront owns a window of 64 columns of
// ALL W rows; per lane it updates the W replicas of its column (local step), sums their new values
// into the average that is launched at this step (MEAN) and folds the average launched d steps ago
// into them (MERGE).  No snapshot and no separate mean kernel: 20 + 8/W bytes per replica-element
// for a step that does all three.  The price is row-strided access: unless P is a multiple of 32 the
// rows are not 128-byte aligned to each other and the kilobytes a wave touches straddle cache lines.
// Same operations in the same order as k_local_step_flat + k_mean + k_merge_flat (identical bits).
template <int WT, bool MEAN, bool MERGE>   // WT > 0: W known at compile time (tree sum); 0: any W
__global__ void __launch_bounds__(kWave)
k_step_all_flat(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g,
                const v4f *__restrict__ A_old, v4f *__restrict__ A_new, int64_t row4, int W,
                float lr, float momentum, float wd, float om, float inv_w)
{
    const int64_t c = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (c >= row4) return;
    v4f a = {0.f, 0.f, 0.f, 0.f};
    if (MERGE) a = ld4<false>(A_old + c);
    if constexpr (WT > 0) {
        v4f y[WT];
        constexpr int JB = WT < 4 ? WT : 4;
#pragma unroll
        for (int j0 = 0; j0 < WT; j0 += JB) {
            v4f vr[JB], gr[JB];
#pragma unroll
            for (int j = 0; j < JB; ++j) {
                const int64_t i = (int64_t)(j0 + j) * row4 + c;
                y[j0 + j] = ld4<true>(x + i);
                vr[j] = ld4<true>(v + i);
                gr[j] = ld4<true>(g + i);
            }
#pragma unroll
            for (int j = 0; j < JB; ++j) {
                const int64_t i = (int64_t)(j0 + j) * row4 + c;
                sgd4(y[j0 + j], vr[j], gr[j], lr, momentum, wd);
                st4<true>(v + i, vr[j]);
                st4<true>(x + i, MERGE ? merge4(y[j0 + j], a, om) : y[j0 + j]);
            }
        }
        if (MEAN) st4<false>(A_new + c, tree_sum<0, WT>(y) * inv_w);
    } else {
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        int j = 0;
        for (; j + 4 <= W; j += 4) {
            v4f y[4], vr[4], gr[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t i = (int64_t)(j + u) * row4 + c;
                y[u] = ld4<true>(x + i);
                vr[u] = ld4<true>(v + i);
                gr[u] = ld4<true>(g + i);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t i = (int64_t)(j + u) * row4 + c;
                sgd4(y[u], vr[u], gr[u], lr, momentum, wd);
                st4<true>(v + i, vr[u]);
                st4<true>(x + i, MERGE ? merge4(y[u], a, om) : y[u]);
            }
            acc += (y[0] + y[1]) + (y[2] + y[3]);
        }
        for (; j < W; ++j) {
            const int64_t i = (int64_t)j * row4 + c;
            v4f y = ld4<true>(x + i), vr = ld4<true>(v + i);
            const v4f gr = ld4<true>(g + i);
            sgd4(y, vr, gr, lr, momentum, wd);
            st4<true>(v + i, vr);
            st4<true>(x + i, MERGE ? merge4(y, a, om) : y);
            acc += y;
        }
        if (MEAN) st4<false>(A_new + c, acc * inv_w);
    }
}

// ------------------------------------------------------------------------------------------------
// Delayed merge: x_j <- y_j + (1 - xi)(A - y_j) for every replica j, where y_j is the value after the
// local step (held in x_j, or in the snapshot when the local step stored only that).
// Table version: grid = chunks; the chunk of A is read once into registers and applied to all W
// replicas: (8 + 4/W) bytes per replica-element.

// FROM_S: the pre-merge value y is read from snapshot rows Y (row stride P_pad, chunk at foff)
// instead of from x (the local step stored only the snapshot).
template <bool FROM_S>
__global__ void __launch_bounds__(kThreads)
k_merge(const Chunk *__restrict__ chunks, float *const *__restrict__ xp, const float *__restrict__ A,
        const float *__restrict__ Y, int64_t P_pad, int n_tensors, int W, float om)
{
    const Chunk c = chunks[blockIdx.x];
    const float *__restrict__ a = A + c.foff;
    const v4f *a4 = reinterpret_cast<const v4f *>(a);
    const int tid = threadIdx.x;
    const int len = c.len;
    const bool full = (len == kChunk);
    const bool a_aligned = (reinterpret_cast<uintptr_t>(a) & 15u) == 0;

    v4f ar[kUnroll];
    if (full && a_aligned) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) ar[u] = ld4<false>(a4 + tid + u * kThreads);
    }
    for (int j = 0; j < W; ++j) {
        float *x = xp[(int64_t)j * n_tensors + c.tensor] + c.off;
        const float *y = FROM_S ? Y + (int64_t)j * P_pad + c.foff : x;
        const bool aligned = a_aligned && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) & 15u) == 0;
        if (aligned) {
            v4f *x4 = reinterpret_cast<v4f *>(x);
            const v4f *y4 = reinterpret_cast<const v4f *>(y);
            if (full) {
                v4f yr[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) yr[u] = ld4<true>(y4 + tid + u * kThreads);
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) st4<true>(x4 + tid + u * kThreads, merge4(yr[u], ar[u], om));
            } else {
                const int n4 = len >> 2;
                for (int i = tid; i < n4; i += kThreads) x4[i] = merge4(y4[i], a4[i], om);
                const int e = (n4 << 2) + tid;
                if (e < len) { const float ys = y[e]; x[e] = fmaf(om, a[e] - ys, ys); }
            }
        } else {
            for (int e = tid; e < len; e += kThreads) { const float ys = y[e]; x[e] = fmaf(om, a[e] - ys, ys); }
        }
    }
}

// Matrix layout merge: X (and Y, the values after the local step: X itself or the snapshot) are W
// rows of row4 128-bit columns back to back, A is one row.  Same decomposition as the folded kernel.
// (8 + 4/W) bytes per replica-element.  Needs n4 = W*P/4 < 2^31.
template <int WT>   // WT > 0: W known at compile time; 0: any W
__global__ void __launch_bounds__(kWave)
k_merge_flat(v4f *__restrict__ X, const v4f *__restrict__ Y, const v4f *__restrict__ A,
             unsigned n4, unsigned row4, int W, unsigned log_band, float om)
{
    unsigned i, c;
    if (!decode_block(blockIdx.x, WT > 0 ? (unsigned)WT : (unsigned)W, row4, n4, log_band, i, c)) return;
    const v4f a = ld4<false>(A + c);
    const v4f y = ld4<true>(Y + i);
    st4<true>(X + i, merge4(y, a, om));
}

// The same one-pass iteration with the W rows of a 64-column window spread over the W wavefronts of
// a workgroup: wavefront j does replica j's local step and merge (three loads in flight per lane
// instead of 3W, W times as many waves), leaves its y in LDS, and after the barrier wavefront 0 adds
// the W values in tree order and stores the average.  Measured on MI355X 4-5 % faster than the
// lane-owns-a-column form at W = 8 (0.72 against 0.75-0.78 ms for the ResNet-50-shaped set).  Same
// operations in the same order (identical bits).  W = WT is a compile-time constant, 2 <= WT <= 16.
template <int WT, bool MERGE>
__global__ void __launch_bounds__(kWave * WT)
k_step_all_rows(v4f *__restrict__ x, v4f *__restrict__ v, const v4f *__restrict__ g,
                const v4f *__restrict__ A_old, v4f *__restrict__ A_new, int64_t row4,
                float lr, float momentum, float wd, float om, float inv_w)
{
    __shared__ v4f part[WT][kWave];
    const int w = threadIdx.x / kWave, l = threadIdx.x % kWave;
    const int64_t c = (int64_t)blockIdx.x * kWave + l;
    if (c < row4) {
        const int64_t i = (int64_t)w * row4 + c;
        v4f y = ld4<true>(x + i), vr = ld4<true>(v + i);
        const v4f gr = ld4<true>(g + i);
        v4f a = {0.f, 0.f, 0.f, 0.f};
        if (MERGE) a = ld4<false>(A_old + c);
        sgd4(y, vr, gr, lr, momentum, wd);
        st4<true>(v + i, vr);
        st4<true>(x + i, MERGE ? merge4(y, a, om) : y);
        part[w][l] = y;
    }
    __syncthreads();
    if (w == 0 && c < row4) {
        v4f p[WT];
#pragma unroll
        for (int k = 0; k < WT; ++k) p[k] = part[k][l];
        st4<false>(A_new + c, tree_sum<0, WT>(p) * inv_w);
    }
}

// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) k_fill_zero(v4f *__restrict__ p, int64_t n4)
{
    const v4f z = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kThreads)
        p[i] = z;
}

}  // namespace dasgd
