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
// Two ways of finding the data.
//   rows     every replica's parameters are ONE contiguous run of P floats (the paper's X_k with one
//            column per worker: a W x P matrix with any row stride, or one arena per replica).  The W
//            base pointers of x, v and g travel in the kernel arguments and are selected by blockIdx.y,
//            so nothing has to be loaded from memory before a wave knows its addresses.
//   records  anything else (one allocation per tensor, odd sizes, unaligned pointers): one 32-byte
//            record per replica and 4096-float piece of a tensor holds the piece's pointers; the 16
//            single-wave workgroups of a piece read the same record (one scalar load, cached).
//
// What measurements on MI355X fixed (a stand-alone study program sits beside this file):
//   * one 64-lane wavefront per workgroup and one 128-bit access per lane per array beats every larger
//     shape by 5-10 % (256 x 1, 256 x 4 unrolled, persistent grid-stride loops);
//   * non-temporal loads and stores: + 7-10 %;
//   * a wave's loads issued ONE AFTER THE OTHER (x, wait, v, wait, g) beat the same loads issued
//     together by 1-3 %: many short-lived waves with one request each keep the memory system more
//     evenly fed than fewer requests per wave in a burst.  The compiler would batch them, so each
//     loaded value passes through arrived(), an empty asm statement that needs the value;
//   * kilobytes that straddle a 1 KiB boundary cost up to 15 %: a row's blocks are aligned to the
//     row's own address (see rows_column);
//   * workgroups are dealt round-robin to the 8 L2 partitions (XCDs) in dispatch order, x fastest,
//     then y, then z.  Kernels that re-read the average for every replica use a three-dimensional
//     grid (8 B, W, bands): a partition sees B windows of replica 0, the same windows of replica 1,
//     ..., and that piece of the average comes from HBM once and from its L2 for the other W - 1.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dasgd {

constexpr int kWave     = 64;                 // lanes of a wavefront
constexpr int kMaxRows  = 32;                 // replicas whose row pointers fit the kernel arguments
constexpr int kPieceLog = 4;                  // a record covers 2^kPieceLog blocks of 64 128-bit elements
constexpr int kPiece    = 256 << kPieceLog;   // = 4096 floats
constexpr int kPad      = 64;                 // tensors start on 256-byte boundaries in padded library rows
constexpr int kThreads  = 256;                // workgroup of the fill kernel

struct RowSet { float *p[kMaxRows]; };
struct ConstRowSet { const float *p[kMaxRows]; };

// One piece (at most kPiece floats) of one tensor of one replica.
struct Rec {
    float *x;
    float *v;
    uint32_t aoff;      // position of the piece in a library-owned row (snapshot, average), in floats
    uint32_t goff;      // position of the piece in its tensor, in floats
    uint32_t len;       // floats in the piece
    uint32_t tensor;
};

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) v4f gv4f;             // pointers read from memory are generic
typedef const __attribute__((address_space(1))) v4f cgv4f;      // to the compiler: say "global" where known
typedef __attribute__((address_space(1))) float gf32;
typedef const __attribute__((address_space(1))) float cgf32;

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
__device__ __forceinline__ v4f gld4(cgv4f *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void gst4(gv4f *p, v4f a) { __builtin_nontemporal_store(a, p); }

// The value must be in its registers here: a load issued before stays before, and the next load is
// issued only after this one has come back.
__device__ __forceinline__ void arrived(v4f &a) { asm volatile("" : "+v"(a)); }

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
__device__ __forceinline__ float merge1(float y, float a, float om) { return fmaf(om, a - y, y); }
__device__ __forceinline__ v4f merge4(v4f x, v4f a, float om) {
    v4f r;
    r.x = merge1(x.x, a.x, om);
    r.y = merge1(x.y, a.y, om);
    r.z = merge1(x.z, a.z, om);
    r.w = merge1(x.w, a.w, om);
    return r;
}

// ------------------------------------------------------------------------------------------------
// Work decomposition of the row kernels.  A row is row4 128-bit columns starting at a 16-byte aligned
// address; block q of the row covers the columns q*64 - head ... q*64 - head + 63 that exist, where
// head = (address / 16) mod 64 is the row's offset from a 1 KiB boundary: every wave then touches one
// whole aligned kilobyte (the first and the last block of a row are partial).  Columns and blocks are
// 32-bit: rows of up to 2^31 columns.
__host__ __device__ __forceinline__ unsigned rows_head(const void *row) {
    return (unsigned)((reinterpret_cast<uintptr_t>(row) >> 4) & 63u);
}
// column handled by `lane` of block q (a value >= row4, possibly by wrap-around, means none)
__host__ __device__ __forceinline__ unsigned rows_column(unsigned q, unsigned lane, unsigned head) {
    return q * 64u + lane - head;
}
// blocks a row can need whatever its head
__host__ __device__ __forceinline__ unsigned rows_blocks(unsigned row4) { return (row4 + 63u + 63u) / 64u; }
// block index of a workgroup in a grid (gx, W, gz)
#define DASGD_BLOCK_OF_WG (blockIdx.z * gridDim.x + blockIdx.x)

// ------------------------------------------------------------------------------------------------
// Local step on every replica, rows addressing.  grid = (gx, W, gz), one wavefront per workgroup.
// 20 bytes per element (24 when both x and the snapshot are stored).
// MERGE: this step's merge is folded in -- the value stored to x is y + om (A - y), the snapshot (if
// any) still receives y (paper Eq. 2, both branches in one pass): 20 + 4/W bytes per element.
// S: snapshot rows (row stride s_stride4 columns, row j column c <-> x_j column c); A: the average.
template <int MODE, bool MERGE>
__global__ void __launch_bounds__(kWave)
k_step_rows(const RowSet x, const RowSet v, const ConstRowSet g, v4f *__restrict__ S, int64_t s_stride4,
            const v4f *__restrict__ A, unsigned row4, float lr, float momentum, float wd, float om)
{
    constexpr bool WX = (MODE != kStoreS), WS = (MODE != kStoreX);
    static_assert(!(MERGE && MODE == kStoreS), "a folded merge always stores x");
    const unsigned j = blockIdx.y;
    v4f *__restrict__ xj = reinterpret_cast<v4f *>(x.p[j]);
    v4f *__restrict__ vj = reinterpret_cast<v4f *>(v.p[j]);
    const v4f *__restrict__ gj = reinterpret_cast<const v4f *>(g.p[j]);
    const unsigned c = rows_column(DASGD_BLOCK_OF_WG, threadIdx.x, rows_head(xj));
    if (c >= row4) return;
    v4f a = {0.f, 0.f, 0.f, 0.f};
    if (MERGE) { a = ld4<false>(A + c); arrived(a); }
    v4f xr = ld4<true>(xj + c); arrived(xr);
    v4f vr = ld4<true>(vj + c); arrived(vr);
    v4f gr = ld4<true>(gj + c); arrived(gr);
    sgd4(xr, vr, gr, lr, momentum, wd);
    st4<true>(vj + c, vr);
    if (WS) st4<true>(S + (int64_t)j * s_stride4 + c, xr);
    if (WX) st4<true>(xj + c, MERGE ? merge4(xr, a, om) : xr);
}

// Delayed merge, rows addressing: x_j <- y_j + (1 - xi)(A - y_j), where y_j is the value after the
// local step (held in x_j, or in the snapshot when the local step stored only that).  Same grid as the
// folded step.  (8 + 4/W) bytes per element.
template <bool FROM_S>
__global__ void __launch_bounds__(kWave)
k_merge_rows(const RowSet x, const v4f *__restrict__ S, int64_t s_stride4, const v4f *__restrict__ A, unsigned row4, float om)
{
    const unsigned j = blockIdx.y;
    v4f *__restrict__ xj = reinterpret_cast<v4f *>(x.p[j]);
    const unsigned c = rows_column(DASGD_BLOCK_OF_WG, threadIdx.x, rows_head(xj));
    if (c >= row4) return;
    v4f a = ld4<false>(A + c); arrived(a);
    const v4f y = FROM_S ? ld4<true>(S + (int64_t)j * s_stride4 + c) : ld4<true>(xj + c);
    st4<true>(xj + c, merge4(y, a, om));
}

// ------------------------------------------------------------------------------------------------
// Sum of r[LO..HI) in pairwise (tree) order: the left part gets the larger half.
template <int LO, int HI> __device__ __forceinline__ v4f tree_sum(const v4f *r) {
    if constexpr (HI - LO == 1) return r[LO];
    else {
        constexpr int MID = LO + (HI - LO + 1) / 2;
        return tree_sum<LO, MID>(r) + tree_sum<MID, HI>(r);
    }
}

// Column windows of the mean kernels: workgroup b takes the 64-column window mean_window(b).  RUNS:
// eight consecutive windows go to the same L2 partition back to back (workgroup b runs on partition
// b mod 8).  When the rows are not 128-byte aligned relative to each other, the cache line two
// neighbouring windows share is then found in that L2 instead of being fetched from HBM twice.
// Aligned rows share no lines and keep the plain order, which is a little faster.  A permutation of
// [0, 64 n) for every n: the grid is rounded up to a multiple of 64 workgroups.
template <bool RUNS> __host__ __device__ __forceinline__ uint64_t mean_window(uint64_t b) {
    return RUNS ? ((b >> 6) * 8 + (b & 7)) * 8 + ((b >> 3) & 7) : b;
}

// W-way replica mean: A[c] = (1/W) sum_j row_j[c].  The rows are split over the NW wavefronts of a
// workgroup: wavefront w sums rows [w R, (w+1) R) of a 64-column window (R = W / NW loads in flight per
// lane), writes its partial sum to LDS, and after the barrier wavefront 0 adds the NW partials in tree
// order and stores the average.  With few rows per wave many more waves are in flight, which measured
// 2-6 % faster than one lane reading all W rows.  Same pairwise order over rows as a plain tree sum.
// (4 + 4/W) bytes per element.
template <int WT, int NW, bool RUNS>
__global__ void __launch_bounds__(kWave * NW)
k_mean_rows(const ConstRowSet rows, v4f *__restrict__ A, unsigned row4, float inv_w)
{
    constexpr int R = WT / NW;
    static_assert(R * NW == WT && R >= 1, "rows must split evenly over the wavefronts");
    __shared__ v4f part[NW][kWave];
    // The mean runs beside whatever the caller has on the main stream (typically dense compute that
    // leaves wave slots free but keeps the issue ports busy): its few instructions go first.
    __builtin_amdgcn_s_setprio(3);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), l = threadIdx.x % kWave;
    const uint64_t c = mean_window<RUNS>(blockIdx.x) * kWave + l;
    if (c < row4) {
        v4f r[R];
#pragma unroll
        for (int j = 0; j < R; ++j) r[j] = ld4<true>(reinterpret_cast<const v4f *>(rows.p[w * R + j]) + c);
        part[w][l] = tree_sum<0, R>(r);
    }
    __syncthreads();
    if (w == 0 && c < row4) {
        v4f p[NW];
#pragma unroll
        for (int k = 0; k < NW; ++k) p[k] = part[k][l];
        st4<false>(A + c, tree_sum<0, NW>(p) * inv_w);
    }
}

// The same for any W up to kMaxRows with one lane reading its column from all rows (W independent
// loads in flight, no cross-lane traffic), in the same pairwise order.
template <int WT> __device__ __forceinline__ v4f column_sum(const ConstRowSet &rows, uint64_t c) {
    v4f r[WT];
#pragma unroll
    for (int j = 0; j < WT; ++j) r[j] = ld4<true>(reinterpret_cast<const v4f *>(rows.p[j]) + c);
    return tree_sum<0, WT>(r);
}
template <bool RUNS>
__global__ void __launch_bounds__(kWave)
k_mean_any(const ConstRowSet rows, v4f *__restrict__ A, unsigned row4, int W, float inv_w)
{
    __builtin_amdgcn_s_setprio(3);
    const uint64_t c = mean_window<RUNS>(blockIdx.x) * kWave + threadIdx.x;
    if (c >= row4) return;
    v4f s;
    switch (W) {
#define DASGD_CASE(N) case N: s = column_sum<N>(rows, c); break;
        DASGD_CASE(1) DASGD_CASE(2) DASGD_CASE(3) DASGD_CASE(4) DASGD_CASE(5) DASGD_CASE(6) DASGD_CASE(7) DASGD_CASE(8)
        DASGD_CASE(9) DASGD_CASE(10) DASGD_CASE(11) DASGD_CASE(12) DASGD_CASE(13) DASGD_CASE(14) DASGD_CASE(15) DASGD_CASE(16)
        DASGD_CASE(17) DASGD_CASE(18) DASGD_CASE(19) DASGD_CASE(20) DASGD_CASE(21) DASGD_CASE(22) DASGD_CASE(23) DASGD_CASE(24)
        DASGD_CASE(25) DASGD_CASE(26) DASGD_CASE(27) DASGD_CASE(28) DASGD_CASE(29) DASGD_CASE(30) DASGD_CASE(31) DASGD_CASE(32)
#undef DASGD_CASE
    default: return;
    }
    st4<false>(A + c, s * inv_w);
}

// More than kMaxRows replicas: the rows are those of a library-owned snapshot (base + j * stride), summed
// four at a time.  Not the pairwise order: equal to it only up to rounding.
__global__ void __launch_bounds__(kWave)
k_mean_strided(const v4f *__restrict__ S, int64_t stride4, v4f *__restrict__ A, unsigned row4, int W, float inv_w)
{
    __builtin_amdgcn_s_setprio(3);
    const uint64_t c = (uint64_t)blockIdx.x * kWave + threadIdx.x;
    if (c >= row4) return;
    v4f acc = {0.f, 0.f, 0.f, 0.f};
    int j = 0;
    for (; j + 4 <= W; j += 4) {
        const v4f a = ld4<true>(S + (int64_t)(j + 0) * stride4 + c);
        const v4f b = ld4<true>(S + (int64_t)(j + 1) * stride4 + c);
        const v4f d = ld4<true>(S + (int64_t)(j + 2) * stride4 + c);
        const v4f e = ld4<true>(S + (int64_t)(j + 3) * stride4 + c);
        acc += (a + b) + (d + e);
    }
    for (; j < W; ++j) acc += ld4<true>(S + (int64_t)j * stride4 + c);
    st4<false>(A + c, acc * inv_w);
}

// Zero-copy snapshot with reconstruction.  When a step both launches an average and merges an older
// one, the folded kernel leaves only the merged weights x'_j = y_j + om (A_old - y_j) = xi y_j + om A_old
// in memory.  The average of the y_j is still recoverable from them, because the merge is affine and
// the same for every replica:   mean_j y_j = (mean_j x'_j - om A_old) / xi .
// The subtraction cancels (operands ~|x|, result ~ xi |x|), so the mean of the x'_j must not be rounded
// at the size of x.  The replicas differ by little, hence single precision suffices on differences:
//     mean_j x'_j = x'_0 + (1/W) sum_j (x'_j - x'_0)            (each difference exact or nearly so)
//     mean_j y_j  = ( fma(-om, A_old, x'_0) + (1/W) sum_j (x'_j - x'_0) ) / xi
// where the fma rounds once, at the size of the result.  What remains is the fp32 rounding of the x'_j
// themselves, averaged over W and amplified by 1/xi.  Wave w takes rows w, w + NW, ... (any W) and
// keeps its first row as its own reference; wave 0 refers the others' to row 0.
template <int NW, bool RUNS>
__global__ void __launch_bounds__(kWave * NW)
k_mean_undo_merge(const ConstRowSet rows, const v4f *__restrict__ A_old, v4f *__restrict__ A_new, unsigned row4, int W,
                  float inv_w, float om, float inv_xi)
{
    __shared__ v4f first[NW][kWave], dsum[NW][kWave];
    __builtin_amdgcn_s_setprio(3);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), l = threadIdx.x % kWave;
    const uint64_t c = mean_window<RUNS>(blockIdx.x) * kWave + l;
    if (c < row4 && w < W) {
        const v4f r0 = ld4<true>(reinterpret_cast<const v4f *>(rows.p[w]) + c);
        v4f d = {0.f, 0.f, 0.f, 0.f};
        for (int j = w + NW; j < W; j += NW) d += ld4<true>(reinterpret_cast<const v4f *>(rows.p[j]) + c) - r0;
        first[w][l] = r0;
        dsum[w][l] = d;
    }
    __syncthreads();
    if (w == 0 && c < row4) {
        const v4f r0 = first[0][l];
        v4f d = dsum[0][l];
#pragma unroll
        for (int k = 1; k < NW; ++k)
            if (k < W) d += dsum[k][l] + (float)((W - k + NW - 1) / NW) * (first[k][l] - r0);   // rows of wave k: each = its reference + ...
        const v4f a = ld4<false>(A_old + c);
        v4f t;
        t.x = fmaf(-om, a.x, r0.x); t.y = fmaf(-om, a.y, r0.y); t.z = fmaf(-om, a.z, r0.z); t.w = fmaf(-om, a.w, r0.w);
        st4<false>(A_new + c, (t + d * inv_w) * inv_xi);
    }
}

// ------------------------------------------------------------------------------------------------
// Everything of one iteration in ONE pass, rows addressing: the W rows of a 64-column window are
// spread over the W wavefronts of a workgroup.  Wavefront j does replica j's local step and merge
// (MERGE), leaves its y in LDS, and after the barrier wavefront 0 adds the W values in tree order and
// stores the average launched at this step.  No snapshot and no separate mean kernel: 20 + 8/W bytes
// per element for a step that does all three.  Same operations in the same order as the separate
// kernels (identical bits).  W = WT is a compile-time constant, 2 <= WT <= 16.
template <int WT, bool MERGE>
__global__ void __launch_bounds__(kWave * WT)
k_step_all_rows(const RowSet x, const RowSet v, const ConstRowSet g, const v4f *__restrict__ A_old, v4f *__restrict__ A_new,
                unsigned row4, float lr, float momentum, float wd, float om, float inv_w)
{
    __shared__ v4f part[WT][kWave];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), l = threadIdx.x % kWave;
    const uint64_t c = (uint64_t)blockIdx.x * kWave + l;
    if (c < row4) {
        v4f *xj = reinterpret_cast<v4f *>(x.p[w]) + c, *vj = reinterpret_cast<v4f *>(v.p[w]) + c;
        v4f a = {0.f, 0.f, 0.f, 0.f};
        if (MERGE) { a = ld4<false>(A_old + c); arrived(a); }
        v4f y = ld4<true>(xj); arrived(y);
        v4f vr = ld4<true>(vj); arrived(vr);
        v4f gr = ld4<true>(reinterpret_cast<const v4f *>(g.p[w]) + c); arrived(gr);
        sgd4(y, vr, gr, lr, momentum, wd);
        st4<true>(vj, vr);
        st4<true>(xj, MERGE ? merge4(y, a, om) : y);
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

// The same for any W up to kMaxRows: one lane updates the W replicas of its column one after the other
// and keeps their new values for the tree sum.
template <int WT> __device__ __forceinline__ v4f column_step(const RowSet &x, const RowSet &v, const ConstRowSet &g, uint64_t c, bool merge,
                                                             v4f a, float lr, float momentum, float wd, float om) {
    v4f y[WT];
#pragma unroll
    for (int j = 0; j < WT; ++j) {
        v4f *xj = reinterpret_cast<v4f *>(x.p[j]) + c, *vj = reinterpret_cast<v4f *>(v.p[j]) + c;
        v4f vr = ld4<true>(vj);
        const v4f gr = ld4<true>(reinterpret_cast<const v4f *>(g.p[j]) + c);
        y[j] = ld4<true>(xj);
        sgd4(y[j], vr, gr, lr, momentum, wd);
        st4<true>(vj, vr);
        st4<true>(xj, merge ? merge4(y[j], a, om) : y[j]);
    }
    return tree_sum<0, WT>(y);
}
template <bool MERGE>
__global__ void __launch_bounds__(kWave)
k_step_all_any(const RowSet x, const RowSet v, const ConstRowSet g, const v4f *__restrict__ A_old, v4f *__restrict__ A_new,
               unsigned row4, int W, float lr, float momentum, float wd, float om, float inv_w)
{
    const uint64_t c = (uint64_t)blockIdx.x * kWave + threadIdx.x;
    if (c >= row4) return;
    v4f a = {0.f, 0.f, 0.f, 0.f};
    if (MERGE) a = ld4<false>(A_old + c);
    v4f s;
    switch (W) {
#define DASGD_CASE(N) case N: s = column_step<N>(x, v, g, c, MERGE, a, lr, momentum, wd, om); break;
        DASGD_CASE(1) DASGD_CASE(2) DASGD_CASE(3) DASGD_CASE(4) DASGD_CASE(5) DASGD_CASE(6) DASGD_CASE(7) DASGD_CASE(8)
        DASGD_CASE(9) DASGD_CASE(10) DASGD_CASE(11) DASGD_CASE(12) DASGD_CASE(13) DASGD_CASE(14) DASGD_CASE(15) DASGD_CASE(16)
        DASGD_CASE(17) DASGD_CASE(18) DASGD_CASE(19) DASGD_CASE(20) DASGD_CASE(21) DASGD_CASE(22) DASGD_CASE(23) DASGD_CASE(24)
        DASGD_CASE(25) DASGD_CASE(26) DASGD_CASE(27) DASGD_CASE(28) DASGD_CASE(29) DASGD_CASE(30) DASGD_CASE(31) DASGD_CASE(32)
#undef DASGD_CASE
    default: return;
    }
    st4<false>(A_new + c, s * inv_w);
}

// ------------------------------------------------------------------------------------------------
// Records addressing.  grid = (gx, W, gz); workgroup q = z gx + x of replica y handles block q mod 16 of
// piece q div 16 (a piece shorter than 16 blocks leaves its last workgroups idle).  A block is 256
// floats: one 128-bit access per lane when the piece's x, v, g (and snapshot / average) addresses are
// 16-byte aligned, four 32-bit accesses per lane otherwise; up to three floats past the last whole
// 128-bit element are done by the lane behind it.
struct Block {
    gf32 *x, *v;
    cgf32 *g;
    gf32 *s;
    cgf32 *a;
    unsigned len, first;        // floats in the piece; first float of this block
    bool live, aligned;
};
template <bool WS, bool MERGE>
__device__ __forceinline__ Block block_of(const Rec *__restrict__ recs, unsigned recs_per_row, unsigned slots,
                                          const float *const *__restrict__ gp, int n_tensors, float *S, int64_t s_stride, const float *A)
{
    Block b;
    b.live = false;
    const unsigned q = DASGD_BLOCK_OF_WG, j = blockIdx.y;
    if (q >= slots) return b;
    const Rec r = recs[(size_t)j * recs_per_row + (q >> kPieceLog)];
    b.len = r.len;
    b.first = (q & ((1u << kPieceLog) - 1u)) * 256u;
    if (b.first >= r.len) return b;
    b.live = true;
    b.x = (gf32 *)r.x;
    b.v = (gf32 *)r.v;
    b.g = gp ? (cgf32 *)(gp[(size_t)j * n_tensors + r.tensor] + r.goff) : nullptr;
    b.s = WS ? (gf32 *)(S + (int64_t)j * s_stride + r.aoff) : nullptr;
    b.a = MERGE ? (cgf32 *)(A + r.aoff) : nullptr;
    b.aligned = ((reinterpret_cast<uintptr_t>(r.x) | reinterpret_cast<uintptr_t>(r.v) | (uintptr_t)b.g | (uintptr_t)b.s | (uintptr_t)b.a) & 15u) == 0;
    return b;
}

template <int MODE, bool MERGE>
__global__ void __launch_bounds__(kWave)
k_step_records(const Rec *__restrict__ recs, unsigned recs_per_row, unsigned slots, const float *const *__restrict__ gp, int n_tensors,
               float *__restrict__ S, int64_t s_stride, const float *__restrict__ A, float lr, float momentum, float wd, float om)
{
    constexpr bool WX = (MODE != kStoreS), WS = (MODE != kStoreX);
    static_assert(!(MERGE && MODE == kStoreS), "a folded merge always stores x");
    const Block b = block_of<WS, MERGE>(recs, recs_per_row, slots, gp, n_tensors, S, s_stride, A);
    if (!b.live) return;
    if (b.aligned) {
        const unsigned c = b.first / 4 + threadIdx.x, n4 = b.len >> 2;
        if (c < n4) {
            v4f a = {0.f, 0.f, 0.f, 0.f};
            if (MERGE) { a = *((cgv4f *)b.a + c); arrived(a); }
            v4f xr = gld4((cgv4f *)b.x + c); arrived(xr);
            v4f vr = gld4((cgv4f *)b.v + c); arrived(vr);
            v4f gr = gld4((cgv4f *)b.g + c); arrived(gr);
            sgd4(xr, vr, gr, lr, momentum, wd);
            gst4((gv4f *)b.v + c, vr);
            if (WS) gst4((gv4f *)b.s + c, xr);
            if (WX) gst4((gv4f *)b.x + c, MERGE ? merge4(xr, a, om) : xr);
        } else if (c == n4) {
            for (unsigned e = n4 * 4; e < b.len; ++e) {
                float xs = b.x[e], vs = b.v[e];
                sgd1(xs, vs, b.g[e], lr, momentum, wd);
                b.v[e] = vs;
                if (WS) b.s[e] = xs;
                if (WX) b.x[e] = MERGE ? merge1(xs, b.a[e], om) : xs;
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned e = b.first + k * kWave + threadIdx.x;
            if (e < b.len) {
                float xs = b.x[e], vs = b.v[e];
                sgd1(xs, vs, b.g[e], lr, momentum, wd);
                b.v[e] = vs;
                if (WS) b.s[e] = xs;
                if (WX) b.x[e] = MERGE ? merge1(xs, b.a[e], om) : xs;
            }
        }
    }
}

// Everything of one iteration in one pass, records addressing: the W replicas' copies of a 256-float block
// on the W wavefronts of a workgroup (grid = slots workgroups; workgroup q handles block q mod 16 of piece
// q div 16).  Wavefront j does replica j's local step and merge exactly as k_step_records does (128-bit
// accesses where that replica's addresses allow, 32-bit ones otherwise), leaves its y in LDS by position in
// the block, and after the barrier wavefront 0 adds the W values in tree order and stores the average.
// Same operations in the same order as the separate kernels (identical bits).  W = WT.
template <int LO, int HI> __device__ __forceinline__ float tree_sum1(const float *r) {
    if constexpr (HI - LO == 1) return r[LO];
    else {
        constexpr int MID = LO + (HI - LO + 1) / 2;
        return tree_sum1<LO, MID>(r) + tree_sum1<MID, HI>(r);
    }
}
template <int WT, bool MERGE>
__global__ void __launch_bounds__(kWave * WT)
k_step_all_records(const Rec *__restrict__ recs, unsigned recs_per_row, unsigned slots, const float *const *__restrict__ gp, int n_tensors,
                   const float *__restrict__ A_old, float *__restrict__ A_new, float lr, float momentum, float wd, float om, float inv_w)
{
    __shared__ __attribute__((aligned(16))) float part[WT][256];
    const unsigned q = blockIdx.x;
    if (q >= slots) return;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), l = threadIdx.x % kWave;
    const unsigned piece = q >> kPieceLog, first = (q & ((1u << kPieceLog) - 1u)) * 256u;
    const unsigned len = recs[piece].len, aoff = recs[piece].aoff;      // replica 0's: the same for every replica
    if (first >= len) return;                                           // (uniform over the workgroup)
    const Rec r = recs[(size_t)w * recs_per_row + piece];
    gf32 *x = (gf32 *)r.x, *v = (gf32 *)r.v;
    cgf32 *g = (cgf32 *)(gp[(size_t)w * n_tensors + r.tensor] + r.goff);
    cgf32 *a = MERGE ? (cgf32 *)(A_old + aoff) : nullptr;
    const bool aligned = ((reinterpret_cast<uintptr_t>(r.x) | reinterpret_cast<uintptr_t>(r.v) | (uintptr_t)g | (uintptr_t)a) & 15u) == 0;
    if (aligned) {
        const unsigned c = first / 4 + l, n4 = len >> 2;
        if (c < n4) {
            v4f av = {0.f, 0.f, 0.f, 0.f};
            if (MERGE) { av = *((cgv4f *)a + c); arrived(av); }
            v4f xr = gld4((cgv4f *)x + c); arrived(xr);
            v4f vr = gld4((cgv4f *)v + c); arrived(vr);
            v4f gr = gld4((cgv4f *)g + c); arrived(gr);
            sgd4(xr, vr, gr, lr, momentum, wd);
            gst4((gv4f *)v + c, vr);
            gst4((gv4f *)x + c, MERGE ? merge4(xr, av, om) : xr);
            *reinterpret_cast<v4f *>(&part[w][4 * l]) = xr;
        } else if (c == n4) {
            for (unsigned e = n4 * 4; e < len; ++e) {
                float xs = x[e], vs = v[e];
                sgd1(xs, vs, g[e], lr, momentum, wd);
                v[e] = vs;
                x[e] = MERGE ? merge1(xs, a[e], om) : xs;
                part[w][e - first] = xs;
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned e = first + k * kWave + l;
            if (e < len) {
                float xs = x[e], vs = v[e];
                sgd1(xs, vs, g[e], lr, momentum, wd);
                v[e] = vs;
                x[e] = MERGE ? merge1(xs, a[e], om) : xs;
                part[w][k * kWave + l] = xs;
            }
        }
    }
    __syncthreads();
    if (w == 0) {
        gf32 *out = (gf32 *)(A_new + aoff);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned e = first + k * kWave + l;
            if (e < len) {
                float p[WT];
#pragma unroll
                for (int j = 0; j < WT; ++j) p[j] = part[j][k * kWave + l];
                out[e] = tree_sum1<0, WT>(p) * inv_w;
            }
        }
    }
}

// Delayed merge, records addressing.  FROM_S: the value after the local step is read from the snapshot.
template <bool FROM_S>
__global__ void __launch_bounds__(kWave)
k_merge_records(const Rec *__restrict__ recs, unsigned recs_per_row, unsigned slots, const float *__restrict__ S, int64_t s_stride,
                const float *__restrict__ A, float om)
{
    const Block b = block_of<FROM_S, true>(recs, recs_per_row, slots, nullptr, 0, const_cast<float *>(S), s_stride, A);
    if (!b.live) return;
    cgf32 *y = FROM_S ? (cgf32 *)b.s : (cgf32 *)b.x;
    if (b.aligned) {
        const unsigned c = b.first / 4 + threadIdx.x, n4 = b.len >> 2;
        if (c < n4) {
            v4f a = *((cgv4f *)b.a + c); arrived(a);
            const v4f yr = gld4((cgv4f *)y + c);
            gst4((gv4f *)b.x + c, merge4(yr, a, om));
        } else if (c == n4) {
            for (unsigned e = n4 * 4; e < b.len; ++e) b.x[e] = merge1(y[e], b.a[e], om);
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const unsigned e = b.first + k * kWave + threadIdx.x;
            if (e < b.len) b.x[e] = merge1(y[e], b.a[e], om);
        }
    }
}

// W-way mean of the live weights, records addressing (zero-copy snapshot when the replicas are not rows):
// workgroup q handles block q mod 16 of piece q div 16, reads that block from every replica's tensor and
// writes it to the average at the piece's position.  Pairwise order over the replicas for W <= kMaxRows,
// four at a time above.  UNDO: the weights already hold the merged values; the merge is undone on the mean
// as in k_mean_undo_merge (differences to replica 0, one fma at the size of the result).
template <typename T> __device__ __forceinline__ T piece_load(const float *base, unsigned i);
template <> __device__ __forceinline__ v4f piece_load<v4f>(const float *base, unsigned i) { return gld4((cgv4f *)base + i); }
template <> __device__ __forceinline__ float piece_load<float>(const float *base, unsigned i) { return ((cgf32 *)base)[i]; }

template <typename T, int LO, int HI>
__device__ __forceinline__ T piece_tree(const Rec *__restrict__ recs, size_t rpr, unsigned piece, unsigned i) {
    if constexpr (HI - LO == 1) return piece_load<T>(recs[(size_t)LO * rpr + piece].x, i);
    else {
        constexpr int MID = LO + (HI - LO + 1) / 2;
        return piece_tree<T, LO, MID>(recs, rpr, piece, i) + piece_tree<T, MID, HI>(recs, rpr, piece, i);
    }
}
template <typename T>
__device__ __forceinline__ T piece_sum(const Rec *__restrict__ recs, size_t rpr, unsigned piece, unsigned i, int W) {
    switch (W) {
#define DASGD_CASE(N) case N: return piece_tree<T, 0, N>(recs, rpr, piece, i);
        DASGD_CASE(1) DASGD_CASE(2) DASGD_CASE(3) DASGD_CASE(4) DASGD_CASE(5) DASGD_CASE(6) DASGD_CASE(7) DASGD_CASE(8)
        DASGD_CASE(9) DASGD_CASE(10) DASGD_CASE(11) DASGD_CASE(12) DASGD_CASE(13) DASGD_CASE(14) DASGD_CASE(15) DASGD_CASE(16)
        DASGD_CASE(17) DASGD_CASE(18) DASGD_CASE(19) DASGD_CASE(20) DASGD_CASE(21) DASGD_CASE(22) DASGD_CASE(23) DASGD_CASE(24)
        DASGD_CASE(25) DASGD_CASE(26) DASGD_CASE(27) DASGD_CASE(28) DASGD_CASE(29) DASGD_CASE(30) DASGD_CASE(31) DASGD_CASE(32)
#undef DASGD_CASE
    default: break;
    }
    T acc = T(0.f);
    int j = 0;
    for (; j + 4 <= W; j += 4) {
        const T a = piece_load<T>(recs[(size_t)(j + 0) * rpr + piece].x, i), b = piece_load<T>(recs[(size_t)(j + 1) * rpr + piece].x, i);
        const T d = piece_load<T>(recs[(size_t)(j + 2) * rpr + piece].x, i), e = piece_load<T>(recs[(size_t)(j + 3) * rpr + piece].x, i);
        acc += (a + b) + (d + e);
    }
    for (; j < W; ++j) acc += piece_load<T>(recs[(size_t)j * rpr + piece].x, i);
    return acc;
}
// mean of the y recovered from the merged weights x' (see k_mean_undo_merge), one element of type T
template <typename T>
__device__ __forceinline__ T piece_undo(const Rec *__restrict__ recs, size_t rpr, unsigned piece, unsigned i, int W, T a_old,
                                        float inv_w, float om, float inv_xi) {
    const T r0 = piece_load<T>(recs[piece].x, i);
    T d = T(0.f);
#pragma unroll 4
    for (int j = 1; j < W; ++j) d += piece_load<T>(recs[(size_t)j * rpr + piece].x, i) - r0;
    T t;
    if constexpr (sizeof(T) == sizeof(float)) t = fmaf(-om, a_old, r0);
    else { t.x = fmaf(-om, a_old.x, r0.x); t.y = fmaf(-om, a_old.y, r0.y); t.z = fmaf(-om, a_old.z, r0.z); t.w = fmaf(-om, a_old.w, r0.w); }
    return (t + d * inv_w) * inv_xi;
}

template <bool UNDO>
__global__ void __launch_bounds__(kWave)
k_mean_records(const Rec *__restrict__ recs, unsigned recs_per_row, unsigned slots, int W, const float *__restrict__ A_old,
               float *__restrict__ A_new, float inv_w, float om, float inv_xi)
{
    __builtin_amdgcn_s_setprio(3);
    const unsigned q = blockIdx.x;
    if (q >= slots) return;
    const unsigned piece = q >> kPieceLog, first = (q & ((1u << kPieceLog) - 1u)) * 256u;
    const Rec r0 = recs[piece];
    if (first >= r0.len) return;
    const size_t rpr = recs_per_row;
    gf32 *out = (gf32 *)(A_new + r0.aoff);
    cgf32 *old = UNDO ? (cgf32 *)(A_old + r0.aoff) : nullptr;
    uintptr_t bits = (uintptr_t)out | (uintptr_t)old;
    for (int j = 0; j < W; ++j) bits |= reinterpret_cast<uintptr_t>(recs[(size_t)j * rpr + piece].x);
    if ((bits & 15u) == 0) {
        const unsigned c = first / 4 + threadIdx.x, n4 = r0.len >> 2;
        if (c < n4) {
            v4f y;
            if (UNDO) y = piece_undo<v4f>(recs, rpr, piece, c, W, *((cgv4f *)old + c), inv_w, om, inv_xi);
            else y = piece_sum<v4f>(recs, rpr, piece, c, W) * inv_w;
            *((gv4f *)out + c) = y;
        } else if (c == n4) {
            for (unsigned e = n4 * 4; e < r0.len; ++e)
                out[e] = UNDO ? piece_undo<float>(recs, rpr, piece, e, W, old[e], inv_w, om, inv_xi) : piece_sum<float>(recs, rpr, piece, e, W) * inv_w;
        }
    } else {
#pragma unroll 1
        for (int k = 0; k < 4; ++k) {
            const unsigned e = first + k * kWave + threadIdx.x;
            if (e < r0.len)
                out[e] = UNDO ? piece_undo<float>(recs, rpr, piece, e, W, old[e], inv_w, om, inv_xi) : piece_sum<float>(recs, rpr, piece, e, W) * inv_w;
        }
    }
}

// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) k_fill_zero(v4f *__restrict__ p, int64_t n4)
{
    const v4f z = {0.f, 0.f, 0.f, 0.f};
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kThreads)
        p[i] = z;
}

// One wavefront that lets about `ticks` ticks of the constant 100 MHz clock pass and exits: launched on
// the side stream in front of a mean, it gives the kernel that the caller enqueued on the main stream
// behind the local step a head start.  Which of two kernels that become ready at the same moment is
// dispatched first decides how they share the chip: a kernel already in place keeps its wave slots and the
// mean fills the rest, but a mean dispatched first takes every slot it can use and the other kernel only
// starts as the mean drains (measured on MI355X: a 0.75 ms kernel took 0.96-1.08 ms behind a 0.16 ms mean
// that won the race by 0.3 us, and 0.75 ms when it was 6 us ahead).  The loop is bounded whatever the
// clock reads.
__global__ void __launch_bounds__(kWave) k_head_start(unsigned ticks)
{
    const uint64_t t0 = wall_clock64();
    for (int i = 0; i < 512; ++i) {
        if (wall_clock64() - t0 >= (uint64_t)ticks) break;
        __builtin_amdgcn_s_sleep(16);               // 16 x 64 clocks, about half a microsecond
    }
}

}  // namespace dasgd
