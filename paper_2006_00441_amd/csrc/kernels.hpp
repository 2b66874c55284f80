// Device code of the DaSGD parameter pipeline for gfx950 (CDNA4, 64-wide wavefronts).
//
// All three kernels are pure streaming passes bound by HBM bandwidth (<= 0.3 flop per byte), so
// the design is about memory traffic only: 128-bit accesses, several independent loads in
// flight per lane before the first use, every byte touched once, no LDS, no MFMA.
//
//   k_local_step   x, v, g -> x, v [, snapshot]        (paper Eq. 2, first branch; Section 4.1)
//   k_mean         snapshot rows -> average             ((X - eta G) J of the matrix form, appendix)
//   k_merge        x, average -> x                      (Eq. 2, second branch)
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

// ------------------------------------------------------------------------------------------------
// Local step on every replica: grid = (chunks, W).  20 bytes per element (24 with the snapshot).
template <bool SNAP, bool NT>
__global__ void __launch_bounds__(kThreads)
k_local_step(const Chunk *__restrict__ chunks, float *const *__restrict__ xp, float *const *__restrict__ vp,
             const float *const *__restrict__ gp, float *__restrict__ S, int64_t P_pad, int n_tensors,
             float lr, float momentum, float wd)
{
    const Chunk c = chunks[blockIdx.x];
    const int j = blockIdx.y;
    const int64_t row = (int64_t)j * n_tensors + c.tensor;
    float *__restrict__ x = xp[row] + c.off;
    float *__restrict__ v = vp[row] + c.off;
    const float *__restrict__ g = gp[row] + c.off;
    float *__restrict__ s = SNAP ? S + (int64_t)j * P_pad + c.foff : nullptr;
    const int tid = threadIdx.x;
    const int len = c.len;

    const bool aligned = ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(v) |
                           reinterpret_cast<uintptr_t>(g)) & 15u) == 0;
    if (aligned) {
        v4f *x4 = reinterpret_cast<v4f *>(x);
        v4f *v4 = reinterpret_cast<v4f *>(v);
        const v4f *g4 = reinterpret_cast<const v4f *>(g);
        v4f *s4 = reinterpret_cast<v4f *>(s);
        if (len == kChunk) {
            v4f xr[kUnroll], vr[kUnroll], gr[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int i = tid + u * kThreads;
                xr[u] = ld4<false>(x4 + i);
                vr[u] = ld4<false>(v4 + i);
                gr[u] = ld4<NT>(g4 + i);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int i = tid + u * kThreads;
                sgd4(xr[u], vr[u], gr[u], lr, momentum, wd);
                st4<false>(x4 + i, xr[u]);
                st4<false>(v4 + i, vr[u]);
                if (SNAP) st4<NT>(s4 + i, xr[u]);
            }
        } else {
            const int n4 = len >> 2;
            for (int i = tid; i < n4; i += kThreads) {
                v4f xr = x4[i], vr = v4[i];
                const v4f gr = g4[i];
                sgd4(xr, vr, gr, lr, momentum, wd);
                x4[i] = xr;
                v4[i] = vr;
                if (SNAP) s4[i] = xr;
            }
            const int e = (n4 << 2) + tid;         // at most 3 leftover elements
            if (e < len) {
                float xs = x[e], vs = v[e];
                sgd1(xs, vs, g[e], lr, momentum, wd);
                x[e] = xs;
                v[e] = vs;
                if (SNAP) s[e] = xs;
            }
        }
    } else {
        for (int e = tid; e < len; e += kThreads) {
            float xs = x[e], vs = v[e];
            sgd1(xs, vs, g[e], lr, momentum, wd);
            x[e] = xs;
            v[e] = vs;
            if (SNAP) s[e] = xs;
        }
    }
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
// needs no cross-lane traffic.  (4 + 4/W) bytes per replica-element.  WT > 0: W known at compile
// time, the whole column set is loaded before the tree sum; WT == 0: any W, four rows at a time.
template <int WT, int U, bool NT>
__global__ void __launch_bounds__(kThreads)
k_mean(const v4f *__restrict__ S, v4f *__restrict__ A, int64_t n4, int64_t row4, int W, float inv_w)
{
    const int64_t base = (int64_t)blockIdx.x * (kThreads * U) + threadIdx.x;
    if constexpr (WT > 0) {
        v4f r[U][WT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * kThreads;
            if (i < n4) {
#pragma unroll
                for (int j = 0; j < WT; ++j) r[u][j] = ld4<NT>(S + (int64_t)j * row4 + i);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * kThreads;
            if (i < n4) st4<false>(A + i, tree_sum<0, WT>(r[u]) * inv_w);
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + (int64_t)u * kThreads;
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

// ------------------------------------------------------------------------------------------------
// Delayed merge: x_j <- x_j + (1 - xi)(A - x_j) for every replica j; grid = chunks.  The chunk of A
// is read once into registers and applied to all W replicas: (8 + 4/W) bytes per replica-element.
__device__ __forceinline__ v4f merge4(v4f x, v4f a, float om) {
    v4f r;
    r.x = fmaf(om, a.x - x.x, x.x);
    r.y = fmaf(om, a.y - x.y, x.y);
    r.z = fmaf(om, a.z - x.z, x.z);
    r.w = fmaf(om, a.w - x.w, x.w);
    return r;
}

template <bool NT>
__global__ void __launch_bounds__(kThreads)
k_merge(const Chunk *__restrict__ chunks, float *const *__restrict__ xp, const float *__restrict__ A,
        int n_tensors, int W, float om)
{
    const Chunk c = chunks[blockIdx.x];
    const float *__restrict__ a = A + c.foff;              // 256-byte aligned by construction
    const v4f *a4 = reinterpret_cast<const v4f *>(a);
    const int tid = threadIdx.x;
    const int len = c.len;
    const bool full = (len == kChunk);

    v4f ar[kUnroll];
    if (full) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) ar[u] = ld4<NT>(a4 + tid + u * kThreads);
    }
    for (int j = 0; j < W; ++j) {
        float *__restrict__ x = xp[(int64_t)j * n_tensors + c.tensor] + c.off;
        const bool aligned = (reinterpret_cast<uintptr_t>(x) & 15u) == 0;
        if (aligned) {
            v4f *x4 = reinterpret_cast<v4f *>(x);
            if (full) {
                v4f xr[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) xr[u] = x4[tid + u * kThreads];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) x4[tid + u * kThreads] = merge4(xr[u], ar[u], om);
            } else {
                const int n4 = len >> 2;
                for (int i = tid; i < n4; i += kThreads) x4[i] = merge4(x4[i], a4[i], om);
                const int e = (n4 << 2) + tid;
                if (e < len) { const float xs = x[e]; x[e] = fmaf(om, a[e] - xs, xs); }
            }
        } else {
            for (int e = tid; e < len; e += kThreads) { const float xs = x[e]; x[e] = fmaf(om, a[e] - xs, xs); }
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

}  // namespace dasgd
