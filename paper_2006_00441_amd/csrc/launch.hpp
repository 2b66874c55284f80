// Launching the W-way mean (the average of Eq. 2, second branch) for every row count and layout, the
// file-scope scratch of the entry point that allocates nothing, and the stand-alone average.
// Included by dasgd.hip only.
#pragma once
#include "context.hpp"

namespace {

// Are the rows 128-byte aligned relative to each other?  (If not, neighbouring column windows of the mean
// kernels share cache lines, and the kernels issue runs of windows on one L2 partition.)
bool rows_share_lines(const ConstRowSet &r, int W)
{
    for (int j = 0; j < W; ++j)
        if ((reinterpret_cast<uintptr_t>(r.p[j]) - reinterpret_cast<uintptr_t>(r.p[0])) & 127u) return true;
    return (reinterpret_cast<uintptr_t>(r.p[0]) & 127u) != 0;
}

inline unsigned mean_grid(unsigned row4) { return ((row4 + kWave - 1) / kWave + 63u) / 64u * 64u; }

// W-way mean of `row_elems` floats per row (a multiple of 4, rows 16-byte aligned) into A.
// rows: the W row pointers (W <= kMaxRows); or strided != nullptr: rows at strided + j * stride floats.
hipError_t launch_mean_of(int W, hipStream_t s, const ConstRowSet *rows, const float *strided, int64_t stride, float *A, int64_t row_elems)
{
    const unsigned row4 = (unsigned)(row_elems / 4);
    v4f *A4 = reinterpret_cast<v4f *>(A);
    const float inv_w = 1.0f / (float)W;
    ConstRowSet r = {};
    if (rows) r = *rows;
    else if (W <= kMaxRows)
        for (int j = 0; j < W; ++j) r.p[j] = strided + (int64_t)j * stride;
    if (W > kMaxRows) {
        hipLaunchKernelGGL(k_mean_strided, dim3((row4 + kWave - 1) / kWave), dim3(kWave), 0, s,
                           reinterpret_cast<const v4f *>(strided), stride / 4, A4, row4, W, inv_w);
        return hipGetLastError();
    }
    const bool runs = rows_share_lines(r, W);
    const dim3 grid(mean_grid(row4));
#define DASGD_LAUNCH_MEAN(WT, NW)                                                                               \
    do {                                                                                                        \
        if (runs) hipLaunchKernelGGL((k_mean_rows<WT, NW, true>), grid, dim3(kWave * NW), 0, s, r, A4, row4, inv_w);  \
        else      hipLaunchKernelGGL((k_mean_rows<WT, NW, false>), grid, dim3(kWave * NW), 0, s, r, A4, row4, inv_w); \
    } while (0)
    switch (W) {                // rows split over wavefronts + LDS where that measured faster
    case 4:  DASGD_LAUNCH_MEAN(4, 4);  break;
    case 8:  DASGD_LAUNCH_MEAN(8, 4);  break;
    case 16: DASGD_LAUNCH_MEAN(16, 8); break;
    default:
        if (runs) hipLaunchKernelGGL((k_mean_any<true>), grid, dim3(kWave), 0, s, r, A4, row4, W, inv_w);
        else      hipLaunchKernelGGL((k_mean_any<false>), grid, dim3(kWave), 0, s, r, A4, row4, W, inv_w);
        break;
    }
#undef DASGD_LAUNCH_MEAN
    return hipGetLastError();
}
int launch_mean(dasgd_ctx *c, hipStream_t s, const ConstRowSet *rows, const float *strided, int64_t stride, float *A, int64_t row_elems)
{
    HIPCHK(c, launch_mean_of(c->W, s, rows, strided, stride, A, row_elems));
    return DASGD_OK;
}

thread_local int g_last_hip = 0;        // HIP error of the latest failed call that has no context

// Scratch memory of dasgd_average_now_static: the average of one call.  Every GPU the library runs on holds
// its own copy of the array, at its own address, until the process ends.  Host code must not use the name
// as an address: the per-device address comes from hipGetSymbolAddress, once per device.
constexpr int64_t kStaticScratchFloats = 32ll << 20;        // 128 MiB
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
float *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
int static_scratch(float **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) return DASGD_EINVAL;
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e == hipSuccess) g_scratch_ptr[dev] = static_cast<float *>(p);
        }
        *out = g_scratch_ptr[dev];
    }
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return DASGD_EHIP;
    }
    return DASGD_OK;
}

// The blocking average of dasgd_average_now: A <- mean of the rows, rows <- xi row + (1 - xi) A.  Launches
// two kernels on `s` and allocates nothing.
int average_now(int W, int64_t P, float *const *x_rows, float xi, float *A, hipStream_t s)
{
    if (W < 1 || W > kMaxRows || P < 4 || P % 4 != 0 || P / 4 > (1ll << 31) - 256) return DASGD_EINVAL;
    if (!x_rows || !A || !(xi >= 0.f && xi <= 1.f)) return DASGD_EINVAL;
    std::pair<uintptr_t, size_t> iv[kMaxRows + 1];
    RowSet xr = {};
    ConstRowSet cr = {};
    for (int j = 0; j < W; ++j) {
        if (!x_rows[j] || (reinterpret_cast<uintptr_t>(x_rows[j]) & 15u)) return DASGD_EINVAL;
        if (!range_ok(x_rows[j], sizeof(float) * (size_t)P)) return DASGD_EINVAL;
        xr.p[j] = x_rows[j];
        cr.p[j] = x_rows[j];
        iv[j] = {reinterpret_cast<uintptr_t>(x_rows[j]), sizeof(float) * (size_t)P};
    }
    iv[W] = {reinterpret_cast<uintptr_t>(A), sizeof(float) * (size_t)P};
    std::sort(iv, iv + W + 1);
    for (int i = 1; i <= W; ++i)
        if (iv[i].first < iv[i - 1].first + iv[i - 1].second) return DASGD_EINVAL;     // rows and scratch must not share bytes
    hipError_t e = launch_mean_of(W, s, &cr, nullptr, 0, A, P);
    if (e == hipSuccess) {
        const unsigned row4 = (unsigned)(P / 4);
        const dim3 grid = band_grid(rows_blocks(row4), W, 9).grid;
        hipLaunchKernelGGL((k_merge_rows<false>), grid, dim3(kWave), 0, s, xr, static_cast<const v4f *>(nullptr), (int64_t)0,
                           reinterpret_cast<const v4f *>(A), row4, 1.0f - xi);
        e = hipGetLastError();
    }
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return DASGD_EHIP;
    }
    return DASGD_OK;
}

}  // namespace
