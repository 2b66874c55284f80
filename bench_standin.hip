// Harness-side kernels used by bench.py only (not part of the library).
//
// 1. A stand-in for a forward/backward pass:
// an ALU-bound kernel that, unlike a maximal-occupancy GEMM, leaves wave slots and registers free on
// every SIMD, the way the many small kernels of a real forward/backward pass do.  It shows what the
// side-stream schedule hides when the hardware can co-schedule the mean at all.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
__global__ void __launch_bounds__(256) k_alu_standin(float *__restrict__ out, int iters)
{
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    float a0 = gid * 1e-6f, a1 = a0 + 1.f, a2 = a0 + 2.f, a3 = a0 + 3.f, a4 = a0 + 4.f, a5 = a0 + 5.f, a6 = a0 + 6.f, a7 = a0 + 7.f;
    const float m = 0.999f, c = 1e-3f;
    for (int i = 0; i < iters; ++i) {          // eight independent FMA chains keep the vector ALU busy
        a0 = fmaf(a0, m, c); a1 = fmaf(a1, m, c); a2 = fmaf(a2, m, c); a3 = fmaf(a3, m, c);
        a4 = fmaf(a4, m, c); a5 = fmaf(a5, m, c); a6 = fmaf(a6, m, c); a7 = fmaf(a7, m, c);
    }
    out[gid] = ((a0 + a1) + (a2 + a3)) + ((a4 + a5) + (a6 + a7));
}

// 2. A plain copy in the launch shape the library's streaming kernels use (one 64-lane wave per workgroup,
// one 128-bit non-temporal load and store per lane): the bandwidth a pure read+write stream reaches on the
// box at hand, reported beside the vendor peak.
typedef float v4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(64) k_copy_stream(v4 *__restrict__ dst, const v4 *__restrict__ src, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}
}  // namespace

// Copy n_floats floats (a multiple of 4, both pointers 16-byte aligned, device memory, at most 2^31-1
// workgroups of 256 floats) from src to dst on `stream`.  Returns the HIP error code of the launch, or 1 for
// a bad size.
extern "C" int bench_copy_stream(void *dst, const void *src, size_t n_floats, void *stream)
{
    if (n_floats == 0 || n_floats % 4 || (n_floats / 256 + 1) > 0x7fffffffull) return 1;
    const size_t n4 = n_floats / 4;
    hipLaunchKernelGGL(k_copy_stream, dim3((unsigned)((n4 + 63) / 64)), dim3(64), 0, static_cast<hipStream_t>(stream),
                       static_cast<v4 *>(dst), static_cast<const v4 *>(src), n4);
    return (int)hipGetLastError();
}

// Launch the stand-in on `stream`: `blocks` workgroups of 256 threads, `iters` loop trips each; out must
// hold blocks*256 floats (device).  Returns the HIP error code of the launch.
extern "C" int bench_alu_standin(void *out, int blocks, int iters, void *stream)
{
    hipLaunchKernelGGL(k_alu_standin, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<float *>(out), iters);
    return (int)hipGetLastError();
}
