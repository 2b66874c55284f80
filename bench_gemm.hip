// Harness-side, used by bench.py only (not part of the library): the overlap-stress workload's
// forward/backward stand-in, one bf16 GEMM n x n x n, issued through hipBLASLt with a chosen algorithm.
//
// torch.matmul takes the algorithm that hipBLASLt's heuristic ranks first for the GEMM alone.  On MI355X
// that kernel holds a whole register file per SIMD, so nothing can run beside it.  hipBLASLt ships many
// more algorithms for the same problem; this file lists them (hipblaslt_ext::getAllAlgos, filtered with
// matmulIsAlgoSupported) and runs any one of them, so that bench.py can pick the algorithm that makes the
// whole step -- GEMM, W-way mean beside it, local step -- fastest rather than the GEMM alone.
#include <hip/hip_runtime.h>
#include <hipblaslt/hipblaslt.h>
#include <hipblaslt/hipblaslt-ext.hpp>

#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

namespace {
struct Gemm {
    hipblasLtHandle_t handle = nullptr;
    hipblasLtMatmulDesc_t desc = nullptr;
    hipblasLtMatrixLayout_t a = nullptr, b = nullptr, c = nullptr;
    std::vector<hipblasLtMatmulHeuristicResult_t> algos;      // supported ones only
    std::vector<size_t> workspace;
    int n = 0, first_by_heuristic = -1;
} G;
const float kOne = 1.0f, kZero = 0.0f;

void close_all()
{
    if (G.a) hipblasLtMatrixLayoutDestroy(G.a);
    if (G.b) hipblasLtMatrixLayoutDestroy(G.b);
    if (G.c) hipblasLtMatrixLayoutDestroy(G.c);
    if (G.desc) hipblasLtMatmulDescDestroy(G.desc);
    if (G.handle) hipblasLtDestroy(G.handle);
    G = Gemm{};
}
}  // namespace

extern "C" {

// Prepare C = op(A) * op(B) for n x n bf16 matrices (column-major, op = transpose if trans_a / trans_b is
// non-zero, fp32 accumulation, bf16 result) and collect every algorithm of the library that supports the
// problem with at most max_workspace bytes of workspace.  Returns the number of algorithms (>= 1) or a
// negative hipBLAS status.
int bench_gemm_open(int n, size_t max_workspace, int trans_a, int trans_b)
{
    close_all();
    if (n < 256 || n % 256) return -1;
    G.n = n;
#define BLT(expr)                                    \
    do {                                             \
        const hipblasStatus_t s_ = (expr);           \
        if (s_ != HIPBLAS_STATUS_SUCCESS) {          \
            close_all();                             \
            return -(int)s_ - 100;                   \
        }                                            \
    } while (0)
    BLT(hipblasLtCreate(&G.handle));
    BLT(hipblasLtMatmulDescCreate(&G.desc, HIPBLAS_COMPUTE_32F, HIP_R_32F));
    const hipblasOperation_t op_a = trans_a ? HIPBLAS_OP_T : HIPBLAS_OP_N, op_b = trans_b ? HIPBLAS_OP_T : HIPBLAS_OP_N;
    BLT(hipblasLtMatmulDescSetAttribute(G.desc, HIPBLASLT_MATMUL_DESC_TRANSA, &op_a, sizeof(op_a)));
    BLT(hipblasLtMatmulDescSetAttribute(G.desc, HIPBLASLT_MATMUL_DESC_TRANSB, &op_b, sizeof(op_b)));
    BLT(hipblasLtMatrixLayoutCreate(&G.a, HIP_R_16BF, n, n, n));
    BLT(hipblasLtMatrixLayoutCreate(&G.b, HIP_R_16BF, n, n, n));
    BLT(hipblasLtMatrixLayoutCreate(&G.c, HIP_R_16BF, n, n, n));

    std::vector<hipblasLtMatmulHeuristicResult_t> all;
    BLT(hipblaslt_ext::getAllAlgos(G.handle, hipblaslt_ext::GemmType::HIPBLASLT_GEMM, op_a, op_b, HIP_R_16BF, HIP_R_16BF,
                                   HIP_R_16BF, HIP_R_16BF, HIPBLAS_COMPUTE_32F, all));
    for (auto &r : all) {
        size_t ws = 0;
        if (hipblaslt_ext::matmulIsAlgoSupported(G.handle, G.desc, &kOne, G.a, G.b, &kZero, G.c, G.c, r.algo, ws) !=
            HIPBLAS_STATUS_SUCCESS)
            continue;
        if (ws > max_workspace) continue;
        G.algos.push_back(r);
        G.workspace.push_back(ws);
    }
    // the algorithm the heuristic ranks first (what a framework's matmul gets)
    hipblasLtMatmulPreference_t pref = nullptr;
    BLT(hipblasLtMatmulPreferenceCreate(&pref));
    hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &max_workspace, sizeof(max_workspace));
    hipblasLtMatmulHeuristicResult_t top[1];
    int got = 0;
    const hipblasStatus_t hs = hipblasLtMatmulAlgoGetHeuristic(G.handle, G.desc, G.a, G.b, G.c, G.c, pref, 1, top, &got);
    hipblasLtMatmulPreferenceDestroy(pref);
    if (hs == HIPBLAS_STATUS_SUCCESS && got == 1) {
        const int want = hipblaslt_ext::getIndexFromAlgo(top[0].algo);
        for (size_t i = 0; i < G.algos.size(); ++i)
            if (hipblaslt_ext::getIndexFromAlgo(G.algos[i].algo) == want) G.first_by_heuristic = (int)i;
    }
#undef BLT
    return G.algos.empty() ? -2 : (int)G.algos.size();
}

// Position (in this file's list) of the algorithm the heuristic ranks first, or -1.
int bench_gemm_first_by_heuristic(void) { return G.first_by_heuristic; }

// Workspace bytes algorithm i needs (0 if i is out of range).
size_t bench_gemm_workspace(int i) { return i >= 0 && (size_t)i < G.workspace.size() ? G.workspace[i] : 0; }

// The library's own index of algorithm i (stable for one library version), or -1.
int bench_gemm_library_index(int i)
{
    return i >= 0 && (size_t)i < G.algos.size() ? hipblaslt_ext::getIndexFromAlgo(G.algos[i].algo) : -1;
}

// Kernel name of algorithm i into buf (truncated to cap-1 characters).  Returns its full length.
int bench_gemm_name(int i, char *buf, int cap)
{
    if (i < 0 || (size_t)i >= G.algos.size() || !buf || cap < 1) return 0;
    const std::string s = hipblaslt_ext::getKernelNameFromAlgo(G.handle, G.algos[i].algo);
    std::snprintf(buf, (size_t)cap, "%s", s.c_str());
    return (int)s.size();
}

// Enqueue C = A * B with algorithm i on `stream`.  A, B, C: n*n bf16 each, device memory; workspace: device
// memory of at least bench_gemm_workspace(i) bytes (may be NULL if that is 0).  Returns 0 or a negative
// hipBLAS status; nothing is enqueued on an error.
int bench_gemm_run(int i, const void *A, const void *B, void *C, void *workspace, size_t workspace_bytes, void *stream)
{
    if (i < 0 || (size_t)i >= G.algos.size() || !A || !B || !C) return -1;
    if (G.workspace[i] > workspace_bytes || (G.workspace[i] && !workspace)) return -3;
    const hipblasStatus_t s = hipblasLtMatmul(G.handle, G.desc, &kOne, A, G.a, B, G.b, &kZero, C, G.c, C, G.c, &G.algos[i].algo,
                                              workspace, workspace_bytes, static_cast<hipStream_t>(stream));
    return s == HIPBLAS_STATUS_SUCCESS ? 0 : -(int)s - 100;
}

void bench_gemm_close(void) { close_all(); }

}  // extern "C"
