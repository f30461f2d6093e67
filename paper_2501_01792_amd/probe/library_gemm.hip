// Measurement aid (libhkprobe_lt.so, a library of its own because it links the vendor GEMM library; not part of
// libhybridkv and no operation of the paper): times the candidate kernels the vendor library offers for a plain
// C[M, N] = A[M, K] x W[N, K]^T on 16-bit operands with fp32 accumulation, the plain-GEMM counterpart of the fused
// K/V projection (Eq. 7), so that the projection kernel can be set beside the best the library has for the shape,
// not only beside the one kernel its heuristic picks first.
#include <stddef.h>
#include <stdint.h>
#include <vector>
#include <hip/hip_runtime.h>
#include <hipblaslt/hipblaslt.h>

// A [M, K], W [N, K], C [M, N] row-major fp16 (bf16 with dtype 1), device; ws: device workspace of ws_bytes for the
// library (candidates that want more are skipped: their time is reported as 0).  Asks the library for up to
// max_candidates kernels in its own order of preference, runs each `iters` times after one warm-up launch and writes
// the mean milliseconds to ms_out[0 .. *n_out).  Synchronises the stream.  Returns 0, -1 null pointer, -2 bad shape,
// -7 a HIP or library call failed.
extern "C" int hkprobe_library_gemm_candidates(const void *A, const void *W, void *C, int64_t M, int32_t N, int32_t K, int32_t dtype,
                                               void *ws, size_t ws_bytes, int32_t max_candidates, int32_t iters,
                                               float *ms_out, int32_t *n_out, void *stream)
{
    if (!A || !W || !C || !ms_out || !n_out) return -1;
    if (M <= 0 || N <= 0 || K <= 0 || max_candidates <= 0 || max_candidates > 256 || iters <= 0 || iters > 100) return -2;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const hipDataType dt = dtype == 1 ? HIP_R_16BF : HIP_R_16F;
    hipblasLtHandle_t h = nullptr;
    hipblasLtMatmulDesc_t desc = nullptr;
    hipblasLtMatrixLayout_t lw = nullptr, la = nullptr, lc = nullptr;
    hipblasLtMatmulPreference_t pref = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = -7;
    *n_out = 0;
    do {
        // column-major view: C^T [N, M] = W (stored [K, N], transposed) x A (stored [K, M])
        if (hipblasLtCreate(&h) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipblasLtMatmulDescCreate(&desc, HIPBLAS_COMPUTE_32F, HIP_R_32F) != HIPBLAS_STATUS_SUCCESS) break;
        const hipblasOperation_t ta = HIPBLAS_OP_T, tb = HIPBLAS_OP_N;
        if (hipblasLtMatmulDescSetAttribute(desc, HIPBLASLT_MATMUL_DESC_TRANSA, &ta, sizeof(ta)) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipblasLtMatmulDescSetAttribute(desc, HIPBLASLT_MATMUL_DESC_TRANSB, &tb, sizeof(tb)) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipblasLtMatrixLayoutCreate(&lw, dt, K, N, K) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipblasLtMatrixLayoutCreate(&la, dt, K, M, K) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipblasLtMatrixLayoutCreate(&lc, dt, N, M, N) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipblasLtMatmulPreferenceCreate(&pref) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &ws_bytes, sizeof(ws_bytes)) !=
            HIPBLAS_STATUS_SUCCESS)
            break;
        std::vector<hipblasLtMatmulHeuristicResult_t> res(max_candidates);
        int got = 0;
        if (hipblasLtMatmulAlgoGetHeuristic(h, desc, lw, la, lc, lc, pref, max_candidates, res.data(), &got) != HIPBLAS_STATUS_SUCCESS) break;
        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) break;
        const float alpha = 1.f, beta = 0.f;
        bool ok = true;
        for (int i = 0; i < got && ok; ++i) {
            ms_out[i] = 0.f;
            if (res[i].workspaceSize > ws_bytes || (res[i].workspaceSize > 0 && !ws)) continue;
            auto run = [&]() {
                return hipblasLtMatmul(h, desc, &alpha, W, lw, A, la, &beta, C, lc, C, lc, &res[i].algo, ws, ws_bytes, s);
            };
            if (run() != HIPBLAS_STATUS_SUCCESS) continue;                   // the library refuses this one for the problem
            ok = hipEventRecord(e0, s) == hipSuccess;
            for (int r = 0; r < iters && ok; ++r) ok = run() == HIPBLAS_STATUS_SUCCESS;
            ok = ok && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
            float ms = 0.f;
            ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
            ms_out[i] = ms / iters;
        }
        if (!ok) break;
        *n_out = got;
        rc = 0;
    } while (false);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (pref) (void)hipblasLtMatmulPreferenceDestroy(pref);
    if (lw) (void)hipblasLtMatrixLayoutDestroy(lw);
    if (la) (void)hipblasLtMatrixLayoutDestroy(la);
    if (lc) (void)hipblasLtMatrixLayoutDestroy(lc);
    if (desc) (void)hipblasLtMatmulDescDestroy(desc);
    if (h) (void)hipblasLtDestroy(h);
    return rc;
}
