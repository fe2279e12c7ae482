// Context measurement, not part of the library: the vendor's 2:4 structured-sparse GEMM (hipSPARSELt) on the
// shapes of the forward product  Y = X (B .* W)^T  of Eq. (3) of arXiv 2302.06058, with the same memory layouts
// this library uses (W row-major I x J, X row-major T x J, Y row-major T x I), bf16 in, fp32 accumulate, bf16 out.
//
//   vendor_sparse_gemm [I J T]...      default: 11008 4096 8192   4096 11008 8192
//
// Per shape and operand layout (the library's own, and W and / or X stored the other way round): W is pruned 2:4 along J by the vendor's own pruning call and compressed by its own compression
// call; the product is planned twice -- with the library's default kernel and after its own search over its
// kernels -- and each plan is timed over 20 launches between two events.  Sixteen outputs are checked against a
// host dot product over the pruned weights.  Prints one line per measurement.
#include <hip/hip_runtime.h>
#include <hipsparselt/hipsparselt.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define HIP_OK(x)                                                                     \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) { std::printf("hip error %d at line %d\n", (int)e_, __LINE__); return 1; } \
    } while (0)
#define SP_OK(x)                                                                      \
    do {                                                                              \
        hipsparseStatus_t s_ = (x);                                                   \
        if (s_ != HIPSPARSE_STATUS_SUCCESS) { std::printf("hipsparselt status %d at line %d (%s)\n", (int)s_, __LINE__, #x); return 2; } \
    } while (0)

static uint16_t f2bf(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}
static float bf2f(uint16_t h) {
    uint32_t u = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

static int run_shape(int64_t I, int64_t J, int64_t T, bool tA, bool tB) {
    // host data: small integers scaled, so that the check is tight
    std::vector<uint16_t> hW(static_cast<size_t>(I) * J), hX(static_cast<size_t>(T) * J);
    uint32_t st = 12345u + static_cast<uint32_t>(I * 7 + J * 3 + T);
    auto rnd = [&]() { st = st * 1664525u + 1013904223u; return static_cast<int>((st >> 9) % 2001) - 1000; };
    for (auto& w : hW) w = f2bf(rnd() * 2e-5f);
    for (auto& x : hX) x = f2bf(rnd() * 1e-3f);
    uint16_t *dW, *dWp, *dX, *dY;
    HIP_OK(hipMalloc(&dW, hW.size() * 2));
    HIP_OK(hipMalloc(&dWp, hW.size() * 2));
    HIP_OK(hipMalloc(&dX, hX.size() * 2));
    HIP_OK(hipMalloc(&dY, static_cast<size_t>(T) * I * 2));
    HIP_OK(hipMemcpy(dW, hW.data(), hW.size() * 2, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dX, hX.data(), hX.size() * 2, hipMemcpyHostToDevice));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    hipsparseLtHandle_t handle;
    SP_OK(hipsparseLtInit(&handle));
    // Column-major descriptors.  tA, !tB is this library's layout: W (I x J row-major) is the column-major J x I
    // matrix with ld = J, taken transposed; X (T x J row-major) is column-major J x T; Y (T x I row-major) is I x T.
    // The other three combinations store W and / or X the other way round (same buffers, same product shape).
    hipsparseLtMatDescriptor_t mA, mB, mC;
    SP_OK(hipsparseLtStructuredDescriptorInit(&handle, &mA, tA ? J : I, tA ? I : J, tA ? J : I, 16, HIP_R_16BF, HIPSPARSE_ORDER_COL,
                                              HIPSPARSELT_SPARSITY_50_PERCENT));
    SP_OK(hipsparseLtDenseDescriptorInit(&handle, &mB, tB ? T : J, tB ? J : T, tB ? T : J, 16, HIP_R_16BF, HIPSPARSE_ORDER_COL));
    SP_OK(hipsparseLtDenseDescriptorInit(&handle, &mC, I, T, I, 16, HIP_R_16BF, HIPSPARSE_ORDER_COL));
    hipsparseLtMatmulDescriptor_t mm;
    SP_OK(hipsparseLtMatmulDescriptorInit(&handle, &mm, tA ? HIPSPARSE_OPERATION_TRANSPOSE : HIPSPARSE_OPERATION_NON_TRANSPOSE,
                                          tB ? HIPSPARSE_OPERATION_TRANSPOSE : HIPSPARSE_OPERATION_NON_TRANSPOSE, &mA, &mB, &mC, &mC,
                                          HIPSPARSELT_COMPUTE_32F));
    hipsparseLtMatmulAlgSelection_t alg;
    SP_OK(hipsparseLtMatmulAlgSelectionInit(&handle, &alg, &mm, HIPSPARSELT_MATMUL_ALG_DEFAULT));
    hipsparseLtMatmulPlan_t plan;
    SP_OK(hipsparseLtMatmulPlanInit(&handle, &plan, &mm, &alg));

    SP_OK(hipsparseLtSpMMAPrune(&handle, &mm, dW, dWp, HIPSPARSELT_PRUNE_SPMMA_STRIP, stream));
    size_t csize = 0, cbuf = 0;
    SP_OK(hipsparseLtSpMMACompressedSize(&handle, &plan, &csize, &cbuf));
    void *dComp = nullptr, *dCbuf = nullptr, *dWs = nullptr;
    HIP_OK(hipMalloc(&dComp, csize));
    if (cbuf) HIP_OK(hipMalloc(&dCbuf, cbuf));
    SP_OK(hipsparseLtSpMMACompress(&handle, &plan, dWp, dComp, dCbuf, stream));
    size_t ws = 0;
    SP_OK(hipsparseLtMatmulGetWorkspace(&handle, &plan, &ws));
    if (ws) HIP_OK(hipMalloc(&dWs, ws));
    HIP_OK(hipStreamSynchronize(stream));

    const float alpha = 1.f, beta = 0.f;
    hipEvent_t e0, e1;
    HIP_OK(hipEventCreate(&e0));
    HIP_OK(hipEventCreate(&e1));
    auto time_plan = [&](const char* what) -> int {
        for (int i = 0; i < 3; ++i) SP_OK(hipsparseLtMatmul(&handle, &plan, &alpha, dComp, dX, &beta, dY, dY, dWs, &stream, 1));
        HIP_OK(hipEventRecord(e0, stream));
        const int reps = 20;
        for (int i = 0; i < reps; ++i) SP_OK(hipsparseLtMatmul(&handle, &plan, &alpha, dComp, dX, &beta, dY, dY, dWs, &stream, 1));
        HIP_OK(hipEventRecord(e1, stream));
        HIP_OK(hipEventSynchronize(e1));
        float ms = 0;
        HIP_OK(hipEventElapsedTime(&ms, e0, e1));
        const double us = ms * 1e3 / reps;
        std::printf("vendor 2:4 GEMM  W %lld x %lld, T = %lld, op(W) = %s, op(X^T) = %s, %s: %.1f us per launch = %.0f TFLOP/s dense-equivalent\n",
                    (long long)I, (long long)J, (long long)T, tA ? "T" : "N", tB ? "T" : "N", what, us, 2.0 * I * J * T / us / 1e6);
        return 0;
    };
    if (int rc = time_plan("default kernel")) return rc;

    // check 16 outputs against the pruned weights (in this library's layout only)
    if (tA && !tB) {
        std::vector<uint16_t> hWp(hW.size()), hY(static_cast<size_t>(4) * I);
        HIP_OK(hipMemcpy(hWp.data(), dWp, hWp.size() * 2, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(hY.data(), dY, hY.size() * 2, hipMemcpyDeviceToHost));
        double worst = 0;
        int64_t kept = 0;
        for (int64_t j = 0; j < J; ++j) kept += hWp[j] != 0 && hWp[j] != 0x8000;
        for (int t = 0; t < 4; ++t)
            for (int i = 0; i < 4; ++i) {
                double ref = 0;
                for (int64_t j = 0; j < J; ++j) ref += static_cast<double>(bf2f(hX[t * J + j])) * bf2f(hWp[i * J + j]);
                const double got = bf2f(hY[t * I + i]);
                const double err = std::fabs(got - ref) / (std::fabs(ref) + 1e-6);
                if (err > worst) worst = err;
            }
        std::printf("   check: 16 outputs, worst relative error %.2e; row 0 of the pruned W keeps %lld of %lld\n", worst,
                    (long long)kept, (long long)J);
    }
    // the library's own search over its kernels, then the same timing
    {
        hipsparseStatus_t s = hipsparseLtMatmulSearch(&handle, &plan, &alpha, dComp, dX, &beta, dY, dY, dWs, &stream, 1);
        if (s == HIPSPARSE_STATUS_SUCCESS) {
            if (int rc = time_plan("after the library's kernel search")) return rc;
        } else {
            std::printf("   kernel search not available (status %d)\n", (int)s);
        }
    }
    hipsparseLtMatmulPlanDestroy(&plan);
    hipsparseLtMatDescriptorDestroy(&mA);
    hipsparseLtMatDescriptorDestroy(&mB);
    hipsparseLtMatDescriptorDestroy(&mC);
    hipsparseLtDestroy(&handle);
    (void)hipFree(dW); (void)hipFree(dWp); (void)hipFree(dX); (void)hipFree(dY); (void)hipFree(dComp);
    if (dCbuf) (void)hipFree(dCbuf);
    if (dWs) (void)hipFree(dWs);
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    (void)hipStreamDestroy(stream);
    return 0;
}

int main(int argc, char** argv) {
    std::vector<int64_t> v;
    for (int i = 1; i < argc; ++i) v.push_back(std::atoll(argv[i]));
    if (v.empty()) v = {11008, 4096, 8192, 4096, 11008, 8192};
    if (v.size() % 3) { std::printf("usage: vendor_sparse_gemm [I J T]...\n"); return 1; }
    int rc = 0;
    for (size_t k = 0; k < v.size(); k += 3)
        for (int lay = 0; lay < 4; ++lay) {
            const int r = run_shape(v[k], v[k + 1], v[k + 2], (lay & 1) == 0, (lay & 2) != 0);
            if (r) rc = r;
        }
    return rc;
}
