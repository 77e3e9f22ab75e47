// hipSPARSE SpMM on the same CSR / row-major B, C: the vendor baseline timed beside the
// PCSR kernels.  Bench infrastructure only; nothing in libpcsr.so depends on it.
#include <hip/hip_runtime.h>
#include <hipsparse/hipsparse.h>

#include <cstdint>
#include <new>

namespace {
struct Ctx {
    hipsparseHandle_t handle = nullptr;
    hipsparseSpMatDescr_t A = nullptr;
    hipsparseDnMatDescr_t B = nullptr, C = nullptr;
    void *buffer = nullptr;
    size_t buffer_bytes = 0;
    hipsparseSpMMAlg_t alg = HIPSPARSE_SPMM_ALG_DEFAULT;
    float alpha = 1.0f, beta = 0.0f;
};
} // namespace

extern "C" {

// alg: 0 default, 4 CSR_ALG1, 6 CSR_ALG2, 12 CSR_ALG3.  All pointers are device memory.
// Returns 0 or 1000 + hipsparseStatus / 2000 + hipError.
int hsp_spmm_create(int64_t n_rows, int64_t n_cols, int64_t nnz, const int32_t *rowptr,
                    const int32_t *colidx, const float *vals, const float *B, float *C, int32_t K,
                    int32_t alg, void *stream, void **out)
{
    Ctx *c = new (std::nothrow) Ctx();
    if (!c) return 1;
    c->alg = (hipsparseSpMMAlg_t)alg;
    hipsparseStatus_t s = hipsparseCreate(&c->handle);
    if (s == HIPSPARSE_STATUS_SUCCESS) s = hipsparseSetStream(c->handle, (hipStream_t)stream);
    if (s == HIPSPARSE_STATUS_SUCCESS)
        s = hipsparseCreateCsr(&c->A, n_rows, n_cols, nnz, (void *)rowptr, (void *)colidx, (void *)vals,
                               HIPSPARSE_INDEX_32I, HIPSPARSE_INDEX_32I, HIPSPARSE_INDEX_BASE_ZERO,
                               HIP_R_32F);
    if (s == HIPSPARSE_STATUS_SUCCESS)
        s = hipsparseCreateDnMat(&c->B, n_cols, K, K, (void *)B, HIP_R_32F, HIPSPARSE_ORDER_ROW);
    if (s == HIPSPARSE_STATUS_SUCCESS)
        s = hipsparseCreateDnMat(&c->C, n_rows, K, K, (void *)C, HIP_R_32F, HIPSPARSE_ORDER_ROW);
    if (s == HIPSPARSE_STATUS_SUCCESS)
        s = hipsparseSpMM_bufferSize(c->handle, HIPSPARSE_OPERATION_NON_TRANSPOSE,
                                     HIPSPARSE_OPERATION_NON_TRANSPOSE, &c->alpha, c->A, c->B, &c->beta,
                                     c->C, HIP_R_32F, c->alg, &c->buffer_bytes);
    if (s != HIPSPARSE_STATUS_SUCCESS) return 1000 + (int)s;
    hipError_t e = hipMalloc(&c->buffer, c->buffer_bytes ? c->buffer_bytes : 16);
    if (e != hipSuccess) return 2000 + (int)e;
    s = hipsparseSpMM_preprocess(c->handle, HIPSPARSE_OPERATION_NON_TRANSPOSE,
                                 HIPSPARSE_OPERATION_NON_TRANSPOSE, &c->alpha, c->A, c->B, &c->beta, c->C,
                                 HIP_R_32F, c->alg, c->buffer);
    if (s != HIPSPARSE_STATUS_SUCCESS) return 1000 + (int)s;
    *out = c;
    return 0;
}

int hsp_spmm_run(void *ctx)
{
    Ctx *c = (Ctx *)ctx;
    hipsparseStatus_t s =
        hipsparseSpMM(c->handle, HIPSPARSE_OPERATION_NON_TRANSPOSE, HIPSPARSE_OPERATION_NON_TRANSPOSE,
                      &c->alpha, c->A, c->B, &c->beta, c->C, HIP_R_32F, c->alg, c->buffer);
    return s == HIPSPARSE_STATUS_SUCCESS ? 0 : 1000 + (int)s;
}

int64_t hsp_spmm_buffer_bytes(void *ctx) { return (int64_t)((Ctx *)ctx)->buffer_bytes; }

int hsp_spmm_destroy(void *ctx)
{
    Ctx *c = (Ctx *)ctx;
    if (!c) return 0;
    if (c->buffer) (void)hipFree(c->buffer);
    if (c->C) hipsparseDestroyDnMat(c->C);
    if (c->B) hipsparseDestroyDnMat(c->B);
    if (c->A) hipsparseDestroySpMat(c->A);
    if (c->handle) hipsparseDestroy(c->handle);
    delete c;
    return 0;
}
}
