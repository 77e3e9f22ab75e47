// Plain CSR SpMM used as the measured baseline and as a cross-check: the basic scheme the
// paper starts from (Section 2, Algorithm 1): a wavefront owns one row of C and 64 of its
// columns, walks the row's nonzeros one at a time straight from the CSR arrays, and every
// lane does one multiply-add per nonzero.  No vector loads, no coarsening, no blocking, no
// balancing, no staging of colIdx/val.  Own code with its own launch scheme (a flat grid of
// wavefront tiles walked with a stride); it is not part of libpcsr.so.
//
// Per output element the nonzeros are added in stored order with one fused multiply-add
// each, which is also what the V=1, S=0 instance of the parameterised kernel does on rows
// that fit one chunk: the two must then agree bit for bit.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

__global__ void __launch_bounds__(512) plain_csr_spmm_kernel(const int32_t *__restrict__ rowptr,
                                                             const int32_t *__restrict__ colidx,
                                                             const float *__restrict__ val,
                                                             const float *__restrict__ B, float *C,
                                                             long n_rows, int K, int slices)
{
    const int lane = threadIdx.x % 64;
    const long waves_per_grid = (long)gridDim.x * (blockDim.x / 64);
    const long tiles = n_rows * slices; // one tile = (row, 64-column slice)
    for (long tile = (long)blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64; tile < tiles;
         tile += waves_per_grid) {
        const long row = tile / slices;
        const int k = (int)(tile - row * slices) * 64 + lane;
        if (k >= K) continue;
        float sum = 0.0f;
        const int end = rowptr[row + 1];
        for (int p = rowptr[row]; p < end; ++p) sum = fmaf(val[p], B[(long)colidx[p] * K + k], sum);
        C[row * K + k] = sum;
    }
}

} // namespace

extern "C" {

// All pointers device.  W = wavefronts per workgroup (1..8).  Returns 0 or a hipError_t.
int alg1_spmm(int64_t n_rows, const int32_t *rowptr, const int32_t *colidx, const float *val,
              const float *B, float *C, int32_t K, int32_t W, void *stream)
{
    if (n_rows <= 0 || K <= 0) return 0;
    if (W < 1 || W > 8) return -1;
    const int slices = (K + 63) / 64;
    const long tiles = n_rows * slices;
    long blocks = (tiles + W - 1) / W;
    if (blocks > (1L << 22)) blocks = 1L << 22; // the stride loop covers the rest
    hipLaunchKernelGGL(plain_csr_spmm_kernel, dim3((unsigned)blocks), dim3(64 * W), 0, (hipStream_t)stream,
                       rowptr, colidx, val, B, C, (long)n_rows, (int)K, slices);
    return (int)hipGetLastError();
}
}
