// The paper's Algorithm 1 ("Basic CSR-based SpMM"), written for 64-lane wavefronts exactly as
// printed: one wavefront per row of C, lane l of block column blk.y owns column blk.y*64 + l,
// the row's nonzeros are walked one by one and each lane does one multiply-accumulate per
// nonzero.  No vector loads, no coarsening, no blocking, no balancing.  It is the baseline the
// parameterised kernel (Algorithm 2) generalises: measurement infrastructure and a bit-exact
// cross-check for the V=1, F=1, S=0 instance on short rows; not part of libpcsr.so.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

__global__ void __launch_bounds__(512) alg1_kernel(const int32_t *__restrict__ rowptr,
                                                   const int32_t *__restrict__ colidx,
                                                   const float *__restrict__ val,
                                                   const float *__restrict__ B, float *C, int n_rows, int K)
{
    const int warp = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int W = blockDim.x >> 6;
    const long crow = (long)blockIdx.x * W + warp;
    const int seg = blockIdx.y * 64 + lane;
    if (crow >= n_rows || seg >= K) return;
    const int head = rowptr[crow], tail = rowptr[crow + 1];
    float res = 0.0f;
    for (int i = head; i < tail; ++i) res = fmaf(val[i], B[(long)colidx[i] * K + seg], res);
    C[crow * K + seg] = res;
}

} // namespace

extern "C" {

// All pointers device.  W = wavefronts per workgroup (1..8).  Returns 0 or a hipError_t.
int alg1_spmm(int64_t n_rows, const int32_t *rowptr, const int32_t *colidx, const float *val,
              const float *B, float *C, int32_t K, int32_t W, void *stream)
{
    if (n_rows <= 0 || K <= 0) return 0;
    if (W < 1 || W > 8) return -1;
    dim3 grid((unsigned)((n_rows + W - 1) / W), (unsigned)((K + 63) / 64));
    hipLaunchKernelGGL(alg1_kernel, grid, dim3(64 * W), 0, (hipStream_t)stream, rowptr, colidx, val, B, C,
                       (int)n_rows, (int)K);
    return (int)hipGetLastError();
}
}
