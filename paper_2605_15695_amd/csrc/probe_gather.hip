// Gather-ceiling probe: how fast can this GPU pull randomly indexed rows of a dense
// row-major fp32 matrix through the cache hierarchy when nothing else is in the way?
// The SpMM kernels are bound by exactly this access on scattered inputs, so the probe
// gives the "second roofline" their cache-level gather rate nnz*K*4/t is compared with.
// Measurement infrastructure only (built into libpcsr_baseline.so).
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

// One group of LPR lanes per gathered row (LPR*4 floats = one row), 64/LPR rows per
// wavefront instruction, U independent gathers in flight per lane, no dependent chain
// other than the (coalesced, prefetched) index stream.
template <int LPR, int U>
__global__ void __launch_bounds__(256) gather_probe_kernel(const float *__restrict__ B, int row_floats,
                                                           const int32_t *__restrict__ idx, long n_idx,
                                                           float *out)
{
    constexpr int G = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int lg = lane & (LPR - 1);
    const long group = ((long)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * G + lane / LPR;
    const long n_groups = (long)gridDim.x * (blockDim.x >> 6) * G;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    // group g takes indices g*U .. g*U+U-1, then strides by n_groups*U
    for (long base = group * U; base < n_idx; base += n_groups * U) {
        int r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = base + u < n_idx ? idx[base + u] : idx[base];
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            v[u] = *reinterpret_cast<const float4 *>(B + (long)r[u] * row_floats + lg * 4);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc.x += v[u].x;
            acc.y += v[u].y;
            acc.z += v[u].z;
            acc.w += v[u].w;
        }
    }
    out[(long)blockIdx.x * blockDim.x + threadIdx.x] = acc.x + acc.y + acc.z + acc.w;
}

template <int LPR> hipError_t launch(const float *B, int row_floats, const int32_t *idx, long n_idx,
                                     float *out, int blocks, hipStream_t s)
{
    hipLaunchKernelGGL((gather_probe_kernel<LPR, 8>), dim3(blocks), dim3(256), 0, s, B, row_floats, idx,
                       n_idx, out);
    return hipGetLastError();
}

} // namespace

extern "C" {

// B: device fp32 [n_rows x row_floats]; row_floats in {16,32,64,128,256}; idx: device
// int32[n_idx], every entry in [0, n_rows); out: device fp32[blocks*256].  Returns 0 or
// a hipError_t / -1 for an unsupported row width.
int probe_gather(const float *B, int32_t row_floats, const int32_t *idx, int64_t n_idx, float *out,
                 int32_t blocks, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    switch (row_floats) {
    case 16: return (int)launch<4>(B, row_floats, idx, n_idx, out, blocks, s);
    case 32: return (int)launch<8>(B, row_floats, idx, n_idx, out, blocks, s);
    case 64: return (int)launch<16>(B, row_floats, idx, n_idx, out, blocks, s);
    case 128: return (int)launch<32>(B, row_floats, idx, n_idx, out, blocks, s);
    case 256: return (int)launch<64>(B, row_floats, idx, n_idx, out, blocks, s);
    }
    return -1;
}
}
