// Plain device kernel for the 4-bit integer product and its dequantisation: one thread
// per output element, a running int32 sum over packed bytes.  Slow by design; it is the
// on-device cross-check for the tiled and streaming kernels (Sec. 3 of the paper:
// low-bit matrix multiplication; Table 1 row O2 for the step sizes).
#include "pq_internal.h"

#include <hip/hip_fp16.h>

namespace pq {
namespace {

__device__ __forceinline__ int nib_lo(uint32_t b) { return (int)(b << 28) >> 28; }
__device__ __forceinline__ int nib_hi(uint32_t b) { return (int)(b << 24) >> 28; }

__global__ __launch_bounds__(256) void k_gemm_simple(const uint8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                                                   const float* __restrict__ sw, float sx, int64_t M, int64_t N,
                                                   int64_t K, __half* __restrict__ out, int32_t* __restrict__ acc)
{
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t m = blockIdx.y;
    if (n >= N || m >= M) return;
    const uint8_t* a = xq + m * (K / 2);
    const uint8_t* b = wq + n * (K / 2);
    int32_t s = 0;
    for (int64_t j = 0; j < K / 2; ++j) {
        const uint32_t pa = a[j], pb = b[j];
        s += nib_lo(pa) * nib_lo(pb) + nib_hi(pa) * nib_hi(pb);
    }
    if (acc) acc[m * N + n] = s;
    if (out) out[m * N + n] = __float2half_rn(mul_rn((float)s, sx * sw[n]));
}

}  // namespace

int launch_gemm_simple(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N,
                       int64_t K, void* out, int32_t* acc, hipStream_t st)
{
    for (int64_t m0 = 0; m0 < M; m0 += 65535) {
        const int64_t mm = (M - m0 < 65535) ? (M - m0) : 65535;
        dim3 grid((unsigned)((N + 255) / 256), (unsigned)mm);
        hipLaunchKernelGGL(k_gemm_simple, grid, dim3(256), 0, st,
                           static_cast<const uint8_t*>(xq) + m0 * (K / 2), static_cast<const uint8_t*>(wq), sw, sx,
                           mm, N, K, out ? static_cast<__half*>(out) + m0 * N : nullptr,
                           acc ? acc + m0 * N : nullptr);
        int rc = hip_status(hipGetLastError());
        if (rc != PQ_OK) return rc;
    }
    return PQ_OK;
}

// corr[n] = (8 - zero_point) * sum_k wq[n,k]: what the zero-point of Eq. 1 adds to every
// accumulator of output channel n (offline work: one wavefront per weight row).
namespace {
__global__ __launch_bounds__(64) void k_zero_point_correction(const uint8_t* __restrict__ wq, int N, int K, int zo8,
                                                             int32_t* __restrict__ corr)
{
    const int n = blockIdx.x, lane = threadIdx.x;
    const uint32_t* row = reinterpret_cast<const uint32_t*>(wq + (int64_t)n * (K >> 1));
    int sum = 0;
    for (int d = lane; d < (K >> 3); d += 64)
        sum = __builtin_amdgcn_sdot8((int)row[d], 0x11111111, sum, false);   // eight signed nibbles times 1
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    if (lane == 0) corr[n] = zo8 * sum;
}
}  // namespace

int launch_zero_point_correction(const void* wq, int64_t N, int64_t K, int32_t zero_point, int32_t* corr, hipStream_t st)
{
    hipLaunchKernelGGL(k_zero_point_correction, dim3((unsigned)N), dim3(64), 0, st, static_cast<const uint8_t*>(wq),
                       (int)N, (int)K, 8 - zero_point, corr);
    return hip_status(hipGetLastError());
}

}  // namespace pq
