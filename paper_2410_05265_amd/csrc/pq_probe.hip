// Two measuring sticks for the rooflines (not part of the path): what this GPU's INT8 matrix pipe
// delivers when nothing but matrix instructions is issued, and what a kernel that only reads a
// buffer gets out of HBM.  The benchmark reports the path's kernels against the nominal peaks and
// against these.
#include "pq_internal.h"

namespace pq {
namespace {

// Every wavefront issues `iters` x 16 independent v_mfma_i32_32x32x32_i8 on operands it loads once
// from `operands` (so their bit patterns are the caller's: zeros, codes times 16, random bytes: the
// matrix pipe's speed depends on them on a power-limited chip).  4 wavefronts per workgroup, one per SIMD.
__global__ __launch_bounds__(256) void k_probe_mfma(const v4i* __restrict__ operands, int n_operands, int iters,
                                                   int* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    v4i a[4], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a[t] = operands[((blockIdx.x * 8 + t) * 64 + lane) % n_operands];
        b[t] = operands[((blockIdx.x * 8 + 4 + t) * 64 + lane) % n_operands];
    }
    v16i c[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) c[i][j][v] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) c[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], c[i][j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s ^= c[i][j][v];
    if (s == 0x5EED5EED) sink[0] = s;   // keeps the results alive; practically never true
}

// One workgroup of 1024 threads per CU; a wavefront-load is 1 KiB contiguous, eight in flight per lane.
__global__ __launch_bounds__(1024) void k_probe_read(const v4i* __restrict__ src, int64_t n16, int* __restrict__ sink)
{
    const int64_t stride = (int64_t)gridDim.x * 1024;
    v4i s = {0, 0, 0, 0};
    int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        v4i v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) { s.x ^= v[u].x; s.y ^= v[u].y; s.z ^= v[u].z; s.w ^= v[u].w; }
    }
    for (; i < n16; i += stride) {
        const v4i v = __builtin_nontemporal_load(src + i);
        s.x ^= v.x; s.y ^= v.y; s.z ^= v.z; s.w ^= v.w;
    }
    if ((s.x ^ s.y ^ s.z ^ s.w) == 0x5EED5EED) sink[0] = s.x;
}

}  // namespace

int launch_probe_mfma(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups, int32_t* sink,
                      hipStream_t st)
{
    hipLaunchKernelGGL(k_probe_mfma, dim3((unsigned)workgroups), dim3(256), 0, st, static_cast<const v4i*>(operands),
                       (int)(operand_bytes / 16), (int)iters, sink);
    return hip_status(hipGetLastError());
}

int launch_probe_read(const void* src, int64_t bytes, int32_t* sink, hipStream_t st)
{
    hipLaunchKernelGGL(k_probe_read, dim3(256), dim3(1024), 0, st, static_cast<const v4i*>(src), bytes / 16, sink);
    return hip_status(hipGetLastError());
}

}  // namespace pq
