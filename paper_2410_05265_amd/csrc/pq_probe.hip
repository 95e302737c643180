// Measuring sticks for the rooflines (not part of the path): what this GPU's INT8 matrix pipe
// delivers when nothing but matrix instructions is issued (and the 6-bit floating-point one, which
// multiplies 4-bit integer codes exactly), and what a kernel that only reads a buffer gets out of HBM.  The benchmark reports the path's kernels against the nominal peaks and
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

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// A 4-bit integer code (and +8) as a 6-bit float with 3 exponent and 2 mantissa bits (bias 3):
// 0, 1, 1.5 x 2, 4 x {1, 1.25, 1.5, 1.75}, 8 are all exact in that format.
__device__ __forceinline__ uint32_t e3m2_of_code(int c)
{
    c = c < -8 ? -8 : (c > 8 ? 8 : c);
    const uint32_t m = (uint32_t)(c < 0 ? -c : c);
    if (m == 0) return 0;
    const uint32_t e = 31u - (uint32_t)__builtin_clz(m);
    return (c < 0 ? 32u : 0u) | ((e + 3u) << 2) | (((m << 2) >> e) & 3u);
}

// The same measuring stick for the 6-bit floating-point matrix instruction (fp32 accumulate; operand
// registers: 32 values of 6 bits in the first six dwords of eight).  Integer codes written in that
// format multiply and add exactly (k_probe_f6_product checks it), at twice the nominal rate of INT8.
__global__ __launch_bounds__(256) void k_probe_mfma_f6(const v8i* __restrict__ operands, int n_operands, int iters,
                                                      int* __restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    v8i a[4], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a[t] = operands[((blockIdx.x * 8 + t) * 64 + lane) % n_operands];
        b[t] = operands[((blockIdx.x * 8 + 4 + t) * 64 + lane) % n_operands];
    }
    v16f c[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) c[i][j][v] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)   // formats 3, 3: both operands E3M2; scale bytes 127: 2^0
                c[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], c[i][j], 3, 3, 0, 127, 0, 127);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += c[i][j][v];
    if (s == 12345.678f) sink[0] = 1;   // keeps the results alive; practically never true
}

// One wavefront: out[i][j] = sum_k a[i][k] b[j][k] for 32 x 32 outputs, codes in [-8, 8] given as int8,
// encoded to E3M2 here and multiplied by the 6-bit matrix instruction.  Lane l holds row l % 32 and, per
// step of 64 channels, the 32 channels of block l / 32 (the same assignment for both operands, so the
// sum over k does not depend on how the instruction numbers k inside a register).
__global__ __launch_bounds__(64) void k_probe_f6_product(const int8_t* __restrict__ a, const int8_t* __restrict__ b,
                                                        int K, int32_t* __restrict__ out)
{
    const int lane = threadIdx.x, row = lane & 31, kb = lane >> 5;
    v16f acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    for (int k0 = 0; k0 < K; k0 += 64) {
        const int8_t* pa = a + (int64_t)row * K + k0 + kb * 32;
        const int8_t* pb = b + (int64_t)row * K + k0 + kb * 32;
        uint64_t wa[3] = {0, 0, 0}, wb[3] = {0, 0, 0};   // 3 x 64 bits = 32 values of 6 bits
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const int bit = 6 * i;
            const uint64_t ea = e3m2_of_code(pa[i]), eb = e3m2_of_code(pb[i]);
            wa[bit / 64] |= ea << (bit % 64);
            wb[bit / 64] |= eb << (bit % 64);
            if (bit % 64 > 58) {
                wa[bit / 64 + 1] |= ea >> (64 - bit % 64);
                wb[bit / 64 + 1] |= eb >> (64 - bit % 64);
            }
        }
        v8i x = {0, 0, 0, 0, 0, 0, 0, 0}, y = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            x[2 * i] = (int)(uint32_t)wa[i]; x[2 * i + 1] = (int)(uint32_t)(wa[i] >> 32);
            y[2 * i] = (int)(uint32_t)wb[i]; y[2 * i + 1] = (int)(uint32_t)(wb[i] >> 32);
        }
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(x, y, acc, 3, 3, 0, 127, 0, 127);
    }
    // lane l, register v: column l % 32 of the second operand, row 8 (v / 4) + 4 (l / 32) + v % 4 of the first
#pragma unroll
    for (int v = 0; v < 16; ++v) out[(8 * (v >> 2) + 4 * kb + (v & 3)) * 32 + row] = (int32_t)acc[v];
}

}  // namespace

int launch_probe_mfma_f6(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups, int32_t* sink,
                         hipStream_t st)
{
    hipLaunchKernelGGL(k_probe_mfma_f6, dim3((unsigned)workgroups), dim3(256), 0, st, static_cast<const v8i*>(operands),
                       (int)(operand_bytes / 32), (int)iters, sink);
    return hip_status(hipGetLastError());
}

int launch_probe_f6_product(const int8_t* a, const int8_t* b, int64_t K, int32_t* out, hipStream_t st)
{
    hipLaunchKernelGGL(k_probe_f6_product, dim3(1), dim3(64), 0, st, a, b, (int)K, out);
    return hip_status(hipGetLastError());
}

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
