// Weight-streaming variant of the 4-bit product for decode (M <= 16 tokens): the packed
// weight matrix is read from HBM exactly once, which is all that matters at these shapes
// (Sec. 3 of the paper: weight quantization speeds up memory-bound computation; the
// decoding column of the inference-speed table in Sec. 5.4).
//
// A workgroup owns 16 consecutive output channels; its wavefronts split K.  Each lane
// loads 16 packed bytes (32 channels) of one weight row per step and the matching 16
// bytes of one token's codes (tokens >= M supply zeros), expands both to int8 * 16 and
// issues two 16x16x64 matrix instructions, so the sum over K needs no cross-lane
// reduction.  Partial tiles of the wavefronts are added through LDS.
//
// v_mfma_i32_16x16x64_i8 layout used (lane l, r = l % 16, g = l / 16):
//   A: row r, bytes k = 16 g .. 16 g + 15;  B: column r, same bytes;
//   D: register v holds D[4 g + v][r].
#include "pq_internal.h"

#include <hip/hip_fp16.h>

namespace pq {
namespace {

constexpr int kWaves = 4;
constexpr int kUnroll = 4;

__global__ __launch_bounds__(kWaves * 64) void k_gemv(const uint8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                                                     const float* __restrict__ sw, float sx, int M, int N, int K,
                                                     __half* __restrict__ out, int32_t* __restrict__ acc_out)
{
    __shared__ int red[kWaves][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int Kb = K >> 1;
    const int steps = (Kb + 63) >> 6;                       // 64 packed bytes per row per step
    const int per = (steps + kWaves - 1) / kWaves;
    const int s_begin = wave * per;
    const int s_end = (s_begin + per < steps) ? (s_begin + per) : steps;

    const uint8_t* wrow = wq + (int64_t)(n0 + r) * Kb + g * 16;
    const uint8_t* xrow = xq + (int64_t)(r < M ? r : 0) * Kb + g * 16;
    const bool has_x = r < M;

    v4i acc = {0, 0, 0, 0};
    for (int s = s_begin; s < s_end; s += kUnroll) {
        v4i w[kUnroll], x[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int off = (s + u) * 64;
            const bool in = (s + u) < s_end && (off + g * 16) < Kb;
            w[u] = (v4i){0, 0, 0, 0};
            x[u] = (v4i){0, 0, 0, 0};
            if (in) w[u] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wrow + off));
            if (in && has_x) x[u] = *reinterpret_cast<const v4i*>(xrow + off);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            v4i we, wo, xe, xo;
            unpack16(w[u], we, wo);
            unpack16(x[u], xe, xo);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(we, xe, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo, acc, 0, 0, 0);
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][v][lane] = acc[v];
    __syncthreads();
    if (wave == 0 && has_x) {
        const int m = r;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            int a = 0;
#pragma unroll
            for (int w2 = 0; w2 < kWaves; ++w2) a += red[w2][v][lane];
            a >>= 8;
            const int n = n0 + 4 * g + v;
            if (acc_out) acc_out[(int64_t)m * N + n] = a;
            if (out) out[(int64_t)m * N + n] = __float2half_rn((float)a * (sx * sw[n]));
        }
    }
}

}  // namespace

int launch_gemv(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                void* out, int32_t* acc, hipStream_t st)
{
    if (M > 16 || N > (1 << 30) || K > (1 << 30)) return PQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_gemv, dim3((unsigned)(N / 16)), dim3(kWaves * 64), 0, st, static_cast<const uint8_t*>(xq),
                       static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N, (int)K, static_cast<__half*>(out),
                       acc);
    return hip_status(hipGetLastError());
}

}  // namespace pq
