// Weight-streaming variant of the 4-bit product for decode (M <= 16 tokens): the packed
// weight matrix is read from HBM exactly once, which is all that matters at these shapes
// (Sec. 3 of the paper: weight quantization speeds up memory-bound computation; the
// decoding column of the inference-speed table in Sec. 5.4).
//
// A workgroup owns 16 consecutive output channels (one contiguous block of the weight
// matrix); its wavefronts split K so that each has about eight 16-byte loads per lane, all
// issued at once: at these sizes (32-112 KB per CU) the kernel is one burst of loads, and
// what counts is that every byte is requested as early as possible.  Each lane
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

constexpr int kMaxWaves = 16;
constexpr int kBatch = 8;   // 16-byte loads a lane has in flight: the whole K slice of most shapes

__global__ __launch_bounds__(kMaxWaves * 64) void k_gemv(const uint8_t* __restrict__ xq, const uint8_t* __restrict__ wq,
                                                        const float* __restrict__ sw, float sx, int M, int N, int K,
                                                        __half* __restrict__ out, int32_t* __restrict__ acc_out)
{
    __shared__ int red[kMaxWaves][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int Kb = K >> 1;
    const int steps = (Kb + 63) >> 6;                       // 64 packed bytes per row per step
    const int per = (steps + nwaves - 1) / nwaves;
    const int s_begin = wave * per;
    const int s_end = (s_begin + per < steps) ? (s_begin + per) : steps;

    const uint8_t* wrow = wq + (int64_t)(n0 + r) * Kb + g * 16;
    const uint8_t* xrow = xq + (int64_t)(r < M ? r : 0) * Kb + g * 16;
    const bool has_x = r < M;

    v4i acc = {0, 0, 0, 0};
    for (int s = s_begin; s < s_end; s += kBatch) {
        v4i w[kBatch], x[kBatch];
        // every weight load of the batch is issued before anything waits
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int off = (s + u) * 64;
            const bool in = (s + u) < s_end && (off + g * 16) < Kb;
            w[u] = (v4i){0, 0, 0, 0};
            if (in) w[u] = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(wrow + off));
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int off = (s + u) * 64;
            const bool in = (s + u) < s_end && (off + g * 16) < Kb;
            x[u] = (v4i){0, 0, 0, 0};
            if (in && has_x) x[u] = *reinterpret_cast<const v4i*>(xrow + off);
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
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
        int a[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            a[v] = 0;
            for (int w2 = 0; w2 < nwaves; ++w2) a[v] += red[w2][v][lane];
            a[v] >>= 8;
        }
        const int n = n0 + 4 * g;   // this lane's four consecutive channels
        if (acc_out) *reinterpret_cast<int4*>(acc_out + (int64_t)m * N + n) = make_int4(a[0], a[1], a[2], a[3]);
        if (out) {
            const float4 sc = *reinterpret_cast<const float4*>(sw + n);
            const __half2 lo = __floats2half2_rn((float)a[0] * (sx * sc.x), (float)a[1] * (sx * sc.y));
            const __half2 hi = __floats2half2_rn((float)a[2] * (sx * sc.z), (float)a[3] * (sx * sc.w));
            uint2 pk;
            pk.x = *reinterpret_cast<const uint32_t*>(&lo);
            pk.y = *reinterpret_cast<const uint32_t*>(&hi);
            *reinterpret_cast<uint2*>(out + (int64_t)m * N + n) = pk;
        }
    }
}

}  // namespace

int launch_gemv(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                void* out, int32_t* acc, hipStream_t st)
{
    if (M > 16 || N > (1 << 30) || K > (1 << 30)) return PQ_ERR_UNSUPPORTED;
    const int steps = (int)((K / 2 + 63) / 64);
    int nwaves = (steps + kBatch - 1) / kBatch;
    nwaves = nwaves < 1 ? 1 : (nwaves > kMaxWaves ? kMaxWaves : nwaves);
    hipLaunchKernelGGL(k_gemv, dim3((unsigned)(N / 16)), dim3(nwaves * 64), 0, st, static_cast<const uint8_t*>(xq),
                       static_cast<const uint8_t*>(wq), sw, sx, (int)M, (int)N, (int)K, static_cast<__half*>(out),
                       acc);
    return hip_status(hipGetLastError());
}

}  // namespace pq
