// Online Hadamard rotation + static per-tensor 4-bit quantization + nibble packing.
//
// Follows App. B "Online Rotation" of the paper (a Walsh-Hadamard transform applied to a
// linear's input at run time) and Eq. 1 in its symmetric form with a step size fixed at
// calibration (Sec. 3 "Dynamic and Static").  One pass over the activations: 2 bytes
// read and half a byte written per element; the rotated values never leave registers.
//
// Work split.  A workgroup of 256 threads owns one chunk of a row: 2048*G consecutive
// channels, thread t holding G groups of 8 consecutive channels (channel = 2048*g + 8*t
// + i).  The butterfly stage with distance d pairs channel e with e ^ d:
//   d = 1, 2, 4            inside a thread's 8 registers
//   d = 8 .. 256           between lanes of a wavefront (DPP / swizzle / permlane swap)
//   d = 512, 1024          between the 4 wavefronts, one radix-4 exchange through LDS
//   d = 2048 ..            between a thread's G groups (registers)
// Butterflies are fp32.  1/sqrt(h) is folded into the reciprocal step size.
#include "pq_internal.h"

#include <hip/hip_fp16.h>

namespace pq {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 2048;  // channels per workgroup per group index

// ---- partner exchange between lanes: returns the value held by lane (id ^ (1 << B)).
template <int B>
__device__ __forceinline__ float lane_xor(float v)
{
    const int iv = __float_as_int(v);
    int r;
    if constexpr (B == 0) {
        r = __builtin_amdgcn_update_dpp(iv, iv, 0xB1, 0xF, 0xF, false);  // quad_perm [1,0,3,2]
    } else if constexpr (B == 1) {
        r = __builtin_amdgcn_update_dpp(iv, iv, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
    } else if constexpr (B == 2) {
        // lanes 0-3 and 8-11 of each row of 16 take lane+4, the others lane-4
        r = __builtin_amdgcn_update_dpp(iv, iv, 0x104, 0xF, 0x5, false);  // row_shl:4
        r = __builtin_amdgcn_update_dpp(r, iv, 0x114, 0xF, 0xA, false);   // row_shr:4
    } else if constexpr (B == 3) {
        r = __builtin_amdgcn_update_dpp(iv, iv, 0x128, 0xF, 0xF, false);  // row_ror:8
    } else if constexpr (B == 4) {
        r = __builtin_amdgcn_ds_swizzle(iv, 0x401F);  // bit-mask mode: and 0x1F, xor 0x10
    } else {
        r = __shfl_xor(iv, 32, 64);
    }
    return __int_as_float(r);
}

template <int B, int NV>
__device__ __forceinline__ void lane_stage(float (&v)[NV], int lane)
{
    const bool upper = (lane >> B) & 1;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const float p = lane_xor<B>(v[i]);
        v[i] = upper ? (p - v[i]) : (p + v[i]);
    }
}

// d = 1, 2, 4 inside one group of 8
__device__ __forceinline__ void reg_stages8(float* v, int nstages)
{
    if (nstages >= 1) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) { float a = v[i], b = v[i + 1]; v[i] = a + b; v[i + 1] = a - b; }
    }
    if (nstages >= 2) {
#pragma unroll
        for (int i = 0; i < 8; i += 4)
#pragma unroll
            for (int j = 0; j < 2; ++j) { float a = v[i + j], b = v[i + j + 2]; v[i + j] = a + b; v[i + j + 2] = a - b; }
    }
    if (nstages >= 3) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { float a = v[j], b = v[j + 4]; v[j] = a + b; v[j + 4] = a - b; }
    }
}

// Round-to-nearest-even of eight scaled values, clamp to [-8,7], pack low nibble first.
// `magic` puts round(t) + 8 into the low mantissa bits of an fp32 in [2^23, 2^24).
constexpr float kMagic = 12582920.0f;            // 1.5 * 2^23 + 8, bit pattern 0x4B400008
constexpr uint32_t kMagicSum = 0x4B400000u * 0x11111111u;  // sum of (pattern - offset part) << 4i

template <bool EXACT>
__device__ __forceinline__ uint32_t quant_pack8(const float* v, const float* raw, float mult, float step)
{
    float t[8];
    uint32_t bits[8];
    bool suspect = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        t[i] = v[i] * mult;
        const float c = __builtin_amdgcn_fmed3f(t[i], -8.0f, 7.0f);
        const float r = c + kMagic;                 // fp32 add rounds to an integer, ties to even
        bits[i] = __float_as_uint(r);
        if constexpr (EXACT) {
            const float f = c - (r - kMagic);       // exact; |f| <= 0.5
            suspect |= (fabsf(f) > 0.5f - 0x1.0p-18f);
        }
    }
    if constexpr (EXACT) {
        // t carries two fp32 roundings (reciprocal and product), so a quotient within
        // ~1e-6 of k + 1/2 may have been rounded to the wrong side.  Decide those from
        // the sign of (k + 1/2) * step - x, which one fused multiply-add gives exactly.
        if (__builtin_expect(suspect, 0)) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float c = __builtin_amdgcn_fmed3f(t[i], -8.0f, 7.0f);
                const float r = c + kMagic;
                const float f = c - (r - kMagic);
                if (fabsf(f) > 0.5f - 0x1.0p-18f) {
                    const float k = floorf(t[i]);
                    const float d = fmaf(k + 0.5f, step, -raw[i]);
                    const int ki = (int)k;
                    int q = d > 0.0f ? ki : (d < 0.0f ? ki + 1 : ((ki & 1) ? ki + 1 : ki));
                    q = q < -8 ? -8 : (q > 7 ? 7 : q);
                    bits[i] = 0x4B400008u + (uint32_t)q;
                }
            }
        }
    }
    uint32_t s = bits[7];
#pragma unroll
    for (int i = 6; i >= 0; --i) s = (s << 4) + bits[i];
    return (s - kMagicSum) ^ 0x88888888u;   // offset-binary nibbles -> two's complement
}

template <int G, bool EXACT>
__global__ __launch_bounds__(kThreads) void k_rotate_quant(const __half* __restrict__ x, int64_t K, int log2h,
                                                          float mult, float step, uint32_t* __restrict__ xq)
{
    __shared__ float xch[(G * kChunk * 4 > 0 && !EXACT) ? G * kChunk : 1];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int64_t row = blockIdx.y;
    const int64_t chunk0 = (int64_t)blockIdx.x * (G * kChunk);

    float v[G][8];
    bool live[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int64_t e0 = chunk0 + (int64_t)g * kChunk + tid * 8;
        live[g] = e0 < K;
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (live[g]) raw = *reinterpret_cast<const uint4*>(x + row * K + e0);
        const __half2* h2 = reinterpret_cast<const __half2*>(&raw);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float2 f = __half22float2(h2[i]);
            v[g][2 * i] = f.x;
            v[g][2 * i + 1] = f.y;
        }
    }

    if constexpr (EXACT) {
        // no rotation: the unrotated value doubles as the exact tie-break operand
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (live[g]) {
                const int64_t e0 = chunk0 + (int64_t)g * kChunk + tid * 8;
                xq[(row * K + e0) >> 3] = quant_pack8<true>(v[g], v[g], mult, step);
            }
        }
    } else {
#pragma unroll
        for (int g = 0; g < G; ++g) reg_stages8(v[g], log2h < 3 ? log2h : 3);
        float(&flat)[G * 8] = reinterpret_cast<float(&)[G * 8]>(v);
        if (log2h > 3) lane_stage<0>(flat, lane);
        if (log2h > 4) lane_stage<1>(flat, lane);
        if (log2h > 5) lane_stage<2>(flat, lane);
        if (log2h > 6) lane_stage<3>(flat, lane);
        if (log2h > 7) lane_stage<4>(flat, lane);
        if (log2h > 8) lane_stage<5>(flat, lane);
        if (log2h > 9) {
            // radix-4 (or radix-2 when h == 1024) exchange between the 4 wavefronts
#pragma unroll
            for (int i = 0; i < G * 8; ++i) xch[(wave * G * 8 + i) * 64 + lane] = flat[i];
            __syncthreads();
            const bool two = log2h > 10;
#pragma unroll
            for (int i = 0; i < G * 8; ++i) {
                const float a = xch[((wave ^ 1) * G * 8 + i) * 64 + lane];
                float r = (wave & 1) ? (a - flat[i]) : (a + flat[i]);
                if (two) {
                    const float b = xch[((wave ^ 2) * G * 8 + i) * 64 + lane];
                    const float c = xch[((wave ^ 3) * G * 8 + i) * 64 + lane];
                    const float rp = (wave & 1) ? (c - b) : (c + b);   // same stage-1 result in the partner pair
                    r = (wave & 2) ? (rp - r) : (rp + r);
                }
                flat[i] = r;
            }
        }
        if constexpr (G > 1) {
            // d = 2048 * 2^j between groups
#pragma unroll
            for (int dg = 1; dg < G; dg <<= 1) {
                if (log2h > 11 + __builtin_ctz(dg)) {
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        if ((g & dg) == 0) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const float a = v[g][i], b = v[g + dg][i];
                                v[g][i] = a + b;
                                v[g + dg][i] = a - b;
                            }
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (live[g]) {
                const int64_t e0 = chunk0 + (int64_t)g * kChunk + tid * 8;
                xq[(row * K + e0) >> 3] = quant_pack8<false>(v[g], v[g], mult, step);
            }
        }
    }
}

}  // namespace

int launch_rotate_quant(const void* x, int64_t M, int64_t K, int32_t h, float act_scale, void* xq,
                        hipStream_t st)
{
    const __half* xp = static_cast<const __half*>(x);
    uint32_t* op = static_cast<uint32_t*>(xq);
    if (M > 65535) {
        // grid.y is limited to 65535 rows per launch
        for (int64_t m0 = 0; m0 < M; m0 += 65535) {
            const int64_t mm = (M - m0 < 65535) ? (M - m0) : 65535;
            int rc = launch_rotate_quant(xp + m0 * K, mm, K, h, act_scale, op + m0 * K / 8, st);
            if (rc != PQ_OK) return rc;
        }
        return PQ_OK;
    }
    if (h <= 1) {
        const float inv = (float)(1.0 / (double)act_scale);
        dim3 grid((unsigned)((K + kChunk - 1) / kChunk), (unsigned)M);
        hipLaunchKernelGGL((k_rotate_quant<1, true>), grid, dim3(kThreads), 0, st, xp, K, 0, inv, act_scale, op);
        return hip_status(hipGetLastError());
    }
    int log2h = 0;
    while ((1 << log2h) < h) ++log2h;
    const float mult = (float)(1.0 / ((double)act_scale * sqrt((double)h)));
    const int G = h <= kChunk ? 1 : h / kChunk;
    dim3 grid((unsigned)((K + (int64_t)G * kChunk - 1) / ((int64_t)G * kChunk)), (unsigned)M);
    switch (G) {
        case 1: hipLaunchKernelGGL((k_rotate_quant<1, false>), grid, dim3(kThreads), 0, st, xp, K, log2h, mult, act_scale, op); break;
        case 2: hipLaunchKernelGGL((k_rotate_quant<2, false>), grid, dim3(kThreads), 0, st, xp, K, log2h, mult, act_scale, op); break;
        case 4: hipLaunchKernelGGL((k_rotate_quant<4, false>), grid, dim3(kThreads), 0, st, xp, K, log2h, mult, act_scale, op); break;
        case 8: hipLaunchKernelGGL((k_rotate_quant<8, false>), grid, dim3(kThreads), 0, st, xp, K, log2h, mult, act_scale, op); break;
        default: return PQ_ERR_UNSUPPORTED;
    }
    return hip_status(hipGetLastError());
}

}  // namespace pq
