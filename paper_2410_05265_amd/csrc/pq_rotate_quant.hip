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
#include "pq_rotate.h"

namespace pq {
namespace {

using rq::kChunk;
using rq::kThreads;

// R rows of one chunk column per workgroup: all R loads of a thread are issued before the
// arithmetic starts (the kernel has 2.5 bytes of traffic per element and little else to hide
// latency with).
template <int G, bool EXACT, int R, int BITS>
__global__ __launch_bounds__(kThreads) void k_rotate_quant(const __half* __restrict__ x, int64_t M, int64_t K,
                                                          int log2h, float mult, float step,
                                                          uint32_t* __restrict__ xq)
{
    __shared__ float xch[EXACT ? 1 : G * kChunk];
    const int64_t row0 = (int64_t)blockIdx.y * R;
    const int64_t chunk0 = (int64_t)blockIdx.x * (G * kChunk);
    v4i raw[R][G];
    bool live[R][G];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool in = row0 + r < M;
        rq::load_chunk<G>(static_cast<const __half*>(x + (in ? row0 + r : 0) * K), K, chunk0, threadIdx.x, in, raw[r],
                          live[r]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
        rq::rotate_quant_regs<G, EXACT, BITS>(raw[r], live[r], chunk0, log2h, mult, step,
                                        static_cast<uint32_t*>(xq + (row0 + r) * (BITS == 8 ? K >> 2 : K >> 3)),
                                        (rq::lds_f32_ptr)xch,
                                        threadIdx.x, row0 + r < M);
}

template <int BITS>
int launch_rq(const __half* xp, int64_t M, int64_t K, int32_t h, float act_scale, uint32_t* op, hipStream_t st)
{
    if (M > 65535) {
        // grid.y is limited to 65535 per launch
        for (int64_t m0 = 0; m0 < M; m0 += 65534) {
            const int64_t mm = (M - m0 < 65534) ? (M - m0) : 65534;
            int rc = launch_rq<BITS>(xp + m0 * K, mm, K, h, act_scale, op + m0 * (BITS == 8 ? K / 4 : K / 8), st);
            if (rc != PQ_OK) return rc;
        }
        return PQ_OK;
    }
    if (h <= 1) {
        const float inv = (float)(1.0 / (double)act_scale);
        dim3 grid((unsigned)((K + kChunk - 1) / kChunk), (unsigned)((M + 1) / 2));
        hipLaunchKernelGGL((k_rotate_quant<1, true, 2, BITS>), grid, dim3(kThreads), 0, st, xp, M, K, 0, inv, act_scale, op);
        return hip_status(hipGetLastError());
    }
    int log2h = 0;
    while ((1 << log2h) < h) ++log2h;
    const float mult = (float)(1.0 / ((double)act_scale * sqrt((double)h)));
    const int G = h <= kChunk ? 1 : h / kChunk;
    const int R = G <= 2 ? 2 : 1;
    dim3 grid((unsigned)((K + (int64_t)G * kChunk - 1) / ((int64_t)G * kChunk)), (unsigned)((M + R - 1) / R));
    switch (G) {
        case 1: hipLaunchKernelGGL((k_rotate_quant<1, false, 2, BITS>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, mult, act_scale, op); break;
        case 2: hipLaunchKernelGGL((k_rotate_quant<2, false, 2, BITS>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, mult, act_scale, op); break;
        case 4: hipLaunchKernelGGL((k_rotate_quant<4, false, 1, BITS>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, mult, act_scale, op); break;
        case 8: hipLaunchKernelGGL((k_rotate_quant<8, false, 1, BITS>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, mult, act_scale, op); break;
        default: return PQ_ERR_UNSUPPORTED;
    }
    return hip_status(hipGetLastError());
}

}  // namespace

int launch_rotate_quant(const void* x, int64_t M, int64_t K, int32_t h, float act_scale, void* xq, hipStream_t st)
{
    return launch_rq<4>(static_cast<const __half*>(x), M, K, h, act_scale, static_cast<uint32_t*>(xq), st);
}

int launch_rotate_quant8(const void* x, int64_t M, int64_t K, int32_t h, float act_scale, void* xq8, hipStream_t st)
{
    return launch_rq<8>(static_cast<const __half*>(x), M, K, h, act_scale, static_cast<uint32_t*>(xq8), st);
}

}  // namespace pq
