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
template <int G, bool EXACT, int R, int BITS, typename STEPS, bool STREAM>
__global__ __launch_bounds__(kThreads) void k_rotate_quant(const __half* __restrict__ x, int64_t M, int64_t K,
                                                          int log2h, STEPS steps, uint32_t* __restrict__ xq)
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
    for (int r = 0; r < R; ++r) {
        uint32_t* row = xq + (row0 + r) * (BITS == 16 ? K >> 1 : (BITS == 8 ? K >> 2 : K >> 3));
        if constexpr (BITS == 16)
            rq::rotate_quant_regs_with<G, EXACT, BITS>(raw[r], live[r], chunk0, log2h, steps, row, (rq::lds_f32_ptr)xch,
                                                       threadIdx.x, row0 + r < M);
        else
            rq::rotate_quant_regs_with<G, EXACT, BITS>(raw[r], live[r], chunk0, log2h, steps, rq::GlobalCodes<STREAM>{row},
                                                       (rq::lds_f32_ptr)xch, threadIdx.x, row0 + r < M);
    }
}

// Producer fusion for down_proj (Sec. 3: static quantization makes operator fusion feasible): the
// layer input silu(gate) * up is formed in registers from the two projections' fp16 outputs and
// goes straight into rotation + quantizer, so the intermediate never exists in memory.
template <int G, int R, bool STREAM>
__global__ __launch_bounds__(kThreads) void k_silu_mul_rotate_quant(const __half* __restrict__ gate,
                                                                   const __half* __restrict__ up, int64_t M,
                                                                   int64_t K, int log2h, rq::StaticStep steps,
                                                                   uint32_t* __restrict__ xq)
{
    __shared__ float xch[G * kChunk];
    const int64_t row0 = (int64_t)blockIdx.y * R;
    const int64_t chunk0 = (int64_t)blockIdx.x * (G * kChunk);
    v4i rawg[R][G], rawu[R][G];
    bool live[R][G];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const bool in = row0 + r < M;
        const int64_t row = in ? row0 + r : 0;
        rq::load_chunk<G>(static_cast<const __half*>(gate + row * K), K, chunk0, threadIdx.x, in, rawg[r], live[r]);
        rq::load_chunk<G>(static_cast<const __half*>(up + row * K), K, chunk0, threadIdx.x, in, rawu[r], live[r]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
        rq::rotate_quant_regs_with<G, false, 4>(rawg[r], live[r], chunk0, log2h, steps,
                                                rq::GlobalCodes<STREAM>{xq + (row0 + r) * (K >> 3)},
                                                (rq::lds_f32_ptr)xch, threadIdx.x, row0 + r < M,
                                                rq::SiluGate{rawu[r]});
}

// Group-wise dynamic steps (Table 1 row O1, KV cache): every group of 2^log2gs consecutive channels
// of a token (gs = 32, 64 or 128: 4, 8 or 16 neighbouring lanes) gets s = fp32(clip * max|y| / 7) of
// its own rotated values; the steps go to scale_row[channel / gs] of the token's row.
template <int G>
struct GroupDynStep {
    double inv_sqrt_h;
    float clip;
    int log2gs;
    float* scale_base;       // [rows][K / gs]
    int64_t groups_per_row;
    int64_t row;
    int lane;
    float mult_[G], step_[G];
    template <int NV>
    __device__ __forceinline__ void prepare(const float (&v)[NV])
    {
        static_assert(NV == G * 8, "one group of 8 values per chunk");
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float a = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[g * 8 + i]));
            a = fmaxf(a, rq::lane_xor<0>(a));
            a = fmaxf(a, rq::lane_xor<1>(a));
            if (log2gs > 5) a = fmaxf(a, rq::lane_xor<2>(a));
            if (log2gs > 6) a = fmaxf(a, rq::lane_xor<3>(a));
            float st = (float)(((double)clip * ((double)a * inv_sqrt_h)) / 7.0);
            if (!(st > 0.0f)) st = 1.0f;
            step_[g] = st;
            mult_[g] = (float)(inv_sqrt_h / (double)st);
        }
    }
    __device__ __forceinline__ void get(int64_t e0, float& m, float& s) const
    {
        const int g = (int)(e0 >> 11) & (G - 1);      // chunks start at multiples of 2048 G
        m = mult_[0];
        s = step_[0];
#pragma unroll
        for (int i = 1; i < G; ++i)
            if (g == i) { m = mult_[i]; s = step_[i]; }
        if ((lane & ((1 << (log2gs - 3)) - 1)) == 0) scale_base[row * groups_per_row + (e0 >> log2gs)] = s;
    }
    __device__ __forceinline__ int zero_offset() const { return 0; }
};

template <int G, bool EXACT>
__global__ __launch_bounds__(kThreads) void k_rotate_quant_groups(const __half* __restrict__ x, int64_t M, int64_t K,
                                                                 int log2h, double inv_sqrt_h, float clip, int log2gs,
                                                                 uint32_t* __restrict__ xq,
                                                                 float* __restrict__ group_scale)
{
    __shared__ float xch[EXACT ? 1 : G * kChunk];
    const int64_t row = blockIdx.y;
    const int64_t chunk0 = (int64_t)blockIdx.x * (G * kChunk);
    v4i raw[G];
    bool live[G];
    rq::load_chunk<G>(static_cast<const __half*>(x + row * K), K, chunk0, threadIdx.x, true, raw, live);
    GroupDynStep<G> steps{inv_sqrt_h, clip, log2gs, group_scale, K >> log2gs, row, (int)(threadIdx.x & 63), {}, {}};
    rq::rotate_quant_regs_with<G, EXACT, 4>(raw, live, chunk0, log2h, steps, static_cast<uint32_t*>(xq + row * (K >> 3)),
                                            (rq::lds_f32_ptr)xch, threadIdx.x, true);
}

// `steps` already carries the 1/sqrt(h) factor of the reciprocal step.
template <int BITS, typename STEPS, bool STREAM>
int launch_rq_s(const __half* xp, int64_t M, int64_t K, int32_t h, STEPS steps, uint32_t* op, hipStream_t st)
{
    if (h <= 1) {
        dim3 grid((unsigned)((K + kChunk - 1) / kChunk), (unsigned)((M + 1) / 2));
        hipLaunchKernelGGL((k_rotate_quant<1, true, 2, BITS, STEPS, STREAM>), grid, dim3(kThreads), 0, st, xp, M, K, 0, steps, op);
        return hip_status(hipGetLastError());
    }
    int log2h = 0;
    while ((1 << log2h) < h) ++log2h;
    const int G = h <= kChunk ? 1 : h / kChunk;
    const int R = G <= 2 ? 2 : 1;
    dim3 grid((unsigned)((K + (int64_t)G * kChunk - 1) / ((int64_t)G * kChunk)), (unsigned)((M + R - 1) / R));
    switch (G) {
        case 1: hipLaunchKernelGGL((k_rotate_quant<1, false, 2, BITS, STEPS, STREAM>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, steps, op); break;
        case 2: hipLaunchKernelGGL((k_rotate_quant<2, false, 2, BITS, STEPS, STREAM>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, steps, op); break;
        case 4: hipLaunchKernelGGL((k_rotate_quant<4, false, 1, BITS, STEPS, STREAM>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, steps, op); break;
        case 8: hipLaunchKernelGGL((k_rotate_quant<8, false, 1, BITS, STEPS, STREAM>), grid, dim3(kThreads), 0, st, xp, M, K, log2h, steps, op); break;
        default: return PQ_ERR_UNSUPPORTED;
    }
    return hip_status(hipGetLastError());
}

template <int BITS, typename STEPS>
int launch_rq(const __half* xp, int64_t M, int64_t K, int32_t h, STEPS steps, uint32_t* op, hipStream_t st)
{
    constexpr int kWordsShift = BITS == 16 ? 1 : (BITS == 8 ? 2 : 3);   // output dwords per row = K >> shift
    if (M > 65535) {
        // grid.y is limited to 65535 per launch
        for (int64_t m0 = 0; m0 < M; m0 += 65534) {
            const int64_t mm = (M - m0 < 65534) ? (M - m0) : 65534;
            int rc = launch_rq<BITS, STEPS>(xp + m0 * K, mm, K, h, steps, op + m0 * (K >> kWordsShift), st);
            if (rc != PQ_OK) return rc;
        }
        return PQ_OK;
    }
    // (all codes of the launch; the fp16 output of the rotation-only mode is never streamed)
    if (BITS != 16 && M * (K >> kWordsShift) * 4 <= rq::kStreamBelow) return launch_rq_s<BITS, STEPS, BITS != 16>(xp, M, K, h, steps, op, st);
    return launch_rq_s<BITS, STEPS, false>(xp, M, K, h, steps, op, st);
}

inline rq::StaticStep static_step(float act_scale, int32_t h)
{
    const double r = h > 1 ? sqrt((double)h) : 1.0;
    return rq::StaticStep{(float)(1.0 / ((double)act_scale * r)), act_scale};
}

// The step of a token: fp32(clip * max|y| / qmax) over the whole row held by the workgroup, with
// max|y| = max|v| / sqrt(h) for the unnormalised butterfly outputs v; a row of zeros gets 1.
template <int BITS>
struct DynamicStep {
    double inv_sqrt_h;
    float clip;
    float* red;        // 4 floats of LDS
    float* step_out;   // this row's slot of row_scale
    int tid;
    float mult_, step_;   // set by prepare()
    template <int NV>
    __device__ __forceinline__ void prepare(const float (&v)[NV])
    {
        float step;
        float amax = 0.0f;   // dead groups hold zeros
#pragma unroll
        for (int i = 0; i < NV; ++i) amax = fmaxf(amax, fabsf(v[i]));
        amax = fmaxf(amax, rq::lane_xor<0>(amax));
        amax = fmaxf(amax, rq::lane_xor<1>(amax));
        amax = fmaxf(amax, rq::lane_xor<2>(amax));
        amax = fmaxf(amax, rq::lane_xor<3>(amax));
        amax = fmaxf(amax, rq::lane_xor<4>(amax));
        amax = fmaxf(amax, rq::lane_xor<5>(amax));
        if ((tid & 63) == 0) red[tid >> 6] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        constexpr double qmax = BITS == 8 ? 127.0 : 7.0;
        step = (float)(((double)clip * ((double)amax * inv_sqrt_h)) / qmax);
        if (!(step > 0.0f)) step = 1.0f;
        step_ = step;
        mult_ = (float)(inv_sqrt_h / (double)step);
        if (tid == 0) *step_out = step;
    }
    __device__ __forceinline__ void get(int64_t, float& m, float& s) const { m = mult_; s = step_; }
    __device__ __forceinline__ int zero_offset() const { return 0; }
};

// Per-token dynamic variant (Table 1 row O1): the step size of a row depends on that row's rotated
// values, so a workgroup owns a whole row: NC chunks of 2048 channels stay in registers
// (K <= 2048 NC) between the rotation, the row maximum and the quantizer.  The row's step goes to
// row_scale[m]; codes as in the static kernels (BITS = 4 packed, 8 grouped bytes).
template <int NC, int BITS>
__global__ __launch_bounds__(kThreads) void k_rotate_quant_dyn(const __half* __restrict__ x, int64_t K, int log2h,
                                                              double inv_sqrt_h, float clip,
                                                              uint32_t* __restrict__ xq, float* __restrict__ row_scale)
{
    extern __shared__ float xch_dyn[];   // 2048 NC floats when log2h > 9, else unused
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    v4i raw[NC];
    bool live[NC];
    rq::load_chunk<NC>(static_cast<const __half*>(x + row * K), K, 0, tid, true, raw, live);
    const DynamicStep<BITS> steps{inv_sqrt_h, clip, red, row_scale + row, tid, 0.0f, 0.0f};
    uint32_t* dst_row = xq + row * (BITS == 8 ? K >> 2 : K >> 3);
    if (log2h == 0)
        rq::rotate_quant_regs_with<NC, true, BITS>(raw, live, 0, 0, steps, dst_row, (rq::lds_f32_ptr)xch_dyn, tid, true);
    else
        rq::rotate_quant_regs_with<NC, false, BITS>(raw, live, 0, log2h, steps, dst_row, (rq::lds_f32_ptr)xch_dyn, tid,
                                                    true);
}

// Producer fusion for qkv / gate / up: RMS normalisation (its learned weight folded into the next
// linear, as rotation absorption requires) followed by the static quantizer.  The step of the
// normalised row is static; what the row supplies is 1 / rms.
struct NormStep {
    double inv_step;   // 1 / s
    double inv_k;      // 1 / K
    float eps, step;
    float* red;        // 4 floats of LDS
    int tid;
    float mult_;
    template <int NV>
    __device__ __forceinline__ void prepare(const float (&v)[NV])
    {
        float ss = 0.0f;   // dead groups hold zeros
#pragma unroll
        for (int i = 0; i < NV; ++i) ss = fmaf(v[i], v[i], ss);
        ss += rq::lane_xor<0>(ss);
        ss += rq::lane_xor<1>(ss);
        ss += rq::lane_xor<2>(ss);
        ss += rq::lane_xor<3>(ss);
        ss += rq::lane_xor<4>(ss);
        ss += rq::lane_xor<5>(ss);
        if ((tid & 63) == 0) red[tid >> 6] = ss;
        __syncthreads();
        const double total = ((double)red[0] + (double)red[1]) + ((double)red[2] + (double)red[3]);
        mult_ = (float)(inv_step / sqrt(total * inv_k + (double)eps));
    }
    __device__ __forceinline__ void get(int64_t, float& m, float& s) const { m = mult_; s = step; }
    __device__ __forceinline__ int zero_offset() const { return 0; }
};

template <int NC>
__global__ __launch_bounds__(kThreads) void k_rmsnorm_quant(const __half* __restrict__ x, int64_t K, double inv_step,
                                                           float eps, float step, uint32_t* __restrict__ xq)
{
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    v4i raw[NC];
    bool live[NC];
    rq::load_chunk<NC>(static_cast<const __half*>(x + row * K), K, 0, tid, true, raw, live);
    const NormStep steps{inv_step, 1.0 / (double)K, eps, step, red, tid, 0.0f};
    rq::rotate_quant_regs_with<NC, false, 4>(raw, live, 0, 0, steps, static_cast<uint32_t*>(xq + row * (K >> 3)),
                                             (rq::lds_f32_ptr) nullptr, tid, true);
}

template <int NC, int BITS>
int launch_dyn_nc(const __half* xp, int64_t M, int64_t K, int log2h, double inv_sqrt_h, float clip, uint32_t* op,
                  float* row_scale, hipStream_t st)
{
    const size_t lds = log2h > 9 ? (size_t)NC * kChunk * sizeof(float) : 0;
    auto kern = k_rotate_quant_dyn<NC, BITS>;
    static std::atomic<uint64_t> lds_ok{0};
    if (lds > 48 * 1024 &&
        allow_dynamic_lds(reinterpret_cast<const void*>(kern), (size_t)NC * kChunk * sizeof(float), lds_ok) != PQ_OK)
        return PQ_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)M), dim3(kThreads), lds, st, xp, K, log2h, inv_sqrt_h, clip, op, row_scale);
    return hip_status(hipGetLastError());
}

template <int BITS>
int launch_dyn(const __half* xp, int64_t M, int64_t K, int32_t h, float clip, uint32_t* op, float* row_scale,
               hipStream_t st)
{
    if (K > 16 * kChunk || M > 0x7fffffff) return PQ_ERR_UNSUPPORTED;
    int log2h = 0;
    while ((1 << log2h) < h) ++log2h;
    const double inv_sqrt_h = h > 1 ? 1.0 / sqrt((double)h) : 1.0;
    const int nc = (int)((K + kChunk - 1) / kChunk);
    if (nc <= 1) return launch_dyn_nc<1, BITS>(xp, M, K, log2h, inv_sqrt_h, clip, op, row_scale, st);
    if (nc <= 2) return launch_dyn_nc<2, BITS>(xp, M, K, log2h, inv_sqrt_h, clip, op, row_scale, st);
    if (nc <= 4) return launch_dyn_nc<4, BITS>(xp, M, K, log2h, inv_sqrt_h, clip, op, row_scale, st);
    if (nc <= 8) return launch_dyn_nc<8, BITS>(xp, M, K, log2h, inv_sqrt_h, clip, op, row_scale, st);
    return launch_dyn_nc<16, BITS>(xp, M, K, log2h, inv_sqrt_h, clip, op, row_scale, st);
}

}  // namespace

int launch_rotate_quant(const void* x, int64_t M, int64_t K, int32_t h, float act_scale, void* xq, hipStream_t st)
{
    // 128-point blocks (down_proj of the Llama models): the rotation runs on the matrix pipe, in the kernel that
    // also writes the prepacked form, so both forms of the layer see the same codes
    if (rotate128_mfma_supported(M, K, h)) return launch_rotate128_mfma(x, M, K, act_scale, nullptr, xq, st);
    return launch_rq<4>(static_cast<const __half*>(x), M, K, h, static_step(act_scale, h), static_cast<uint32_t*>(xq), st);
}

// Eq. 1 with a zero-point: stored code = clamp(round(y / s) + z, 0, 15) - 8.
int launch_rotate_quant_zp(const void* x, int64_t M, int64_t K, int32_t h, float act_scale, int32_t zero_point, void* xq,
                           hipStream_t st)
{
    const rq::StaticStep b = static_step(act_scale, h);
    return launch_rq<4>(static_cast<const __half*>(x), M, K, h, rq::StaticStepZp{b.mult, b.step, zero_point - 8},
                        static_cast<uint32_t*>(xq), st);
}

int launch_rotate_quant8(const void* x, int64_t M, int64_t K, int32_t h, float act_scale, void* xq8, hipStream_t st)
{
    return launch_rq<8>(static_cast<const __half*>(x), M, K, h, static_step(act_scale, h), static_cast<uint32_t*>(xq8), st);
}

// Per-head static steps (Table 1 row O2, KV cache): head = channel / head_dim.
int launch_rotate_quant_heads(const void* x, int64_t M, int64_t K, int32_t head_dim, int32_t h, const float* head_scale,
                              void* xq, hipStream_t st)
{
    int log2d = 0;
    while ((1 << log2d) < head_dim) ++log2d;
    const rq::HeadStep steps{head_scale, log2d, h > 1 ? 1.0 / sqrt((double)h) : 1.0};
    return launch_rq<4>(static_cast<const __half*>(x), M, K, h, steps, static_cast<uint32_t*>(xq), st);
}

// Rotation only, fp16 out (queries after RoPE, which are rotated like the keys but not quantized).
int launch_rotate_f16(const void* x, int64_t M, int64_t K, int32_t h, void* y, hipStream_t st)
{
    return launch_rq<16>(static_cast<const __half*>(x), M, K, h, static_step(1.0f, h), static_cast<uint32_t*>(y), st);
}

int launch_rotate_quant_dynamic(const void* x, int64_t M, int64_t K, int32_t h, float clip, int32_t bits, void* xq,
                                float* row_scale, hipStream_t st)
{
    if (bits == 8)
        return launch_dyn<8>(static_cast<const __half*>(x), M, K, h, clip, static_cast<uint32_t*>(xq), row_scale, st);
    return launch_dyn<4>(static_cast<const __half*>(x), M, K, h, clip, static_cast<uint32_t*>(xq), row_scale, st);
}

int launch_silu_mul_rotate_quant(const void* gate, const void* up, int64_t M, int64_t K, int32_t h, float act_scale,
                                 void* xq, hipStream_t st)
{
    const __half* g = static_cast<const __half*>(gate);
    const __half* u = static_cast<const __half*>(up);
    uint32_t* op = static_cast<uint32_t*>(xq);
    for (int64_t m0 = 0; m0 < M; m0 += 65534) {   // grid.y is limited to 65535 per launch
        const int64_t mm = (M - m0 < 65534) ? (M - m0) : 65534;
        int log2h = 0;
        while ((1 << log2h) < h) ++log2h;
        const int G = h <= kChunk ? 1 : h / kChunk;
        const rq::StaticStep steps = static_step(act_scale, h);
        dim3 grid((unsigned)((K + (int64_t)G * kChunk - 1) / ((int64_t)G * kChunk)), (unsigned)((mm + (G <= 2 ? 1 : 0)) / (G <= 2 ? 2 : 1)));
        const __half* gp = g + m0 * K;
        const __half* upp = u + m0 * K;
        uint32_t* o = op + m0 * (K >> 3);
        auto launch = [&](auto streamc) {
            constexpr bool S = decltype(streamc)::value;
            switch (G) {
                case 1: hipLaunchKernelGGL((k_silu_mul_rotate_quant<1, 2, S>), grid, dim3(kThreads), 0, st, gp, upp, mm, K, log2h, steps, o); return true;
                case 2: hipLaunchKernelGGL((k_silu_mul_rotate_quant<2, 2, S>), grid, dim3(kThreads), 0, st, gp, upp, mm, K, log2h, steps, o); return true;
                case 4: hipLaunchKernelGGL((k_silu_mul_rotate_quant<4, 1, S>), grid, dim3(kThreads), 0, st, gp, upp, mm, K, log2h, steps, o); return true;
                case 8: hipLaunchKernelGGL((k_silu_mul_rotate_quant<8, 1, S>), grid, dim3(kThreads), 0, st, gp, upp, mm, K, log2h, steps, o); return true;
                default: return false;
            }
        };
        const bool known = mm * (K >> 1) <= rq::kStreamBelow ? launch(std::true_type{}) : launch(std::false_type{});
        if (!known) return PQ_ERR_UNSUPPORTED;
        const int rc = hip_status(hipGetLastError());
        if (rc != PQ_OK) return rc;
    }
    return PQ_OK;
}

int launch_rmsnorm_quant(const void* x, int64_t M, int64_t K, float eps, float act_scale, void* xq, hipStream_t st)
{
    if (K > 16 * kChunk || M > 0x7fffffff) return PQ_ERR_UNSUPPORTED;
    const __half* xp = static_cast<const __half*>(x);
    uint32_t* op = static_cast<uint32_t*>(xq);
    const double inv_step = 1.0 / (double)act_scale;
    const int nc = (int)((K + kChunk - 1) / kChunk);
    const dim3 grid((unsigned)M), block(kThreads);
    if (nc <= 1) hipLaunchKernelGGL(k_rmsnorm_quant<1>, grid, block, 0, st, xp, K, inv_step, eps, act_scale, op);
    else if (nc <= 2) hipLaunchKernelGGL(k_rmsnorm_quant<2>, grid, block, 0, st, xp, K, inv_step, eps, act_scale, op);
    else if (nc <= 4) hipLaunchKernelGGL(k_rmsnorm_quant<4>, grid, block, 0, st, xp, K, inv_step, eps, act_scale, op);
    else if (nc <= 8) hipLaunchKernelGGL(k_rmsnorm_quant<8>, grid, block, 0, st, xp, K, inv_step, eps, act_scale, op);
    else hipLaunchKernelGGL(k_rmsnorm_quant<16>, grid, block, 0, st, xp, K, inv_step, eps, act_scale, op);
    return hip_status(hipGetLastError());
}

int launch_rotate_quant_groups(const void* x, int64_t M, int64_t K, int32_t group, int32_t h, float clip, void* xq,
                               float* group_scale, hipStream_t st)
{
    const __half* xp = static_cast<const __half*>(x);
    uint32_t* op = static_cast<uint32_t*>(xq);
    int log2gs = 0, log2h = 0;
    while ((1 << log2gs) < group) ++log2gs;
    while ((1 << log2h) < h) ++log2h;
    const double inv_sqrt_h = h > 1 ? 1.0 / sqrt((double)h) : 1.0;
    const int G = h <= kChunk ? 1 : h / kChunk;
    for (int64_t m0 = 0; m0 < M; m0 += 65535) {   // grid.y is limited to 65535 per launch
        const int64_t mm = (M - m0 < 65535) ? (M - m0) : 65535;
        dim3 grid((unsigned)((K + (int64_t)G * kChunk - 1) / ((int64_t)G * kChunk)), (unsigned)mm);
        const __half* xs = xp + m0 * K;
        uint32_t* os = op + m0 * (K >> 3);
        float* gs = group_scale + m0 * (K >> log2gs);
        if (h <= 1) hipLaunchKernelGGL((k_rotate_quant_groups<1, true>), grid, dim3(kThreads), 0, st, xs, mm, K, 0, inv_sqrt_h, clip, log2gs, os, gs);
        else if (G == 1) hipLaunchKernelGGL((k_rotate_quant_groups<1, false>), grid, dim3(kThreads), 0, st, xs, mm, K, log2h, inv_sqrt_h, clip, log2gs, os, gs);
        else return PQ_ERR_UNSUPPORTED;
        const int rc = hip_status(hipGetLastError());
        if (rc != PQ_OK) return rc;
    }
    return PQ_OK;
}

}  // namespace pq
