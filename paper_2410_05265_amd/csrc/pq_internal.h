// Internal declarations shared by the translation units of libpq (gfx950 only).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/pq.h"

namespace pq {

// Launchers: arguments are already validated by the C entry points.
int launch_rotate_quant(const void* x, int64_t M, int64_t K, int32_t h, float act_scale,
                        void* xq, hipStream_t st);
int launch_rotate_quant_zp(const void* x, int64_t M, int64_t K, int32_t h, float act_scale, int32_t zero_point,
                           void* xq, hipStream_t st);
int launch_rotate_quant8(const void* x, int64_t M, int64_t K, int32_t h, float act_scale,
                         void* xq8, hipStream_t st);
// (ws, ws_bytes, force of the three widened products: as for launch_gemm_mfma_ws below)
int launch_gemm_w4a8(const void* xq8, const void* wq, const float* sw, float sx, int64_t M,
                     int64_t N, int64_t K, void* out, int32_t* acc, hipStream_t st, void* ws = nullptr,
                     size_t ws_bytes = 0, bool force = false);
int launch_rotate_quant_dynamic(const void* x, int64_t M, int64_t K, int32_t h, float clip, int32_t bits,
                                void* xq, float* row_scale, hipStream_t st);
int launch_gemm_dynamic(const void* xq, int32_t bits, const void* wq, const float* sw, const float* srow,
                        int64_t M, int64_t N, int64_t K, void* out, int32_t* acc, hipStream_t st,
                        void* ws = nullptr, size_t ws_bytes = 0, bool force = false);
int launch_rotate_quant_heads(const void* x, int64_t M, int64_t K, int32_t head_dim, int32_t h,
                              const float* head_scale, void* xq, hipStream_t st);
int launch_rotate_f16(const void* x, int64_t M, int64_t K, int32_t h, void* y, hipStream_t st);
int launch_silu_mul_rotate_quant(const void* gate, const void* up, int64_t M, int64_t K, int32_t h,
                                 float act_scale, void* xq, hipStream_t st);
int launch_rmsnorm_quant(const void* x, int64_t M, int64_t K, float eps, float act_scale, void* xq,
                         hipStream_t st);
int launch_rotate_quant_groups(const void* x, int64_t M, int64_t K, int32_t group, int32_t h, float clip, void* xq,
                               float* group_scale, hipStream_t st);
int max_calibration_grid();
int launch_calibrate(const void* x, int64_t T, int64_t K, int32_t h, int32_t bits, int32_t n_grid, float gamma_min,
                     float* result, float* ws, hipStream_t st);
int launch_gemm_zp(const void* xq, const void* wq, const float* sw, float sx, const int32_t* zcorr, int64_t M,
                   int64_t N, int64_t K, void* out, int32_t* acc, hipStream_t st, void* ws = nullptr,
                   size_t ws_bytes = 0, bool force = false);
int launch_zero_point_correction(const void* wq, int64_t N, int64_t K, int32_t zero_point, int32_t* corr,
                                 hipStream_t st);
int launch_calibrate_zp(const void* x, int64_t T, int64_t K, int32_t h, int32_t ng, int32_t nb, float gamma_min,
                        float beta_min, float* result, float* ws, hipStream_t st);
int launch_gemm_simple(const void* xq, const void* wq, const float* sw, float sx, int64_t M,
                       int64_t N, int64_t K, void* out, int32_t* acc, hipStream_t st);
int launch_gemm_mfma(const void* xq, const void* wq, const float* sw, float sx, int64_t M,
                     int64_t N, int64_t K, void* out, int32_t* acc, hipStream_t st);
// The tiled kernel with K split over workgroups where a cost model finds that cheaper (few tokens
// per CU); ws holds the partial planes (gemm_splitk_workspace_bytes; 0 = never splits for the shape),
// a smaller one gets fewer planes or the unsplit launch.  force: split whenever K has two runs of two
// stages and ws holds two planes (tests); PQ_ERR_UNSUPPORTED if not.
size_t gemm_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, bool force = false);
// the cost model's microseconds for the unsplit tiled launch (used to choose between kernels)
double gemm_unsplit_cost_us(int64_t M, int64_t N, int64_t K);
int launch_gemm_mfma_ws(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                        void* out, int32_t* acc, void* ws, size_t ws_bytes, bool force, hipStream_t st);
int launch_probe_mfma(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups, int32_t* sink,
                      hipStream_t st);
int launch_probe_read(const void* src, int64_t bytes, int32_t* sink, hipStream_t st);
int launch_probe_mfma_f6(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups, int32_t* sink,
                         hipStream_t st);
// f6 tiles: the register images of the 6-bit matrix instruction, see pq_gemm_f6.hip
size_t f6_tiles_bytes(int64_t R, int64_t K);
bool rotate128_mfma_supported(int64_t R, int64_t K, int32_t h);
int launch_rotate128_mfma(const void* x, int64_t R, int64_t K, float act_scale, void* tiles, void* nibbles, hipStream_t st);
bool quant_f6_supported(int64_t R, int64_t K, int32_t h);
int launch_quant_f6(const void* x, int64_t R, int64_t K, int32_t h, float act_scale, void* out, void* nibbles, hipStream_t st);
int launch_repack_f6(const void* codes, int64_t R, int64_t K, void* out, hipStream_t st);
int launch_gemm_f6(const void* x6, const void* w6, const float* sw, float sx, int64_t M, int64_t N, int64_t K, void* out,
                   int32_t* acc, hipStream_t st);
int launch_probe_f6_product(const int8_t* a, const int8_t* b, int64_t K, int32_t* out, hipStream_t st);

// forced tile configurations (sweeps and tests): previous value, or -2 for an unknown one
int set_gemm_tile(int tile);
int set_gemm_f6_tile(int tile);

bool stream_mfma_supported(int64_t M, int64_t N, int64_t K, int32_t abits = 4);
int stream_mfma_launches(int64_t M, int64_t N, int64_t K, int32_t abits = 4);   // for a supported shape
int launch_stream_mfma(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
                       void* out, int32_t* acc, hipStream_t st, const float* srow = nullptr, int32_t abits = 4,
                       const int32_t* zcorr = nullptr);

// A second weight matrix for the same tokens in the same launch (gate and up of an MLP): its rows follow the
// n1 rows of the first (n1 % 16 == 0), N of launch_decode counts both, and its product goes to an output of
// its own, [M, N - n1].  Only with plain fp16 outputs (no accumulators, per-token steps or zero-point).
struct DecodeSecond {
    const uint8_t* wq;
    const float* sw;
    __half* out;
    int n1;
};

bool decode_supported(int64_t M, int64_t N, int64_t K, int32_t h, int32_t abits = 4);
int launch_decode(const void* x_f16, const void* xq_in, const void* wq, const float* sw, float sx, int32_t h,
                  int64_t M, int64_t N, int64_t K, void* out, int32_t* acc, void* xq_out, hipStream_t st,
                  const float* srow = nullptr, int32_t abits = 4, const int32_t* zcorr = nullptr,
                  const DecodeSecond* second = nullptr);

inline int hip_status(hipError_t e) { return e == hipSuccess ? PQ_OK : PQ_ERR_HIP; }

// A kernel may use more than the default amount of dynamic LDS only after the runtime has been told,
// once per kernel and device.  `done` is that kernel's mask of devices already served (a static of
// the caller; two first calls racing is harmless, the setting is idempotent).
inline int allow_dynamic_lds(const void* kern, size_t bytes, std::atomic<uint64_t>& done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PQ_ERR_HIP;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return PQ_OK;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return PQ_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
    return PQ_OK;
}

// A product rounded to fp32 on its own.  Written as a plain a * b the compiler merges the
// multiplication with the conversion to fp16 that follows (one rounding instead of two) in some
// kernels and not in others, and then the kernels of this library would differ from one another in
// an output's last bit.  The empty asm makes the fp32 value opaque.
__device__ __forceinline__ float mul_rn(float a, float b)
{
    float p = a * b;
    asm("" : "+v"(p));
    return p;
}

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Eight packed 4-bit codes (one dword) become two dwords of int8, each byte equal to
// 16 * code: the odd-channel nibbles already sit in the high half of their byte, the
// even-channel nibbles are shifted there.  No sign extension is needed, and a product of
// two such operands is 256 * (code * code), undone exactly by an arithmetic shift.
__device__ __forceinline__ void unpack16(const v4i p, v4i& even, v4i& odd)
{
    const int m = (int)0xF0F0F0F0u;
    even.x = (p.x << 4) & m; even.y = (p.y << 4) & m; even.z = (p.z << 4) & m; even.w = (p.w << 4) & m;
    odd.x = p.x & m; odd.y = p.y & m; odd.z = p.z & m; odd.w = p.w & m;
}

}  // namespace pq
