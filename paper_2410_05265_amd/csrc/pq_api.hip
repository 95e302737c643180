// C entry points of libpq: argument checking and kernel choice.  No device memory is
// allocated here and nothing synchronises; every kernel goes to the caller's stream.
#include "pq_internal.h"

#include <math.h>

#include <atomic>

// Scratch memory of pq_linear_noalloc: the packed activation codes between the quantizer and the
// product (and, behind them, the partial-sum planes of a split launch).  One copy per GPU, at an
// address of its own, alive until the process ends.  In host code this name is only a stand-in for
// the symbol: the device address comes from hipGetSymbolAddress (scratch_base below).
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) uint8_t scratch[kScratchBytes];

namespace {

// Device address of `scratch` on the current device; looked up once per device, with that device
// current, then kept.  Two first calls racing store the same value twice.
constexpr int kMaxDevices = 64;
std::atomic<uint8_t*> g_scratch_ptr[kMaxDevices];

int scratch_base(uint8_t** base)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PQ_ERR_HIP;
    uint8_t* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void* sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return PQ_ERR_HIP;
        p = static_cast<uint8_t*>(sym);
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *base = p;
    return PQ_OK;
}

std::atomic<int> g_variant{0};  // 0 auto, 1 streaming MFMA (M <= 32), 2 MFMA tiled, 3 simple, 4 streaming dot (M <= 8), 5 tiled, K split

// Kernel for a product with given codes and few tokens: 4 = weight-streaming dot products
// (k_decode), 1 = weight-streaming matrix tiles (k_stream_mfma), 2 = the tiled kernel, -1 = the
// forced variant does not support the shape.  The dot-product kernel costs more with every token,
// the matrix kernel costs the same for any count up to 16 but has a higher floor; where they cross
// depends on the size of the matrix (measured on the Llama-3-8B shapes, 8 / 12.6 / 29 MB of
// weights): 4-bit codes from 5 tokens on (9 on small matrices), int8 codes from 3, 5 and 7.
// 17 to 32 tokens are two launches of the matrix kernel where a cost estimate puts that ahead of
// the tiled kernel (8B shapes: everything but gate/up; 70B: not gate/up either, 224 tiles).
int pick_few_tokens(int64_t M, int64_t N, int64_t K, int32_t abits)
{
    const bool dot = M <= 8 && pq::decode_supported(M, N, K, -1, abits);
    const bool mat = M <= 32 && pq::stream_mfma_supported(M, N, K, abits);
    if (g_variant == 4) return dot ? 4 : -1;
    if (g_variant == 1) return mat ? 1 : -1;
    if (g_variant != 0) return 2;
    const int64_t weight_bytes = N * (K / 2);
    const int size = weight_bytes >= 24000000 ? 2 : (weight_bytes >= 12000000 ? 1 : 0);
    const int64_t dot_limit = abits == 8 ? (size == 2 ? 2 : (size == 1 ? 4 : 6)) : (size >= 1 ? 4 : 8);
    if (dot && (M <= dot_limit || !mat)) return 4;
    if (mat) {
        // one launch of up to 16 tokens always; several launches (17..32 tokens, or rows too long for 16
        // tokens' codes in LDS) that each stream the matrix (2.5 us + bytes at ~5 TB/s) against the tiled
        // kernel, whose time there is a walk over K by however many tiles the output has
        const int launches = pq::stream_mfma_launches(M, N, K, abits);
        if (launches == 1) return 1;
        const double stream_us = launches * (2.5 + (double)weight_bytes / 5.0e6);
        if (stream_us < pq::gemm_unsplit_cost_us(M, N, K)) return 1;
    }
    return 2;
}

// The same choice when the call brings scratch memory for partial-sum planes (timings: 4-bit codes).
// Where the matrix streaming kernel needs two or more launches (17 to 32 tokens, or rows too long
// for 16 tokens' codes in LDS), the split tiled launch with its planes in place beats them on
// matrices of 8 MB and more (8B shapes at 24 tokens: 8-13 us against 9-16; not measured below 8 MB).
int pick_with_planes(int64_t M, int64_t N, int64_t K, size_t plane_bytes, int32_t abits = 4)
{
    const int kernel = pick_few_tokens(M, N, K, abits);
    if (g_variant == 0 && kernel == 1 && N * (K / 2) >= 8000000 && pq::stream_mfma_launches(M, N, K, abits) > 1) {
        const size_t want = pq::gemm_splitk_workspace_bytes(M, N, K);
        if (want > 0 && plane_bytes >= want) return 2;
    }
    return kernel;
}

// Whether pq_linear takes the fused launch (every workgroup rotates and quantizes the few rows for itself)
// when the shape allows it, rather than a quantizer launch and a product launch.  Measured with cold weights
// on 8 to 117 MB matrices: without rotation the fused launch is level or ahead up to 32768 channels in all
// (the rows then pass through the quantizer in the registers they were loaded into; 4 tokens of 8192: 10.1
// against 12.6 us); with rotation a CU spends about 0.2 us per 1024 channels, level for one token up to
// 16384 channels (7.4 us both ways at 14336), behind from two tokens on (11.3 against 10.2 us).
inline bool fused_few_tokens(int64_t M, int64_t K, int32_t had_block)
{
    const int64_t total = M * K;
    if (had_block <= 1) return total <= 32768;
    return total <= 8192 || (M == 1 && total <= 16384);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool good_scale(float s) { return isfinite(s) && s > 0.0f; }

int check_gemm(const void* xq, const void* wq, const float* sw, float sx, int64_t M, int64_t N, int64_t K,
               const void* out, const int32_t* acc)
{
    if (M < 0 || N <= 0 || K <= 0 || (K % 32) != 0 || (N % 16) != 0) return PQ_ERR_SHAPE;
    if (!xq || !wq || !sw || (!out && !acc)) return PQ_ERR_NULL;
    if (!aligned16(xq) || !aligned16(wq) || !aligned16(out) || !aligned16(acc) || !aligned16(sw))
        return PQ_ERR_ALIGN;    // (the epilogues load four channel steps at a time)
    if (!good_scale(sx)) return PQ_ERR_SCALE;
    return PQ_OK;
}

}  // namespace

extern "C" {

int pq_version(void) { return 100; }

const char* pq_status_str(int status)
{
    switch (status) {
        case PQ_OK: return "PQ_OK";
        case PQ_ERR_NULL: return "PQ_ERR_NULL";
        case PQ_ERR_SHAPE: return "PQ_ERR_SHAPE";
        case PQ_ERR_ALIGN: return "PQ_ERR_ALIGN";
        case PQ_ERR_SCALE: return "PQ_ERR_SCALE";
        case PQ_ERR_WORKSPACE: return "PQ_ERR_WORKSPACE";
        case PQ_ERR_HIP: return "PQ_ERR_HIP";
        case PQ_ERR_UNSUPPORTED: return "PQ_ERR_UNSUPPORTED";
        default: return "PQ_ERR_UNKNOWN";
    }
}

int pq_rotate_quant(const void* x_f16, int64_t M, int64_t K, int32_t had_block, float act_scale,
                    void* xq_packed, void* stream)
{
    if (M < 0 || K <= 0 || (K % 32) != 0) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!x_f16 || !xq_packed) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(xq_packed)) return PQ_ERR_ALIGN;
    if (!good_scale(act_scale)) return PQ_ERR_SCALE;
    if (M == 0) return PQ_OK;
    return pq::launch_rotate_quant(x_f16, M, K, had_block, act_scale, xq_packed, static_cast<hipStream_t>(stream));
}

int pq_w4a4_gemm_ws(const void* xq_packed, const void* wq_packed, const float* w_scale, float act_scale, int64_t M,
                    int64_t N, int64_t K, void* out_f16, int32_t* acc_i32, void* workspace, size_t workspace_bytes,
                    void* stream)
{
    int rc = check_gemm(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32);
    if (rc != PQ_OK) return rc;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_ALIGN;
    if (M == 0) return PQ_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (g_variant == 3)
        return pq::launch_gemm_simple(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32, st);
    switch (pick_with_planes(M, N, K, workspace ? workspace_bytes : 0)) {
        case 4:
            return pq::launch_decode(nullptr, xq_packed, wq_packed, w_scale, act_scale, 1, M, N, K, out_f16, acc_i32,
                                     nullptr, st);
        case 1: return pq::launch_stream_mfma(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32, st);
        case 2:
            return pq::launch_gemm_mfma_ws(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32,
                                           workspace, workspace ? workspace_bytes : 0, g_variant == 5, st);
        default: return PQ_ERR_UNSUPPORTED;
    }
}

int pq_w4a4_gemm(const void* xq_packed, const void* wq_packed, const float* w_scale, float act_scale, int64_t M,
                 int64_t N, int64_t K, void* out_f16, int32_t* acc_i32, void* stream)
{
    return pq_w4a4_gemm_ws(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32, nullptr, 0, stream);
}

size_t pq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int32_t act_bits)
{
    if (M <= 0 || N <= 0 || K <= 0 || (K % 32) != 0 || (N % 16) != 0 || (act_bits != 4 && act_bits != 8)) return 0;
    if (g_variant == 3 || pick_with_planes(M, N, K, ~(size_t)0, act_bits) != 2) return 0;
    return pq::gemm_splitk_workspace_bytes(M, N, K, g_variant == 5);
}

size_t pq_w4a4_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) { return pq_gemm_workspace_bytes(M, N, K, 4); }

int pq_w4a4_gemm_simple(const void* xq_packed, const void* wq_packed, const float* w_scale, float act_scale,
                        int64_t M, int64_t N, int64_t K, void* out_f16, int32_t* acc_i32, void* stream)
{
    int rc = check_gemm(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32);
    if (rc != PQ_OK) return rc;
    if (M == 0) return PQ_OK;
    return pq::launch_gemm_simple(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32,
                                  static_cast<hipStream_t>(stream));
}

size_t pq_linear_workspace_bytes(int64_t M, int64_t K)
{
    if (M <= 0 || K <= 0) return 0;
    const size_t b = (size_t)M * (size_t)(K / 2);
    return (b + 255) & ~(size_t)255;
}

int pq_linear(const void* x_f16, const void* wq_packed, const float* w_scale, float act_scale, int32_t had_block,
              int64_t M, int64_t N, int64_t K, void* out_f16, void* workspace, size_t workspace_bytes, void* stream)
{
    if (M < 0 || N <= 0 || K <= 0 || (K % 32) != 0 || (N % 16) != 0) return PQ_ERR_SHAPE;
    if (!x_f16 || !wq_packed || !w_scale || !out_f16) return PQ_ERR_NULL;
    if (M == 0) return PQ_OK;
    if (!workspace || workspace_bytes < pq_linear_workspace_bytes(M, K)) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    // check the second stage's arguments before anything is enqueued
    int rc = check_gemm(workspace, wq_packed, w_scale, act_scale, M, N, K, out_f16, nullptr);
    if (rc != PQ_OK) return rc;
    if (had_block < 0 || had_block > 16384 ||
        (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)))
        return PQ_ERR_SHAPE;
    if (!aligned16(x_f16)) return PQ_ERR_ALIGN;
    // decode: one fused launch (rotate + quantize per workgroup, weights streamed once)
    if (((g_variant == 0 && fused_few_tokens(M, K, had_block)) || g_variant == 4) &&
        pq::decode_supported(M, N, K, had_block))
        return pq::launch_decode(x_f16, nullptr, wq_packed, w_scale, act_scale, had_block, M, N, K, out_f16, nullptr,
                                 workspace, static_cast<hipStream_t>(stream));
    rc = pq_rotate_quant(x_f16, M, K, had_block, act_scale, workspace, stream);
    if (rc != PQ_OK) return rc;
    // whatever the workspace holds beyond the codes serves the product's split launch
    const size_t codes = pq_linear_workspace_bytes(M, K);
    return pq_w4a4_gemm_ws(workspace, wq_packed, w_scale, act_scale, M, N, K, out_f16, nullptr,
                           static_cast<uint8_t*>(workspace) + codes, workspace_bytes - codes, stream);
}

int pq_linear2(const void* x_f16, const void* wq_a, const float* w_scale_a, int64_t N_a, void* out_a_f16,
               const void* wq_b, const float* w_scale_b, int64_t N_b, void* out_b_f16, float act_scale,
               int32_t had_block, int64_t M, int64_t K, void* workspace, size_t workspace_bytes, void* stream)
{
    if (M < 0 || N_a <= 0 || N_b <= 0 || K <= 0 || (K % 32) != 0 || (N_a % 16) != 0 || (N_b % 16) != 0) return PQ_ERR_SHAPE;
    if (!x_f16 || !wq_a || !w_scale_a || !out_a_f16 || !wq_b || !w_scale_b || !out_b_f16) return PQ_ERR_NULL;
    if (M == 0) return PQ_OK;
    if (!workspace || workspace_bytes < pq_linear_workspace_bytes(M, K)) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    int rc = check_gemm(workspace, wq_a, w_scale_a, act_scale, M, N_a, K, out_a_f16, nullptr);
    if (rc == PQ_OK) rc = check_gemm(workspace, wq_b, w_scale_b, act_scale, M, N_b, K, out_b_f16, nullptr);
    if (rc != PQ_OK) return rc;
    if (had_block < 0 || had_block > 16384 ||
        (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)))
        return PQ_ERR_SHAPE;
    if (!aligned16(x_f16)) return PQ_ERR_ALIGN;
    // few tokens: one launch streams both matrices (the rule of pq_linear, on the rows of both)
    if (((g_variant == 0 && fused_few_tokens(M, K, had_block)) || g_variant == 4) &&
        N_a + N_b <= (1 << 30) && pq::decode_supported(M, N_a + N_b, K, had_block)) {
        const pq::DecodeSecond second{static_cast<const uint8_t*>(wq_b), w_scale_b, static_cast<__half*>(out_b_f16), (int)N_a};
        return pq::launch_decode(x_f16, nullptr, wq_a, w_scale_a, act_scale, had_block, M, N_a + N_b, K, out_a_f16, nullptr,
                                 workspace, static_cast<hipStream_t>(stream), nullptr, 4, nullptr, &second);
    }
    rc = pq_rotate_quant(x_f16, M, K, had_block, act_scale, workspace, stream);
    if (rc != PQ_OK) return rc;
    const size_t codes = pq_linear_workspace_bytes(M, K);
    uint8_t* planes = static_cast<uint8_t*>(workspace) + codes;
    rc = pq_w4a4_gemm_ws(workspace, wq_a, w_scale_a, act_scale, M, N_a, K, out_a_f16, nullptr, planes, workspace_bytes - codes, stream);
    if (rc != PQ_OK) return rc;
    return pq_w4a4_gemm_ws(workspace, wq_b, w_scale_b, act_scale, M, N_b, K, out_b_f16, nullptr, planes, workspace_bytes - codes, stream);
}

size_t pq_linear_workspace_bytes_split(int64_t M, int64_t N, int64_t K)
{
    return pq_linear_workspace_bytes(M, K) + pq_w4a4_gemm_workspace_bytes(M, N, K);
}

int pq_rotate_quant8(const void* x_f16, int64_t M, int64_t K, int32_t had_block, float act_scale,
                     void* xq8_grouped, void* stream)
{
    if (M < 0 || K <= 0 || (K % 128) != 0) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!x_f16 || !xq8_grouped) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(xq8_grouped)) return PQ_ERR_ALIGN;
    if (!good_scale(act_scale)) return PQ_ERR_SCALE;
    if (M == 0) return PQ_OK;
    return pq::launch_rotate_quant8(x_f16, M, K, had_block, act_scale, xq8_grouped, static_cast<hipStream_t>(stream));
}

int pq_w4a8_gemm_ws(const void* xq8_grouped, const void* wq_packed, const float* w_scale, float act_scale, int64_t M,
                    int64_t N, int64_t K, void* out_f16, int32_t* acc_i32, void* workspace, size_t workspace_bytes,
                    void* stream)
{
    int rc = check_gemm(xq8_grouped, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32);
    if (rc != PQ_OK) return rc;
    if ((K % 128) != 0) return PQ_ERR_SHAPE;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_ALIGN;
    if (M == 0) return PQ_OK;
    const int few = pick_with_planes(M, N, K, workspace ? workspace_bytes : 0, 8);
    if (few == 4)
        return pq::launch_decode(nullptr, xq8_grouped, wq_packed, w_scale, act_scale, 1, M, N, K, out_f16, acc_i32,
                                 nullptr, static_cast<hipStream_t>(stream), nullptr, 8);
    if (few == 1)
        return pq::launch_stream_mfma(xq8_grouped, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32,
                                      static_cast<hipStream_t>(stream), nullptr, 8);
    return pq::launch_gemm_w4a8(xq8_grouped, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32,
                                static_cast<hipStream_t>(stream), workspace, workspace ? workspace_bytes : 0,
                                g_variant == 5);
}

int pq_w4a8_gemm(const void* xq8_grouped, const void* wq_packed, const float* w_scale, float act_scale, int64_t M,
                 int64_t N, int64_t K, void* out_f16, int32_t* acc_i32, void* stream)
{
    return pq_w4a8_gemm_ws(xq8_grouped, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32, nullptr, 0, stream);
}

size_t pq_linear_w4a8_workspace_bytes(int64_t M, int64_t K)
{
    if (M <= 0 || K <= 0) return 0;
    const size_t b = (size_t)M * (size_t)K;
    return (b + 255) & ~(size_t)255;
}

int pq_linear_w4a8(const void* x_f16, const void* wq_packed, const float* w_scale, float act_scale,
                   int32_t had_block, int64_t M, int64_t N, int64_t K, void* out_f16, void* workspace,
                   size_t workspace_bytes, void* stream)
{
    if (M < 0 || N <= 0 || K <= 0 || (K % 128) != 0 || (N % 16) != 0) return PQ_ERR_SHAPE;
    if (!x_f16 || !wq_packed || !w_scale || !out_f16) return PQ_ERR_NULL;
    if (M == 0) return PQ_OK;
    if (!workspace || workspace_bytes < pq_linear_w4a8_workspace_bytes(M, K)) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    int rc = check_gemm(workspace, wq_packed, w_scale, act_scale, M, N, K, out_f16, nullptr);
    if (rc != PQ_OK) return rc;
    if (had_block < 0 || had_block > 16384 ||
        (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)))
        return PQ_ERR_SHAPE;
    if (!aligned16(x_f16)) return PQ_ERR_ALIGN;
    if (K > 65536 || M * K >= ((int64_t)1 << 32)) return PQ_ERR_UNSUPPORTED;
    rc = pq_rotate_quant8(x_f16, M, K, had_block, act_scale, workspace, stream);
    if (rc != PQ_OK) return rc;
    const size_t codes = pq_linear_w4a8_workspace_bytes(M, K);
    return pq_w4a8_gemm_ws(workspace, wq_packed, w_scale, act_scale, M, N, K, out_f16, nullptr,
                           static_cast<uint8_t*>(workspace) + codes, workspace_bytes - codes, stream);
}

size_t pq_linear_w4a8_workspace_bytes_split(int64_t M, int64_t N, int64_t K)
{
    return pq_linear_w4a8_workspace_bytes(M, K) + pq_gemm_workspace_bytes(M, N, K, 8);
}

int pq_rotate_quant_dynamic(const void* x_f16, int64_t M, int64_t K, int32_t had_block, float clip, int32_t bits,
                            void* xq, float* row_scale, void* stream)
{
    if (M < 0 || K <= 0 || (K % 128) != 0 || (bits != 4 && bits != 8)) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!x_f16 || !xq || !row_scale) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(xq) || (reinterpret_cast<uintptr_t>(row_scale) & 3u)) return PQ_ERR_ALIGN;
    if (!(isfinite(clip) && clip > 0.0f && clip <= 1.0f)) return PQ_ERR_SCALE;
    if (K > 32768) return PQ_ERR_UNSUPPORTED;
    if (M == 0) return PQ_OK;
    return pq::launch_rotate_quant_dynamic(x_f16, M, K, had_block, clip, bits, xq, row_scale,
                                           static_cast<hipStream_t>(stream));
}

int pq_gemm_dynamic_ws(const void* xq, int32_t bits, const void* wq_packed, const float* w_scale,
                       const float* row_scale, int64_t M, int64_t N, int64_t K, void* out_f16, int32_t* acc_i32,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    if (bits != 4 && bits != 8) return PQ_ERR_SHAPE;
    int rc = check_gemm(xq, wq_packed, w_scale, 1.0f, M, N, K, out_f16, acc_i32);
    if (rc != PQ_OK) return rc;
    if ((K % 128) != 0) return PQ_ERR_SHAPE;
    if (!row_scale) return PQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(row_scale) & 3u) return PQ_ERR_ALIGN;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_ALIGN;
    if (M == 0) return PQ_OK;
    // decode: a weight-streaming kernel with the token's step in its epilogue
    const int few = pick_with_planes(M, N, K, workspace ? workspace_bytes : 0, bits);
    if (few == 4)
        return pq::launch_decode(nullptr, xq, wq_packed, w_scale, 1.0f, 1, M, N, K, out_f16, acc_i32, nullptr,
                                 static_cast<hipStream_t>(stream), row_scale, bits);
    if (few == 1)
        return pq::launch_stream_mfma(xq, wq_packed, w_scale, 1.0f, M, N, K, out_f16, acc_i32,
                                      static_cast<hipStream_t>(stream), row_scale, bits);
    return pq::launch_gemm_dynamic(xq, bits, wq_packed, w_scale, row_scale, M, N, K, out_f16, acc_i32,
                                   static_cast<hipStream_t>(stream), workspace, workspace ? workspace_bytes : 0,
                                   g_variant == 5);
}

int pq_gemm_dynamic(const void* xq, int32_t bits, const void* wq_packed, const float* w_scale, const float* row_scale,
                    int64_t M, int64_t N, int64_t K, void* out_f16, int32_t* acc_i32, void* stream)
{
    return pq_gemm_dynamic_ws(xq, bits, wq_packed, w_scale, row_scale, M, N, K, out_f16, acc_i32, nullptr, 0, stream);
}

size_t pq_linear_dynamic_workspace_bytes(int64_t M, int64_t K, int32_t bits)
{
    if (M <= 0 || K <= 0 || (bits != 4 && bits != 8)) return 0;
    const size_t codes = bits == 8 ? (size_t)M * (size_t)K : (size_t)M * (size_t)(K / 2);
    return ((codes + 255) & ~(size_t)255) + (((size_t)M * 4 + 255) & ~(size_t)255);
}

int pq_linear_dynamic(const void* x_f16, const void* wq_packed, const float* w_scale, float clip, int32_t had_block,
                      int32_t bits, int64_t M, int64_t N, int64_t K, void* out_f16, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    if (M < 0 || N <= 0 || K <= 0 || (K % 128) != 0 || (N % 16) != 0 || (bits != 4 && bits != 8)) return PQ_ERR_SHAPE;
    if (!x_f16 || !wq_packed || !w_scale || !out_f16) return PQ_ERR_NULL;
    if (M == 0) return PQ_OK;
    const size_t need = pq_linear_dynamic_workspace_bytes(M, K, bits);
    if (!workspace || workspace_bytes < need) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    float* row_scale = reinterpret_cast<float*>(static_cast<uint8_t*>(workspace) + need -
                                                (((size_t)M * 4 + 255) & ~(size_t)255));
    int rc = check_gemm(workspace, wq_packed, w_scale, 1.0f, M, N, K, out_f16, nullptr);
    if (rc != PQ_OK) return rc;
    if (K > 32768 || M * K >= ((int64_t)1 << 32)) return PQ_ERR_UNSUPPORTED;
    rc = pq_rotate_quant_dynamic(x_f16, M, K, had_block, clip, bits, workspace, row_scale, stream);
    if (rc != PQ_OK) return rc;
    return pq_gemm_dynamic_ws(workspace, bits, wq_packed, w_scale, row_scale, M, N, K, out_f16, nullptr,
                              static_cast<uint8_t*>(workspace) + need, workspace_bytes - need, stream);
}

size_t pq_linear_dynamic_workspace_bytes_split(int64_t M, int64_t N, int64_t K, int32_t bits)
{
    const size_t base = pq_linear_dynamic_workspace_bytes(M, K, bits);
    return base ? base + pq_gemm_workspace_bytes(M, N, K, bits) : 0;
}

int pq_rotate_quant_heads(const void* x_f16, int64_t T, int32_t n_heads, int32_t head_dim, int32_t rotate,
                          const float* head_scale, void* xq_packed, void* stream)
{
    if (T < 0 || n_heads <= 0 || head_dim < 32 || head_dim > 2048 || (head_dim & (head_dim - 1)) != 0)
        return PQ_ERR_SHAPE;
    if (!x_f16 || !head_scale || !xq_packed) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(xq_packed) || (reinterpret_cast<uintptr_t>(head_scale) & 3u))
        return PQ_ERR_ALIGN;
    if (T == 0) return PQ_OK;
    return pq::launch_rotate_quant_heads(x_f16, T, (int64_t)n_heads * head_dim, head_dim, rotate ? head_dim : 1,
                                         head_scale, xq_packed, static_cast<hipStream_t>(stream));
}

int pq_rotate_quant_groups(const void* x_f16, int64_t T, int32_t n_heads, int32_t head_dim, int32_t rotate,
                           int32_t group, float clip, void* xq_packed, float* group_scale, void* stream)
{
    if (T < 0 || n_heads <= 0 || head_dim < 32 || head_dim > 2048 || (head_dim & (head_dim - 1)) != 0)
        return PQ_ERR_SHAPE;
    if ((group != 32 && group != 64 && group != 128) || (head_dim % group) != 0) return PQ_ERR_SHAPE;
    if (!x_f16 || !xq_packed || !group_scale) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(xq_packed) || (reinterpret_cast<uintptr_t>(group_scale) & 3u))
        return PQ_ERR_ALIGN;
    if (!(isfinite(clip) && clip > 0.0f && clip <= 1.0f)) return PQ_ERR_SCALE;
    if (T == 0) return PQ_OK;
    return pq::launch_rotate_quant_groups(x_f16, T, (int64_t)n_heads * head_dim, group, rotate ? head_dim : 1, clip,
                                          xq_packed, group_scale, static_cast<hipStream_t>(stream));
}

int pq_rotate_f16(const void* x_f16, int64_t M, int64_t K, int32_t had_block, void* y_f16, void* stream)
{
    if (M < 0 || K <= 0 || (K % 32) != 0) return PQ_ERR_SHAPE;
    if (had_block < 2 || had_block > 16384 || (had_block & (had_block - 1)) != 0 || (K % had_block) != 0)
        return PQ_ERR_SHAPE;
    if (!x_f16 || !y_f16) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(y_f16)) return PQ_ERR_ALIGN;
    if (M == 0) return PQ_OK;
    return pq::launch_rotate_f16(x_f16, M, K, had_block, y_f16, static_cast<hipStream_t>(stream));
}

int pq_silu_mul_rotate_quant(const void* gate_f16, const void* up_f16, int64_t M, int64_t K, int32_t had_block,
                             float act_scale, void* xq_packed, void* stream)
{
    if (M < 0 || K <= 0 || (K % 32) != 0) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!gate_f16 || !up_f16 || !xq_packed) return PQ_ERR_NULL;
    if (!aligned16(gate_f16) || !aligned16(up_f16) || !aligned16(xq_packed)) return PQ_ERR_ALIGN;
    if (!good_scale(act_scale)) return PQ_ERR_SCALE;
    if (M == 0) return PQ_OK;
    return pq::launch_silu_mul_rotate_quant(gate_f16, up_f16, M, K, had_block, act_scale, xq_packed,
                                            static_cast<hipStream_t>(stream));
}

int pq_rmsnorm_quant(const void* x_f16, int64_t M, int64_t K, float eps, float act_scale, void* xq_packed,
                     void* stream)
{
    if (M < 0 || K <= 0 || (K % 32) != 0) return PQ_ERR_SHAPE;
    if (!x_f16 || !xq_packed) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(xq_packed)) return PQ_ERR_ALIGN;
    if (!good_scale(act_scale) || !(isfinite(eps) && eps >= 0.0f)) return PQ_ERR_SCALE;
    if (K > 32768) return PQ_ERR_UNSUPPORTED;
    if (M == 0) return PQ_OK;
    return pq::launch_rmsnorm_quant(x_f16, M, K, eps, act_scale, xq_packed, static_cast<hipStream_t>(stream));
}

int pq_rotate_quant_zp(const void* x_f16, int64_t M, int64_t K, int32_t had_block, float act_scale, int32_t zero_point,
                       void* xq_packed, void* stream)
{
    if (M < 0 || K <= 0 || (K % 32) != 0 || zero_point < 0 || zero_point > 15) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!x_f16 || !xq_packed) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(xq_packed)) return PQ_ERR_ALIGN;
    if (!good_scale(act_scale)) return PQ_ERR_SCALE;
    if (M == 0) return PQ_OK;
    return pq::launch_rotate_quant_zp(x_f16, M, K, had_block, act_scale, zero_point, xq_packed,
                                      static_cast<hipStream_t>(stream));
}

int pq_zero_point_correction(const void* wq_packed, int64_t N, int64_t K, int32_t zero_point, int32_t* zp_corr,
                             void* stream)
{
    if (N <= 0 || N > (1 << 30) || K <= 0 || K > (1 << 24) || (K % 32) != 0 || zero_point < 0 || zero_point > 15)
        return PQ_ERR_SHAPE;
    if (!wq_packed || !zp_corr) return PQ_ERR_NULL;
    if (!aligned16(wq_packed) || !aligned16(zp_corr)) return PQ_ERR_ALIGN;
    return pq::launch_zero_point_correction(wq_packed, N, K, zero_point, zp_corr, static_cast<hipStream_t>(stream));
}

int pq_w4a4_gemm_zp_ws(const void* xq_packed, const void* wq_packed, const float* w_scale, float act_scale,
                       const int32_t* zp_corr, int64_t M, int64_t N, int64_t K, void* out_f16, int32_t* acc_i32,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    int rc = check_gemm(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32);
    if (rc != PQ_OK) return rc;
    if ((K % 128) != 0) return PQ_ERR_SHAPE;
    if (!zp_corr) return PQ_ERR_NULL;
    if (!aligned16(zp_corr)) return PQ_ERR_ALIGN;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) return PQ_ERR_ALIGN;
    if (K > 32768) return PQ_ERR_UNSUPPORTED;
    if (M == 0) return PQ_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int few = pick_with_planes(M, N, K, workspace ? workspace_bytes : 0, 4);
    if (few == 4)
        return pq::launch_decode(nullptr, xq_packed, wq_packed, w_scale, act_scale, 1, M, N, K, out_f16, acc_i32,
                                 nullptr, st, nullptr, 4, zp_corr);
    if (few == 1)
        return pq::launch_stream_mfma(xq_packed, wq_packed, w_scale, act_scale, M, N, K, out_f16, acc_i32, st, nullptr,
                                      4, zp_corr);
    return pq::launch_gemm_zp(xq_packed, wq_packed, w_scale, act_scale, zp_corr, M, N, K, out_f16, acc_i32, st,
                              workspace, workspace ? workspace_bytes : 0, g_variant == 5);
}

int pq_w4a4_gemm_zp(const void* xq_packed, const void* wq_packed, const float* w_scale, float act_scale,
                    const int32_t* zp_corr, int64_t M, int64_t N, int64_t K, void* out_f16, int32_t* acc_i32,
                    void* stream)
{
    return pq_w4a4_gemm_zp_ws(xq_packed, wq_packed, w_scale, act_scale, zp_corr, M, N, K, out_f16, acc_i32, nullptr, 0,
                              stream);
}

size_t pq_calibrate_workspace_bytes(int64_t T, int32_t n_grid)
{
    if (T <= 0 || n_grid < 2 || n_grid > pq::max_calibration_grid()) return 0;
    return (((size_t)T * (size_t)(n_grid + 1)) * 4 + 255) & ~(size_t)255;
}

int pq_calibrate_static(const void* x_cal_f16, int64_t T, int64_t K, int32_t had_block, int32_t bits, int32_t n_grid,
                        float gamma_min, float* result, void* workspace, size_t workspace_bytes, void* stream)
{
    if (T <= 0 || K <= 0 || (K % 32) != 0 || (bits != 4 && bits != 8)) return PQ_ERR_SHAPE;
    if (n_grid < 2 || n_grid > pq::max_calibration_grid()) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!x_cal_f16 || !result) return PQ_ERR_NULL;
    if (!aligned16(x_cal_f16) || (reinterpret_cast<uintptr_t>(result) & 3u)) return PQ_ERR_ALIGN;
    if (!(gamma_min > 0.0f && gamma_min < 1.0f)) return PQ_ERR_SCALE;
    if (!workspace || workspace_bytes < pq_calibrate_workspace_bytes(T, n_grid)) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    if (K > 32768) return PQ_ERR_UNSUPPORTED;
    return pq::launch_calibrate(x_cal_f16, T, K, had_block, bits, n_grid, gamma_min, result,
                                static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
}

size_t pq_calibrate_zp_workspace_bytes(int64_t T, int32_t n_candidates)
{
    if (T <= 0 || n_candidates < 2 || n_candidates > pq::max_calibration_grid()) return 0;
    return (((size_t)T * (size_t)(n_candidates + 2)) * 4 + 255) & ~(size_t)255;
}

int pq_calibrate_static_zp(const void* x_cal_f16, int64_t T, int64_t K, int32_t had_block, int32_t n_gamma,
                           int32_t n_beta, float gamma_min, float beta_min, float* result, void* workspace,
                           size_t workspace_bytes, void* stream)
{
    if (T <= 0 || K <= 0 || (K % 32) != 0 || n_gamma < 1 || n_beta < 1) return PQ_ERR_SHAPE;
    const int64_t n = (int64_t)n_gamma * n_beta;
    if (n < 2 || n > pq::max_calibration_grid()) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!x_cal_f16 || !result) return PQ_ERR_NULL;
    if (!aligned16(x_cal_f16) || (reinterpret_cast<uintptr_t>(result) & 3u)) return PQ_ERR_ALIGN;
    if (!(gamma_min > 0.0f && gamma_min < 1.0f) || !(beta_min > 0.0f && beta_min < 1.0f)) return PQ_ERR_SCALE;
    if (!workspace || workspace_bytes < pq_calibrate_zp_workspace_bytes(T, (int32_t)n)) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    if (K > 32768) return PQ_ERR_UNSUPPORTED;
    return pq::launch_calibrate_zp(x_cal_f16, T, K, had_block, n_gamma, n_beta, gamma_min, beta_min, result,
                                   static_cast<float*>(workspace), static_cast<hipStream_t>(stream));
}

int pq_probe_mfma_i8(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups, int32_t* sink,
                     void* stream)
{
    if (!operands || !sink) return PQ_ERR_NULL;
    if (!aligned16(operands) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return PQ_ERR_ALIGN;
    if (operand_bytes < 16 || (operand_bytes % 16) != 0 || operand_bytes > ((int64_t)1 << 34) || iters < 0 || iters > (1 << 24) ||
        workgroups < 1 || workgroups > (1 << 20))
        return PQ_ERR_SHAPE;
    return pq::launch_probe_mfma(operands, operand_bytes, iters, workgroups, sink, static_cast<hipStream_t>(stream));
}

int pq_probe_mfma_f6(const void* operands, int64_t operand_bytes, int64_t iters, int32_t workgroups, int32_t* sink,
                     void* stream)
{
    if (!operands || !sink) return PQ_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(operands) & 31u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return PQ_ERR_ALIGN;
    if (operand_bytes < 32 || (operand_bytes % 32) != 0 || operand_bytes > ((int64_t)1 << 34) || iters < 0 || iters > (1 << 24) ||
        workgroups < 1 || workgroups > (1 << 20))
        return PQ_ERR_SHAPE;
    return pq::launch_probe_mfma_f6(operands, operand_bytes, iters, workgroups, sink, static_cast<hipStream_t>(stream));
}

int pq_probe_f6_product(const int8_t* a_codes, const int8_t* b_codes, int64_t K, int32_t* out_i32, void* stream)
{
    if (!a_codes || !b_codes || !out_i32) return PQ_ERR_NULL;
    if (!aligned16(a_codes) || !aligned16(b_codes) || !aligned16(out_i32)) return PQ_ERR_ALIGN;
    if (K < 64 || (K % 64) != 0 || K > 262080) return PQ_ERR_SHAPE;    // |sum| <= 64 K < 2^24: exact in fp32
    return pq::launch_probe_f6_product(a_codes, b_codes, K, out_i32, static_cast<hipStream_t>(stream));
}

size_t pq_f6_tiles_bytes(int64_t rows, int64_t K)
{
    if (rows <= 0 || K <= 0 || (K % 128) != 0) return 0;
    return pq::f6_tiles_bytes(rows, K);
}

int pq_repack_f6(const void* codes_packed, int64_t rows, int64_t K, void* tiles, void* stream)
{
    if (rows < 0 || K <= 0 || (K % 128) != 0) return PQ_ERR_SHAPE;
    if (!codes_packed || !tiles) return PQ_ERR_NULL;
    if (!aligned16(codes_packed) || !aligned16(tiles)) return PQ_ERR_ALIGN;
    if (rows == 0) return PQ_OK;
    if (K > 262080 || pq::f6_tiles_bytes(rows, K) >= ((size_t)1 << 32)) return PQ_ERR_UNSUPPORTED;
    return pq::launch_repack_f6(codes_packed, rows, K, tiles, static_cast<hipStream_t>(stream));
}

int pq_w4a4_gemm_f6(const void* x_tiles, const void* w_tiles, const float* w_scale, float act_scale, int64_t M,
                    int64_t N, int64_t K, void* out_f16, int32_t* acc_i32, void* stream)
{
    int rc = check_gemm(x_tiles, w_tiles, w_scale, act_scale, M, N, K, out_f16, acc_i32);
    if (rc != PQ_OK) return rc;
    if ((K % 128) != 0) return PQ_ERR_SHAPE;
    if (M == 0) return PQ_OK;
    if (K > 262080 || M > (1 << 30) || N > (1 << 30) || pq::f6_tiles_bytes(M, K) >= ((size_t)1 << 32) ||
        pq::f6_tiles_bytes(N, K) >= ((size_t)1 << 32))
        return PQ_ERR_UNSUPPORTED;
    return pq::launch_gemm_f6(x_tiles, w_tiles, w_scale, act_scale, M, N, K, out_f16, acc_i32,
                              static_cast<hipStream_t>(stream));
}

int pq_rotate_quant_f6(const void* x_f16, int64_t M, int64_t K, int32_t had_block, float act_scale, void* x_tiles,
                       void* xq_packed, void* stream)
{
    if (M < 0 || K <= 0 || (K % 128) != 0) return PQ_ERR_SHAPE;
    if (had_block < 0 || had_block > 16384) return PQ_ERR_SHAPE;
    if (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)) return PQ_ERR_SHAPE;
    if (!x_f16 || !x_tiles) return PQ_ERR_NULL;
    if (!aligned16(x_f16) || !aligned16(x_tiles) || !aligned16(xq_packed)) return PQ_ERR_ALIGN;
    if (!good_scale(act_scale)) return PQ_ERR_SCALE;
    if (M == 0) return PQ_OK;
    if (K > 262080 || pq::f6_tiles_bytes(M, K) >= ((size_t)1 << 32) || M * K >= ((int64_t)1 << 32) ||
        !pq::quant_f6_supported(M, K, had_block))
        return PQ_ERR_UNSUPPORTED;
    return pq::launch_quant_f6(x_f16, M, K, had_block, act_scale, x_tiles, xq_packed, static_cast<hipStream_t>(stream));
}

// rotation blocks beyond what the tile-writing quantizer handles go through the canonical codes
static bool f6_needs_codes(int64_t M, int64_t K, int32_t had_block) { return !pq::quant_f6_supported(M, K, had_block); }

size_t pq_linear_f6_workspace_bytes(int64_t M, int64_t K, int32_t had_block)
{
    if (M <= 0 || K <= 0 || (K % 128) != 0) return 0;
    const size_t tiles = (pq::f6_tiles_bytes(M, K) + 255) & ~(size_t)255;
    return tiles + (f6_needs_codes(M, K, had_block) ? pq_linear_workspace_bytes(M, K) : 0);
}

int pq_linear_f6(const void* x_f16, const void* w_tiles, const float* w_scale, float act_scale, int32_t had_block,
                 int64_t M, int64_t N, int64_t K, void* out_f16, void* workspace, size_t workspace_bytes, void* stream)
{
    if (M < 0 || N <= 0 || K <= 0 || (K % 128) != 0 || (N % 16) != 0) return PQ_ERR_SHAPE;
    if (!x_f16 || !w_tiles || !w_scale || !out_f16) return PQ_ERR_NULL;
    if (M == 0) return PQ_OK;
    if (had_block < 0 || had_block > 16384 ||
        (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)))
        return PQ_ERR_SHAPE;
    if (!workspace || workspace_bytes < pq_linear_f6_workspace_bytes(M, K, had_block)) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    int rc = check_gemm(workspace, w_tiles, w_scale, act_scale, M, N, K, out_f16, nullptr);
    if (rc != PQ_OK) return rc;
    if (!aligned16(x_f16)) return PQ_ERR_ALIGN;
    if (K > 262080 || M > (1 << 30) || N > (1 << 30) || pq::f6_tiles_bytes(M, K) >= ((size_t)1 << 32) ||
        pq::f6_tiles_bytes(N, K) >= ((size_t)1 << 32) || M * K >= ((int64_t)1 << 32))
        return PQ_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* tiles = static_cast<uint8_t*>(workspace);
    if (!f6_needs_codes(M, K, had_block)) {
        // rotation blocks up to 512 channels (or none): one launch rotates, quantizes and writes the tiles
        rc = pq::launch_quant_f6(x_f16, M, K, had_block, act_scale, tiles, nullptr, st);
    } else {
        uint8_t* nibbles = tiles + ((pq::f6_tiles_bytes(M, K) + 255) & ~(size_t)255);
        rc = pq_rotate_quant(x_f16, M, K, had_block, act_scale, nibbles, stream);
        if (rc == PQ_OK) rc = pq::launch_repack_f6(nibbles, M, K, tiles, st);
    }
    if (rc != PQ_OK) return rc;
    return pq::launch_gemm_f6(tiles, w_tiles, w_scale, act_scale, M, N, K, out_f16, nullptr, st);
}

int pq_linear2_f6(const void* x_f16, const void* w_tiles_a, const float* w_scale_a, int64_t N_a, void* out_a_f16,
                  const void* w_tiles_b, const float* w_scale_b, int64_t N_b, void* out_b_f16, float act_scale,
                  int32_t had_block, int64_t M, int64_t K, void* workspace, size_t workspace_bytes, void* stream)
{
    if (M < 0 || N_a <= 0 || N_b <= 0 || K <= 0 || (K % 128) != 0 || (N_a % 16) != 0 || (N_b % 16) != 0) return PQ_ERR_SHAPE;
    if (!x_f16 || !w_tiles_a || !w_scale_a || !out_a_f16 || !w_tiles_b || !w_scale_b || !out_b_f16) return PQ_ERR_NULL;
    if (M == 0) return PQ_OK;
    if (had_block < 0 || had_block > 16384 ||
        (had_block > 1 && ((had_block & (had_block - 1)) != 0 || (K % had_block) != 0)))
        return PQ_ERR_SHAPE;
    if (!workspace || workspace_bytes < pq_linear_f6_workspace_bytes(M, K, had_block)) return PQ_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return PQ_ERR_ALIGN;
    int rc = check_gemm(workspace, w_tiles_a, w_scale_a, act_scale, M, N_a, K, out_a_f16, nullptr);
    if (rc == PQ_OK) rc = check_gemm(workspace, w_tiles_b, w_scale_b, act_scale, M, N_b, K, out_b_f16, nullptr);
    if (rc != PQ_OK) return rc;
    if (!aligned16(x_f16)) return PQ_ERR_ALIGN;
    const int64_t n_max = N_a > N_b ? N_a : N_b;
    if (K > 262080 || M > (1 << 30) || n_max > (1 << 30) || pq::f6_tiles_bytes(M, K) >= ((size_t)1 << 32) ||
        pq::f6_tiles_bytes(n_max, K) >= ((size_t)1 << 32) || M * K >= ((int64_t)1 << 32))
        return PQ_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* tiles = static_cast<uint8_t*>(workspace);
    if (!f6_needs_codes(M, K, had_block)) {
        rc = pq::launch_quant_f6(x_f16, M, K, had_block, act_scale, tiles, nullptr, st);
    } else {
        uint8_t* nibbles = tiles + ((pq::f6_tiles_bytes(M, K) + 255) & ~(size_t)255);
        rc = pq_rotate_quant(x_f16, M, K, had_block, act_scale, nibbles, stream);
        if (rc == PQ_OK) rc = pq::launch_repack_f6(nibbles, M, K, tiles, st);
    }
    if (rc != PQ_OK) return rc;
    rc = pq::launch_gemm_f6(tiles, w_tiles_a, w_scale_a, act_scale, M, N_a, K, out_a_f16, nullptr, st);
    if (rc != PQ_OK) return rc;
    return pq::launch_gemm_f6(tiles, w_tiles_b, w_scale_b, act_scale, M, N_b, K, out_b_f16, nullptr, st);
}

size_t pq_prepacked_bytes(int64_t N, int64_t K) { return pq_f6_tiles_bytes(N, K); }

int pq_prepack_weights(const void* wq_packed, int64_t N, int64_t K, void* wq_tiled, void* stream)
{
    return pq_repack_f6(wq_packed, N, K, wq_tiled, stream);
}

int pq_linear_prepacked(const void* x_f16, const void* wq_tiled, const float* w_scale, float act_scale, int32_t had_block,
                        int64_t M, int64_t N, int64_t K, void* out_f16, void* workspace, size_t workspace_bytes, void* stream)
{
    return pq_linear_f6(x_f16, wq_tiled, w_scale, act_scale, had_block, M, N, K, out_f16, workspace, workspace_bytes, stream);
}

int pq_probe_stream_read(const void* src, int64_t bytes, int32_t* sink, void* stream)
{
    if (!src || !sink) return PQ_ERR_NULL;
    if (!aligned16(src) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return PQ_ERR_ALIGN;
    if (bytes < 16 || (bytes % 16) != 0) return PQ_ERR_SHAPE;
    return pq::launch_probe_read(src, bytes, sink, static_cast<hipStream_t>(stream));
}

int pq_set_gemm_tile(int tile) { return pq::set_gemm_tile(tile); }

int pq_set_gemm_f6_tile(int tile) { return pq::set_gemm_f6_tile(tile); }

size_t pq_linear_noalloc_max_bytes(void) { return kScratchBytes; }

int pq_linear_noalloc(const void* x_f16, const void* wq_packed, const float* w_scale, float act_scale,
                      int32_t had_block, int64_t M, int64_t N, int64_t K, void* out_f16, void* stream)
{
    if (M < 0 || N <= 0 || K <= 0 || (K % 32) != 0 || (N % 16) != 0) return PQ_ERR_SHAPE;
    if (M == 0) return PQ_OK;
    // the codes must fit the built-in array (M and K are bounded first so that the product cannot wrap)
    if (M > (int64_t)kScratchBytes || K > 2 * (int64_t)kScratchBytes ||
        pq_linear_workspace_bytes(M, K) > kScratchBytes)
        return PQ_ERR_WORKSPACE;
    uint8_t* base = nullptr;
    const int rc = scratch_base(&base);
    if (rc != PQ_OK) return rc;
    // everything else is pq_linear's business: the same checks, the same kernels, `base` as their workspace
    // (codes first; what lies behind them may hold the planes of a split launch)
    return pq_linear(x_f16, wq_packed, w_scale, act_scale, had_block, M, N, K, out_f16, base, kScratchBytes, stream);
}

int pq_set_gemm_variant(int variant)
{
    if (variant < 0 || variant > 5) return -1;
    return g_variant.exchange(variant);
}

}  // extern "C"
