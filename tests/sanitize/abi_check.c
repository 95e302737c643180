/* Host sanitizer run of the library's argument checking and host-side planning: linked against a
 * build of the library whose host code is compiled with -fsanitize=address,undefined (the GPU code
 * is not instrumented and nothing is launched: every call below fails validation, is a no-op, or is
 * a host-only query).  Written in C so that include/pq.h is also compiled as C.  Run by
 * tests/test_host_sanitizers.py on a machine without a GPU.  Exit code 0 = clean. */
#include <stdio.h>
#include <string.h>

#include "pq.h"

static int failures = 0;
#define EXPECT(call, want)                                                              \
    do {                                                                                \
        const long long got_ = (long long)(call);                                       \
        if (got_ != (long long)(want)) {                                                \
            fprintf(stderr, "abi_check: %s = %lld, expected %lld\n", #call, got_, (long long)(want)); \
            ++failures;                                                                 \
        }                                                                               \
    } while (0)

int main(void)
{
    void* p = (void*)0x1000;      /* never dereferenced: validation comes first */
    void* p256 = (void*)0x10000;
    void* odd = (void*)0x1008;
    const float* pf = (const float*)0x1000;
    int32_t* pi = (int32_t*)0x1000;

    EXPECT(pq_version() >= 100, 1);
    for (int s = -2; s < 12; ++s) EXPECT(strlen(pq_status_str(s)) > 0, 1);

    /* host-only planning over a grid of shapes: cost models, tile choice, mixed-width search */
    static const int64_t Ms[] = {-1, 0, 1, 4, 8, 9, 16, 17, 24, 32, 33, 40, 64, 100, 128, 256, 384, 512, 1024, 2048, 8192};
    static const int64_t Ns[] = {16, 64, 400, 1024, 4096, 6144, 8192, 10240, 11008, 14336, 28672};
    static const int64_t Ks[] = {32, 128, 160, 256, 384, 512, 4096, 8192, 11008, 14336, 28672, 65536, 131072};
    size_t total = 0;
    for (unsigned a = 0; a < sizeof Ms / sizeof *Ms; ++a)
        for (unsigned b = 0; b < sizeof Ns / sizeof *Ns; ++b)
            for (unsigned c = 0; c < sizeof Ks / sizeof *Ks; ++c) {
                const int64_t M = Ms[a], N = Ns[b], K = Ks[c];
                total += pq_w4a4_gemm_workspace_bytes(M, N, K) + pq_gemm_workspace_bytes(M, N, K, 8);
                total += pq_linear_workspace_bytes(M, K) + pq_linear_workspace_bytes_split(M, N, K);
                total += pq_linear_w4a8_workspace_bytes(M, K) + pq_linear_w4a8_workspace_bytes_split(M, N, K);
                total += pq_linear_dynamic_workspace_bytes(M, K, 4) + pq_linear_dynamic_workspace_bytes_split(M, N, K, 8);
                total += pq_f6_tiles_bytes(M, K) + pq_linear_f6_workspace_bytes(M, K, 128) + pq_linear_f6_workspace_bytes(M, K, 4096);
            }
    EXPECT(total > 0, 1);
    EXPECT(pq_calibrate_workspace_bytes(256, 50), 256 * 51 * 4);
    EXPECT(pq_calibrate_zp_workspace_bytes(256, 64), 256 * 66 * 4);
    EXPECT(pq_linear_noalloc_max_bytes(), 32 << 20);

    /* the switches */
    EXPECT(pq_set_gemm_variant(9), -1);
    EXPECT(pq_set_gemm_tile(99), -2);
    EXPECT(pq_set_gemm_f6_tile(7), -2);
    for (int v = 0; v <= 5; ++v) {
        const int prev = pq_set_gemm_variant(v);
        total += pq_w4a4_gemm_workspace_bytes(100, 256, 2048);
        EXPECT(pq_w4a4_gemm(p, p, pf, 0.1f, 0, 64, 512, p, NULL, NULL), PQ_OK);
        EXPECT(pq_set_gemm_variant(prev), v);
    }

    /* argument errors: nothing is enqueued, nothing is dereferenced */
    EXPECT(pq_rotate_quant(NULL, 4, 512, 128, 0.1f, p, NULL), PQ_ERR_NULL);
    EXPECT(pq_rotate_quant(p, 4, 500, 1, 0.1f, p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_rotate_quant(p, 4, 512, 96, 0.1f, p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_rotate_quant(odd, 4, 512, 128, 0.1f, p, NULL), PQ_ERR_ALIGN);
    EXPECT(pq_rotate_quant(p, 4, 512, 128, 0.0f, p, NULL), PQ_ERR_SCALE);
    EXPECT(pq_rotate_quant(p, 0, 512, 128, 0.1f, p, NULL), PQ_OK);
    EXPECT(pq_w4a4_gemm(NULL, p, pf, 0.1f, 4, 64, 512, p, NULL, NULL), PQ_ERR_NULL);
    EXPECT(pq_w4a4_gemm(p, p, pf, 0.1f, 4, 60, 512, p, NULL, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_w4a4_gemm(p, odd, pf, 0.1f, 4, 64, 512, p, NULL, NULL), PQ_ERR_ALIGN);
    EXPECT(pq_w4a4_gemm(p, p, (const float*)0x1004, 0.1f, 4, 64, 512, p, NULL, NULL), PQ_ERR_ALIGN);
    EXPECT(pq_w4a4_gemm(p, p, pf, -2.0f, 4, 64, 512, p, NULL, NULL), PQ_ERR_SCALE);
    EXPECT(pq_w4a4_gemm(p, p, pf, 0.1f, 40, 64, 131072, p, NULL, NULL), PQ_ERR_UNSUPPORTED);
    EXPECT(pq_w4a4_gemm_ws(p, p, pf, 0.1f, 64, 64, 512, p, NULL, odd, 1 << 20, NULL), PQ_ERR_ALIGN);
    EXPECT(pq_w4a4_gemm_simple(p, p, pf, 0.1f, 4, 64, 48, p, NULL, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_linear(p, p, pf, 0.1f, 128, 4, 64, 512, p, NULL, 0, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_linear(p, p, pf, 0.1f, 128, 4, 64, 512, p, p, 1023, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_linear(p, p, pf, 0.1f, 100, 4, 64, 512, p, p256, 4096, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_linear(p, p, pf, 0.1f, 128, 0, 64, 512, p, NULL, 0, NULL), PQ_OK);
    EXPECT(pq_linear_noalloc(p, p, pf, 0.1f, 1, (int64_t)1 << 40, 64, 64, p, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_linear_noalloc(p, p, pf, 0.1f, 1, 4, 64, (int64_t)1 << 40, p, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_linear_noalloc(p, p, pf, 0.1f, 1, 4, 60, 64, p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_rotate_quant8(p, 4, 160, 1, 0.1f, p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_w4a8_gemm(p, p, pf, 0.1f, 40, 64, 131072, p, NULL, NULL), PQ_ERR_UNSUPPORTED);
    EXPECT(pq_linear_w4a8(p, p, pf, 0.1f, 128, 4, 64, 256, p, p256, 512, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_rotate_quant_dynamic(p, 4, 256, 1, 1.25f, 4, p, (float*)p, NULL), PQ_ERR_SCALE);
    EXPECT(pq_gemm_dynamic(p, 3, p, pf, pf, 4, 64, 256, p, NULL, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_linear_dynamic(p, p, pf, 1.0f, 1, 4, 4, 64, 256, p, p256, 512, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_rotate_quant_heads(p, 4, 8, 48, 1, pf, p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_rotate_quant_groups(p, 4, 8, 128, 1, 48, 1.0f, p, (float*)p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_rotate_f16(p, 4, 256, 96, p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_silu_mul_rotate_quant(p, NULL, 4, 256, 128, 0.1f, p, NULL), PQ_ERR_NULL);
    EXPECT(pq_rmsnorm_quant(p, 4, 65536, 1e-6f, 0.1f, p, NULL), PQ_ERR_UNSUPPORTED);
    EXPECT(pq_rotate_quant_zp(p, 4, 256, 1, 0.1f, 16, p, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_zero_point_correction(p, 16, 256, 3, NULL, NULL), PQ_ERR_NULL);
    EXPECT(pq_w4a4_gemm_zp(p, p, pf, 0.1f, NULL, 64, 64, 512, p, NULL, NULL), PQ_ERR_NULL);
    EXPECT(pq_calibrate_static(p, 4, 256, 1, 4, 8, 0.5f, (float*)p, p256, 16, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_calibrate_static_zp(p, 4, 256, 1, 8, 8, 0.5f, 1.5f, (float*)p, p256, 1 << 20, NULL), PQ_ERR_SCALE);
    EXPECT(pq_probe_mfma_i8(p, 1000, 10, 256, pi, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_probe_stream_read(odd, 1024, pi, NULL), PQ_ERR_ALIGN);
    EXPECT(pq_probe_mfma_f6(p, 48, 1, 1, pi, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_probe_f6_product((const int8_t*)p, (const int8_t*)p, 96, pi, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_repack_f6(p, 32, 262144, p, NULL), PQ_ERR_UNSUPPORTED);
    EXPECT(pq_w4a4_gemm_f6(p, p, pf, 0.1f, 32, 16, 160, p, NULL, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_linear_f6(p, p, pf, 0.1f, 1, 32, 16, 128, p, p256, 100, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_rotate_quant_f6(p, 32, 2048, 1024, 0.1f, p, NULL, NULL), PQ_ERR_UNSUPPORTED);
    EXPECT(pq_rotate_quant_f6(p, 32, 96, 1, 0.1f, p, NULL, NULL), PQ_ERR_SHAPE);
    /* two matrices on one quantized input, canonical and prepacked */
    EXPECT(pq_linear2(p, p, pf, 64, p, p, pf, 32, p, 0.1f, 128, 0, 512, p256, 4096, NULL), PQ_OK);
    EXPECT(pq_linear2(p, p, pf, 64, p, NULL, pf, 32, p, 0.1f, 128, 4, 512, p256, 4096, NULL), PQ_ERR_NULL);
    EXPECT(pq_linear2(p, p, pf, 64, p, p, pf, 40, p, 0.1f, 128, 4, 512, p256, 4096, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_linear2(p, p, pf, 64, p, p, pf, 32, p, 0.1f, 128, 4, 512, p256, 16, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_linear2(p, p, pf, 64, p, p, pf, 32, p, -1.0f, 128, 4, 512, p256, 4096, NULL), PQ_ERR_SCALE);
    EXPECT(pq_linear2_f6(p, p, pf, 64, p, p, pf, 32, p, 0.1f, 128, 0, 512, p256, 1 << 20, NULL), PQ_OK);
    EXPECT(pq_linear2_f6(p, p, pf, 64, p, p, NULL, 32, p, 0.1f, 128, 4, 512, p256, 1 << 20, NULL), PQ_ERR_NULL);
    EXPECT(pq_linear2_f6(p, p, pf, 64, p, p, pf, 32, p, 0.1f, 128, 4, 480, p256, 1 << 20, NULL), PQ_ERR_SHAPE);
    EXPECT(pq_linear2_f6(p, p, pf, 64, p, p, pf, 32, p, 0.1f, 128, 4, 512, p256, 64, NULL), PQ_ERR_WORKSPACE);
    EXPECT(pq_linear2_f6(p, p, pf, 64, p, p, pf, 32, p, 0.1f, 1, 4, 262144, p256, (size_t)1 << 30, NULL), PQ_ERR_UNSUPPORTED);

    printf(failures ? "abi_check: %d FAILED\n" : "abi_check: ok\n", failures);
    return failures != 0;
}
