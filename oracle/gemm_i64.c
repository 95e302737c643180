/* CPU oracle, C part (TEST INFRASTRUCTURE ONLY; never linked into the HIP library).
 *
 * The integer product of the quantized linear layer, written as its definition:
 *   acc[m][n] = sum_k (int64) q[m][k] * (int64) wq[n][k]
 * (Sec. 3 of the paper: weight and activation quantization together allow low-bit
 * matrix multiplication).  Codes arrive unpacked, one int8 per element, both operands
 * with the reduction index contiguous.  No blocking, no reordering: one dot product
 * per output, summed in index order; rows of the output are spread over OpenMP threads.
 *
 * Returns 0, or 1 if some |acc| does not fit a signed 32-bit integer (the GPU path
 * accumulates in int32, so the oracle refuses inputs for which that would overflow).
 */
#include <stdint.h>
#include <omp.h>

int pqo_threads(void) { return omp_get_max_threads(); }

int pqo_gemm_i64(const int8_t* q, const int8_t* wq, int64_t M, int64_t N, int64_t K, int64_t* acc)
{
    int overflow = 0;
#pragma omp parallel for schedule(static) reduction(| : overflow)
    for (int64_t m = 0; m < M; ++m) {
        const int8_t* a = q + m * K;
        for (int64_t n = 0; n < N; ++n) {
            const int8_t* b = wq + n * K;
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int64_t)a[k] * (int64_t)b[k];
            if (s > INT32_MAX || s < INT32_MIN) overflow = 1;
            acc[m * N + n] = s;
        }
    }
    return overflow;
}
