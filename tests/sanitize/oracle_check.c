/* Host sanitizer run of the oracle's C part: compiled together with oracle/gemm_i64.c under
 * -fsanitize=address,undefined and run by tests/test_host_sanitizers.py.  Shapes are small and
 * ragged so that any read or write one element past a row or past the output trips the sanitizer;
 * values are checked against a second, differently ordered sum.  Exit code 0 = clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int pqo_threads(void);
int pqo_gemm_i64(const int8_t* q, const int8_t* wq, int64_t M, int64_t N, int64_t K, int64_t* acc);

static uint32_t rng_state = 12345u;
static int8_t next_code(int lo, int hi)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (int8_t)(lo + (int)((rng_state >> 8) % (uint32_t)(hi - lo + 1)));
}

static int check(int64_t M, int64_t N, int64_t K, int lo, int hi, int want_overflow)
{
    /* exact-size heap blocks: the sanitizer's red zones sit right behind the last element */
    int8_t* q = malloc((size_t)(M * K ? M * K : 1));
    int8_t* w = malloc((size_t)(N * K ? N * K : 1));
    int64_t* acc = malloc(sizeof(int64_t) * (size_t)(M * N ? M * N : 1));
    for (int64_t i = 0; i < M * K; ++i) q[i] = next_code(lo, hi);
    for (int64_t i = 0; i < N * K; ++i) w[i] = next_code(lo, hi);
    const int overflow = pqo_gemm_i64(q, w, M, N, K, acc);
    int bad = overflow != want_overflow;
    for (int64_t m = 0; m < M && !bad; ++m)
        for (int64_t n = 0; n < N && !bad; ++n) {
            int64_t s = 0;
            for (int64_t k = K - 1; k >= 0; --k) s += (int64_t)w[n * K + k] * (int64_t)q[m * K + k];
            if (s != acc[m * N + n]) bad = 1;
        }
    if (bad) fprintf(stderr, "oracle_check: mismatch at M=%lld N=%lld K=%lld\n", (long long)M, (long long)N, (long long)K);
    free(q); free(w); free(acc);
    return bad;
}

int main(void)
{
    int bad = pqo_threads() < 1;
    bad |= check(1, 1, 1, -8, 7, 0);
    bad |= check(3, 5, 7, -8, 7, 0);
    bad |= check(17, 33, 129, -8, 7, 0);
    bad |= check(64, 48, 512, -128, 127, 0);
    bad |= check(0, 4, 32, -8, 7, 0);
    bad |= check(4, 0, 32, -8, 7, 0);
    bad |= check(2, 3, 0, -8, 7, 0);
    bad |= check(2, 2, 200000, 127, 127, 1);      /* 127 * 127 * 200000 > 2^31: reported, sums still exact in int64 */
    bad |= check(2, 2, 28672, -8, -8, 0);         /* the largest magnitude of the 4-bit path: 1 835 008 */
    printf(bad ? "oracle_check: FAILED\n" : "oracle_check: ok\n");
    return bad;
}
