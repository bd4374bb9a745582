/* Runs every entry point of the CPU oracle under -fsanitize=address,undefined (tests/test_sanitizers.py) on
 * small heap arrays that are exactly as long as the calls may touch: ragged last blocks, blocks of one element,
 * one block for the whole array, all four data types, with and without a local term.  Exits 0 when every call
 * succeeds and a few identities hold; an out-of-bounds access or undefined operation aborts the run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int dq8o_set_threads(int t);
int dq8o_codebook(int kind, float *cb);
int dq8o_absmax(const float *x, size_t n, size_t block, float *scales);
int dq8o_encode(int kind, const float *x, size_t n, size_t block, float *scales, uint8_t *codes, int scales_given);
int dq8o_decode(int kind, const uint8_t *codes, const float *scales, size_t n, size_t block, float *out);
int dq8o_decode_accumulate_avg(int kind, const uint8_t *const *codes, const float *const *scales, int K, size_t n,
                               size_t block, float *out);
int dq8o_decode_accumulate_avg_local(int kind, const uint8_t *const *codes, const float *const *scales, int K,
                                     const float *local, size_t n, size_t block, float *out);
int dq8o_decode_avg_encode(int kind, const uint8_t *const *codes, const float *const *scales, int K, const float *local,
                           size_t n, size_t block, float *out_scales, uint8_t *out_codes);
int dq8o_error_stats(int kind, const float *x, size_t n, size_t block, float *scales, int scales_given, double *stats,
                     double *means);

static int failures = 0;
#define CHECK(cond, what)                                                              \
    do {                                                                               \
        if (!(cond)) {                                                                 \
            ++failures;                                                                \
            printf("FAIL %s (%s, line %d)\n", #cond, what, __LINE__);                  \
        }                                                                              \
    } while (0)

static uint32_t lcg(uint32_t *s) { return *s = *s * 1664525u + 1013904223u; }

static void run(int kind, size_t n, size_t block, int K)
{
    const size_t B = block == 0 ? n : block, nb = (n + B - 1) / B;
    uint32_t seed = (uint32_t)(kind * 7919 + n * 31 + block * 17 + K);
    float *x = malloc(n * sizeof(float)), *local = malloc(n * sizeof(float));
    float *amax = malloc(nb * sizeof(float)), *out = malloc(n * sizeof(float)), *mean = malloc(n * sizeof(float));
    float *rs = malloc(nb * sizeof(float)), *rs2 = malloc(nb * sizeof(float));
    uint8_t *rc = malloc(n), *rc2 = malloc(n);
    double *stats = malloc(4 * nb * sizeof(double)), means[2];
    const uint8_t *cp[8];
    const float *sp[8];
    uint8_t *codes[8];
    float *scales[8];
    char what[96];
    size_t i;
    int k;
    snprintf(what, sizeof(what), "kind %d n %zu block %zu K %d", kind, n, block, K);
    for (i = 0; i < n; ++i) {
        const uint32_t r = lcg(&seed);
        x[i] = (r % 11 == 0) ? 0.0f : ((float)(int32_t)r) * (1.0f / 2147483648.0f) * ((r >> 3) % 5 == 0 ? 1e-6f : 3.0f);
        local[i] = ((float)(int32_t)lcg(&seed)) * (1.0f / 2147483648.0f);
    }
    CHECK(dq8o_absmax(x, n, block, amax) == 0, what);
    for (k = 0; k < K; ++k) {
        codes[k] = malloc(n);
        scales[k] = malloc(nb * sizeof(float));
        for (i = 0; i < n; ++i) local[i] = -local[i] * 0.5f + x[i];
        CHECK(dq8o_encode(kind, k == 0 ? x : local, n, block, scales[k], codes[k], 0) == 0, what);
        cp[k] = codes[k];
        sp[k] = scales[k];
    }
    CHECK(memcmp(amax, scales[0], nb * sizeof(float)) == 0, what);
    CHECK(dq8o_encode(kind, x, n, block, amax, rc, 1) == 0 && memcmp(rc, codes[0], n) == 0, what);
    CHECK(dq8o_decode(kind, codes[0], scales[0], n, block, out) == 0, what);
    CHECK(dq8o_decode_accumulate_avg(kind, cp, sp, K, n, block, mean) == 0, what);
    CHECK(dq8o_encode(kind, mean, n, block, rs, rc, 0) == 0, what);
    CHECK(dq8o_decode_avg_encode(kind, cp, sp, K, NULL, n, block, rs2, rc2) == 0, what);
    CHECK(memcmp(rs, rs2, nb * sizeof(float)) == 0 && memcmp(rc, rc2, n) == 0, what);
    CHECK(dq8o_decode_accumulate_avg_local(kind, cp, sp, K, local, n, block, mean) == 0, what);
    CHECK(dq8o_decode_avg_encode(kind, cp, sp, K, local, n, block, rs2, rc2) == 0, what);
    CHECK(dq8o_decode_accumulate_avg_local(kind, NULL, NULL, 0, local, n, block, mean) == 0, what);
    CHECK(dq8o_error_stats(kind, x, n, block, rs, 0, stats, means) == 0, what);
    CHECK(memcmp(rs, amax, nb * sizeof(float)) == 0 && means[0] >= 0.0 && means[1] >= 0.0, what);
    CHECK(dq8o_error_stats(kind, x, n, block, amax, 1, stats, NULL) == 0, what);
    for (i = 0; i < nb; ++i) CHECK(stats[4 * i + 3] <= (double)amax[i] && stats[4 * i + 2] <= (double)B, what);
    for (k = 0; k < K; ++k) {
        free(codes[k]);
        free(scales[k]);
    }
    free(x); free(local); free(amax); free(out); free(mean); free(rs); free(rs2); free(rc); free(rc2); free(stats);
}

int main(void)
{
    static const size_t sizes[] = {1, 2, 3, 7, 64, 100, 257, 1000};
    static const size_t blocks[] = {0, 1, 3, 64, 100, 4096};
    float cb[256];
    int kind, t;
    size_t a, b;
    CHECK(dq8o_codebook(4, cb) != 0 && dq8o_codebook(-1, cb) != 0, "unknown kinds are rejected");
    for (t = 1; t <= 3; t += 2) {
        dq8o_set_threads(t);
        for (kind = 0; kind < 4; ++kind) {
            CHECK(dq8o_codebook(kind, cb) == 0, "codebook");
            for (a = 0; a < sizeof(sizes) / sizeof(sizes[0]); ++a)
                for (b = 0; b < sizeof(blocks) / sizeof(blocks[0]); ++b) run(kind, sizes[a], blocks[b], 1 + (int)((a + b) % 5));
        }
    }
    /* n == 0 touches nothing */
    CHECK(dq8o_absmax(NULL, 0, 0, NULL) == 0 && dq8o_encode(0, NULL, 0, 0, NULL, NULL, 0) == 0, "empty input");
    CHECK(dq8o_decode(0, NULL, NULL, 0, 0, NULL) == 0, "empty input");
    if (failures) {
        printf("%d checks failed\n", failures);
        return 1;
    }
    printf("oracle checks ok\n");
    return 0;
}
