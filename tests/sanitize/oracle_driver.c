/* Runs the CPU oracle (oracle/pvq_oracle.c, compiled into this program with AddressSanitizer and
 * UndefinedBehaviorSanitizer) over small seeded inputs through every entry point: size table, K from a
 * budget, quantiser, rank / unrank round trips (one-, two- and twelve-word indices), matrix encode / decode
 * with float32 amplitudes and with codes, least-squares amplitudes, rotation, error correction.  It checks
 * only what makes a wrong result visible here (round trips, invariants): the values themselves are pinned
 * by the Python tests.  Exit status 0 = no sanitizer report and all checks held. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int pvqo_table(int D, int K, uint32_t *out);
int pvqo_words_per_integer(void);
int pvqo_index_bits(int D, int K);
int pvqo_max_k(int D, int bit_budget);
void pvqo_quantize_group(const float *w, int D, int K, int32_t *y, float *ss_out);
int pvqo_rank_many(int D, int K, int64_t n, const int32_t *x, uint32_t *c_words);
int pvqo_unrank_many(int D, int K, int64_t n, const uint32_t *c_words, int32_t *x, int omit_negative_update);
int64_t pvqo_row_words(int64_t groups, int bits);
float pvqo_ls_amplitude(const float *w, const int32_t *y, int D);
int pvqo_encode(const float *W, int64_t rows, int64_t cols, int D, int K, int scale_bits, int amp_mode,
                const float *edges, uint32_t *index_out, void *scale_out, float *rowss_out, int8_t *pulses_out,
                int nthreads);
int pvqo_correct(float *W, int64_t rows, int64_t cols, int D, int K, int amp_mode, const float *U, float *Q_out,
                 int nthreads);
int pvqo_hadamard_rows(const float *X, int64_t rows, int64_t cols, int64_t block, const uint8_t *signs,
                       int signs_after, float *Y);
int pvqo_decode(const uint32_t *index, const void *scale, const float *rowss, int64_t rows, int64_t cols, int D,
                int K, int scale_bits, const double *centers, double *W_out, int8_t *pulses_out, const double *x,
                int batch, double *out, int nthreads);

static uint64_t state = 20241016;
static double uniform(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0;
}
static float gauss(void) { return (float)(sqrt(-2.0 * log(uniform() + 1e-300)) * cos(6.283185307179586 * uniform())); }

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); exit(1); } } while (0)

static void round_trip(int D, int K, int n)
{
    const int NW = pvqo_words_per_integer();
    float *w = malloc(sizeof(float) * D);
    int32_t *y = malloc(sizeof(int32_t) * (size_t)n * D), *back = malloc(sizeof(int32_t) * (size_t)n * D);
    uint32_t *c = calloc((size_t)n * NW, 4);
    for (int p = 0; p < n; p++) {
        for (int i = 0; i < D; i++) w[i] = gauss();
        float ss;
        pvqo_quantize_group(w, D, K, y + (size_t)p * D, &ss);
        int sum = 0;
        for (int i = 0; i < D; i++) sum += abs(y[(size_t)p * D + i]);
        CHECK(sum == K);
    }
    CHECK(pvqo_rank_many(D, K, n, y, c) == 0);
    CHECK(pvqo_unrank_many(D, K, n, c, back, 0) == 0);
    CHECK(memcmp(y, back, sizeof(int32_t) * (size_t)n * D) == 0);
    free(w); free(y); free(back); free(c);
}

static void matrix(int rows, int cols, int D, int K, int scale_bits, int amp_mode, int threads)
{
    const int64_t G = cols / D;
    const int bits = pvqo_index_bits(D, K);
    const int64_t iw = pvqo_row_words(G, bits), sw = scale_bits ? pvqo_row_words(G, scale_bits) : G;
    float *W = malloc(sizeof(float) * (size_t)rows * cols);
    for (int64_t i = 0; i < (int64_t)rows * cols; i++) W[i] = 0.02f * gauss();
    const int n = 1 << scale_bits;
    float *edges = malloc(sizeof(float) * n);
    double *centers = malloc(sizeof(double) * n);
    for (int j = 0; j < n; j++) { edges[j] = (float)((j + 1.0) / (n * (double)G)); centers[j] = (j + 0.5) / (n * (double)G); }
    uint32_t *index = calloc((size_t)rows * iw, 4);
    uint32_t *scale = calloc((size_t)rows * sw, 4);
    float *rowss = calloc(rows, sizeof(float));
    /* the optional pulse plane is int8: only up to K = 127 */
    int8_t *pulses = K <= 127 ? malloc((size_t)rows * cols) : NULL, *pulses2 = K <= 127 ? malloc((size_t)rows * cols) : NULL;
    CHECK(pvqo_encode(W, rows, cols, D, K, scale_bits, amp_mode, scale_bits ? edges : NULL, index, scale, rowss, pulses, threads) == 0);
    double *Wd = malloc(sizeof(double) * (size_t)rows * cols), *x = malloc(sizeof(double) * 2 * cols), *out = malloc(sizeof(double) * 2 * rows);
    for (int i = 0; i < 2 * cols; i++) x[i] = gauss();
    CHECK(pvqo_decode(index, scale, rowss, rows, cols, D, K, scale_bits, scale_bits ? centers : NULL, Wd, pulses2, x, 2, out, threads) == 0);
    if (pulses) CHECK(memcmp(pulses, pulses2, (size_t)rows * cols) == 0);
    for (int64_t i = 0; i < (int64_t)rows * cols; i++) CHECK(isfinite(Wd[i]));
    free(W); free(edges); free(centers); free(index); free(scale); free(rowss); free(pulses); free(pulses2); free(Wd); free(x); free(out);
}

int main(void)
{
    const int NW = pvqo_words_per_integer();
    uint32_t *tab = malloc(sizeof(uint32_t) * NW * 9 * 17);
    CHECK(pvqo_table(8, 16, tab) == 0);
    CHECK(tab[(8 * 17 + 16) * NW] == 15158272u);
    free(tab);
    CHECK(pvqo_index_bits(8, 16) == 24 && pvqo_max_k(8, 24) == 16 && pvqo_max_k(16, 52) == 33 && pvqo_max_k(128, 384) == 187);
    CHECK(pvqo_index_bits(0, 3) < 0 && pvqo_max_k(8, 0) < 0);
    round_trip(8, 16, 2000); round_trip(16, 33, 1000); round_trip(32, 60, 500); round_trip(128, 187, 50);
    round_trip(3, 1, 50); round_trip(1, 5, 10);
    matrix(7, 8 * 37, 8, 16, 0, 0, 1); matrix(9, 8 * 64, 8, 16, 2, 0, 3); matrix(5, 16 * 33, 16, 33, 4, 1, 2);
    matrix(3, 32 * 9, 32, 60, 8, 1, 8); matrix(2, 128 * 3, 128, 187, 0, 1, 1);
    {   /* rotation there and back; the error correction on a small well-conditioned factor */
        const int rows = 5, cols = 256;
        float *X = malloc(sizeof(float) * rows * cols), *Y = malloc(sizeof(float) * rows * cols), *Z = malloc(sizeof(float) * rows * cols);
        uint8_t *signs = malloc(cols);
        for (int i = 0; i < rows * cols; i++) X[i] = gauss();
        for (int i = 0; i < cols; i++) signs[i] = uniform() < 0.5;
        CHECK(pvqo_hadamard_rows(X, rows, cols, 64, signs, 0, Y) == 0);
        CHECK(pvqo_hadamard_rows(Y, rows, cols, 64, signs, 1, Z) == 0);
        for (int i = 0; i < rows * cols; i++) CHECK(fabsf(Z[i] - X[i]) < 1e-4f);
        CHECK(pvqo_hadamard_rows(X, rows, cols, 48, signs, 0, Y) != 0);
        float *U = calloc((size_t)cols * cols, sizeof(float)), *Q = malloc(sizeof(float) * rows * cols);
        for (int i = 0; i < cols; i++) { U[i * cols + i] = 1.0f; for (int j = i + 1; j < cols; j++) U[i * cols + j] = 0.01f * gauss(); }
        CHECK(pvqo_correct(X, rows, cols, 8, 16, 0, U, Q, 2) == 0);
        CHECK(pvqo_correct(Y, rows, cols, 16, 33, 1, U, Q, 1) == 0);
        for (int i = 0; i < rows * cols; i++) CHECK(isfinite(X[i]) && isfinite(Y[i]));
        free(X); free(Y); free(Z); free(signs); free(U); free(Q);
    }
    puts("oracle: ok");
    return 0;
}
