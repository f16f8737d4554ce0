/*
 * CPU oracle for group-wise Pyramid Vector Quantization (PVQ) of weight matrices.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU library is
 * checked against.  It shares no code with the GPU path, is never called by it, and is
 * only loaded by the tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * What is written out here, step by step and in the paper's order and notation
 * (arXiv 2410.16926):
 *   - the size table N(D,K) of the integer pyramid P(D,K)      (Sec. 2.4, recurrence eq.)
 *   - the choice of the pulse count K from a bit budget         (Sec. 3.3, Step 2)
 *   - quantising a direction onto P(D,K)                        (Sec. 2.5 "Quantizing the direction")
 *   - pyramid encoding  (point -> integer index)                (App. B.2, Alg. 2)
 *   - pyramid decoding  (integer index -> point), corrected     (App. B.3, Alg. 3)
 *   - the group amplitude s = ||w||_2                            (Sec. 2.3)
 *     or the least-squares amplitude for the quantised direction (Sec. 3.3 Step 4)
 *   - amplitude codes against Beta quantile edges               (Sec. 3.3 Step 5, Sec. 3.4)
 *   - dequantisation: point -> unit sphere -> times amplitude   (Sec. 2.4 eq. for S(D,K), Sec. 3.4)
 *   - the randomised Hadamard rotation along the rows           (Sec. 2.3, Sec. 3.3 Step 1)
 *   - the group-by-group correction of the quantisation error   (Sec. 3.3 Step 6)
 *   - the reference product  out = W_hat x                       (float64 textbook matmul)
 *
 * Arithmetic.  Index arithmetic uses the fixed-width multi-word integers below (NW 32-bit
 * words, little-endian), so that the 52- and 104-bit indices of D=16/32 are exact.  The
 * encoder's floating point is IEEE binary32 with the evaluation order stated at each
 * function (the build's contract fixes it so that two implementations can agree bit for
 * bit); the file must be compiled with -ffp-contract=off and without -ffast-math.  The
 * decoder and the product are float64.
 *
 * Readings taken where the printed text is garbled or silent are marked "Reading:".
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NW 16 /* words per integer: 512 bits */

typedef struct {
    uint32_t w[NW];
} big_t;

/* ------------------------------------------------------------------ */
/* multi-word unsigned integers                                        */
/* ------------------------------------------------------------------ */

static void big_set(big_t *a, uint32_t v)
{
    memset(a, 0, sizeof *a);
    a->w[0] = v;
}

/* r = a + b; returns the carry out of the top word */
static uint32_t big_add(big_t *r, const big_t *a, const big_t *b)
{
    uint64_t carry = 0;
    for (int i = 0; i < NW; i++) {
        uint64_t s = (uint64_t)a->w[i] + b->w[i] + carry;
        r->w[i] = (uint32_t)s;
        carry = s >> 32;
    }
    return (uint32_t)carry;
}

/* r = a - b (caller guarantees a >= b) */
static void big_sub(big_t *r, const big_t *a, const big_t *b)
{
    uint64_t borrow = 0;
    for (int i = 0; i < NW; i++) {
        uint64_t d = (uint64_t)a->w[i] - b->w[i] - borrow;
        r->w[i] = (uint32_t)d;
        borrow = (d >> 32) & 1u;
    }
}

/* -1, 0, +1 for a < b, a == b, a > b */
static int big_cmp(const big_t *a, const big_t *b)
{
    for (int i = NW - 1; i >= 0; i--) {
        if (a->w[i] < b->w[i]) return -1;
        if (a->w[i] > b->w[i]) return 1;
    }
    return 0;
}

/* number of bits needed to write a (0 for a == 0) */
static int big_bitlen(const big_t *a)
{
    for (int i = NW - 1; i >= 0; i--) {
        if (a->w[i]) {
            int n = 0;
            uint32_t v = a->w[i];
            while (v) { n++; v >>= 1; }
            return 32 * i + n;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* size table N(d,k), 0 <= d <= D, 0 <= k <= K          (Sec. 2.4)      */
/* ------------------------------------------------------------------ */

typedef struct {
    int D, K;
    big_t *n; /* n[d*(K+1)+k] */
    int overflow;
} table_t;

static const big_t *tab_at(const table_t *t, int d, int k)
{
    return &t->n[(size_t)d * (t->K + 1) + k];
}

/*
 * N(d,0) = 1 for all d >= 0, N(0,k) = 0 for k >= 1, and
 * N(d,k) = N(d-1,k) + N(d,k-1) + N(d-1,k-1).
 * Reading: the printed recurrence ends in "N(D,K)", which would be circular; the last
 * term is N(D-1,K-1), as the closed form and the worked size N(2,7)=28 require.
 */
static table_t *tab_build(int D, int K)
{
    table_t *t = malloc(sizeof *t);
    t->D = D;
    t->K = K;
    t->overflow = 0;
    t->n = malloc(sizeof(big_t) * (size_t)(D + 1) * (K + 1));
    for (int d = 0; d <= D; d++) {
        for (int k = 0; k <= K; k++) {
            big_t *e = &t->n[(size_t)d * (K + 1) + k];
            if (k == 0) {
                big_set(e, 1);
            } else if (d == 0) {
                big_set(e, 0);
            } else {
                big_t s;
                uint32_t c1 = big_add(&s, tab_at(t, d - 1, k), tab_at(t, d, k - 1));
                uint32_t c2 = big_add(e, &s, tab_at(t, d - 1, k - 1));
                if (c1 || c2) t->overflow = 1;
            }
        }
    }
    return t;
}

static void tab_free(table_t *t)
{
    free(t->n);
    free(t);
}

/* Copy the whole table out, NW words per entry, row-major in (d,k). Returns 0, or -1 on
 * overflow of the NW-word integers. */
int pvqo_table(int D, int K, uint32_t *out)
{
    if (D < 0 || K < 0) return -1;
    table_t *t = tab_build(D, K);
    int bad = t->overflow;
    memcpy(out, t->n, sizeof(big_t) * (size_t)(D + 1) * (K + 1));
    tab_free(t);
    return bad ? -1 : 0;
}

int pvqo_words_per_integer(void) { return NW; }

/* Bits of a codeword index: indices run over [0, N(D,K)-1] (the worked example of the
 * paper's Fig. 2 has C(2,7) = [0,27]), so the width is bit_length(N(D,K)-1). */
static int tab_index_bits(const table_t *t)
{
    big_t one, top;
    big_set(&one, 1);
    big_sub(&top, tab_at(t, t->D, t->K), &one);
    return big_bitlen(&top);
}

int pvqo_index_bits(int D, int K)
{
    if (D < 1 || K < 1) return -1;
    table_t *t = tab_build(D, K);
    int b = t->overflow ? -1 : tab_index_bits(t);
    tab_free(t);
    return b;
}

/*
 * Sec. 3.3 Step 2: the largest K whose index still fits the bit budget.
 * Reading: the printed test "ceil(log2(N)/D) < b" is garbled; the budget is the total
 * number of index bits of one group, and the width is computed exactly, not with log2.
 */
int pvqo_max_k(int D, int bit_budget)
{
    if (D < 1 || bit_budget < 1 || bit_budget > 32 * NW - 2) return -1;
    int best = -1;
    for (int K = 1; K <= 4096; K++) {
        int b = pvqo_index_bits(D, K);
        if (b < 0 || b > bit_budget) break;
        best = K;
    }
    return best;
}

/* ------------------------------------------------------------------ */
/* fixed-order float32 sums                                            */
/* ------------------------------------------------------------------ */

/*
 * Sum by levels of adjacent pairs: (v0+v1), (v2+v3), ...; an odd last element moves up
 * unchanged; repeat until one value is left.  For a power-of-two count this is the
 * balanced binary tree ((v0+v1)+(v2+v3))+...  buf is overwritten.
 */
static float sum_pair_levels(float *buf, int n)
{
    if (n <= 0) return 0.0f;
    while (n > 1) {
        int h = n / 2;
        for (int i = 0; i < h; i++) buf[i] = buf[2 * i] + buf[2 * i + 1];
        if (n & 1) buf[h] = buf[n - 1];
        n = h + (n & 1);
    }
    return buf[0];
}

/* ------------------------------------------------------------------ */
/* quantising the direction                       (Sec. 2.5)           */
/* ------------------------------------------------------------------ */

/*
 * One group w[0..D-1]  ->  y on P(D,K), plus ss = sum of squares (float32, pair levels,
 * each square rounded first).
 *
 * Project onto the l1 ball of radius K and round:  t_i = |w_i| * (K / ||w||_1),
 * y_i = round(t_i) (to nearest, ties to even).  If sum(y) != K, lower (or raise) by one
 * the element with the biggest deviation from its projected value, until the sum is K.
 * Ties go to the lowest coordinate.  Signs of w are applied at the end.
 *
 * Reading: the appendix listing of this routine disagrees with the section text and
 * need not terminate; the text is followed.  "Closest point" is closest in Euclidean
 * distance to the projected point t.
 * Reading: an all-zero group (or one so small that K/||w||_1 is not finite) has no
 * direction; it is sent to (0,...,0,+K), which has index 0.
 */
void pvqo_quantize_group(const float *w, int D, int K, int32_t *y, float *ss_out)
{
    float *a = malloc(sizeof(float) * D);
    float *t = malloc(sizeof(float) * D);
    float *buf = malloc(sizeof(float) * D);

    for (int i = 0; i < D; i++) a[i] = fabsf(w[i]);
    memcpy(buf, a, sizeof(float) * D);
    float l1 = sum_pair_levels(buf, D);
    for (int i = 0; i < D; i++) buf[i] = w[i] * w[i];
    float ss = sum_pair_levels(buf, D);
    if (ss_out) *ss_out = ss;

    float g = (float)K / l1;
    if (!(l1 > 0.0f) || !isfinite(g)) {
        for (int i = 0; i < D; i++) y[i] = 0;
        y[D - 1] = K;
        free(a); free(t); free(buf);
        return;
    }

    int S = 0;
    for (int i = 0; i < D; i++) {
        t[i] = a[i] * g;
        y[i] = (int32_t)rintf(t[i]);
        S += y[i];
    }
    while (S > K) {
        int best = -1;
        float dev = 0.0f;
        for (int i = 0; i < D; i++) {
            if (y[i] <= 0) continue;
            float e = (float)y[i] - t[i]; /* how far above its projected value */
            if (best < 0 || e > dev) { best = i; dev = e; }
        }
        y[best] -= 1;
        S -= 1;
    }
    while (S < K) {
        int best = -1;
        float dev = 0.0f;
        for (int i = 0; i < D; i++) {
            float e = t[i] - (float)y[i]; /* how far below its projected value */
            if (best < 0 || e > dev) { best = i; dev = e; }
        }
        y[best] += 1;
        S += 1;
    }
    for (int i = 0; i < D; i++)
        if (w[i] < 0.0f) y[i] = -y[i];

    free(a); free(t); free(buf);
}

/* ------------------------------------------------------------------ */
/* pyramid encoding                                (App. B.2, Alg. 2)  */
/* ------------------------------------------------------------------ */

/*
 * c = 0, k = K; for coordinate i (d = D - i dimensions still open) with m = |x_i| >= 1:
 *   c += N(d-1,k) + 2 * sum_{j=1}^{m-1} N(d-1,k-j) + [x_i < 0] * N(d-1,k-m);  k -= m.
 * The listing's separate branch for |x_i| = 1 is this expression with an empty sum.
 * Returns 0, or -1 if x is not on P(D,K).
 */
static int rank_point(const table_t *t, const int32_t *x, big_t *c)
{
    int D = t->D, k = t->K;
    big_set(c, 0);
    for (int i = 0; i < D; i++) {
        int d = D - i;
        int m = x[i] < 0 ? -x[i] : x[i];
        if (m > k) return -1;
        if (m >= 1) {
            big_add(c, c, tab_at(t, d - 1, k));
            for (int j = 1; j <= m - 1; j++) {
                big_add(c, c, tab_at(t, d - 1, k - j));
                big_add(c, c, tab_at(t, d - 1, k - j));
            }
            if (x[i] < 0) big_add(c, c, tab_at(t, d - 1, k - m));
            k -= m;
        }
    }
    return k == 0 ? 0 : -1;
}

/* ------------------------------------------------------------------ */
/* pyramid decoding                                (App. B.3, Alg. 3)  */
/* ------------------------------------------------------------------ */

/*
 * z = 0, k = K; for coordinate i with d = D - i:
 *   if k == 0 or c < z + N(d-1,k):  x_i = 0
 *   else z += N(d-1,k); j = 1;
 *        while j < k and c >= z + 2 N(d-1,k-j):  z += 2 N(d-1,k-j); j++
 *        if c < z + N(d-1,k-j):  x_i = +j   else  x_i = -j, z += N(d-1,k-j)
 *   k -= |x_i|
 * Reading: the listing has an undefined "cb" (it is z), an update of z after x_i = -j
 * printed without its assignment, and no updates of i, d, k; these are restored.  Its
 * "c = z" shortcut (all remaining pulses on the last coordinate) is what the general
 * branch yields anyway and is left out.  The guard j < k keeps k-j >= 0.
 *
 * omit_negative_update = 1 reproduces the mistake of the original 1986 description that
 * the paper's Sec. 2.5 reports (no update of z after x_i = -j); it exists so that a test
 * can show the round-trip checks catch exactly that mistake.  Always 0 otherwise.
 */
static void unrank_index(const table_t *t, const big_t *c, int32_t *x, int omit_negative_update)
{
    int D = t->D, k = t->K;
    big_t z, lim, two;
    big_set(&z, 0);
    for (int i = 0; i < D; i++) {
        int d = D - i;
        x[i] = 0;
        if (k == 0) continue;
        big_add(&lim, &z, tab_at(t, d - 1, k));
        if (big_cmp(c, &lim) < 0) continue; /* x_i = 0 */
        z = lim;
        int j = 1;
        for (;;) {
            if (j >= k) break;
            big_add(&two, tab_at(t, d - 1, k - j), tab_at(t, d - 1, k - j));
            big_add(&lim, &z, &two);
            if (big_cmp(c, &lim) < 0) break;
            z = lim;
            j++;
        }
        big_add(&lim, &z, tab_at(t, d - 1, k - j));
        if (big_cmp(c, &lim) < 0) {
            x[i] = j;
        } else {
            x[i] = -j;
            if (!omit_negative_update) z = lim;
        }
        k -= j;
    }
}

/* Single-point entry points for the tests.  c is NW words. */
int pvqo_rank(int D, int K, const int32_t *x, uint32_t *c_words)
{
    table_t *t = tab_build(D, K);
    big_t c;
    int rc = rank_point(t, x, &c);
    memcpy(c_words, c.w, sizeof c.w);
    tab_free(t);
    return rc;
}

int pvqo_unrank(int D, int K, const uint32_t *c_words, int32_t *x, int omit_negative_update)
{
    table_t *t = tab_build(D, K);
    big_t c;
    memcpy(c.w, c_words, sizeof c.w);
    int rc = big_cmp(&c, tab_at(t, D, K)) < 0 ? 0 : -1;
    if (rc == 0) unrank_index(t, &c, x, omit_negative_update);
    tab_free(t);
    return rc;
}

/* Many points at once (tests enumerate whole pyramids). x is [n][D], c is [n][NW]. */
int pvqo_rank_many(int D, int K, int64_t n, const int32_t *x, uint32_t *c_words)
{
    table_t *t = tab_build(D, K);
    int rc = 0;
    for (int64_t p = 0; p < n; p++) {
        big_t c;
        if (rank_point(t, x + p * D, &c)) rc = -1;
        memcpy(c_words + p * NW, c.w, sizeof c.w);
    }
    tab_free(t);
    return rc;
}

int pvqo_unrank_many(int D, int K, int64_t n, const uint32_t *c_words, int32_t *x,
                     int omit_negative_update)
{
    table_t *t = tab_build(D, K);
    int rc = 0;
    for (int64_t p = 0; p < n; p++) {
        big_t c;
        memcpy(c.w, c_words + p * NW, sizeof c.w);
        if (big_cmp(&c, tab_at(t, D, K)) >= 0) { rc = -1; continue; }
        unrank_index(t, &c, x + p * D, omit_negative_update);
    }
    tab_free(t);
    return rc;
}

/* ------------------------------------------------------------------ */
/* packed layout                                                        */
/* ------------------------------------------------------------------ */

/*
 * Reading: the paper does not fix a storage layout.  Each row is a little-endian bit
 * stream over 32-bit words: the field of group g occupies bits [g*b, (g+1)*b), least
 * significant bit first; every row starts on a word boundary.
 */
static int64_t row_words(int64_t groups, int bits)
{
    return (groups * bits + 31) / 32;
}

int64_t pvqo_row_words(int64_t groups, int bits) { return row_words(groups, bits); }

static void put_bits(uint32_t *row, int64_t bitpos, int nbits, const uint32_t *value_words)
{
    for (int b = 0; b < nbits; b++) {
        uint32_t bit = (value_words[b >> 5] >> (b & 31)) & 1u;
        int64_t p = bitpos + b;
        if (bit) row[p >> 5] |= (uint32_t)1 << (p & 31);
    }
}

static void get_bits(const uint32_t *row, int64_t bitpos, int nbits, uint32_t *value_words)
{
    for (int i = 0; i < NW; i++) value_words[i] = 0;
    for (int b = 0; b < nbits; b++) {
        int64_t p = bitpos + b;
        uint32_t bit = (row[p >> 5] >> (p & 31)) & 1u;
        value_words[b >> 5] |= bit << (b & 31);
    }
}

/* ------------------------------------------------------------------ */
/* whole-matrix encode                                                  */
/* ------------------------------------------------------------------ */

typedef struct {
    const table_t *tab;
    const float *W;
    int64_t rows, cols, r0, r1;
    int D, K, index_bits, scale_bits;
    int amp_mode;       /* 0: s_g = ||w_g||_2; 1: least-squares amplitude */
    const float *edges; /* 2^scale_bits - 1 ascending float32 edges, or NULL */
    uint32_t *index_out;
    void *scale_out;
    float *rowss_out;
    int8_t *pulses_out;
} enc_job_t;

/*
 * Least-squares amplitude of a group for its quantised direction (Sec. 3.3 Step 4).
 * The group is rebuilt as s * y / ||y||_2; the s that minimises ||w - s y/||y||_2||_2 is
 *     s = (y . w) / ||y||_2 .
 * Reading: the section prints the ratio of the two inner products upside down; the
 * minimiser of the stated distance is the one above (a test checks it against a
 * least-squares solve).
 * float32, fixed order: products (float)y_i * w_i rounded one by one, summed over pair
 * levels; sum of y_i^2 as an integer; one square root, one division.
 */
float pvqo_ls_amplitude(const float *w, const int32_t *y, int D)
{
    float *buf = malloc(sizeof(float) * D);
    int32_t n2 = 0;
    for (int i = 0; i < D; i++) {
        buf[i] = (float)y[i] * w[i];
        n2 += y[i] * y[i];
    }
    float dot = sum_pair_levels(buf, D);
    free(buf);
    return dot / sqrtf((float)n2);
}

/*
 * Rows r0..r1-1 of W (row-major float32, cols = G*D; a bf16 source is widened exactly
 * by the caller).  Per group: quantise, rank, pack, and the amplitude s_g: sqrtf(ss_g)
 * with ss_g the group's sum of squares, or (amp_mode 1) the least-squares amplitude, for
 * which ss_g = s_g * s_g below.
 *   scale_bits == 0: s_g is stored as float32 [rows][G].
 *   scale_bits  > 0 (Sec. 3.3 Step 5 / Sec. 3.4): rowss = sum_g ss_g (pair levels),
 *       u_g = ss_g / rowss, code q_g = number of edges <= u_g, which is
 *       floor(CDF(u_g) * 2^b) when edges[j-1] = PPF(j / 2^b); codes are packed like the
 *       indices, rowss is stored per row.
 */
static void *encode_rows(void *arg)
{
    enc_job_t *J = arg;
    int D = J->D, K = J->K;
    int64_t G = J->cols / D;
    int64_t iw = row_words(G, J->index_bits);
    int64_t sw = J->scale_bits ? row_words(G, J->scale_bits) : 0;
    int32_t *y = malloc(sizeof(int32_t) * D);
    float *ss = malloc(sizeof(float) * G);
    float *amp = malloc(sizeof(float) * G);
    float *buf = malloc(sizeof(float) * G);
    int nedges = J->scale_bits ? (1 << J->scale_bits) - 1 : 0;

    for (int64_t r = J->r0; r < J->r1; r++) {
        const float *wrow = J->W + r * J->cols;
        uint32_t *irow = J->index_out + r * iw;
        memset(irow, 0, sizeof(uint32_t) * iw);
        for (int64_t g = 0; g < G; g++) {
            big_t c;
            pvqo_quantize_group(wrow + g * D, D, K, y, &ss[g]);
            if (J->amp_mode == 1) {
                amp[g] = pvqo_ls_amplitude(wrow + g * D, y, D);
                ss[g] = amp[g] * amp[g];
            } else {
                amp[g] = sqrtf(ss[g]);
            }
            rank_point(J->tab, y, &c);
            put_bits(irow, g * J->index_bits, J->index_bits, c.w);
            if (J->pulses_out)
                for (int i = 0; i < D; i++) J->pulses_out[r * J->cols + g * D + i] = (int8_t)y[i];
        }
        if (J->scale_bits == 0) {
            float *srow = (float *)J->scale_out + r * G;
            for (int64_t g = 0; g < G; g++) srow[g] = amp[g];
            if (J->rowss_out) {
                memcpy(buf, ss, sizeof(float) * G);
                J->rowss_out[r] = sum_pair_levels(buf, (int)G);
            }
        } else {
            uint32_t *srow = (uint32_t *)J->scale_out + r * sw;
            memset(srow, 0, sizeof(uint32_t) * sw);
            memcpy(buf, ss, sizeof(float) * G);
            float rowss = sum_pair_levels(buf, (int)G);
            J->rowss_out[r] = rowss;
            for (int64_t g = 0; g < G; g++) {
                float u = ss[g] / rowss;
                uint32_t q = 0;
                for (int j = 0; j < nedges; j++)
                    if (J->edges[j] <= u) q++;
                put_bits(srow, g * J->scale_bits, J->scale_bits, &q);
            }
        }
    }
    free(y); free(ss); free(amp); free(buf);
    return NULL;
}

/* Rows are split into nthreads contiguous blocks (plain static split; 1 = serial). */
int pvqo_encode(const float *W, int64_t rows, int64_t cols, int D, int K, int scale_bits,
                int amp_mode, const float *edges, uint32_t *index_out, void *scale_out,
                float *rowss_out, int8_t *pulses_out, int nthreads)
{
    if (D < 1 || K < 1 || K > 1023 || cols % D || scale_bits < 0 || scale_bits > 8) return -1;
    if (K > 127 && pulses_out) return -1; /* the optional pulse plane is int8 */
    if (amp_mode != 0 && amp_mode != 1) return -1;
    if (scale_bits > 0 && (!edges || !rowss_out)) return -1;
    table_t *t = tab_build(D, K);
    if (t->overflow) { tab_free(t); return -1; }
    int ib = tab_index_bits(t);
    if (nthreads < 1) nthreads = 1;
    if (nthreads > rows) nthreads = rows > 0 ? (int)rows : 1;
    pthread_t *th = malloc(sizeof(pthread_t) * nthreads);
    enc_job_t *jobs = malloc(sizeof(enc_job_t) * nthreads);
    for (int i = 0; i < nthreads; i++) {
        enc_job_t j = { t, W, rows, cols, rows * i / nthreads, rows * (i + 1) / nthreads,
                        D, K, ib, scale_bits, amp_mode, edges, index_out, scale_out, rowss_out,
                        pulses_out };
        jobs[i] = j;
        if (nthreads == 1) encode_rows(&jobs[i]);
        else pthread_create(&th[i], NULL, encode_rows, &jobs[i]);
    }
    if (nthreads > 1)
        for (int i = 0; i < nthreads; i++) pthread_join(th[i], NULL);
    free(th); free(jobs);
    tab_free(t);
    return 0;
}

/* ------------------------------------------------------------------ */
/* correcting the quantisation error, group after group   (Sec. 3.3 Step 6) */
/* ------------------------------------------------------------------ */

/*
 * Every row w of W (float32 [rows][cols], in place) goes through the groups g = 0 .. G-1 in
 * order.  At group g (columns gD .. gD+D-1):
 *   1. the group's current values are quantised as in Steps 3 and 4: point y on P(D,K),
 *      amplitude s (norm, or amp_mode 1: least squares), and its quantised value
 *          q_i = (s / sqrtf((float) sum y_i^2)) * (float) y_i            (float32, as written);
 *   2. e = w_g - q (float32) is the error that the columns not yet quantised take up:
 *          w_rest <- w_rest - e (A_gg)^-1 A_g,rest,
 *      A the inverse of the Hessian restricted to the columns from g on.  (Reading: the section
 *      prints the two sub-matrices with their indices mixed up; this is the update that
 *      minimises the proxy loss of Sec. 2.1 over the remaining columns with the columns up to
 *      g held at their quantised values, the block form of the update of the work it cites.)
 *      With H^-1 = U^T U, U upper triangular (the Cholesky factor that the section points to),
 *      A = U_{g:,g:}^T U_{g:,g:}, so (A_gg)^-1 A_g,rest = U_gg^-1 U_g,rest:
 *          t U_gg = e          by substitution, j = 0 .. D-1:
 *                              t_j = (e_j - t_0 U[gD+0][gD+j] - ... - t_{j-1} U[gD+j-1][gD+j]) / U[gD+j][gD+j]
 *          w_c <- w_c - t_0 U[gD][c] - ... - t_{D-1} U[gD+D-1][c]     for every column c >= (g+1) D.
 *      float32; each "- t_i U" is one fused multiply-add fmaf(-t_i, U, .), applied in the
 *      order i = 0, 1, ... to the running value (a fixed order, so that two implementations
 *      that decide roundings from these values can agree bit for bit).
 * The columns of group g are not written again after step g: on return W holds, for every
 * group, the values that were quantised, so that encoding W reproduces y and s.
 * Reading: the amplitude in the error is the float32 amplitude of Step 4 also when amplitude
 * codes (Step 5) are stored afterwards: their row normaliser needs the amplitudes of the whole
 * row, which exist only after the last group.
 * U: float32 [cols][cols], row-major; only its upper triangle is read.  Q_out (optional,
 * float32 [rows][cols]) receives the quantised values q.
 */
typedef struct {
    float *W; float *Q_out; const float *U;
    int64_t cols, r0, r1;
    int D, K, amp_mode;
} corr_job_t;

static void *correct_rows(void *arg)
{
    corr_job_t *J = arg;
    int D = J->D;
    int64_t C = J->cols, G = C / D;
    int32_t *y = malloc(sizeof(int32_t) * D);
    float *t = malloc(sizeof(float) * D);
    for (int64_t r = J->r0; r < J->r1; r++) {
        float *w = J->W + r * C;
        for (int64_t g = 0; g < G; g++) {
            float *wg = w + g * D;
            const float *Ug = J->U + (g * D) * C;   /* row gD of U */
            float ss, s;
            pvqo_quantize_group(wg, D, J->K, y, &ss);
            s = J->amp_mode == 1 ? pvqo_ls_amplitude(wg, y, D) : sqrtf(ss);
            int32_t n2 = 0;
            for (int i = 0; i < D; i++) n2 += y[i] * y[i];
            float gain = s / sqrtf((float)n2);
            for (int j = 0; j < D; j++) {
                float q = gain * (float)y[j];
                if (J->Q_out) J->Q_out[r * C + g * D + j] = q;
                float acc = wg[j] - q;
                for (int i = 0; i < j; i++) acc = fmaf(-t[i], Ug[i * C + g * D + j], acc);
                t[j] = acc / Ug[j * C + g * D + j];
            }
            for (int64_t c = (g + 1) * D; c < C; c++) {
                float acc = w[c];
                for (int i = 0; i < D; i++) acc = fmaf(-t[i], Ug[i * C + c], acc);
                w[c] = acc;
            }
        }
    }
    free(y); free(t);
    return NULL;
}

int pvqo_correct(float *W, int64_t rows, int64_t cols, int D, int K, int amp_mode,
                 const float *U, float *Q_out, int nthreads)
{
    if (D < 1 || K < 1 || K > 1023 || cols % D || !W || !U) return -1;
    if (amp_mode != 0 && amp_mode != 1) return -1;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > rows) nthreads = rows > 0 ? (int)rows : 1;
    pthread_t *th = malloc(sizeof(pthread_t) * nthreads);
    corr_job_t *jobs = malloc(sizeof(corr_job_t) * nthreads);
    for (int i = 0; i < nthreads; i++) {
        corr_job_t j = { W, Q_out, U, cols, rows * i / nthreads, rows * (i + 1) / nthreads,
                         D, K, amp_mode };
        jobs[i] = j;
        if (nthreads == 1) correct_rows(&jobs[i]);
        else pthread_create(&th[i], NULL, correct_rows, &jobs[i]);
    }
    if (nthreads > 1)
        for (int i = 0; i < nthreads; i++) pthread_join(th[i], NULL);
    free(th); free(jobs);
    return 0;
}

/* ------------------------------------------------------------------ */
/* randomised Hadamard rotation along the rows    (Sec. 2.3, Sec. 3.3 Step 1) */
/* ------------------------------------------------------------------ */

/*
 * Every row of X (float32 [rows][cols]) is cut into blocks of `block` consecutive values
 * (block a power of two dividing cols) and each block x is replaced by
 *     signs_after == 0:   H (s . x) / sqrt(block)        (the rotation applied before quantising)
 *     signs_after == 1:   s . (H x) / sqrt(block)        (its inverse: H is symmetric, H H = block I)
 * with H the Sylvester-Hadamard matrix in natural order and s_i = -1 where signs[i] != 0, else +1
 * (signs has cols entries, NULL = all +1).
 * float32 throughout: the transform is the in-place butterfly a,b -> a+b, a-b over strides
 * 1, 2, 4, ..., block/2 in that order (every value of a stage is one rounded sum or difference
 * of two values of the stage before, so the result does not depend on how a stage is scheduled),
 * then one multiplication by the float32 nearest to 1/sqrt(block).
 * Reading: the paper takes its rotation from the works it cites and gives no arithmetic; this
 * is the plain fast Walsh-Hadamard transform, block diagonal when cols is not a power of two.
 */
int pvqo_hadamard_rows(const float *X, int64_t rows, int64_t cols, int64_t block,
                       const uint8_t *signs, int signs_after, float *Y)
{
    if (block < 1 || (block & (block - 1)) || cols % block) return -1;
    float scale = (float)(1.0 / sqrt((double)block));
    float *v = malloc(sizeof(float) * block);
    for (int64_t r = 0; r < rows; r++)
        for (int64_t b0 = 0; b0 < cols; b0 += block) {
            const float *x = X + r * cols + b0;
            for (int64_t i = 0; i < block; i++)
                v[i] = (!signs_after && signs && signs[b0 + i]) ? -x[i] : x[i];
            for (int64_t h = 1; h < block; h *= 2)
                for (int64_t i = 0; i < block; i += 2 * h)
                    for (int64_t j = i; j < i + h; j++) {
                        float a = v[j], b = v[j + h];
                        v[j] = a + b;
                        v[j + h] = a - b;
                    }
            float *y = Y + r * cols + b0;
            for (int64_t i = 0; i < block; i++) {
                float t = v[i] * scale;
                y[i] = (signs_after && signs && signs[b0 + i]) ? -t : t;
            }
        }
    free(v);
    return 0;
}

/* ------------------------------------------------------------------ */
/* whole-matrix decode and the reference product                        */
/* ------------------------------------------------------------------ */

typedef struct {
    const table_t *tab;
    const uint32_t *index;
    const void *scale;
    const float *rowss;
    int64_t rows, cols, r0, r1;
    int D, K, index_bits, scale_bits;
    const double *centers; /* 2^scale_bits values PPF((q+0.5)/2^b), or NULL */
    double *W_out;         /* [rows][cols] or NULL */
    int8_t *pulses_out;    /* [rows][cols] or NULL */
    const double *x;       /* [batch][cols] or NULL */
    int batch;
    double *out;           /* [batch][rows] */
} dec_job_t;

/*
 * Index -> point p (Alg. 3) -> direction p / ||p||_2 on the unit sphere (the spherical
 * code S(D,K) of Sec. 2.4) -> times the amplitude:
 *   scale_bits == 0: the stored float32 s_g;
 *   scale_bits  > 0: s_g^2 = PPF((q+0.5)/2^b) * rowss  (Sec. 3.4 dequantize; the quantised
 *       quantity is the squared amplitude normalised by the row's sum of squares).
 * All in float64.  If x is given, out[b][r] = sum_c W_hat[r][c] * x[b][c] as well.
 */
static void *decode_rows(void *arg)
{
    dec_job_t *J = arg;
    int D = J->D;
    int64_t G = J->cols / D;
    int64_t iw = row_words(G, J->index_bits);
    int64_t sw = J->scale_bits ? row_words(G, J->scale_bits) : 0;
    int32_t *p = malloc(sizeof(int32_t) * D);
    double *wrow = malloc(sizeof(double) * J->cols);

    for (int64_t r = J->r0; r < J->r1; r++) {
        const uint32_t *irow = J->index + r * iw;
        for (int64_t g = 0; g < G; g++) {
            big_t c;
            get_bits(irow, g * J->index_bits, J->index_bits, c.w);
            if (big_cmp(&c, tab_at(J->tab, D, J->K)) >= 0) {
                /* not a codeword: decoded as zeros */
                for (int i = 0; i < D; i++) { p[i] = 0; wrow[g * D + i] = 0.0; }
            } else {
                unrank_index(J->tab, &c, p, 0);
                double n2 = 0.0;
                for (int i = 0; i < D; i++) n2 += (double)p[i] * (double)p[i];
                double s;
                if (J->scale_bits == 0) {
                    s = (double)((const float *)J->scale)[r * G + g];
                } else {
                    uint32_t q[NW];
                    get_bits((const uint32_t *)J->scale + r * sw, g * J->scale_bits,
                             J->scale_bits, q);
                    s = sqrt(J->centers[q[0]] * (double)J->rowss[r]);
                }
                for (int i = 0; i < D; i++) wrow[g * D + i] = s * (double)p[i] / sqrt(n2);
            }
            if (J->pulses_out)
                for (int i = 0; i < D; i++) J->pulses_out[r * J->cols + g * D + i] = (int8_t)p[i];
        }
        if (J->W_out) memcpy(J->W_out + r * J->cols, wrow, sizeof(double) * J->cols);
        for (int b = 0; b < J->batch; b++) {
            double acc = 0.0;
            const double *xb = J->x + (int64_t)b * J->cols;
            for (int64_t c = 0; c < J->cols; c++) acc += wrow[c] * xb[c];
            J->out[(int64_t)b * J->rows + r] = acc;
        }
    }
    free(p); free(wrow);
    return NULL;
}

int pvqo_decode(const uint32_t *index, const void *scale, const float *rowss, int64_t rows,
                int64_t cols, int D, int K, int scale_bits, const double *centers,
                double *W_out, int8_t *pulses_out, const double *x, int batch, double *out,
                int nthreads)
{
    if (D < 1 || K < 1 || K > 1023 || cols % D || scale_bits < 0 || scale_bits > 8) return -1;
    if (K > 127 && pulses_out) return -1; /* the optional pulse plane is int8 */
    if (scale_bits > 0 && (!centers || !rowss)) return -1;
    if (batch > 0 && (!x || !out)) return -1;
    table_t *t = tab_build(D, K);
    if (t->overflow) { tab_free(t); return -1; }
    int ib = tab_index_bits(t);
    if (nthreads < 1) nthreads = 1;
    if (nthreads > rows) nthreads = rows > 0 ? (int)rows : 1;
    pthread_t *th = malloc(sizeof(pthread_t) * nthreads);
    dec_job_t *jobs = malloc(sizeof(dec_job_t) * nthreads);
    for (int i = 0; i < nthreads; i++) {
        dec_job_t j = { t, index, scale, rowss, rows, cols, rows * i / nthreads,
                        rows * (i + 1) / nthreads, D, K, ib, scale_bits, centers, W_out,
                        pulses_out, x, batch, out };
        jobs[i] = j;
        if (nthreads == 1) decode_rows(&jobs[i]);
        else pthread_create(&th[i], NULL, decode_rows, &jobs[i]);
    }
    if (nthreads > 1)
        for (int i = 0; i < nthreads; i++) pthread_join(th[i], NULL);
    free(th); free(jobs);
    tab_free(t);
    return 0;
}
