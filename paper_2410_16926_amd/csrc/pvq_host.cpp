// Host side of libpvq: status codes, exact size tables, the choice of K, Beta quantile tables,
// the context, and argument validation in front of the kernel launchers.
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "pvq_internal.h"
#include "pvq_diagnostics.h"
#include "pvq_walk.h"

// ------------------------------------------------------------------------------------------
// status
// ------------------------------------------------------------------------------------------

static thread_local int g_last_hip_error = 0;

static int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return PVQ_E_HIP;
}

extern "C" const char *pvq_strerror(int status)
{
    switch (status) {
    case PVQ_OK: return "ok";
    case PVQ_E_INVALID_ARG: return "invalid argument";
    case PVQ_E_UNSUPPORTED: return "unsupported configuration";
    case PVQ_E_ALIGNMENT: return "pointer or leading dimension not aligned as required";
    case PVQ_E_HIP: return "HIP runtime error (see pvq_last_hip_error)";
    case PVQ_E_NOMEM: return "out of host memory";
    default: return "unknown status";
    }
}

extern "C" int pvq_last_hip_error(void) { return g_last_hip_error; }

// ------------------------------------------------------------------------------------------
// 512-bit unsigned integers (eight 64-bit limbs) for the size tables
// ------------------------------------------------------------------------------------------

namespace {

struct U512 {
    uint64_t limb[8] = {0, 0, 0, 0, 0, 0, 0, 0};

    static U512 of(uint64_t v)
    {
        U512 r;
        r.limb[0] = v;
        return r;
    }
    // returns true when the sum left 512 bits
    bool add(const U512 &o)
    {
        unsigned __int128 carry = 0;
        for (int i = 0; i < 8; i++) {
            unsigned __int128 s = (unsigned __int128)limb[i] + o.limb[i] + carry;
            limb[i] = (uint64_t)s;
            carry = s >> 64;
        }
        return carry != 0;
    }
    void decrement()  // value > 0
    {
        for (int i = 0; i < 8; i++)
            if (limb[i]-- != 0) break;
    }
    int bit_length() const
    {
        for (int i = 7; i >= 0; i--)
            if (limb[i]) return 64 * i + 64 - __builtin_clzll(limb[i]);
        return 0;
    }
    uint32_t word(int i) const { return (uint32_t)(limb[i >> 1] >> (32 * (i & 1))); }
};

// Pyramid sizes N(d,k) for d <= D, k <= K (Sec. 2.4).  Rolling rows would do for a single count,
// but the kernels need every row, so the whole table is kept.
struct SizeTable {
    int D, K;
    int first_bad_k;      // smallest k with an entry that left 512 bits (K+1 if none); columns
                          // below it are exact, because N(d,k) only depends on columns <= k
    bool overflow;
    std::vector<U512> n;  // (D+1) x (K+1)

    SizeTable(int D_, int K_) : D(D_), K(K_), first_bad_k(K_ + 1), n((size_t)(D_ + 1) * (K_ + 1))
    {
        for (int k = 0; k <= K; k++) at(0, k) = U512::of(k == 0 ? 1 : 0);
        for (int d = 1; d <= D; d++) {
            at(d, 0) = U512::of(1);
            for (int k = 1; k <= K; k++) {
                U512 v = at(d - 1, k);
                bool bad = v.add(at(d, k - 1));
                bad |= v.add(at(d - 1, k - 1));
                if (bad && k < first_bad_k) first_bad_k = k;
                at(d, k) = v;
            }
        }
        overflow = first_bad_k <= K;
    }
    U512 &at(int d, int k) { return n[(size_t)d * (K + 1) + k]; }
    const U512 &at(int d, int k) const { return n[(size_t)d * (K + 1) + k]; }
    int index_bits() const
    {
        U512 top = at(D, K);
        top.decrement();
        return top.bit_length();
    }
};

}  // namespace

extern "C" int pvq_count(int D, int K, uint32_t *count_words, int *index_bits)
{
    if (D < 1 || D > 256 || K < 0 || K > 1024) return PVQ_E_INVALID_ARG;
    SizeTable t(D, K);
    if (t.overflow) return PVQ_E_UNSUPPORTED;
    if (count_words)
        for (int i = 0; i < 16; i++) count_words[i] = t.at(D, K).word(i);
    if (index_bits) *index_bits = t.index_bits();
    return PVQ_OK;
}

extern "C" int pvq_max_k(int D, int bit_budget, int *K)
{
    if (D < 1 || D > 256 || bit_budget < 1 || bit_budget > 511 || !K) return PVQ_E_INVALID_ARG;
    // One table with a generous K bound; N(D,k) grows with k, so the first k that does not fit
    // (or that left the 512-bit integers) ends the search.
    int kmax = 1024;
    SizeTable t(D, kmax);
    int best = 0;
    for (int k = 1; k <= kmax && k < t.first_bad_k; k++) {
        U512 top = t.at(D, k);
        top.decrement();
        if (top.bit_length() > bit_budget) break;
        best = k;
    }
    if (best < 1) return PVQ_E_UNSUPPORTED;
    *K = best;
    return PVQ_OK;
}

// ------------------------------------------------------------------------------------------
// Beta(a, b) quantiles for integer a (D even): Sec. 3.4
// ------------------------------------------------------------------------------------------

namespace {

// For integer a the upper tail of Beta(a, b) is a short sum of positive terms,
//   P[X > x] = (1-x)^b * sum_{j < a} C(b+j-1, j) x^j,
// evaluated in long double.  The lower tail is 1 minus it; the probabilities asked for are
// multiples of 2^-9 at the finest, so the subtraction costs nothing that matters at 64 mantissa bits.
long double beta_upper_tail(long double x, int a, long double b)
{
    if (x <= 0) return 1.0L;
    if (x >= 1) return 0.0L;
    long double lead = expl(b * log1pl(-x));
    long double term = 1.0L;  // C(b+j-1, j) x^j at j = 0
    long double sum = 0.0L;
    for (int j = 0; j < a; j++) {
        sum += term;
        term *= (b + j) * x / (long double)(j + 1);
    }
    return lead * sum;
}

// PPF(p) by bisection: the upper tail decreases in x.
double beta_ppf(long double p, int a, long double b)
{
    long double lo = 0.0L, hi = 1.0L;
    long double target = 1.0L - p;
    for (int it = 0; it < 400; it++) {
        long double mid = 0.5L * (lo + hi);
        if (mid == lo || mid == hi) break;
        if (beta_upper_tail(mid, a, b) > target) lo = mid; else hi = mid;
    }
    return (double)(0.5L * (lo + hi));
}

bool scale_bits_ok(int sb) { return sb == 0 || sb == 1 || sb == 2 || sb == 4 || sb == 8; }

}  // namespace

extern "C" int pvq_beta_tables(int D, int64_t G, int scale_bits, double *edges, double *centers)
{
    if (!edges || !centers || D < 2 || G < 2) return PVQ_E_INVALID_ARG;
    if ((D & 1) || !scale_bits_ok(scale_bits) || scale_bits == 0) return PVQ_E_UNSUPPORTED;
    int a = D / 2;
    long double b = (long double)D * (long double)(G - 1) / 2.0L;
    int n = 1 << scale_bits;
    for (int j = 1; j < n; j++) edges[j - 1] = beta_ppf((long double)j / n, a, b);
    for (int q = 0; q < n; q++) centers[q] = beta_ppf(((long double)q + 0.5L) / n, a, b);
    return PVQ_OK;
}

// ------------------------------------------------------------------------------------------
// tables of the coordinate-by-coordinate decoder (pvq_walk.hip)
// ------------------------------------------------------------------------------------------

namespace {

U512 shifted_left(const U512 &v, int n)   // n < 512; bits shifted out are lost
{
    U512 r;
    const int limbs = n / 64, bits = n % 64;
    for (int i = 7; i >= limbs; i--) {
        uint64_t x = v.limb[i - limbs] << bits;
        if (bits && i - limbs - 1 >= 0) x |= v.limb[i - limbs - 1] >> (64 - bits);
        r.limb[i] = x;
    }
    return r;
}

bool less_or_equal(const U512 &a, const U512 &b)
{
    for (int i = 7; i >= 0; i--)
        if (a.limb[i] != b.limb[i]) return a.limb[i] < b.limb[i];
    return true;
}

// Lays the blob out (pvq_walk.h has the layout's formulas) and fills it: rows d' = 1 .. D-1 of U(d',x),
// x = -1 .. K+1; guess rows for d' >= 2: entry 0 for q/2 = 0, entry 1 + (e << mb) + f for q/2 in
// [2^e (1 + f / 2^mb), 2^e (1 + (f+1) / 2^mb)) = the number of x in [0, K] with U(d',x) <= that bucket's lower edge.
bool build_walk_tables(const SizeTable &t, int D, int K, int words, std::vector<unsigned char> &blob, pvq_walk_params &p)
{
    using namespace pvq_walk;
    if (D > 32 || K > 253) return false;
    memset(&p, 0, sizeof p);
    int fit_half = 0, fit_quarter = 0;
    for (int d = 1; d < D; d++) {
        if (words >= 2 && t.at(d, K).bit_length() <= 16 * words) fit_half = d;
        if (words >= 4 && t.at(d, K).bit_length() <= 8 * words) fit_quarter = d;
    }
    pvq_walk_schedule(D, words, fit_half, fit_quarter, &p.dA, &p.dB);
    if (p.dA > fit_half || p.dB > fit_quarter || p.dB > p.dA) return false;
    p.K = K;
    for (int cls = 0; cls < 3; cls++) p.row_bytes[cls] = (uint32_t)(((size_t)(K + 3) * ((4 * words) >> cls) + 15) / 16 * 16);
    blob.clear();
    // cumulative rows
    std::vector<std::vector<U512>> U(D);
    for (int dp = 1; dp < D; dp++) {
        const int es = pvq_walk_entry_bits(dp, words, p.dA, p.dB) / 8;
        U512 run;
        for (int x = 0; x <= K; x++) { run.add(t.at(dp, x)); U[dp].push_back(run); }
        if (run.bit_length() > 8 * es) return false;
        const size_t first = blob.size();
        blob.resize(first + p.row_bytes[pvq_walk_class(dp, p.dA, p.dB)], 0);
        for (int x = 0; x <= K; x++)
            for (int w = 0; w < es / 4; w++) {
                const uint32_t v = U[dp][x].word(w);
                memcpy(&blob[first + (size_t)(x + 1) * es + 4 * w], &v, 4);
            }
        memset(&blob[first + (size_t)(K + 2) * es], 0xFF, es);        // never <= q/2
    }
    // guess rows
    p.guess_base = (uint32_t)blob.size();
    for (int dp = 2; dp < D; dp++) {
        const int mb = pvq_walk_mb(dp);
        const int n = (int)pvq_walk_guess_entries(dp, pvq_walk_entry_bits(dp, words, p.dA, p.dB));
        if (blob.size() != p.guess_base + pvq_walk_guess_offset(dp, words, p.dA, p.dB)) return false;
        for (int idx = 0; idx < n; idx++) {
            int count = 0;
            if (idx >= 1) {
                const int e = (idx - 1) >> mb, f = (idx - 1) & ((1 << mb) - 1);
                // U <= (2^mb + f) 2^(e - mb)   <=>   U 2^mb <= (2^mb + f) 2^e
                const U512 edge = shifted_left(U512::of((uint64_t)((1 << mb) + f)), e);
                for (int x = 0; x <= K; x++)
                    if (less_or_equal(shifted_left(U[dp][x], mb), edge)) count = x + 1;
            }
            blob.push_back((unsigned char)count);
        }
    }
    blob.resize((blob.size() + 15) / 16 * 16);
    p.bytes = (uint32_t)blob.size();
    return true;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// context
// ------------------------------------------------------------------------------------------

extern "C" int pvq_ctx_create(pvq_ctx **out, int D, int K, int scale_bits, const double *edges,
                              const double *centers)
{
    if (!out) return PVQ_E_INVALID_ARG;
    *out = nullptr;
    // groups of 64 and 128 values (the on-the-fly activation setting) go to the kernels of pvq_wide.hip:
    // a wave per group, tables of up to 16-word integers streamed from device memory
    const bool wide = D == 64 || D == 128;
    if (!wide && D != 8 && D != 16 && D != 32) return PVQ_E_UNSUPPORTED;
    if (K < 1 || K > (wide ? 1023 : 127)) return PVQ_E_UNSUPPORTED;
    if (!scale_bits_ok(scale_bits) || (wide && scale_bits != 0)) return PVQ_E_UNSUPPORTED;
    if (scale_bits > 0 && (!edges || !centers)) return PVQ_E_INVALID_ARG;

    SizeTable t(D, K);
    if (t.overflow) return PVQ_E_UNSUPPORTED;
    int bits = t.index_bits();
    if (bits < 1 || bits > (wide ? 512 : 128)) return PVQ_E_UNSUPPORTED;
    int words = bits <= 32 ? 1 : (bits <= 64 ? 2 : 4);
    if (wide) words = 4 * ((std::max(t.at(D, K).bit_length(), 1) + 127) / 128);   // N(D,K) itself is an entry
    // the decoders form N(D,K) - 1 - index in `words` words: N(D,K) must fit them (it fails to only when it
    // is exactly 2^(32 words), which no supported (D,K) gives)
    if (t.at(D, K).bit_length() > 32 * words) return PVQ_E_UNSUPPORTED;

    int n = scale_bits ? (1 << scale_bits) : 0;
    std::vector<float> e32, sc32;
    if (scale_bits) {
        for (int j = 0; j + 1 < n; j++) {
            if (!(edges[j] >= 0.0) || (j > 0 && !(edges[j] >= edges[j - 1]))) return PVQ_E_INVALID_ARG;
            e32.push_back((float)edges[j]);
        }
        for (int q = 0; q < n; q++) {
            if (!(centers[q] >= 0.0)) return PVQ_E_INVALID_ARG;
            sc32.push_back((float)std::sqrt(centers[q]));
        }
    }

    // tab_n[dp][k] = N(dp,k); tab_u[dp][k+1] = N(dp,0) + ... + N(dp,k), tab_u[dp][0] = 0.
    // Every entry is below N(D,K) (the pyramid of one more dimension contains all of them), so it
    // fits `words` words.
    std::vector<uint32_t> hn, hu, hc, hkey;
    if (wide) {
        // tab_n[d][k] = N(d,k), d = 0..D;  tab_u[d][k] = 2 (N(d,0) + ... + N(d,k)) mod 2^(32 words), d = 0..D-1
        hn.resize((size_t)(D + 1) * (K + 1) * words);
        hu.resize((size_t)D * (K + 1) * words);
        for (int d = 0; d <= D; d++) {
            U512 run;
            for (int k = 0; k <= K; k++) {
                const U512 &v = t.at(d, k);
                run.add(v);
                U512 twice = run;
                twice.add(run);
                for (int w = 0; w < words; w++) {
                    hn[((size_t)d * (K + 1) + k) * words + w] = v.word(w);
                    if (d < D) hu[((size_t)d * (K + 1) + k) * words + w] = twice.word(w);
                }
            }
        }
        hkey.resize((size_t)D * (K + 1));
        for (size_t i = 0; i < hkey.size(); i++) hkey[i] = pvq_wide_key(&hu[i * words], words);
        // The encoders' table: what a cell (d,k) of the walk adds to the index, in its four forms
        //   N,  -E,  N - E,  2N - E   (modulo 2^(32 words); E = 0 in row D, whose cell only ever adds N),
        // entry ((d (K+1) + k) 4 + form) of `words` words.
        hc.resize((size_t)(D + 1) * (K + 1) * 4 * words);
        for (int d = 0; d <= D; d++)
            for (int k = 0; k <= K; k++) {
                const uint32_t *n = &hn[((size_t)d * (K + 1) + k) * words];
                const uint32_t *ev = d < D ? &hu[((size_t)d * (K + 1) + k) * words] : nullptr;
                uint32_t *out = &hc[((size_t)d * (K + 1) + k) * 4 * words];
                for (int form = 0; form < 4; form++) {
                    const int times = form == 0 ? 1 : form - 1;          // how often N counts: 1, 0, 1, 2
                    uint64_t carry = 0;
                    int64_t borrow = 0;
                    for (int w = 0; w < words; w++) {
                        const uint64_t add = (uint64_t)n[w] * (uint64_t)times + carry;
                        carry = add >> 32;
                        const int64_t sub = (int64_t)(add & 0xFFFFFFFFu) - (form > 0 && ev ? (int64_t)ev[w] : 0) - borrow;
                        borrow = sub < 0 ? 1 : 0;
                        out[(size_t)form * words + w] = (uint32_t)sub;
                    }
                }
            }
    } else {
        hn.resize((size_t)D * (K + 1) * words);
        hu.resize((size_t)D * (K + 2) * words);
    }
    for (int dp = 0; dp < D && !wide; dp++) {
        U512 run;  // running sum
        for (int w = 0; w < words; w++) hu[((size_t)dp * (K + 2)) * words + w] = 0;
        for (int k = 0; k <= K; k++) {
            const U512 &v = t.at(dp, k);
            run.add(v);
            for (int w = 0; w < words; w++) {
                hn[((size_t)dp * (K + 1) + k) * words + w] = v.word(w);
                hu[((size_t)dp * (K + 2) + k + 1) * words + w] = run.word(w);
            }
        }
    }

    pvq_ctx *c = new (std::nothrow) pvq_ctx();
    if (!c) return PVQ_E_NOMEM;
    c->D = D; c->K = K; c->index_bits = bits; c->words = words; c->scale_bits = scale_bits; c->wide = wide ? 1 : 0;
    c->tab_n = c->tab_u = c->tab_c = c->tab_key = nullptr; c->edges = c->sqrtc = nullptr; c->fast8_blob = c->fast8g_blob = nullptr; c->enc8_offs = nullptr; c->amplitude = PVQ_AMP_NORM;
    c->tab_n_bytes = hn.size() * 4; c->tab_u_bytes = hu.size() * 4;

    hipError_t e = hipGetDevice(&c->device);
    if (e == hipSuccess) e = hipMalloc((void **)&c->tab_n, c->tab_n_bytes);
    if (e == hipSuccess) e = hipMalloc((void **)&c->tab_u, c->tab_u_bytes);
    if (e == hipSuccess) e = hipMemcpy(c->tab_n, hn.data(), c->tab_n_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->tab_u, hu.data(), c->tab_u_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess && !hc.empty()) {
        e = hipMalloc((void **)&c->tab_c, hc.size() * 4);
        if (e == hipSuccess) e = hipMemcpy(c->tab_c, hc.data(), hc.size() * 4, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMalloc((void **)&c->tab_key, hkey.size() * 4);
        if (e == hipSuccess) e = hipMemcpy(c->tab_key, hkey.data(), hkey.size() * 4, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && scale_bits) {
        // the edge table is padded to 2^b entries with +inf so that kernels may read a full table
        e32.push_back(INFINITY);
        e = hipMalloc((void **)&c->edges, sizeof(float) * n);
        if (e == hipSuccess) e = hipMalloc((void **)&c->sqrtc, sizeof(float) * n);
        if (e == hipSuccess) e = hipMemcpy(c->edges, e32.data(), sizeof(float) * n, hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMemcpy(c->sqrtc, sc32.data(), sizeof(float) * n, hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && D == 8 && words == 1) {
        std::vector<unsigned char> blob;
        if (pvq_fast8_build(K, kFast8MaxBytes, false, blob, c->fast8)) {
            e = pvq_fast8_prepare();
            if (e == hipSuccess) e = hipMalloc((void **)&c->fast8_blob, blob.size());
            if (e == hipSuccess) e = hipMemcpy(c->fast8_blob, blob.data(), blob.size(), hipMemcpyHostToDevice);
            if (e == hipSuccess && pvq_fast8_build(K, kFast8MaxBytes, true, blob, c->fast8g)) {
                e = hipMalloc((void **)&c->fast8g_blob, blob.size());
                if (e == hipSuccess) e = hipMemcpy(c->fast8g_blob, blob.data(), blob.size(), hipMemcpyHostToDevice);
            }
        }
    }
    if (e == hipSuccess && !wide) {
        std::vector<unsigned char> blob;
        // the decoders of pvq_walk.hip keep these in LDS: every supported (D, K) fits
        if (!build_walk_tables(t, D, K, words, blob, c->walk)) { pvq_ctx_destroy(c); return PVQ_E_UNSUPPORTED; }
        e = hipMalloc((void **)&c->walk_blob, blob.size());
        if (e == hipSuccess) e = hipMemcpy(c->walk_blob, blob.data(), blob.size(), hipMemcpyHostToDevice);
        if (e == hipSuccess && !pvq_walk_usable(c)) { pvq_ctx_destroy(c); return PVQ_E_UNSUPPORTED; }
    }
    if (e == hipSuccess && D == 8 && bits == 24) {
        // What coordinate i (7-i dimensions after it) adds to the index when k pulses are left and it
        // takes magnitude m with the given sign (App. B.2):
        //   N(7-i,k) [m>0] + 2 sum_{j=1}^{m-1} N(7-i,k-j) + [negative] N(7-i,k-m)
        const int K1 = K + 1;
        std::vector<uint32_t> offs((size_t)7 * K1 * K1 * 2, 0u);
        for (int i = 0; i < 7; i++)
            for (int k = 0; k <= K; k++)
                for (int m = 1; m <= k; m++) {
                    uint64_t v = t.at(7 - i, k).limb[0];
                    for (int j = 1; j < m; j++) v += 2 * t.at(7 - i, k - j).limb[0];
                    const size_t at = (((size_t)i * K1 + k) * K1 + m) * 2;
                    offs[at] = (uint32_t)v;
                    offs[at + 1] = (uint32_t)(v + t.at(7 - i, k - m).limb[0]);
                }
        e = hipMalloc((void **)&c->enc8_offs, offs.size() * 4);
        if (e == hipSuccess) e = hipMemcpy(c->enc8_offs, offs.data(), offs.size() * 4, hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        pvq_ctx_destroy(c);
        return hip_fail(e);
    }
    *out = c;
    return PVQ_OK;
}

extern "C" int pvq_ctx_destroy(pvq_ctx *c)
{
    if (!c) return PVQ_OK;
    hipError_t first = hipSuccess;
    void *ptrs[10] = {c->tab_key, c->tab_n, c->tab_u, c->tab_c, c->edges, c->sqrtc, c->fast8_blob, c->fast8g_blob, c->walk_blob, c->enc8_offs};
    for (void *p : ptrs) {
        if (!p) continue;
        hipError_t e = hipFree(p);
        if (first == hipSuccess) first = e;
    }
    delete c;
    return first == hipSuccess ? PVQ_OK : hip_fail(first);
}

extern "C" int pvq_ctx_info(const pvq_ctx *c, int *D, int *K, int *index_bits, int *scale_bits)
{
    if (!c) return PVQ_E_INVALID_ARG;
    if (D) *D = c->D;
    if (K) *K = c->K;
    if (index_bits) *index_bits = c->index_bits;
    if (scale_bits) *scale_bits = c->scale_bits;
    return PVQ_OK;
}

extern "C" int pvq_size_table_device(int D, int K, int words, uint32_t *table, uint32_t *overflow, void *stream)
{
    if (D < 0 || K < 0 || words < 1 || !table || !overflow) return PVQ_E_INVALID_ARG;
    if (D > 1024 || K > 1023 || words > 16) return PVQ_E_UNSUPPORTED;
    const hipError_t e = pvq_launch_size_table(D, K, words, table, overflow, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

extern "C" int pvq_hadamard(const void *X, int dtype, int64_t rows, int64_t cols, int64_t ldx, int block,
                            const uint8_t *signs, int inverse, void *Y, int out_dtype, int64_t ldy, void *stream)
{
    if (rows < 0 || cols < 0 || ldx < cols || ldy < cols) return PVQ_E_INVALID_ARG;
    if ((dtype != PVQ_F32 && dtype != PVQ_BF16) || (out_dtype != PVQ_F32 && out_dtype != PVQ_BF16))
        return PVQ_E_UNSUPPORTED;
    if (block < 8 || block > 8192 || (block & (block - 1)) || cols % block) return PVQ_E_UNSUPPORTED;
    if (rows == 0 || cols == 0) return PVQ_OK;
    if (!X || !Y) return PVQ_E_INVALID_ARG;
    const int64_t isz = dtype == PVQ_F32 ? 4 : 2, osz = out_dtype == PVQ_F32 ? 4 : 2;
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 15) || (ldx * isz) % 16 || (ldy * osz) % 16 || ((uintptr_t)signs & 7))
        return PVQ_E_ALIGNMENT;
    if (rows * ((cols + 511) / 512) > 0x7FFFFFFF) return PVQ_E_UNSUPPORTED;
    const hipError_t e = pvq_launch_hadamard(X, dtype, rows, cols, ldx, block, signs, inverse ? 1 : 0, Y, out_dtype,
                                             ldy, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

extern "C" int pvq_ctx_set_amplitude(pvq_ctx *c, int amplitude)
{
    if (!c || (amplitude != PVQ_AMP_NORM && amplitude != PVQ_AMP_LS)) return PVQ_E_INVALID_ARG;
    c->amplitude = amplitude;
    return PVQ_OK;
}

static int64_t stream_words(int64_t groups, int bits) { return (groups * bits + 31) / 32; }

static int check_shape(const pvq_ctx *c, int64_t rows, int64_t cols)
{
    if (!c || rows < 0 || cols < 0) return PVQ_E_INVALID_ARG;
    if (cols % c->D) return PVQ_E_UNSUPPORTED;
    // 32-bit bit offsets inside a row and 31-bit element counts per launch dimension
    if (cols > (int64_t)1 << 24 || rows > (int64_t)1 << 30) return PVQ_E_UNSUPPORTED;
    return PVQ_OK;
}

extern "C" int pvq_packed_sizes(const pvq_ctx *c, int64_t rows, int64_t cols, size_t *index_bytes,
                                size_t *scale_bytes, size_t *rownorm_bytes)
{
    int rc = check_shape(c, rows, cols);
    if (rc) return rc;
    int64_t G = cols / c->D;
    if (index_bytes) *index_bytes = (size_t)(rows * stream_words(G, c->index_bits) * 4);
    if (scale_bytes)
        *scale_bytes = (size_t)(c->scale_bits ? rows * stream_words(G, c->scale_bits) * 4 : rows * G * 4);
    if (rownorm_bytes) *rownorm_bytes = (size_t)(rows * 4);
    return PVQ_OK;
}

// ------------------------------------------------------------------------------------------
// the hot path: validation, then launch
// ------------------------------------------------------------------------------------------

static bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

static int check_device(const pvq_ctx *c)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    return dev == c->device ? PVQ_OK : PVQ_E_INVALID_ARG;
}

extern "C" int pvq_encode(const pvq_ctx *c, const void *W, int dtype, int64_t rows, int64_t cols,
                          int64_t ldw, uint32_t *index_out, void *scale_out, float *rownorm_out,
                          int8_t *pulses_out, void *stream)
{
    int rc = check_shape(c, rows, cols);
    if (rc) return rc;
    if (dtype != PVQ_F32 && dtype != PVQ_BF16) return PVQ_E_INVALID_ARG;
    if (rows == 0 || cols == 0) return PVQ_OK;
    if (!W || !index_out || !scale_out || ldw < cols) return PVQ_E_INVALID_ARG;
    if (c->scale_bits > 0 && !rownorm_out) return PVQ_E_INVALID_ARG;
    size_t esz = dtype == PVQ_F32 ? 4 : 2;
    if (!aligned(W, 16) || (ldw * esz) % 16 || !aligned(index_out, 4) || !aligned(scale_out, 4) ||
        (rownorm_out && !aligned(rownorm_out, 4)) || (pulses_out && !aligned(pulses_out, 16)))
        return PVQ_E_ALIGNMENT;
    if ((rc = check_device(c))) return rc;

    pvq_encode_args a;
    a.ls_amplitude = c->amplitude == PVQ_AMP_LS ? 1 : 0;
    a.W = W; a.rows = rows; a.cols = cols; a.ldw = ldw; a.groups = cols / c->D;
    a.index_out = index_out; a.scale_out = scale_out; a.rownorm_out = rownorm_out;
    a.pulses_out = pulses_out;
    a.index_row_words = stream_words(a.groups, c->index_bits);
    a.scale_row_words = c->scale_bits ? stream_words(a.groups, c->scale_bits) : 0;
    if (c->wide && pulses_out && c->K > 127) return PVQ_E_UNSUPPORTED;   // int8 cannot hold such pulses
    if (!c->wide && !pvq_encode8_usable(c, a) && !pvq_encode_fits(c, a)) return PVQ_E_UNSUPPORTED;   // rows too long for LDS
    hipError_t e = c->wide ? pvq_wide_launch_encode(c, a, dtype, (hipStream_t)stream)
                   : pvq_encode8_usable(c, a) ? pvq_encode8_launch(c, a, dtype, (hipStream_t)stream)
                                              : pvq_launch_encode(c, a, dtype, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

extern "C" int pvq_rotate_encode(const pvq_ctx *c, const void *X, int dtype, int64_t rows, int64_t cols,
                                 int64_t ldx, int block, const uint8_t *signs, uint32_t *index_out,
                                 void *scale_out, float *rownorm_out, void *stream)
{
    int rc = check_shape(c, rows, cols);
    if (rc) return rc;
    if (dtype != PVQ_F32 && dtype != PVQ_BF16) return PVQ_E_INVALID_ARG;
    const bool long_groups = c->wide && c->D == 128 && c->words <= 12;
    const bool groups_of_8 = !c->wide && c->D == 8 && c->index_bits == 24;
    if (!long_groups && !groups_of_8) return PVQ_E_UNSUPPORTED;
    if (block < (long_groups ? 128 : 8) || block > 8192 || (block & (block - 1)) || cols % block) return PVQ_E_UNSUPPORTED;
    const int lanes = std::min(1024, std::max(256, block / 8));   // of a workgroup: whole blocks of the rotation
    if (long_groups) {
        // a workgroup's groups must fill whole words of the index plane
        if (((int64_t)(lanes / 16) * c->index_bits) % 32) return PVQ_E_UNSUPPORTED;
    }
    pvq_encode_args a;
    a.ls_amplitude = c->amplitude == PVQ_AMP_LS ? 1 : 0;
    a.W = X; a.rows = rows; a.cols = cols; a.ldw = ldx; a.groups = cols / c->D;
    a.index_out = index_out; a.scale_out = scale_out; a.rownorm_out = rownorm_out; a.pulses_out = nullptr;
    a.index_row_words = stream_words(a.groups, c->index_bits);
    a.scale_row_words = c->scale_bits ? stream_words(a.groups, c->scale_bits) : 0;
    // groups of 8: rows of whole chunks of `lanes` groups, at most 4096 groups
    if (groups_of_8 && cols > 0 && !pvq_rotate_encode8_usable(c, a, block)) return PVQ_E_UNSUPPORTED;
    if (rows == 0 || cols == 0) return PVQ_OK;
    if (!X || !index_out || !scale_out || ldx < cols) return PVQ_E_INVALID_ARG;
    if (c->scale_bits > 0 && !rownorm_out) return PVQ_E_INVALID_ARG;
    const size_t esz = dtype == PVQ_F32 ? 4 : 2;
    if (!aligned(X, 16) || (ldx * esz) % 16 || !aligned(index_out, 4) || !aligned(scale_out, 4) || !aligned(signs, 8) ||
        (rownorm_out && !aligned(rownorm_out, 4)))
        return PVQ_E_ALIGNMENT;
    if ((rc = check_device(c))) return rc;
    const hipError_t e = long_groups ? pvq_wide_launch_rotate_encode(c, a, dtype, block, signs, (hipStream_t)stream)
                                     : pvq_rotate_encode8_launch(c, a, dtype, block, signs, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

extern "C" int pvq_correct_work_bytes(int64_t rows, size_t *bytes)
{
    if (rows < 0 || rows > (int64_t)1 << 30 || !bytes) return PVQ_E_INVALID_ARG;
    *bytes = (size_t)rows * 256 * sizeof(float);   // two buffers of 128 t values per row, used in turn
    return PVQ_OK;
}

// what pvq_correct and pvq_correct_static check alike; *nothing_to_do for an empty matrix
static int check_correct_args(const pvq_ctx *c, const float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                              int64_t ldu, bool *nothing_to_do)
{
    *nothing_to_do = false;
    int rc = check_shape(c, rows, cols);
    if (rc) return rc;
    // (column tiles of 128 are the second grid dimension of the update kernel: at most 65535 of them)
    if (c->wide || (c->D != 8 && c->D != 16 && c->D != 32) || cols % 64 || cols > (int64_t)1 << 22) return PVQ_E_UNSUPPORTED;
    if (rows == 0 || cols == 0) { *nothing_to_do = true; return PVQ_OK; }
    if (!W || !U || ldw < cols || ldu < cols) return PVQ_E_INVALID_ARG;
    if (!aligned(W, 16) || ldw % 4 || !aligned(U, 16) || ldu % 4) return PVQ_E_ALIGNMENT;
    return PVQ_OK;
}

extern "C" int pvq_correct(const pvq_ctx *c, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                           int64_t ldu, void *work, size_t work_bytes, void *stream)
{
    bool empty;
    int rc = check_correct_args(c, W, rows, cols, ldw, U, ldu, &empty);
    if (rc || empty) return rc;
    if (!work || work_bytes < (size_t)rows * 256 * sizeof(float)) return PVQ_E_INVALID_ARG;
    if (!aligned(work, 16)) return PVQ_E_ALIGNMENT;
    if ((rc = check_device(c))) return rc;
    const hipError_t e = pvq_launch_correct(c, W, rows, cols, ldw, U, ldu, (float *)work, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

extern "C" int pvq_correct_set_front_tiles(int64_t tiles, int64_t *previous)
{
    if (tiles < 0) return PVQ_E_INVALID_ARG;
    const int64_t old = pvq_correct_front_tiles(tiles);
    if (previous) *previous = old;
    return PVQ_OK;
}

extern "C" int pvq_correct_static_max_rows(int64_t *rows)
{
    if (!rows) return PVQ_E_INVALID_ARG;
    *rows = pvq_correct_static_max_rows();
    return PVQ_OK;
}

extern "C" int pvq_correct_static(const pvq_ctx *c, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                                  int64_t ldu, void *stream)
{
    bool empty;
    int rc = check_correct_args(c, W, rows, cols, ldw, U, ldu, &empty);
    if (rc || empty) return rc;
    if (rows > pvq_correct_static_max_rows()) return PVQ_E_UNSUPPORTED;   // more rows than the static buffer holds
    if ((rc = check_device(c))) return rc;
    const hipError_t e = pvq_launch_correct_static(c, W, rows, cols, ldw, U, ldu, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

static int fill_decode_args(const pvq_ctx *c, pvq_decode_args &a, const uint32_t *index,
                            const void *scale, const float *rownorm, int64_t rows, int64_t cols)
{
    if (!index || !scale) return PVQ_E_INVALID_ARG;
    if (c->scale_bits > 0 && !rownorm) return PVQ_E_INVALID_ARG;
    if (!aligned(index, 4) || !aligned(scale, 4) || (rownorm && !aligned(rownorm, 4))) return PVQ_E_ALIGNMENT;
    memset(&a, 0, sizeof a);
    a.index = index; a.scale = scale; a.rownorm = rownorm;
    a.rows = rows; a.cols = cols; a.groups = cols / c->D;
    a.index_row_words = stream_words(a.groups, c->index_bits);
    a.scale_row_words = c->scale_bits ? stream_words(a.groups, c->scale_bits) : 0;
    return PVQ_OK;
}

// The table decoder for groups of 8 copies 155 KB of tables into every unit's LDS before its first group (about
// 13 us a launch); the coordinate-by-coordinate decoder starts with 3 KB.  Measured to bf16: 1024 x 8192 (1.0 M
// groups) 22.2 against 17.8 us, 512 x 512 27 against 14 us, 2048 x 8192 (2.1 M groups) 24.1 against 25.4 us.
static std::atomic<int64_t> g_table_decoder_min_groups{1572864};

static bool table_decoder_pays(const pvq_ctx *c, const pvq_decode_args &a)
{
    return pvq_fast8_decode_usable(c, a) && a.rows * a.groups >= g_table_decoder_min_groups.load(std::memory_order_relaxed);
}

extern "C" int pvq_decode_set_table_decoder_min_groups(int64_t groups, int64_t *previous)
{
    if (groups < 0) return PVQ_E_INVALID_ARG;
    const int64_t old = g_table_decoder_min_groups.exchange(groups);
    if (previous) *previous = old;
    return PVQ_OK;
}

extern "C" int pvq_decode(const pvq_ctx *c, const uint32_t *index, const void *scale,
                          const float *rownorm, int64_t rows, int64_t cols, void *W_out,
                          int out_dtype, int64_t ldw, void *stream)
{
    int rc = check_shape(c, rows, cols);
    if (rc) return rc;
    if (out_dtype != PVQ_F32 && out_dtype != PVQ_F16 && out_dtype != PVQ_BF16) return PVQ_E_INVALID_ARG;
    if (rows == 0 || cols == 0) return PVQ_OK;
    if (!W_out || ldw < cols) return PVQ_E_INVALID_ARG;
    size_t esz = out_dtype == PVQ_F32 ? 4 : 2;
    if (!aligned(W_out, 16) || (ldw * esz) % 16) return PVQ_E_ALIGNMENT;
    pvq_decode_args a;
    if ((rc = fill_decode_args(c, a, index, scale, rownorm, rows, cols))) return rc;
    if ((rc = check_device(c))) return rc;
    a.W_out = W_out; a.ldw = ldw;
    hipError_t e = c->wide ? pvq_wide_launch_decode(c, a, out_dtype, (hipStream_t)stream)
                   : table_decoder_pays(c, a) ? pvq_fast8_launch_decode(c, a, out_dtype, (hipStream_t)stream)
                                              : pvq_walk_launch_decode(c, a, out_dtype, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

extern "C" int pvq_decode_gemv(const pvq_ctx *c, const uint32_t *index, const void *scale,
                               const float *rownorm, int64_t rows, int64_t cols, const void *x,
                               int batch, int64_t ldx, float *y, int64_t ldy, void *stream)
{
    int rc = check_shape(c, rows, cols);
    if (rc) return rc;
    if (batch < 0) return PVQ_E_INVALID_ARG;
    if (batch > 16 || (c && c->wide)) return PVQ_E_UNSUPPORTED;
    if (rows == 0 || batch == 0) return PVQ_OK;
    if (!y || ldy < rows) return PVQ_E_INVALID_ARG;
    if (!aligned(y, 4)) return PVQ_E_ALIGNMENT;
    pvq_decode_args a;
    if (cols == 0) {
        // an empty sum: y = 0
        hipError_t e = hipSuccess;
        for (int b = 0; b < batch && e == hipSuccess; b++)
            e = pvq_launch_fill_zero(y + (int64_t)b * ldy, rows, (hipStream_t)stream);
        return e == hipSuccess ? PVQ_OK : hip_fail(e);
    }
    if (!x || ldx < cols) return PVQ_E_INVALID_ARG;
    if (!aligned(x, 16) || ldx % 8) return PVQ_E_ALIGNMENT;
    if ((rc = fill_decode_args(c, a, index, scale, rownorm, rows, cols))) return rc;
    if ((rc = check_device(c))) return rc;
    a.x = x; a.batch = batch; a.ldx = ldx; a.y = y; a.ldy = ldy;
    hipError_t e = pvq_fast8_gemv_usable(c, a) ? pvq_fast8_launch_gemv(c, a, (hipStream_t)stream)
                                               : pvq_walk_launch_gemv(c, a, (hipStream_t)stream);
    return e == hipSuccess ? PVQ_OK : hip_fail(e);
}

extern "C" int pvq_decode_gemv_plan(const pvq_ctx *c, int64_t rows, int64_t cols, int batch, int *kinds, int *nvecs,
                                    int max_passes, int *passes)
{
    int rc = check_shape(c, rows, cols);
    if (rc) return rc;
    if (!kinds || !nvecs || !passes || batch < 1 || batch > 16 || max_passes < 1) return PVQ_E_INVALID_ARG;
    if (c->wide) return PVQ_E_UNSUPPORTED;
    pvq_decode_args a;
    memset(&a, 0, sizeof a);
    a.rows = rows; a.cols = cols; a.groups = cols / c->D; a.batch = batch;
    pvq_gemv_pass plan[16];
    int n = 1;
    plan[0] = {PVQ_PASS_GENERIC, batch};
    if (pvq_fast8_gemv_usable(c, a)) n = pvq_fast8_plan_gemv(c, a, plan);
    if (n > max_passes) return PVQ_E_INVALID_ARG;
    for (int i = 0; i < n; i++) { kinds[i] = plan[i].kind; nvecs[i] = plan[i].nvec; }
    *passes = n;
    return PVQ_OK;
}

// ------------------------------------------------------------------------------------------
// host replay of the coordinate-by-coordinate decoder's tables
// ------------------------------------------------------------------------------------------

namespace {

typedef unsigned __int128 u128;

u128 low128(const U512 &v) { return ((u128)v.limb[1] << 64) | v.limb[0]; }

// App. B.3 as printed (with the corrections of the boundary's decode contract), in 128-bit integers
void plain_unrank(const SizeTable &t, int D, int K, u128 c, int *y)
{
    int k = K;
    u128 r = c;
    for (int i = 0; i < D - 1; i++) {
        const int dp = D - 1 - i;
        y[i] = 0;
        if (k == 0) continue;
        if (r < low128(t.at(dp, k))) continue;
        r -= low128(t.at(dp, k));
        int j = 1;
        while (j < k && r >= 2 * low128(t.at(dp, k - j))) { r -= 2 * low128(t.at(dp, k - j)); j++; }
        if (r < low128(t.at(dp, k - j))) y[i] = j; else { y[i] = -j; r -= low128(t.at(dp, k - j)); }
        k -= j;
    }
    y[D - 1] = r == 0 ? k : -k;
}

template <int D, int W, int DA, int DB>
uint64_t replay_walk(const SizeTable &t, int K, const std::vector<unsigned char> &blob, const pvq_walk_params &p,
                     uint64_t seed, uint64_t count)
{
    using T = typename pvq_walk::wide<W>::type;
    const u128 total = low128(t.at(D, K));
    uint64_t bad = 0, state = seed;
    auto next64 = [&]() {   // splitmix64
        uint64_t z = (state += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    };
    for (uint64_t n = 0; n < count; n++) {
        u128 c;
        if (n < 4) c = n == 0 ? 0 : n == 1 ? total - 1 : n == 2 ? total / 2 : total / 3;   // ends and middles first
        else {
            c = (((u128)next64() << 64) | next64()) % total;
            // a third of the samples near the start of the range, where long runs of equal coordinates lie
            if (n % 3 == 0) c >>= (next64() % 100);
        }
        int want[D], got[D];
        plain_unrank(t, D, K, c, want);
        int n2w = 0;
        for (int i = 0; i < D; i++) n2w += want[i] * want[i];
        const int n2 = pvq_walk::unrank_walk<D, W, DA, DB>((T)c, blob.data(), p, [&](int i, uint32_t m, bool negative) { got[i] = negative ? -(int)m : (int)m; });
        bool same = n2 == n2w;
        for (int i = 0; i < D; i++) same = same && got[i] == want[i];
        bad += !same;
    }
    return bad;
}

}  // namespace

extern "C" int pvq_walk_tables_selftest(int D, int K, uint64_t seed, uint64_t count, uint64_t *mismatches,
                                        int *schedule, uint32_t *table_bytes)
{
    if (!mismatches) return PVQ_E_INVALID_ARG;
    if ((D != 8 && D != 16 && D != 32) || K < 1 || K > 127) return PVQ_E_UNSUPPORTED;
    SizeTable t(D, K);
    if (t.overflow) return PVQ_E_UNSUPPORTED;
    const int bits = t.index_bits();
    if (bits < 1 || bits > 128 || t.at(D, K).bit_length() > 128) return PVQ_E_UNSUPPORTED;
    const int words = bits <= 32 ? 1 : (bits <= 64 ? 2 : 4);
    if (t.at(D, K).bit_length() > 32 * words) return PVQ_E_UNSUPPORTED;
    std::vector<unsigned char> blob;
    pvq_walk_params p;
    if (!build_walk_tables(t, D, K, words, blob, p)) return PVQ_E_UNSUPPORTED;
    if (schedule) { schedule[0] = p.dA; schedule[1] = p.dB; }
    if (table_bytes) *table_bytes = p.bytes;
#define PVQ_WALK_REPLAY(D_, W_, DA_, DB_) (*mismatches = replay_walk<D_, W_, DA_, DB_>(t, K, blob, p, seed, count), PVQ_OK)
    PVQ_WALK_DISPATCH(PVQ_WALK_REPLAY, D, words, p.dA, p.dB);
#undef PVQ_WALK_REPLAY
}
