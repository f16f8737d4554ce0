// Runs the host-only part of libpvq (pvq_host.cpp, pvq_fast8_tables.cpp: exact size tables, K from a budget,
// Beta quantiles, the decoders' table builders and their host replays; none of it needs a GPU) compiled into
// this program with AddressSanitizer and UndefinedBehaviorSanitizer.  The kernels' launch functions are
// stubs that abort: nothing here may reach them.  Exit status 0 = no sanitizer report and all checks held.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "pvq.h"
#include "pvq_diagnostics.h"
#include "pvq_internal.h"   // pvq_wide_key

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); exit(1); } } while (0)

int main()
{
    uint32_t words[16];
    int bits = 0, K = 0;
    CHECK(pvq_count(8, 16, words, &bits) == PVQ_OK && words[0] == 15158272u && bits == 24);
    CHECK(pvq_count(128, 187, words, &bits) == PVQ_OK && bits == 384);
    CHECK(pvq_count(256, 1024, words, &bits) == PVQ_E_UNSUPPORTED);
    CHECK(pvq_count(0, 3, words, &bits) == PVQ_E_INVALID_ARG);
    CHECK(pvq_max_k(8, 24, &K) == PVQ_OK && K == 16);
    CHECK(pvq_max_k(16, 52, &K) == PVQ_OK && K == 33);
    CHECK(pvq_max_k(32, 104, &K) == PVQ_OK && K == 60);
    CHECK(pvq_max_k(128, 384, &K) == PVQ_OK && K == 187);
    CHECK(pvq_max_k(8, 3, &K) == PVQ_E_UNSUPPORTED);
    for (int sb : {1, 2, 4, 8}) {
        std::vector<double> edges((1 << sb) - 1 + 1), centers(1 << sb);
        CHECK(pvq_beta_tables(8, 1024, sb, edges.data(), centers.data()) == PVQ_OK);
        for (int j = 1; j + 1 < (1 << sb); j++) CHECK(edges[j] > edges[j - 1]);
        CHECK(pvq_beta_tables(16, 256, sb, edges.data(), centers.data()) == PVQ_OK);
    }
    CHECK(pvq_beta_tables(7, 16, 2, nullptr, nullptr) != PVQ_OK);
    uint64_t bad = 1;
    for (int k : {1, 2, 5, 9}) { CHECK(pvq_fast_tables_selftest(k, 0, 1ull << 40, &bad) == PVQ_OK && bad == 0); }
    CHECK(pvq_fast_tables_selftest(16, 0, 300000, &bad) == PVQ_OK && bad == 0);            // a stretch of the 24-bit setting
    CHECK(pvq_fast_tables_selftest(16, 15158272 - 300000, 300000, &bad) == PVQ_OK && bad == 0);
    CHECK(pvq_fast_tables_selftest(40, 0, 10, &bad) == PVQ_E_UNSUPPORTED);
    int sched[2];
    uint32_t nbytes = 0;
    for (auto dk : {std::pair<int, int>{16, 33}, {32, 60}, {8, 40}, {32, 9}, {16, 60}, {32, 100}, {8, 1}}) {
        CHECK(pvq_walk_tables_selftest(dk.first, dk.second, 7, 20000, &bad, sched, &nbytes) == PVQ_OK && bad == 0 && nbytes > 0);
    }
    CHECK(pvq_walk_tables_selftest(64, 10, 7, 10, &bad, sched, &nbytes) == PVQ_E_UNSUPPORTED);
    // the long-group decoder's search keys: keys that differ order the integers as the integers themselves do
    {
        uint64_t state = 12345;
        auto next = [&]() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(state >> 32); };
        auto less = [](const uint32_t *a, const uint32_t *b, int n) {
            for (int i = n - 1; i >= 0; i--) if (a[i] != b[i]) return a[i] < b[i];
            return false;
        };
        for (int trial = 0; trial < 200000; trial++) {
            const int n = 4 * (1 + (int)(next() % 4));
            uint32_t a[16] = {0}, b[16] = {0};
            const int top = (int)(next() % (uint32_t)n);                 // highest word that may be set
            for (int i = 0; i <= top; i++) { a[i] = next(); b[i] = next(); }
            const uint32_t kind = next() % 4;
            if (kind == 0) for (int i = top; i >= 0 && i > top - 2; i--) b[i] = a[i];    // agree in the leading words
            if (kind == 1) { a[top] >>= next() % 32; b[top] >>= next() % 32; }                // any bit length
            if (kind == 2) { for (int i = 0; i <= top; i++) b[i] = a[i]; b[0] ^= 1u; }      // neighbours
            const uint32_t ka = pvq_wide_key(a, n), kb = pvq_wide_key(b, n);
            if (ka < kb) CHECK(less(a, b, n));
            if (ka > kb) CHECK(less(b, a, n));
        }
        const uint32_t zero[4] = {0, 0, 0, 0}, one[4] = {1, 0, 0, 0}, big[4] = {0, 0, 0, 0x80000000u};
        CHECK(pvq_wide_key(zero, 4) == 0 && pvq_wide_key(one, 4) == ((1u << 22) | (1u << 21)));
        CHECK(pvq_wide_key(big, 4) == ((128u << 22) | (1u << 21)));
    }
    // argument checks that return before any device call
    pvq_ctx *ctx = nullptr;
    CHECK(pvq_ctx_create(&ctx, 7, 16, 0, nullptr, nullptr) == PVQ_E_UNSUPPORTED && ctx == nullptr);
    CHECK(pvq_ctx_create(&ctx, 8, 0, 0, nullptr, nullptr) == PVQ_E_UNSUPPORTED);
    CHECK(pvq_ctx_create(&ctx, 8, 16, 2, nullptr, nullptr) == PVQ_E_INVALID_ARG);
    CHECK(pvq_ctx_create(nullptr, 8, 16, 0, nullptr, nullptr) == PVQ_E_INVALID_ARG);
    CHECK(pvq_ctx_destroy(nullptr) == PVQ_OK);
    size_t n = 0;
    CHECK(pvq_correct_work_bytes(1000, &n) == PVQ_OK && n == 1000u * 256 * 4);
    CHECK(pvq_strerror(PVQ_E_UNSUPPORTED) != nullptr);
    puts("host: ok");
    return 0;
}
