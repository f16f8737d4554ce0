// Host construction of the tables used by the D = 8 table-driven decoder (see pvq_fast8.h), and a
// host self-test that replays the device walk over a range of indices.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "pvq.h"
#include "pvq_diagnostics.h"
#include "pvq_fast8.h"
#include "pvq_small_table.h"

namespace {

using namespace pvq_small;

struct Block {
    uint64_t start, size;
    uint32_t values, n2x4;
    int next_k;
};

// Bucket row over one row of blocks: entry j describes indices [j << shift, (j+1) << shift).
template <typename E>
void build_bucket_row(const std::vector<Block> &blocks, uint32_t first_index, uint64_t total, int shift,
                      int thr_bits, int db_bits, std::vector<E> &out)
{
    const uint64_t width = (uint64_t)1 << shift;
    const uint64_t nb = (total + width - 1) / width;
    size_t a = 0;
    for (uint64_t j = 0; j < nb; j++) {
        const uint64_t lo = j * width, hi = lo + width;
        while (a + 1 < blocks.size() && blocks[a + 1].start <= lo) a++;
        uint32_t db = 0, thr = 0;
        uint64_t best = 0;
        for (size_t b = a + 1; b < blocks.size() && blocks[b].start < hi && b - a < ((size_t)1 << db_bits); b++) {
            const uint64_t cover = std::min(hi, blocks[b].start + blocks[b].size) - blocks[b].start;
            if (cover > best) { best = cover; db = (uint32_t)(b - a); thr = (uint32_t)(blocks[b].start - lo); }
        }
        out.push_back((E)(thr | (db << thr_bits) | ((first_index + (uint32_t)a) << (thr_bits + db_bits))));
    }
}

// Bucket row in the next-block form: (index of A - bucket number) << shift, plus 2^shift minus the
// start of the block after A inside the bucket (nothing if it starts beyond the bucket).  The bucket
// number counts over all rows of the stage, as the biased residuals do (see write_blocks).
template <typename E>
void build_next_bucket_row(const std::vector<Block> &blocks, uint32_t first_index, uint64_t total, int shift,
                           std::vector<E> &out)
{
    const uint64_t row_bucket = out.size();   // the row's first bucket, counted over the whole stage
    const uint64_t width = (uint64_t)1 << shift;
    const uint64_t nb = (total + width - 1) / width;
    size_t a = 0;
    for (uint64_t j = 0; j < nb; j++) {
        const uint64_t lo = j * width, hi = lo + width;
        while (a + 1 < blocks.size() && blocks[a + 1].start <= lo) a++;
        uint64_t low = 0;
        if (a + 1 < blocks.size() && blocks[a + 1].start < hi) low = width - (blocks[a + 1].start - lo);
        const uint64_t high = (uint64_t)first_index + a - (row_bucket + j);   // modulo the entry width
        out.push_back((E)((high << shift) + low));
    }
}

void align16(std::vector<unsigned char> &blob) { blob.resize((blob.size() + 15) & ~(size_t)15); }

template <typename T>
uint32_t append(std::vector<unsigned char> &blob, const std::vector<T> &v)
{
    align16(blob);
    const uint32_t off = (uint32_t)blob.size();
    blob.resize(off + v.size() * sizeof(T));
    if (!v.empty()) memcpy(blob.data() + off, v.data(), v.size() * sizeof(T));
    return off;
}

bool build_with_shifts(int K, const SmallTable &N, int s0, int s1, int s2, uint32_t max_bytes, bool s0_outside,
                       std::vector<unsigned char> &blob, pvq_fast8_params &p)
{
    // ---- block lists --------------------------------------------------------------------
    auto pair_blocks = [&](int rest_dims, int k) {
        std::vector<Block> v;
        uint64_t start = 0;
        for (int a : visiting_order(k))
            for (int b : visiting_order(k - abs(a))) {
                const int m = abs(a) + abs(b);
                Block blk{start, N.at(rest_dims, k - m), bf16_of_int(a) | (bf16_of_int(b) << 16),
                          (uint32_t)(4 * (a * a + b * b)), k - m};
                v.push_back(blk);
                start += blk.size;
            }
        return v;
    };
    auto single_blocks = [&](int rest_dims, int k) {
        std::vector<Block> v;
        uint64_t start = 0;
        for (int a : visiting_order(k)) {
            Block blk{start, N.at(rest_dims, k - abs(a)), bf16_of_int(a), (uint32_t)(4 * a * a), k - abs(a)};
            v.push_back(blk);
            start += blk.size;
        }
        return v;
    };

    std::vector<std::vector<Block>> rows0{pair_blocks(6, K)}, rows1, rows2;
    for (int k = 0; k <= K; k++) { rows1.push_back(pair_blocks(4, k)); rows2.push_back(single_blocks(3, k)); }

    // ---- T3: every (k, r) of the last three coordinates ---------------------------------------
    std::vector<uint32_t> t3;  // two words per entry
    std::vector<uint32_t> t3_row(K + 1);
    for (int k = 0; k <= K; k++) {
        t3_row[k] = (uint32_t)t3.size() * 4;
        for (int a : visiting_order(k))
            for (int b : visiting_order(k - abs(a))) {
                const int rem = k - abs(a) - abs(b);
                for (int sgn = 0; sgn < (rem ? 2 : 1); sgn++) {
                    const int c = sgn ? -rem : rem;
                    t3.push_back((bf16_of_int(a) << 16) | (uint32_t)(4 * (a * a + b * b + c * c)));
                    t3.push_back(bf16_of_int(b) | (bf16_of_int(c) << 16));
                }
            }
        if ((t3.size() * 4 - t3_row[k]) / 8 != N.at(3, k)) return false;
    }

    // ---- bucket rows --------------------------------------------------------------------------
    std::vector<uint32_t> bk0, bk1;
    std::vector<uint16_t> bk2;
    std::vector<uint32_t> bk1_row(K + 1), bk2_row(K + 1);
    // S0's blocks read from LDS: next-block entries (a step to the following block is cheap there);
    // read through the vector cache: two-candidate entries, which need such steps five times less often
    if (!s0_outside) build_next_bucket_row<uint32_t>(rows0[0], 0, N.at(8, K), s0, bk0);
    else build_bucket_row<uint32_t>(rows0[0], 0, N.at(8, K), s0, kFast8ThrBits, kFast8DbBits, bk0);
    uint32_t first = 0;
    for (int k = 0; k <= K; k++) {
        bk1_row[k] = (uint32_t)bk1.size() * 4;
        build_bucket_row<uint32_t>(rows1[k], first, N.at(6, k), s1, kFast8ThrBits, kFast8DbBits, bk1);
        first += (uint32_t)rows1[k].size();
    }
    first = 0;
    for (int k = 0; k <= K; k++) {
        bk2_row[k] = (uint32_t)bk2.size() * 2;
        build_next_bucket_row<uint16_t>(rows2[k], first, N.at(4, k), s2, bk2);
        first += (uint32_t)rows2[k].size();
    }
    if (first >= (1u << (16 - s2))) return false;   // S2's block numbers must fit the 16-bit entries

    // ---- lay the blob out ---------------------------------------------------------------------
    // sizes are known now; offsets of the rows that `meta` words point to must be fixed before the
    // block tables are written
    auto up16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
    size_t off = 0;
    const size_t o_bk0 = off; off = up16(off + bk0.size() * 4);
    const size_t o_bk1 = off; off = up16(off + bk1.size() * 4);
    const size_t o_bk2 = off; off = up16(off + bk2.size() * 2);
    const size_t o_t3 = off;  off = up16(off + t3.size() * 4);
    size_t nblk0 = rows0[0].size(), nblk1 = 0, nblk2 = 0;
    for (auto &r : rows1) nblk1 += r.size();
    for (auto &r : rows2) nblk2 += r.size();
    size_t o_bl0 = 0;
    if (!s0_outside) { o_bl0 = off; off = up16(off + nblk0 * 16); }
    const size_t o_bl1 = off; off = up16(off + nblk1 * 16);
    const size_t o_bl2 = off; off = up16(off + nblk2 * 16);
    // 1/sqrt(n2) comes last of what goes to LDS: a kernel that builds its own gain table leaves it out
    const size_t lds_bytes = off;
    const size_t o_invs = off; off = up16(off + (size_t)(K * K + 1) * 4);
    const size_t tab_bytes = off;
    if (s0_outside) { o_bl0 = off; off = up16(off + nblk0 * 16); }
    if (tab_bytes > max_bytes || off >= ((size_t)1 << 18)) return false;

    // Residuals travel biased: inside stage S a residual r of row k is kept as r + (first bucket of
    // row k, counted over the stage) << shift_S, so that r >> shift_S is the bucket's place in the
    // stage's whole bucket table and no row offset has to be carried or added.  A block entry's
    // `start` therefore holds start + this row's bias - the next stage's row bias, and `end` holds
    // end + this row's bias.  For T3 the bias is the row's first entry (shift 0).
    auto write_blocks = [&](const std::vector<std::vector<Block>> &rows, auto row_bias, auto next_bias) {
        std::vector<pvq_fast8_block> v;
        for (size_t k = 0; k < rows.size(); k++) {
            const auto &row = rows[k];
            // S0 has a single row, reached with k = K pulses and no bias
            const uint32_t bias = row_bias((int)k);
            for (size_t i = 0; i < row.size(); i++) {
                pvq_fast8_block e;
                e.start = (uint32_t)row[i].start + bias - next_bias(row[i].next_k);
                e.end = i + 1 < row.size() ? (uint32_t)(row[i].start + row[i].size) + bias : 0xFFFFFFFFu;
                e.values = row[i].values;
                e.meta = row[i].n2x4;
                v.push_back(e);
            }
        }
        return v;
    };
    auto bias1 = [&](int k) { return (bk1_row[k] / 4u) << s1; };
    auto bias2 = [&](int k) { return (bk2_row[k] / 2u) << s2; };
    auto bias3 = [&](int k) { return t3_row[k] / 8u; };
    const auto bl0 = write_blocks(rows0, [&](int) { return 0u; }, bias1);
    const auto bl1 = write_blocks(rows1, bias1, bias2);
    const auto bl2 = write_blocks(rows2, bias2, bias3);
    std::vector<float> invs((size_t)K * K + 1);
    invs[0] = 0.0f;
    for (int n2 = 1; n2 <= K * K; n2++) invs[n2] = (float)(1.0 / std::sqrt((double)n2));

    blob.clear();
    bool ok = append(blob, bk0) == o_bk0 && append(blob, bk1) == o_bk1 && append(blob, bk2) == o_bk2 &&
              append(blob, t3) == o_t3;
    if (!s0_outside) ok = ok && append(blob, bl0) == o_bl0;
    ok = ok && append(blob, bl1) == o_bl1 && append(blob, bl2) == o_bl2 && append(blob, invs) == o_invs;
    if (s0_outside) ok = ok && append(blob, bl0) == o_bl0;
    align16(blob);
    if (!ok || blob.size() != off) return false;

    p.blob_bytes = (uint32_t)blob.size();
    p.lds_bytes = (uint32_t)lds_bytes;
    p.tab_bytes = (uint32_t)tab_bytes;
    p.s0_outside = s0_outside ? 1u : 0u;
    p.n_minus_1 = (uint32_t)(N.at(8, K) - 1);
    p.bk0 = (uint32_t)o_bk0; p.bk1 = (uint32_t)o_bk1; p.bk2 = (uint32_t)o_bk2; p.t3 = (uint32_t)o_t3;
    p.bl0 = (uint32_t)o_bl0; p.bl1 = (uint32_t)o_bl1; p.bl2 = (uint32_t)o_bl2;
    p.invs = (uint32_t)o_invs;
    p.s0 = s0; p.s1 = s1; p.s2 = s2;
    p.k2max = (uint32_t)(K * K);
    return true;
}

}  // namespace

bool pvq_fast8_build(int K, uint32_t max_bytes, bool s0_outside, std::vector<unsigned char> &blob,
                     pvq_fast8_params &p)
{
    if (K < 1 || K > 22) return false;  // 4*K*K must stay below 2^11
    SmallTable N(K);
    if (N.at(8, K) > ((uint64_t)1 << 32)) return false;
    int bits = 0;
    while (((uint64_t)1 << bits) < N.at(8, K)) bits++;
    // Finer buckets mean fewer block-by-block steps; take the finest combination that fits.  The
    // base shifts follow the index width (for 24 bits: 12 / 8 / 3); S2 is coarsened first (its
    // blocks are the most regular), then S0, and S1 last.
    static const int steps[][3] = {{0, 0, 0}, {0, 0, 1}, {1, 0, 1}, {1, 0, 2}, {1, 1, 2}, {2, 1, 2}, {2, 2, 2}, {3, 3, 2}};
    for (const auto &st : steps) {
        const int s0 = std::min(std::max(1, bits - 12) + st[0], (int)kFast8MaxShift);
        const int s1 = std::min(std::max(1, bits - 16) + st[1], (int)kFast8MaxShift);
        const int s2 = std::min(std::max(1, bits - 21) + st[2], 6);
        if (build_with_shifts(K, N, s0, s1, s2, max_bytes, s0_outside, blob, p)) return true;
    }
    return false;
}

// Replays the table walk on the host for indices [first, first + count) of (8, K) and compares the
// decoded point with the plain coordinate-by-coordinate walk of App. B.3.
extern "C" int pvq_fast_tables_selftest(int K, uint64_t first, uint64_t count, uint64_t *mismatches)
{
    if (!mismatches) return PVQ_E_INVALID_ARG;
    SmallTable N(K);
    const uint64_t total = N.at(8, K);
    uint64_t bad = 0;
    // both table flavours: everything in one place, and S0's block table kept apart
    for (int flavour = 0; flavour < 2; flavour++)
    {
    std::vector<unsigned char> blob;
    pvq_fast8_params p;
    if (!pvq_fast8_build(K, kFast8MaxBytes, flavour == 1, blob, p)) return PVQ_E_UNSUPPORTED;
    for (uint64_t c = first; c < first + count && c < total; c++) {
        uint32_t cc[1] = {(uint32_t)c}, pr[1][4], nn[1];
        if (flavour == 0) pvq_fast8_decode<1, false>(blob.data(), blob.data(), p, cc, pr, nn);
        else pvq_fast8_decode<1, true>(blob.data(), blob.data(), p, cc, pr, nn);
        const uint32_t *pairs = pr[0];
        const uint32_t n2x4 = nn[0];
        int y[8];
        plain_walk(N, K, c, y);
        int n2 = 0;
        bool same = true;
        for (int i = 0; i < 8; i++) {
            n2 += y[i] * y[i];
            const uint32_t h = (pairs[i / 2] >> (16 * (i & 1))) & 0xFFFFu;
            same = same && h == bf16_of_int(y[i]);
        }
        same = same && n2x4 == (uint32_t)(4 * n2);
        bad += !same;
    }
    }
    *mismatches = bad;
    return PVQ_OK;
}
