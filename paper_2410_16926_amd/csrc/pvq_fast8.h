// Table-driven decoder for D = 8 with single-word indices.
//
// App. B.3 walks one coordinate at a time and, inside a coordinate, one magnitude at a time: about
// D + K dependent table reads per group.  The same enumeration order can be inverted in a few
// steps if whole pairs of coordinates are located at once.  In the sub-pyramid with d open
// dimensions and k pulses, the points that share the next two coordinates (a, b) form one
// contiguous block of N(d-2, k-|a|-|b|) indices, and blocks follow each other in the visiting order
// of a, then of b (0, +1, -1, +2, -2, ...).  So a stage is: find the block that holds the residual
// index r, emit (a, b), subtract the block's start, continue with d-2 dimensions.
//
// Stages for D = 8:
//   S0  (d=8, k=K)   pair (y0,y1)  -> residual in (6, k1)
//   S1  (d=6, k1)    pair (y2,y3)  -> residual in (4, k2)
//   S2  (d=4, k2)    single y4     -> residual in (3, k3)
//   T3  (d=3, k3)    direct table over every (k3, r): y5, y6, y7
// Finding a block: a bucket table indexed by (row k, r >> shift) names the block that holds the
// bucket's first index (candidate A) and a second block starting inside the bucket (candidate B, with
// its start relative to the bucket).  The block table entry carries the block's start and end; if
// r lies beyond the end (a bucket with several small blocks) the lane steps on block by block.
// Residuals are carried with a per-row bias that makes r >> shift the bucket's place in the stage's
// whole bucket table (see the block entry).  All tables sit in one blob that a workgroup copies into
// LDS; a second flavour keeps S0's block table outside for a kernel that reads it from device memory.
//
// Values are emitted as packed bf16 pairs (exact for |y| <= 256) ready for v_dot2_f32_bf16, plus
// 4 * sum(y^2) accumulated from the block entries' `meta` words.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define PVQ_HD __host__ __device__ inline
#else
#define PVQ_HD inline
#endif

// Keeps a 16-byte table entry together: without it the compiler reads the one field a loop tests
// first and the other three later, which costs a second LDS round trip per stage.
#if defined(__HIP_DEVICE_COMPILE__)
#define PVQ_KEEP_TOGETHER(q) asm volatile("" : "+v"(q))
#else
#define PVQ_KEEP_TOGETHER(q) ((void)0)
#endif

// a block entry as one 16-byte value (one register tuple on the device)
typedef uint32_t pvq_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t pvq_u32x2 __attribute__((ext_vector_type(2)));

struct pvq_fast8_params {
    uint32_t blob_bytes;  // whole blob
    uint32_t tab_bytes;   // what a workgroup copies into LDS: all but an S0 block table kept outside
    uint32_t lds_bytes;   // tab_bytes without its last table, 1/sqrt(n2) (a kernel with its own gain
                          // table leaves that out)
    uint32_t s0_outside;  // 1: S0's block table lies behind tab_bytes and is read from the blob in
                          // device memory (and S0's bucket entries are two-candidate ones)
    uint32_t n_minus_1;   // N(8,K) - 1: stored indices are clamped to it
    uint32_t bk0, bk1, bk2, t3;   // byte offsets of the three bucket tables and of T3
    uint32_t bl0, bl1, bl2;       // ... and of the three block tables
    uint32_t invs;        // float [K*K + 1]: 1 / sqrt(n2), indexed by n2 (entry 0 = 0)
    uint32_t s0, s1, s2;  // bucket shifts of the three searched stages
    uint32_t k2max;       // n2 <= K*K
};

// Two bucket-entry forms.
// "two-candidate" (S1, 32 bits): bits 0..12 start of candidate B inside the bucket, bits 13..16 index
// distance from A to B (0 = no B), bits 17..31 index of A in the stage's block table.  B is the block
// starting inside the bucket that covers most of it.
// "next-block" (S0 32 bits, S2 16 bits): B is always the block after A, which lets one addition do
// the whole selection: entry = ((index of A - bucket number) << shift) + (2^shift - start of B inside
// the bucket), so that (entry + r) >> shift = index of A, plus one exactly when r has reached B (the
// low parts carry).  In the 16-bit form the arithmetic is modulo 2^16.
constexpr uint32_t kFast8ThrBits = 13;
constexpr uint32_t kFast8DbBits = 4;
constexpr uint32_t kFast8MaxShift = 13;   // all bucket shifts stay at or below this
// LDS left for the blob: the 160 KiB of a compute unit minus 5 KiB for the kernels' own buffers
// (partial sums: 2 KiB; amplitude table: 1 KiB, or a fused gain table in place of 1/sqrt(n2))
constexpr uint32_t kFast8MaxBytes = 160 * 1024 - 5120;

// block entry (16 bytes, read as one uint4): x = start, y = end (0xFFFFFFFF for the last block of a
// row), z = values as bf16 pair, w = meta = 4*(a^2+b^2).  start and end are biased: a residual is
// carried as r + (its row's first bucket in the stage's bucket table) << shift, so that r >> shift
// finds the bucket without a row offset; x = start + this row's bias - the next stage's row bias.
struct pvq_fast8_block {
    uint32_t start, end, values, meta;
};

// A searched stage for NG independent groups at once, in two halves so that all bucket reads are
// issued together and then all block reads (the latencies of the groups overlap instead of adding up).
//
// First half: the bucket lookups in the stage's bucket table at byte offset `bk` (r is biased with
// its row, see the block entry); returns in addr[j] the byte offset of the block entry chosen for r[j].
// MODE 0: two-candidate 32-bit entries; 1: next-block 32-bit entries; 2: next-block 16-bit entries.
template <int NG, int MODE>
PVQ_HD void pvq_fast8_find(const unsigned char *lds, uint32_t bk, uint32_t shift, uint32_t bl,
                           const uint32_t (&r)[NG], uint32_t (&addr)[NG])
{
    uint32_t e[NG];
#pragma unroll
    for (int j = 0; j < NG; j++) {
        if constexpr (MODE == 2) e[j] = *reinterpret_cast<const uint16_t *>(lds + bk + (r[j] >> shift) * 2u);
        else e[j] = *reinterpret_cast<const uint32_t *>(lds + bk + (r[j] >> shift) * 4u);
    }
#pragma unroll
    for (int j = 0; j < NG; j++) {
        uint32_t idx;
        if constexpr (MODE == 0) {
            const uint32_t rlow = r[j] & ((1u << shift) - 1u);
            const uint32_t thr = e[j] & ((1u << kFast8ThrBits) - 1u);
            const uint32_t db = (e[j] >> kFast8ThrBits) & ((1u << kFast8DbBits) - 1u);
            idx = (e[j] >> (kFast8ThrBits + kFast8DbBits)) + (rlow >= thr ? db : 0u);
        } else if constexpr (MODE == 1) {
            idx = (e[j] + r[j]) >> shift;
        } else {
            idx = (uint32_t)(uint16_t)(e[j] + r[j]) >> shift;
        }
        addr[j] = bl + (idx << 4);
    }
}

// Second half, after b[j] has been read from `mem + addr[j]`: a bucket with several small blocks
// makes the few lanes concerned move on block by block; then r[j] becomes the residual inside the
// block found.  `mem` is the memory that holds the block table (the LDS copy of the blob, or the
// blob in device memory).  `addr_of(addr)` fills in the entries' addresses when they are needed: a
// caller that did not keep them looks them up again, which only the rare groups that move on pay for.
template <int NG, typename AddrOf>
PVQ_HD void pvq_fast8_settle(const unsigned char *mem, uint32_t (&r)[NG], pvq_u32x4 (&b)[NG], AddrOf &&addr_of)
{
    bool miss = false, mj[NG];
#pragma unroll
    for (int j = 0; j < NG; j++) {
        PVQ_KEEP_TOGETHER(b[j]);
        mj[j] = r[j] >= b[j].y;
        miss = miss || mj[j];
    }
    if (miss) {
        // (stepping all NG groups together, one round trip per step of the furthest group, measured
        // slower than one short loop per group)
        uint32_t addr[NG];
        addr_of(addr);
#pragma unroll
        for (int j = 0; j < NG; j++) {
            if (mj[j]) {
                do {
                    addr[j] += 16;
                    b[j] = *reinterpret_cast<const pvq_u32x4 *>(mem + addr[j]);
                    PVQ_KEEP_TOGETHER(b[j]);
                } while (r[j] >= b[j].y);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NG; j++) r[j] -= b[j].x;
}

// both halves, block table in LDS
template <int NG, int MODE>
PVQ_HD void pvq_fast8_stage(const unsigned char *lds, uint32_t bk, uint32_t shift, uint32_t bl,
                            uint32_t (&r)[NG], pvq_u32x4 (&b)[NG])
{
    uint32_t addr[NG];
    pvq_fast8_find<NG, MODE>(lds, bk, shift, bl, r, addr);
#pragma unroll
    for (int j = 0; j < NG; j++) b[j] = *reinterpret_cast<const pvq_u32x4 *>(lds + addr[j]);
    pvq_fast8_settle<NG>(lds, r, b, [&](uint32_t (&out)[NG]) {
#pragma unroll
        for (int j = 0; j < NG; j++) out[j] = addr[j];
    });
}

// S0 for NG stored indices, up to the addresses of the block entries (in `blob` when OUTSIDE, else in
// `lds`): a caller that reads those entries from device memory can start S0 of its next indices
// while it still decodes the current ones.  r = the indices, clamped to the last valid one.
template <int NG, bool OUTSIDE>
PVQ_HD void pvq_fast8_s0_find(const unsigned char *lds, const pvq_fast8_params &p, const uint32_t (&c)[NG],
                              uint32_t (&r)[NG], uint32_t (&addr)[NG])
{
#pragma unroll
    for (int j = 0; j < NG; j++) r[j] = c[j] < p.n_minus_1 ? c[j] : p.n_minus_1;
    pvq_fast8_find<NG, OUTSIDE ? 0 : 1>(lds, p.bk0, p.s0, p.bl0, r, addr);
}

// The rest of the decoder, from S0's block entries b (as read from the addresses that
// pvq_fast8_s0_find gave for the clamped indices r) on.  Per index:
// four bf16 pairs (y0,y1) (y2,y3) (y4,y5) (y6,y7) and n2x4 = 4 * sum y^2.  Each pair is handed to
// `emit(j, pair number, word)` as soon as its stage has found it, so that a consumer that folds
// pairs into sums (the fused product) keeps one accumulator per group alive instead of the block
// entries.
template <int NG, bool OUTSIDE, typename Emit>
PVQ_HD void pvq_fast8_rest(const unsigned char *lds, const unsigned char *blob, const pvq_fast8_params &p,
                           uint32_t (&r)[NG], pvq_u32x4 (&b)[NG], Emit &&emit, uint32_t (&n2x4)[NG])
{
    uint32_t acc[NG], y4[NG];
    pvq_fast8_settle<NG>(OUTSIDE ? blob : lds, r, b, [&](uint32_t (&out)[NG]) {
        uint32_t same[NG];
        pvq_fast8_s0_find<NG, OUTSIDE>(lds, p, r, same, out);
    });
#pragma unroll
    for (int j = 0; j < NG; j++) { emit(j, 0, b[j].z); acc[j] = b[j].w; }
    pvq_fast8_stage<NG, 0>(lds, p.bk1, p.s1, p.bl1, r, b);
#pragma unroll
    for (int j = 0; j < NG; j++) { emit(j, 1, b[j].z); acc[j] += b[j].w; }
    pvq_fast8_stage<NG, 2>(lds, p.bk2, p.s2, p.bl2, r, b);
#pragma unroll
    for (int j = 0; j < NG; j++) { y4[j] = b[j].z; acc[j] += b[j].w; }
    pvq_u32x2 t[NG];
#pragma unroll
    for (int j = 0; j < NG; j++) t[j] = *reinterpret_cast<const pvq_u32x2 *>(lds + p.t3 + (r[j] << 3));
#pragma unroll
    for (int j = 0; j < NG; j++) {
        emit(j, 2, (t[j].x & 0xFFFF0000u) | y4[j]);
        emit(j, 3, t[j].y);
        n2x4[j] = (acc[j] + t[j].x) & 0x7FFu;
    }
}

// Whole decoder, one index set after the other.  `lds` holds the first tab_bytes of the blob (on the
// device: their copy in LDS), `blob` the whole blob (used for S0's block table when OUTSIDE).
template <int NG, bool OUTSIDE, typename Emit>
PVQ_HD void pvq_fast8_decode_emit(const unsigned char *lds, const unsigned char *blob, const pvq_fast8_params &p,
                                  const uint32_t (&c)[NG], Emit &&emit, uint32_t (&n2x4)[NG])
{
    uint32_t r[NG], addr[NG];
    pvq_u32x4 b[NG];
    const unsigned char *s0mem = OUTSIDE ? blob : lds;
    pvq_fast8_s0_find<NG, OUTSIDE>(lds, p, c, r, addr);
#pragma unroll
    for (int j = 0; j < NG; j++) b[j] = *reinterpret_cast<const pvq_u32x4 *>(s0mem + addr[j]);
    pvq_fast8_rest<NG, OUTSIDE>(lds, blob, p, r, b, emit, n2x4);
}

// The same with the pairs stored.
template <int NG, bool OUTSIDE>
PVQ_HD void pvq_fast8_decode(const unsigned char *lds, const unsigned char *blob, const pvq_fast8_params &p,
                             const uint32_t (&c)[NG], uint32_t (&pairs)[NG][4], uint32_t (&n2x4)[NG])
{
    pvq_fast8_decode_emit<NG, OUTSIDE>(lds, blob, p, c, [&](int j, int pair, uint32_t w) { pairs[j][pair] = w; }, n2x4);
}

// Host side: builds the blob for (8, K) if what goes to LDS fits `max_bytes`; returns false otherwise.
// s0_outside: keep S0's block table behind the part copied to LDS.
#include <vector>
bool pvq_fast8_build(int K, uint32_t max_bytes, bool s0_outside, std::vector<unsigned char> &blob,
                     pvq_fast8_params &p);
