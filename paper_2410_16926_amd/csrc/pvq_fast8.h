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
// bucket's first index (candidate A) and the block starting inside the bucket that covers most of it
// (candidate B, with its start relative to the bucket).  The block table entry carries the block's
// start and end; if r lies beyond the end (a bucket with several small blocks) the walk moves on
// block by block.  All tables sit in one blob that a workgroup copies into LDS.
//
// Values are emitted as packed bf16 pairs (exact for |y| <= 256) ready for v_dot2_f32_bf16, plus
// 4 * sum(y^2) accumulated in the low bits of the block entries' `meta` words.
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
#define PVQ_KEEP_TOGETHER(q) asm volatile("" : "+v"((q).x), "+v"((q).y), "+v"((q).z), "+v"((q).w))
#else
#define PVQ_KEEP_TOGETHER(q) ((void)0)
#endif

struct pvq_fast8_params {
    uint32_t blob_bytes;
    uint32_t n_minus_1;   // N(8,K) - 1: stored indices are clamped to it
    uint32_t bk0, bl0;    // byte offsets of S0's bucket table and block table
    uint32_t bl1, bl2;    // S1 / S2 block tables (their bucket rows are reached through meta)
    uint32_t invs;        // float [K*K + 1]: 1 / sqrt(n2), indexed by n2 (entry 0 = 0)
    uint32_t s0, s1, s2;  // bucket shifts of the three searched stages
    uint32_t k2max;       // n2 <= K*K
};

// 32-bit bucket entry (S0, S1): bits 0..12 start of candidate B inside the bucket, bits 13..16 index
// distance from A to B (0 = no B), bits 17..31 index of A in the stage's block table.
// 16-bit bucket entry (S2, few blocks): 5 / 2 / 9 bits.
constexpr uint32_t kFast8ThrBits = 13;
constexpr uint32_t kFast8DbBits = 4;
constexpr uint32_t kFast8S2ThrBits = 5;
constexpr uint32_t kFast8S2DbBits = 2;
// LDS left for the blob: the 160 KiB of a compute unit minus 4 KiB for the kernels' own buffers
constexpr uint32_t kFast8MaxBytes = 160 * 1024 - 4096;

// block entry (16 bytes): start, end (0xFFFFFFFF for the last block of a row), values as bf16 pair,
// meta = 4*(a^2+b^2) in bits 0..10 | byte offset of the next stage's row << 14
struct pvq_fast8_block {
    uint32_t start, end, values, meta;
};

// One searched stage for NG independent groups at once: all bucket reads are issued together, then
// all block reads, so that the LDS latencies of the groups overlap instead of adding up.
// `row[j]` = byte offset of the bucket row for group j's current k; r[j] is replaced by the residual
// inside the block found; the block is returned in b[j].
// E is the bucket entry type (uint32_t or uint16_t) with THR / DB bits for its first two fields.
// `blmem` is the memory the block table is read from (the LDS copy of the blob or the blob itself).
template <int NG, typename E, uint32_t THR, uint32_t DB>
PVQ_HD void pvq_fast8_stage(const unsigned char *lds, const unsigned char *blmem, const uint32_t (&row)[NG],
                            uint32_t shift, uint32_t bl, uint32_t (&r)[NG], pvq_fast8_block (&b)[NG])
{
    uint32_t e[NG], addr[NG];
#pragma unroll
    for (int j = 0; j < NG; j++)
        e[j] = *reinterpret_cast<const E *>(lds + row[j] + (r[j] >> shift) * (uint32_t)sizeof(E));
#pragma unroll
    for (int j = 0; j < NG; j++) {
        const uint32_t rlow = r[j] & ((1u << shift) - 1u);
        const uint32_t thr = e[j] & ((1u << THR) - 1u);
        const uint32_t db = (e[j] >> THR) & ((1u << DB) - 1u);
        const uint32_t idx = (e[j] >> (THR + DB)) + (rlow >= thr ? db : 0u);
        addr[j] = bl + (idx << 4);
    }
    bool miss = false;
    uint4 q[NG];
#pragma unroll
    for (int j = 0; j < NG; j++) q[j] = *reinterpret_cast<const uint4 *>(blmem + addr[j]);
#pragma unroll
    for (int j = 0; j < NG; j++) {
        PVQ_KEEP_TOGETHER(q[j]);
        b[j].start = q[j].x; b[j].end = q[j].y; b[j].values = q[j].z; b[j].meta = q[j].w;
        miss = miss || r[j] >= q[j].y;
    }
    // a bucket with several small blocks: the few lanes concerned move on block by block
    if (miss) {
#pragma unroll
        for (int j = 0; j < NG; j++) {
            while (r[j] >= b[j].end) {
                addr[j] += 16;
                uint4 n = *reinterpret_cast<const uint4 *>(blmem + addr[j]);
                PVQ_KEEP_TOGETHER(n);
                b[j].start = n.x; b[j].end = n.y; b[j].values = n.z; b[j].meta = n.w;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NG; j++) r[j] -= b[j].start;
}

// NG indices -> per index four bf16 pairs (y0,y1) (y2,y3) (y4,y5) (y6,y7) and n2x4 = 4 * sum y^2.
// `lds` holds the blob; `bl0mem` is where S0's block table is read from: either `lds` again, or the
// blob in global memory, which moves one 16-byte lookup per group from LDS to the vector cache (S0's
// block table is small enough to stay there).
template <int NG>
PVQ_HD void pvq_fast8_decode(const unsigned char *lds, const unsigned char *bl0mem, const pvq_fast8_params &p,
                             const uint32_t (&c)[NG], uint32_t (&pairs)[NG][4], uint32_t (&n2x4)[NG])
{
    uint32_t r[NG], row[NG];
    pvq_fast8_block b0[NG], b1[NG], b2[NG];
#pragma unroll
    for (int j = 0; j < NG; j++) {
        r[j] = c[j] < p.n_minus_1 ? c[j] : p.n_minus_1;
        row[j] = p.bk0;
    }
    pvq_fast8_stage<NG, uint32_t, kFast8ThrBits, kFast8DbBits>(lds, bl0mem, row, p.s0, p.bl0, r, b0);
#pragma unroll
    for (int j = 0; j < NG; j++) row[j] = b0[j].meta >> 14;
    pvq_fast8_stage<NG, uint32_t, kFast8ThrBits, kFast8DbBits>(lds, lds, row, p.s1, p.bl1, r, b1);
#pragma unroll
    for (int j = 0; j < NG; j++) row[j] = b1[j].meta >> 14;
    pvq_fast8_stage<NG, uint16_t, kFast8S2ThrBits, kFast8S2DbBits>(lds, lds, row, p.s2, p.bl2, r, b2);
#pragma unroll
    for (int j = 0; j < NG; j++) {
        const uint2 t = *reinterpret_cast<const uint2 *>(lds + (b2[j].meta >> 14) + (r[j] << 3));
        pairs[j][0] = b0[j].values;
        pairs[j][1] = b1[j].values;
        pairs[j][2] = (t.x & 0xFFFF0000u) | b2[j].values;
        pairs[j][3] = t.y;
        n2x4[j] = (b0[j].meta + b1[j].meta + b2[j].meta + t.x) & 0x7FFu;
    }
}

// Host side: builds the blob for (8, K) if it fits `max_bytes`; returns false otherwise.
#include <vector>
bool pvq_fast8_build(int K, uint32_t max_bytes, std::vector<unsigned char> &blob, pvq_fast8_params &p);
