// Internal interface between the host side of libpvq (argument checks, size tables, context) and
// its kernels.  Not installed; the public contract is include/pvq.h.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>
#include <stdint.h>

#include "pvq.h"
#include "pvq_fast8.h"

// Tables of the coordinate-by-coordinate decoder (pvq_walk.hip), one blob copied to LDS by every workgroup:
// rows of the cumulative size table U(d', x) = N(d',0) + ... + N(d',x) for d' = 1 .. D-1 in this order, entries
// x = -1 .. K+1 (U(d',-1) = 0; the entry behind the row is all ones), each row in the width of its dimension's
// arithmetic and padded to a multiple of 16 bytes; behind them a guess row of bytes per d' >= 2.  Where a row
// lies follows from the schedule (known when the kernels are compiled) and three row sizes, so that the
// kernels carry a handful of scalars rather than an offset per row (pvq_walk.h: pvq_walk_row, pvq_walk_guess).
struct pvq_walk_params {
    uint32_t bytes;         // of the blob (a multiple of 16)
    int K;
    int dA, dB;             // the width schedule: dimensions above dA in `words` words, above dB in half, the rest in a quarter
    uint32_t row_bytes[3];  // bytes of a cumulative row in full, half and quarter width
    uint32_t guess_base;    // byte offset of the first guess row (d' = 2)
};

// A multi-word integer (w[0] the lowest word) as 32 bits that order like the integer wherever they differ: its
// bit length in the upper 10 bits, below them the 22 leading bits (0 for 0).  key(a) < key(b) implies a < b;
// equal keys decide nothing.
#if defined(__HIPCC__)
__host__ __device__
#endif
inline uint32_t pvq_wide_key(const uint32_t *w, int words)
{
    uint32_t hi = 0, lo = 0;
    int t = -1;
    for (int i = 0; i < words; i++)
        if (w[i] != 0) { t = i; hi = w[i]; lo = i > 0 ? w[i - 1] : 0u; }
    if (t < 0) return 0;
    const int lead = __builtin_clz(hi);
    const uint32_t top = lead ? (hi << lead) | (lo >> (32 - lead)) : hi;
    return ((uint32_t)(32 * t + 32 - lead) << 22) | (top >> 10);
}

struct pvq_ctx {
    int D, K;
    int index_bits;
    int words;       // 32-bit words of one table entry / one index in registers: 1, 2 or 4 (wide: 4..16)
    int wide;        // 1: D = 64 or 128; tab_n[d][k] = N(d,k) for d = 0..D, tab_u[d][k] = 2 (N(d,0)+...+N(d,k))
                     //    mod 2^(32 words) for d = 0..D-1, both [.][K+1][words]; kernels in pvq_wide.hip
    int scale_bits;  // 0 = float32 amplitudes
    int device;
    // Device tables.  Entries are `words` little-endian 32-bit words.
    //   tab_n[dp][k]  = N(dp, k),                      dp = 0..D-1, k = 0..K        (App. B.3 walks it)
    //   tab_u[dp][k+1] = sum_{i=0..k} N(dp, i), tab_u[dp][0] = 0,  k = -1..K         (cumulative form of
    //                    App. C.2's V table, shifted so that the empty sum is an entry)
    uint32_t *tab_n;
    uint32_t *tab_u;
    uint32_t *tab_c;   // wide only: [D+1][K+1][4][words], the four forms N, -E, N-E, 2N-E of a cell (encoders)
    uint32_t *tab_key; // wide only: [D][K+1], pvq_wide_key of tab_u's entries (the decoder's search)
    float *edges;   // 2^scale_bits - 1 float32 edges (or nullptr)
    float *sqrtc;   // 2^scale_bits float32 sqrt(centers) (or nullptr)
    size_t tab_n_bytes, tab_u_bytes;
    // Table-driven decoder (D = 8, one-word indices, tables that fit LDS); fast8_blob == nullptr
    // when the configuration has none.  Two flavours of the tables: all of them in one LDS copy (the
    // decode kernel), and S0's block table kept in device memory (the fused product; nullptr if
    // that flavour does not fit).
    unsigned char *fast8_blob, *fast8g_blob;
    pvq_fast8_params fast8, fast8g;
    // Coordinate-by-coordinate decoder's tables (every context with D <= 32); nullptr if they were not made.
    unsigned char *walk_blob = nullptr;
    pvq_walk_params walk;
    int amplitude;   // PVQ_AMP_NORM or PVQ_AMP_LS
    // Per-coordinate index offsets for the D = 8 / 24-bit encoder: [7][K+1][K+1][2] words
    // (coordinate, pulses left, magnitude, sign); nullptr when the configuration has none.
    uint32_t *enc8_offs;
};

struct pvq_encode_args {
    int ls_amplitude;   // 1: least-squares amplitudes instead of norms
    const void *W;
    int64_t rows, cols, ldw, groups;
    uint32_t *index_out;
    void *scale_out;
    float *rownorm_out;
    int8_t *pulses_out;
    int64_t index_row_words, scale_row_words;
};

struct pvq_decode_args {
    const uint32_t *index;
    const void *scale;
    const float *rownorm;
    int64_t rows, cols, groups;
    int64_t index_row_words, scale_row_words;
    void *W_out;
    int64_t ldw;
    const void *x;  // gemv only
    int batch;
    int64_t ldx;
    float *y;
    int64_t ldy;
};

// Least-squares amplitude of a group for its point y (Sec. 3.3 Step 4): (y . w) / ||y||_2 in float32,
// products rounded one by one and summed over adjacent pairs, level by level.
template <int D>
__device__ inline float pvq_ls_amplitude(const float (&w)[D], const int (&y)[D])
{
    float p[D];
    int n2 = 0;
#pragma unroll
    for (int i = 0; i < D; i++) {
        p[i] = (float)y[i] * w[i];
        n2 += y[i] * y[i];
    }
#pragma unroll
    for (int s = 1; s < D; s *= 2)
#pragma unroll
        for (int i = 0; i < D; i += 2 * s) p[i] = p[i] + p[i + s];
    return p[0] / sqrtf((float)n2);
}

// Each returns a hipError_t from the launch (hipSuccess if enqueued).
// false: a row's share of LDS (size table, and with amplitude codes the row's amplitudes) exceeds 64 KB
bool pvq_encode_fits(const pvq_ctx *ctx, const pvq_encode_args &a);
hipError_t pvq_launch_encode(const pvq_ctx *ctx, const pvq_encode_args &a, int dtype, hipStream_t s);

hipError_t pvq_launch_fill_zero(float *p, int64_t n, hipStream_t s);   // p[0..n) = 0 by a kernel

// error correction of Sec. 3.3 Step 6 (pvq_correct.hip): W rows x cols float32 in place, cols a multiple
// of 64, U cols x cols upper triangular, work rows x 128 floats
hipError_t pvq_launch_correct(const pvq_ctx *ctx, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                              int64_t ldu, float *work, hipStream_t s);
// the same with the library's static work buffer (at most pvq_correct_static_max_rows() rows), on `s` alone
int64_t pvq_correct_static_max_rows(void);
// sets the number of update tiles from which a launch does the narrow update inside its panel workgroups; returns the old one
int64_t pvq_correct_front_tiles(int64_t tiles);
hipError_t pvq_launch_correct_static(const pvq_ctx *ctx, float *W, int64_t rows, int64_t cols, int64_t ldw,
                                     const float *U, int64_t ldu, hipStream_t s);

// size table on the GPU (pvq_size_table.hip): (D+1) x (K+1) entries of `words` words, one workgroup
hipError_t pvq_launch_size_table(int D, int K, int words, uint32_t *table, uint32_t *overflow, hipStream_t s);

// randomised Hadamard rotation of rows (pvq_hadamard.hip); arguments already validated
hipError_t pvq_launch_hadamard(const void *X, int in_dtype, int64_t rows, int64_t cols, int64_t ldx, int block,
                               const uint8_t *signs, int signs_after, void *Y, int out_dtype, int64_t ldy,
                               hipStream_t s);

// groups of 64 / 128 values, indices of up to 512 bits (pvq_wide.hip); for contexts with wide == 1
hipError_t pvq_wide_launch_encode(const pvq_ctx *ctx, const pvq_encode_args &a, int dtype, hipStream_t s);
hipError_t pvq_wide_launch_decode(const pvq_ctx *ctx, const pvq_decode_args &a, int out_dtype, hipStream_t s);
// rotation of rows (blocks of `block` values, optional signs) and encoding in one kernel; D = 128, words <= 12
hipError_t pvq_wide_launch_rotate_encode(const pvq_ctx *ctx, const pvq_encode_args &a, int dtype, int block,
                                         const uint8_t *signs, hipStream_t s);

// coordinate-by-coordinate decoder with one table probe per coordinate (pvq_walk.hip)
bool pvq_walk_usable(const pvq_ctx *ctx);
hipError_t pvq_walk_launch_decode(const pvq_ctx *ctx, const pvq_decode_args &a, int out_dtype, hipStream_t s);
hipError_t pvq_walk_launch_gemv(const pvq_ctx *ctx, const pvq_decode_args &a, hipStream_t s);

// D = 8 / 24-bit encoder (pvq_encode8.hip)
bool pvq_encode8_usable(const pvq_ctx *ctx, const pvq_encode_args &a);
hipError_t pvq_encode8_launch(const pvq_ctx *ctx, const pvq_encode_args &a, int dtype, hipStream_t s);
// ... with the rotation of the rows (blocks of `block` values, optional signs) fused in front
bool pvq_rotate_encode8_usable(const pvq_ctx *ctx, const pvq_encode_args &a, int block);
hipError_t pvq_rotate_encode8_launch(const pvq_ctx *ctx, const pvq_encode_args &a, int dtype, int block,
                                     const uint8_t *signs, hipStream_t s);

// D = 8 table-driven kernels (pvq_fast8.hip).  `*_usable` says whether the shape qualifies.
bool pvq_fast8_decode_usable(const pvq_ctx *ctx, const pvq_decode_args &a);
bool pvq_fast8_gemv_usable(const pvq_ctx *ctx, const pvq_decode_args &a);
hipError_t pvq_fast8_launch_decode(const pvq_ctx *ctx, const pvq_decode_args &a, int out_dtype, hipStream_t s);
hipError_t pvq_fast8_launch_gemv(const pvq_ctx *ctx, const pvq_decode_args &a, hipStream_t s);
// The passes of a fused product: which kind of kernel takes how many vectors (a batch of up to 16 vectors
// is at most 16 passes).  pvq_fast8_plan_gemv fills out[] and returns the number of passes.
enum {
    PVQ_PASS_GENERIC = 0,     // pvq_kernels.hip: coordinate-by-coordinate decoder, vector ALU, one pass per call
    PVQ_PASS_VALU = 1,        // gemv8_kernel: 1, 2 or 4 vectors, float32 multiply-adds on the vector ALU
    PVQ_PASS_VALU_ROWS = 2,   // gemv8_row_kernel: one vector, every wave owns whole rows
    PVQ_PASS_VALU16 = 3,      // gemv8_wide_kernel: up to 16 vectors on the vector ALU
    PVQ_PASS_MFMA = 4,        // gemv8_mfma_kernel: 3..16 vectors, the groups' dot products on the matrix cores
};
struct pvq_gemv_pass { int kind, nvec; };
int pvq_fast8_plan_gemv(const pvq_ctx *ctx, const pvq_decode_args &a, pvq_gemv_pass *out);
hipError_t pvq_fast8_prepare(void);  // one-time device queries
