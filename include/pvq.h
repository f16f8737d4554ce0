/*
 * libpvq — group-wise Pyramid Vector Quantization of weight matrices on AMD MI355X (gfx950).
 *
 * The method is that of "Pyramid Vector Quantization for LLMs" (arXiv 2410.16926).  A weight
 * matrix W [rows x cols], cols = G*D, is cut into groups of D consecutive weights of a row.
 * Each group is stored as
 *   - the index of its direction on the integer pyramid P(D,K) = { p in Z^D : sum |p_d| = K }
 *     (Sec. 2.4), an integer in [0, N(D,K)) produced by the pyramid enumeration of App. B.2, and
 *   - its amplitude ||w||_2 (Sec. 2.3), either as a float32 or as a scale_bits-bit code against
 *     quantiles of the Beta(D/2, D(G-1)/2) distribution of the normalised squared amplitudes
 *     (Sec. 3.3 Step 5, Sec. 3.4), plus one float32 normaliser per row.
 *
 * Conventions for every call
 *   - Plain C ABI; no exceptions cross it.  Every function returns PVQ_OK (0) or a negative
 *     pvq_status; pvq_strerror() names it.  On error nothing has been launched.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     memory.  The library never allocates, frees or keeps caller-visible device memory.  A context
 *     owns small read-only device tables of its own.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  encode / decode /
 *     decode_gemv enqueue kernels on it and return without synchronising.  Outputs are overwritten
 *     in full; inputs are never modified.  Concurrent calls on different streams are safe.
 *   - Matrices are row-major; `ld*` arguments are the distance between rows in ELEMENTS.
 *
 * Packed layout (fixed; it is the storage format of the codes)
 *   - Index plane: for every row a little-endian bit stream over 32-bit words.  The index of group g
 *     occupies bits [g*b, (g+1)*b) of its row's stream, least significant bit first, b = index_bits =
 *     bit_length(N(D,K)-1).  Every row starts on a word boundary: row stride =
 *     ceil(G*b/32) words.  Unused high bits of a row's last word are written as zero.
 *   - Scale plane, scale_bits == 0: float32 [rows][G], the amplitudes.
 *     Scale plane, scale_bits in {1,2,4,8}: bit stream per row exactly like the index plane with
 *     b = scale_bits.
 *   - Row normaliser: float32 [rows], the row's sum of squared weights (only used with codes).
 */
#ifndef PVQ_H
#define PVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pvq_ctx pvq_ctx;

typedef enum {
    PVQ_OK = 0,
    PVQ_E_INVALID_ARG = -1, /* null pointer, negative size, ld < cols, bad enum value ...          */
    PVQ_E_UNSUPPORTED = -2, /* D not in {8,16,32,64,128}; K out of range; index wider than 128 (512) bits;
                               cols not a multiple of D; scale_bits not in {0,1,2,4,8}; batch > 16 */
    PVQ_E_ALIGNMENT = -3,   /* a device pointer or ld breaks the alignment stated at the call      */
    PVQ_E_HIP = -4,         /* a HIP runtime call failed; see pvq_last_hip_error()                 */
    PVQ_E_NOMEM = -5        /* host allocation failed                                              */
} pvq_status;

typedef enum { PVQ_F32 = 0, PVQ_F16 = 1, PVQ_BF16 = 2 } pvq_dtype;

/* Text for a status code (static storage). */
const char *pvq_strerror(int status);

/* The hipError_t value of the last failing HIP call made by this thread through the library
 * (0 if none). */
int pvq_last_hip_error(void);

/* ---- host-only helpers (exact integer arithmetic, no GPU needed) ------------------------- */

/*
 * N(D,K), the number of points of P(D,K) (Sec. 2.4: N(D,0)=1, N(0,K>=1)=0,
 * N(D,K) = N(D-1,K) + N(D,K-1) + N(D-1,K-1)), as 16 little-endian 32-bit words in count_words
 * (host, may be NULL), and the width of an index, bit_length(N-1), in index_bits (host, may be NULL).
 * 1 <= D <= 256, 0 <= K <= 1024; PVQ_E_UNSUPPORTED if N does not fit 512 bits.
 */
int pvq_count(int D, int K, uint32_t *count_words, int *index_bits);

/*
 * The whole size table on the GPU (App. C.2: every row is a prefix sum over k of the row before; one
 * workgroup, a multi-word scan through LDS): N(d,k) for d = 0..D, k = 0..K, written to
 * table[(d*(K+1) + k)*words + i], i = 0..words-1 little-endian 32-bit words (device memory,
 * (D+1)*(K+1)*words words, owned by the caller).  *overflow (device, one word) is set to 0, or to 1 if
 * some entry did not fit `words` words (the entries are then the true values modulo 2^(32*words)).
 * Asynchronous on `stream`; uses no memset, so it may be captured.  0 <= D <= 1024, 0 <= K <= 1023,
 * 1 <= words <= 16, else PVQ_E_UNSUPPORTED; NULL pointers PVQ_E_INVALID_ARG.
 */
int pvq_size_table_device(int D, int K, int words, uint32_t *table, uint32_t *overflow, void *stream);

/*
 * Sec. 3.3 Step 2: the largest K >= 1 whose index fits in bit_budget bits (1..511).
 * PVQ_E_UNSUPPORTED if not even K = 1 fits.
 */
int pvq_max_k(int D, int bit_budget, int *K);

/*
 * Quantile tables of the amplitude quantiser (Sec. 3.4) for Beta(D/2, D(G-1)/2), D even, G >= 2:
 *   edges[j-1]  = PPF(j / 2^b),        j = 1 .. 2^b - 1   (quantize(u) = floor(CDF(u) 2^b)
 *                                                           = number of edges <= u)
 *   centers[q]  = PPF((q + 0.5) / 2^b), q = 0 .. 2^b - 1   (dequantize)
 * Both host float64 arrays written by the call.  scale_bits in {1,2,4,8}.
 */
int pvq_beta_tables(int D, int64_t G, int scale_bits, double *edges, double *centers);

/* ---- context ------------------------------------------------------------------------------- */

/*
 * Builds the size tables for (D,K) on the host, uploads them (and the amplitude tables) to the
 * current HIP device, and returns a context usable from any thread and stream of that device; its tables
 * never change, its one setting (pvq_ctx_set_amplitude) is meant to be chosen before the context is shared.  D in {8,16,32}: 1 <= K <= 127, index_bits <= 128.
 * D in {64,128} (long groups, the setting of on-the-fly quantisation of activations, Sec. 3.2 and
 *   Sec. 4.3; e.g. D = 128, K = 187 for 3 bits per value): 1 <= K <= 1023, N(D,K) <= 2^512, float32
 *   amplitudes only (scale_bits == 0; Sec. 3.3 Step 5 quantises amplitudes for small groups);
 *   pvq_encode and pvq_decode work on such a context, pvq_decode_gemv returns PVQ_E_UNSUPPORTED.
 * scale_bits == 0: amplitudes are float32, edges/centers are ignored (may be NULL).
 * scale_bits in {1,2,4,8}: edges (2^b - 1 ascending values) and centers (2^b values), host float64,
 *   e.g. from pvq_beta_tables.  Encoding compares float32(u) with float32(edges[j]); decoding
 *   uses float32(sqrt(centers[q])).
 * This call synchronises (it copies tables); the others do not.
 */
int pvq_ctx_create(pvq_ctx **out, int D, int K, int scale_bits, const double *edges,
                   const double *centers);
int pvq_ctx_destroy(pvq_ctx *ctx);

/* Any of the out pointers may be NULL. */
int pvq_ctx_info(const pvq_ctx *ctx, int *D, int *K, int *index_bits, int *scale_bits);

/*
 * Which amplitude pvq_encode gives a group (host call, takes effect for later pvq_encode calls on
 * this context; not to be changed while an encode of this context is being enqueued by another thread):
 *   PVQ_AMP_NORM  the group's Euclidean norm (Sec. 2.3); the default.
 *   PVQ_AMP_LS    the least-squares amplitude for the quantised direction, s = (y . w) / ||y||_2
 *                 (Sec. 3.3 Step 4: the s that minimises ||w - s y/||y||_2||_2; the section prints the
 *                 ratio of the two inner products upside down).  float32: the products y_i * w_i rounded
 *                 one by one and summed over adjacent pairs, one square root, one division.
 * With amplitude codes the quantised quantity is s^2 over the row's sum of s^2 in both cases
 * (Sec. 3.3 Step 5), so decoding is the same.  PVQ_E_INVALID_ARG for another value.
 */
typedef enum { PVQ_AMP_NORM = 0, PVQ_AMP_LS = 1 } pvq_amplitude;
int pvq_ctx_set_amplitude(pvq_ctx *ctx, int amplitude);

/*
 * Sizes in bytes of the three planes for a rows x cols matrix (host out pointers, may be NULL):
 * index plane rows*ceil(G*index_bits/32)*4; scale plane rows*G*4 (scale_bits == 0) or
 * rows*ceil(G*scale_bits/32)*4; row normaliser rows*4.
 */
int pvq_packed_sizes(const pvq_ctx *ctx, int64_t rows, int64_t cols, size_t *index_bytes,
                     size_t *scale_bytes, size_t *rownorm_bytes);

/*
 * Randomised Hadamard rotation along the rows (Sec. 2.3 "Hadamard coherence processing", Sec. 3.3
 * Step 1), the step in front of pvq_encode, and its inverse, the step behind pvq_decode.
 * Every row of X is cut into blocks of `block` consecutive values and each block x becomes
 *     inverse == 0:   H (s . x) / sqrt(block)
 *     inverse != 0:   s . (H x) / sqrt(block)        (undoes the former: H is symmetric, H H = block I)
 * with H the Sylvester-Hadamard matrix in natural order and s_i = -1 where signs[i] != 0, else +1.
 * float32 arithmetic in a fixed order (butterflies over strides 1, 2, 4, ..., then one multiplication
 * by float32(1/sqrt(block))), one rounding to out_dtype at the end.
 *   X      device, [rows][ldx] of dtype (PVQ_F32 or PVQ_BF16), 16-byte aligned rows (ldx*size % 16 == 0)
 *   Y      device, [rows][ldy] of out_dtype (PVQ_F32 or PVQ_BF16), aligned likewise; Y may be X when the
 *          two types are the same
 *   block  a power of two, 8 <= block <= 8192, dividing cols (a block-diagonal rotation when cols is not
 *          a power of two, e.g. 7 blocks of 4096 for 28672 columns)
 *   signs  device, cols bytes, 8-byte aligned, or NULL for all +1
 * PVQ_E_INVALID_ARG: negative sizes, ldx/ldy < cols, NULL X or Y (unless rows or cols is 0: nothing is
 * done then); PVQ_E_UNSUPPORTED: block or a dtype outside the above, cols not a multiple of block;
 * PVQ_E_ALIGNMENT.
 */
int pvq_hadamard(const void *X, int dtype, int64_t rows, int64_t cols, int64_t ldx, int block,
                 const uint8_t *signs, int inverse, void *Y, int out_dtype, int64_t ldy, void *stream);

/* ---- the hot path --------------------------------------------------------------------------- */

/*
 * Encode a matrix: Sec. 2.5 "Quantizing the direction" (project each group onto the l1 ball of
 * radius K, round, repair the pulse count by +-1 on the coordinates of largest deviation), App. B.2
 * (enumerate the point to its index), Sec. 2.3 (amplitude = l2 norm) and, with scale_bits > 0,
 * Sec. 3.3 Step 5 (amplitude code = floor(CDF(||w_g||^2 / ||w_row||^2) 2^b)).
 *
 *   W           device, [rows][ldw] of `dtype` (PVQ_F32 or PVQ_BF16), 16-byte aligned, ldw >= cols and
 *               ldw*sizeof(element) a multiple of 16.
 *   index_out   device, index plane (see layout), 4-byte aligned.
 *   scale_out   device, scale plane, 4-byte aligned.
 *   rownorm_out device, float32 [rows]; required and written when scale_bits > 0, ignored (may be
 *               NULL) otherwise.
 *   pulses_out  device, int8 [rows][cols], 16-byte aligned, or NULL: the integer points themselves,
 *               for checking.  Must be NULL when K > 127 (PVQ_E_UNSUPPORTED otherwise).
 *
 * Arithmetic is float32 in a fixed order (pairwise sums of |w| and w*w over adjacent elements,
 * one correctly rounded division K/||w||_1, products, round-to-nearest-even; ties in the repair go
 * to the lowest coordinate), so results do not depend on the launch shape.  A group of zeros (or so
 * small that K/||w||_1 overflows) gets the point (0,...,0,+K), index 0.  Non-finite weights give
 * unspecified codes (never an out-of-bounds access).
 * PVQ_E_UNSUPPORTED besides: with amplitude codes a workgroup keeps its row's amplitudes in LDS (7 bytes per
 * group beside the size table, 64 KB in all), so rows of more than about 8000 groups are refused.
 */
int pvq_encode(const pvq_ctx *ctx, const void *W, int dtype, int64_t rows, int64_t cols,
               int64_t ldw, uint32_t *index_out, void *scale_out, float *rownorm_out,
               int8_t *pulses_out, void *stream);

/*
 * Correcting the quantisation error (Sec. 3.3 Step 6, with the proxy loss of Sec. 2.1): the rows of W are
 * taken through their groups in order; every group is quantised as pvq_encode would quantise it (point
 * and amplitude of the context's kind, Steps 3 and 4), and its error e = w_g - q_g is handed on to the
 * columns behind it,
 *     w_rest <- w_rest - e (A_gg)^-1 A_g,rest,   A = inverse of the Hessian restricted to the columns from g on,
 * which minimises the loss over those columns.  The caller gives the upper triangular U with
 * U^T U = H^-1 (from any LAPACK: inverse, then Cholesky), for which (A_gg)^-1 A_g,rest = U_gg^-1 U_g,rest.
 * On return W holds, for every group, the values that were quantised at its step: pvq_encode of W gives
 * the corrected code (amplitude codes, Step 5, are formed there, after the last group).
 *
 *   W      device, float32 [rows][ldw], 16-byte aligned, ldw >= cols, ldw a multiple of 4; overwritten.
 *   U      device, float32 [cols][ldu], 16-byte aligned, ldu >= cols, ldu a multiple of 4; only the upper
 *          triangle is used (what lies below the diagonal may be anything).  Not modified.
 *   work   device, 16-byte aligned scratch of at least pvq_correct_work_bytes(rows) bytes (two buffers of 128
 *          floats per row), owned by the caller, contents undefined afterwards.
 *
 * float32 throughout; q = (s / sqrt(sum y^2)) * y; the substitution and the updates are fused multiply-adds
 * applied one at a time in the order of the rows of U, so the result does not depend on the launch shape.
 * Contexts with D = 8, 16 or 32 and cols a multiple of 64, else PVQ_E_UNSUPPORTED.  A zero on the
 * diagonal of U gives non-finite weights (then encoded as pvq_encode encodes them), never a fault.
 * Launches 2 ceil(cols/128) - 1 kernels on `stream`, nothing else (no other stream, no event, no allocation), so
 * the call can be captured in a graph; asynchronous.
 */
int pvq_correct_work_bytes(int64_t rows, size_t *bytes);
int pvq_correct(const pvq_ctx *ctx, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                int64_t ldu, void *work, size_t work_bytes, void *stream);

/*
 * pvq_correct for callers that cannot allocate device memory or let a library allocate it: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels
 * and results as pvq_correct (bit for bit), without `work`: the t values of the panels go to a buffer that is
 * part of the library's image on every GPU (static device memory, 8 MiB, held until the process ends),
 * which bounds the rows of one call: rows <= *pvq_correct_static_max_rows (8192), else PVQ_E_UNSUPPORTED
 * (rows are independent: a taller matrix is corrected in slices of rows, one call after the other).
 * The call makes no hipMalloc / hipFree, no stream and no event: all kernels run on `stream`.
 * Nothing in the buffer has to start at zero: every value read has been written by the same call.
 * All calls on one GPU share that GPU's buffer: two calls that overlap in time on one GPU (different
 * streams or threads) race and give wrong results; calls on one stream, or ordered by events, are safe.
 */
int pvq_correct_static_max_rows(int64_t *rows);
int pvq_correct_static(const pvq_ctx *ctx, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                       int64_t ldu, void *stream);

/*
 * Rotation and encoding in one pass (Sec. 3.3 Step 1 in front of Sec. 2.5 / App. B.2): every row of X is rotated as
 * by pvq_hadamard(X, ..., block, signs, inverse = 0, float32 result) and the rotated float32 values are encoded as
 * by pvq_encode, without being written: index_out, scale_out and rownorm_out receive exactly what those two calls
 * in a row would give (the context's amplitude kind applies).  Two kinds of context:
 *   D = 128 with N(D,K) < 2^384 (activations, float32 amplitudes): block 128 .. 8192;
 *   D = 8 with 24-bit indices (weights; float32 amplitudes or amplitude codes): block 8 .. 8192, rows of at most
 *     4096 groups that are whole chunks of max(256, min(1024, block / 8)) groups (e.g. 8192 columns with any
 *     block, 4096 columns with blocks up to 4096).
 *
 *   X          device, [rows][ldx] of `dtype` (PVQ_F32 or PVQ_BF16), 16-byte aligned, ldx >= cols,
 *              ldx*sizeof(element) a multiple of 16.
 *   block      a power of two dividing cols.
 *   signs      device, uint8 [cols] (non-zero = -1), 8-byte aligned, or NULL.
 *   index_out, scale_out, rownorm_out   device, the planes of pvq_encode for this context and shape (4-byte
 *              aligned); rownorm_out is required with amplitude codes and ignored (may be NULL) otherwise.
 *
 * PVQ_E_UNSUPPORTED: another context, block or shape outside the above, or (D = 128) an index width for which
 * the groups of one workgroup (16, 32 or 64 of them, for blocks up to 2048, of 4096, of 8192) do not fill
 * whole words.
 */
int pvq_rotate_encode(const pvq_ctx *ctx, const void *X, int dtype, int64_t rows, int64_t cols, int64_t ldx,
                      int block, const uint8_t *signs, uint32_t *index_out, void *scale_out, float *rownorm_out,
                      void *stream);

/*
 * Decode a matrix: App. B.3 (index -> point p), Sec. 2.4 (direction p/||p||_2 on the unit sphere),
 * times the amplitude (the stored float32, or sqrt(centers[q] * rownorm[row]) per Sec. 3.4).
 *
 *   index, scale, rownorm   device, the planes written by pvq_encode (rownorm may be NULL when
 *                           scale_bits == 0).
 *   W_out       device, [rows][ldw] of out_dtype (PVQ_F32, PVQ_F16 or PVQ_BF16), 16-byte aligned,
 *               ldw >= cols and ldw*sizeof(element) a multiple of 16.  Float32 arithmetic, one
 *               round-to-nearest-even conversion to the output type.  For D = 8 with 24-bit indices small
 *               matrices (fewer than about 1.5 M groups) and large ones run on different decoders, whose
 *               float32 gains amplitude / ||p||_2 can differ in the last place (a division by the square
 *               root, or a multiplication by its tabulated reciprocal): values are deterministic for a
 *               given shape and within the stated 1e-6 of the exact ones on either.
 * A stored index >= N(D,K) (corrupt data) decodes to unspecified values without any out-of-bounds
 * access.
 */
int pvq_decode(const pvq_ctx *ctx, const uint32_t *index, const void *scale, const float *rownorm,
               int64_t rows, int64_t cols, void *W_out, int out_dtype, int64_t ldw, void *stream);

/*
 * Decode fused into a matrix-vector product, without materialising the weights:
 *   y[b][r] = sum_c W_hat[r][c] * x[b][c],   W_hat as produced by pvq_decode in float32.
 * Not in the paper; it is the inference-side use of the decoder (Sec. 2.3: the rotated, quantised
 * weights multiply the activations directly).  PVQ_E_UNSUPPORTED for contexts with D = 64 or 128.
 *
 *   x   device, bf16 [batch][ldx], 16-byte aligned, ldx >= cols, ldx a multiple of 8; 1 <= batch <= 16.
 *   y   device, float32 [batch][ldy], ldy >= rows.  Float32 accumulation in a fixed order
 *       (deterministic for a given shape and batch).  A group contributes gain * (y . x): the
 *       products of the integer pulses with bf16 activations are exact in float32, their sum over the group
 *       and the multiplication by the float32 gain are rounded to float32.  The pass that takes 3..16 vectors
 *       at once (D = 8 with 24-bit indices and rows of 256 or more groups, a multiple of 64) forms y . x on
 *       the matrix cores, the pulses being exact in bf16, and applies the float32 gain on the vector ALUs as
 *       the other passes do.  What depends on the batch size a vector is submitted in is the order of the
 *       float32 additions only: y[b] of the same x can differ between batch sizes by rounding (about 1e-7 of
 *       the root sum of squares of the terms), never by the weights used.
 */
int pvq_decode_gemv(const pvq_ctx *ctx, const uint32_t *index, const void *scale,
                    const float *rownorm, int64_t rows, int64_t cols, const void *x, int batch,
                    int64_t ldx, float *y, int64_t ldy, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PVQ_H */
