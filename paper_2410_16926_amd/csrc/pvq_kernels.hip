// gfx950 kernels of libpvq: encode, decode, decode fused into a matrix-vector product.
//
// Work mapping (wave64): one lane owns one group of D weights from load to store, so the group's
// float32 sums are plain register trees with a fixed order, and the index arithmetic is a carry
// chain in that lane's registers.  The size tables live in LDS.  Bit-packed planes are assembled
// in LDS with ds_or and written out as whole words.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pvq_internal.h"
#include "pvq_quantize_dev.h"

namespace {

using namespace pvq_quantize_dev;

constexpr int kThreads = 256;
constexpr int kWave = 64;

template <int W> struct wide;
template <> struct wide<1> { using type = uint32_t; };
template <> struct wide<2> { using type = uint64_t; };
template <> struct wide<4> { using type = unsigned __int128; };

struct tables_t {
    const uint32_t *tab_n;  // [D][K+1] entries of W words
    const uint32_t *tab_u;  // [D][K+2]
    const float *edges;     // 2^scale_bits (last = +inf)
    const float *sqrtc;     // 2^scale_bits
    int K, index_bits, scale_bits;
};

// ---------------------------------------------------------------------------------------------
// bit streams
// ---------------------------------------------------------------------------------------------

// The `bits`-wide field at bit `pos` of a little-endian stream of 32-bit words.  Only words that
// hold part of the field are read.
template <int W>
__device__ inline typename wide<W>::type load_field(const uint32_t *__restrict__ row, uint32_t pos, int bits)
{
    using T = typename wide<W>::type;
    const uint32_t w0 = pos >> 5, sh = pos & 31;
    const int span = (int)sh + bits;  // bits from the start of word w0 to the end of the field
    T v = (T)(row[w0] >> sh);
#pragma unroll
    for (int i = 1; i <= W; i++) {
        if (32 * i < span) {
            const int off = 32 * i - (int)sh;  // 1 .. 32*W
            if (off < 32 * W) v |= (T)row[w0 + i] << off;
        }
    }
    if (bits < 32 * W) v &= (((T)1) << bits) - 1;
    return v;
}

// OR a `bits`-wide value into an LDS word stream at bit `pos` (the stream was zeroed before).
template <int W>
__device__ inline void stage_field(uint32_t *stage, uint32_t pos, int bits, typename wide<W>::type v)
{
    const uint32_t w0 = pos >> 5, sh = pos & 31;
    const int span = (int)sh + bits;
    atomicOr(&stage[w0], (uint32_t)v << sh);
#pragma unroll
    for (int i = 1; i <= W; i++) {
        if (32 * i < span) {
            const int off = 32 * i - (int)sh;
            const uint32_t part = off < 32 * W ? (uint32_t)(v >> off) : 0u;
            atomicOr(&stage[w0 + i], part);
        }
    }
}

template <typename T>
__device__ inline void copy_to_lds(T *dst, const T *__restrict__ src, int n)
{
    for (int i = threadIdx.x; i < n; i += kThreads) dst[i] = src[i];
}

__device__ inline float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// v_cvt_pk_bf16_f32 (round to nearest even) on the value paired with zero
__device__ inline uint32_t f32_to_bf16_rne(float f)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    const f32x2_t pair = {f, 0.0f};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t)) & 0xFFFFu;
}

// v_cvt_f16_f32 rounds to nearest even
__device__ inline uint16_t f32_to_f16_rne(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// ---------------------------------------------------------------------------------------------
// encode
// ---------------------------------------------------------------------------------------------

template <int D, typename TIn>
__device__ inline void load_group(const TIn *__restrict__ p, float (&w)[D])
{
    if constexpr (sizeof(TIn) == 4) {
#pragma unroll
        for (int i = 0; i < D; i += 4) {
            float4 q = *reinterpret_cast<const float4 *>(p + i);
            w[i] = q.x; w[i + 1] = q.y; w[i + 2] = q.z; w[i + 3] = q.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < D; i += 8) {
            uint4 q = *reinterpret_cast<const uint4 *>(p + i);
            uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                w[i + 2 * j] = bf16_to_f32(u[j] & 0xFFFFu);
                w[i + 2 * j + 1] = __uint_as_float(u[j] & 0xFFFF0000u);
            }
        }
    }
}

// App. B.2 with the inner sum taken from the cumulative table (App. C.2): with
// U(d,k) = N(d,0)+...+N(d,k) and U(d,-1) = 0, a coordinate of magnitude m >= 1 adds
//   N(d,k) + 2 (U(d,k-1) - U(d,k-m)) + [x<0] N(d,k-m)  =  U(k) + U(k-1) - U(k-m) - U(k-m-[x<0]).
// tab_u rows are shifted by one entry so that U(-1) is stored.
template <int D, int W>
__device__ inline typename wide<W>::type rank_point(const int (&y)[D], int K,
                                                    const typename wide<W>::type *tab_u)
{
    using T = typename wide<W>::type;
    T c = 0;
    int k = K;
#pragma unroll
    for (int i = 0; i < D - 1; i++) {
        const T *u = tab_u + (D - 1 - i) * (K + 2) + 1;  // u[j] = U(D-1-i, j), j >= -1
        const int m = y[i] < 0 ? -y[i] : y[i];
        if (m > 0) {
            const int neg = y[i] < 0;
            c += u[k] + u[k - 1] - u[k - m] - u[k - m - neg];
            k -= m;
        }
    }
    // last coordinate: +k is first, -k second (k > 0); nothing to add when k == 0
    c += (y[D - 1] < 0) ? 1 : 0;
    return c;
}

template <int D, int W, typename TIn>
__global__ __launch_bounds__(kThreads) void encode_kernel(tables_t tb, pvq_encode_args a)
{
    using T = typename wide<W>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = tb.K, b = tb.index_bits, sb = tb.scale_bits;
    const int G = (int)a.groups;
    const int tab_entries = D * (K + 2);
    T *tab_u = reinterpret_cast<T *>(smem);
    uint32_t *stage = reinterpret_cast<uint32_t *>(tab_u + tab_entries);  // 8*b words
    uint32_t *sstage = stage + 8 * b;                                      // 8*sb words
    float *edges = reinterpret_cast<float *>(sstage + 8 * 8);              // 256 floats
    float *ss_row = edges + 256;                                           // G floats   (sb > 0)
    float *red0 = ss_row + G;                                              // (G+1)/2
    float *red1 = red0 + (G + 1) / 2;                                      // (G+3)/4

    copy_to_lds(tab_u, reinterpret_cast<const T *>(tb.tab_u), tab_entries);
    if (sb > 0) copy_to_lds(edges, tb.edges, 1 << sb);

    const int tid = threadIdx.x;
    const int ntiles = (G + kThreads - 1) / kThreads;
    const int tile_words = 8 * b;  // 256 groups * b bits / 32

    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const TIn *wrow = reinterpret_cast<const TIn *>(a.W) + row * a.ldw;
        uint32_t *irow = a.index_out + row * a.index_row_words;
        for (int tile = 0; tile < ntiles; tile++) {
            for (int i = tid; i < tile_words; i += kThreads) stage[i] = 0;
            __syncthreads();
            const int g = tile * kThreads + tid;
            if (g < G) {
                float w[D];
                int y[D];
                load_group<D, TIn>(wrow + (int64_t)g * D, w);
                float ss = quantize_group<D>(w, K, y);
                const T c = rank_point<D, W>(y, K, tab_u);
                stage_field<W>(stage, (uint32_t)tid * (uint32_t)b, b, c);
                // the amplitude: the norm, or the least-squares one, whose square then stands for
                // the sum of squares in the codes (Sec. 3.3 Steps 4 and 5)
                float amp;
                if (a.ls_amplitude) { amp = pvq_ls_amplitude<D>(w, y); ss = amp * amp; }
                else amp = sqrtf(ss);
                if (sb > 0) ss_row[g] = ss;
                else reinterpret_cast<float *>(a.scale_out)[row * G + g] = amp;
                if (a.pulses_out) {
                    int8_t *p = a.pulses_out + row * a.cols + (int64_t)g * D;
#pragma unroll
                    for (int i = 0; i < D; i += 8) {
                        uint32_t lo = 0, hi = 0;
#pragma unroll
                        for (int j = 0; j < 4; j++) {
                            lo |= ((uint32_t)y[i + j] & 0xFFu) << (8 * j);
                            hi |= ((uint32_t)y[i + 4 + j] & 0xFFu) << (8 * j);
                        }
                        *reinterpret_cast<uint2 *>(p + i) = make_uint2(lo, hi);
                    }
                }
            }
            __syncthreads();
            const int64_t w0 = (int64_t)tile * tile_words;
            const int nw = (int)min((int64_t)tile_words, a.index_row_words - w0);
            for (int i = tid; i < nw; i += kThreads) irow[w0 + i] = stage[i];
            __syncthreads();
        }
        // Row normaliser (code mode only): sum of the groups' sums of squares, adjacent pairs
        // level by level, an odd last element moving up unchanged.
        if (sb > 0) {
            int n = G;
            const float *src = ss_row;
            float *dst = red0;
            while (n > 1) {
                const int h = n >> 1, odd = n & 1;
                for (int i = tid; i < h + odd; i += kThreads)
                    dst[i] = i < h ? src[2 * i] + src[2 * i + 1] : src[n - 1];
                __syncthreads();
                n = h + odd;
                src = dst;
                dst = (dst == red0) ? red1 : red0;
            }
            const float rowss = src[0];
            if (tid == 0) a.rownorm_out[row] = rowss;
            // Sec. 3.3 Step 5: code = floor(CDF(u) 2^b) = number of quantile edges <= u,
            // u = ss_g / rowss.  The edges ascend, so the count is found by bisection.
            uint32_t *srow = reinterpret_cast<uint32_t *>(a.scale_out) + row * a.scale_row_words;
            const int stile_words = 8 * sb;
            const int nedges = (1 << sb) - 1;
            for (int tile = 0; tile < ntiles; tile++) {
                for (int i = tid; i < stile_words; i += kThreads) sstage[i] = 0;
                __syncthreads();
                const int g = tile * kThreads + tid;
                if (g < G) {
                    const float u = ss_row[g] / rowss;
                    int lo = 0, hi = nedges;
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if (edges[mid] <= u) lo = mid + 1; else hi = mid;
                    }
                    atomicOr(&sstage[(tid * sb) >> 5], (uint32_t)lo << ((tid * sb) & 31));
                }
                __syncthreads();
                const int64_t w0 = (int64_t)tile * stile_words;
                const int nw = (int)min((int64_t)stile_words, a.scale_row_words - w0);
                for (int i = tid; i < nw; i += kThreads) srow[w0 + i] = sstage[i];
                __syncthreads();
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// decode
// ---------------------------------------------------------------------------------------------

// App. B.3 over the cumulative table alone.  With U(d,x) = N(d,0) + ... + N(d,x) (U(d,-1) = 0), the points
// of P(d,k) whose first coordinate has magnitude below m >= 1 number  N(d,k) - 2 U(d-1,k-m)  (all points
// minus those of magnitude m or more, two signs each), and N(d,k) = U(d-1,k) + U(d-1,k-1).  The lane keeps
// q = N(d,k) - 1 - r for the residual r in the sub-pyramid still open.  The coordinate's magnitude is the
// smallest m with 2 U(d-1,k-1-m) <= q, that is  m = k - #{x in [0,k-1] : U(d-1,x) <= q/2}: a binary search
// in a row of the table (the same number of steps in every lane, whatever the magnitudes), instead of
// one step per unit of magnitude.  For m = 0 the next q is q - 2 U(d-1,k-1); for m >= 1, with x = k-m and
// N' = N(d-1,x) = U(d-1,x) - U(d-1,x-1):  v = q - 2 U(d-1,x) + N'  is the place inside the block of +-m counted
// from the end of its first half: v >= 0 means +m and the next q is v, v < 0 means -m and the next q is
// v + N'.  (|v| < N' <= N(D,K)/3, so the top bit of the W-word integer is a sign bit.)
// tab_u is the LDS copy of the rows U(d', .), d' = 0..D-1, each shifted by one entry so that U(-1) is stored.
// Every table read stays inside its row whatever the stored field holds.  Returns the sum of squares.
template <int D, int W>
__device__ inline int unrank_point(typename wide<W>::type c, int K,
                                   const typename wide<W>::type *tab_u, int (&y)[D])
{
    using T = typename wide<W>::type;
    int top = 1;                                   // largest power of two <= K (K >= 1)
    while (2 * top <= K) top *= 2;
    const T *u0 = tab_u + (D - 1) * (K + 2) + 1;   // u0[x] = U(D-1, x)
    T q = u0[K] + u0[K - 1] - 1 - c;               // N(D,K) - 1 - c
    int k = K;
    int n2 = 0;
#pragma unroll
    for (int i = 0; i < D - 1; i++) {
        const T *u = tab_u + (D - 1 - i) * (K + 2) + 1;
        int v = 0;
        if (k > 0) {
            const T h = q >> 1;
            int count = 0;
            for (int step = top; step > 0; step >>= 1) {
                const int np = count + step;
                const int at = np <= k ? np - 1 : k - 1;          // inside the row either way
                if (np <= k && u[at] <= h) count = np;
            }
            const int m = k - count;
            if (m == 0) {
                q -= u[k - 1] + u[k - 1];
            } else {
                const T ux = u[count], np1 = ux - u[count - 1];   // U(d-1,x), N(d-1,x) with x = k - m
                T vv = q - ux - ux + np1;
                const bool negative = (vv >> (32 * W - 1)) != 0;
                if (negative) vv += np1;
                q = vv;
                v = negative ? -m : m;
                k = count;
            }
        }
        y[i] = v;
        n2 += v * v;
    }
    y[D - 1] = (q == 0) ? -k : k;                  // the two points +k, -k of P(1,k): q = 1, 0
    n2 += k * k;
    return n2;
}

// amplitude of group g of a row: the stored float32, or sqrt(center[q]) * sqrt(row normaliser)
__device__ inline float load_amplitude(const tables_t &tb, const pvq_decode_args &a, int64_t row,
                                       int g, float sqrt_rownorm, const float *sqrtc_lds)
{
    if (tb.scale_bits == 0) return reinterpret_cast<const float *>(a.scale)[row * a.groups + g];
    const uint32_t *srow = reinterpret_cast<const uint32_t *>(a.scale) + row * a.scale_row_words;
    const uint32_t pos = (uint32_t)g * (uint32_t)tb.scale_bits;
    const uint32_t q = (srow[pos >> 5] >> (pos & 31)) & ((1u << tb.scale_bits) - 1u);
    return sqrtc_lds[q] * sqrt_rownorm;
}

template <int D, int W, int OUT>
__global__ __launch_bounds__(kThreads) void decode_kernel(tables_t tb, pvq_decode_args a)
{
    using T = typename wide<W>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = tb.K;
    T *tab_u = reinterpret_cast<T *>(smem);
    float *sqrtc = reinterpret_cast<float *>(tab_u + D * (K + 2));
    copy_to_lds(tab_u, reinterpret_cast<const T *>(tb.tab_u), D * (K + 2));
    if (tb.scale_bits > 0) copy_to_lds(sqrtc, tb.sqrtc, 1 << tb.scale_bits);
    __syncthreads();

    const int G = (int)a.groups;
    const int g = blockIdx.x * kThreads + threadIdx.x;
    if (g >= G) return;
    for (int64_t row = blockIdx.y; row < a.rows; row += gridDim.y) {
        const uint32_t *irow = a.index + row * a.index_row_words;
        const T c = load_field<W>(irow, (uint32_t)g * (uint32_t)tb.index_bits, tb.index_bits);
        int y[D];
        const int n2 = unrank_point<D, W>(c, K, tab_u, y);
        const float srn = tb.scale_bits > 0 ? sqrtf(a.rownorm[row]) : 0.0f;
        const float amp = load_amplitude(tb, a, row, g, srn, sqrtc);
        // direction on the unit sphere times the amplitude (Sec. 2.4): w = amp * y / ||y||_2
        const float gain = amp / sqrtf((float)n2);
        if constexpr (OUT == PVQ_F32) {
            float *o = reinterpret_cast<float *>(a.W_out) + row * a.ldw + (int64_t)g * D;
#pragma unroll
            for (int i = 0; i < D; i += 4)
                *reinterpret_cast<float4 *>(o + i) = make_float4(gain * (float)y[i], gain * (float)y[i + 1],
                                                                 gain * (float)y[i + 2], gain * (float)y[i + 3]);
        } else {
            uint16_t *o = reinterpret_cast<uint16_t *>(a.W_out) + row * a.ldw + (int64_t)g * D;
#pragma unroll
            for (int i = 0; i < D; i += 8) {
                uint32_t p[4];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float f0 = gain * (float)y[i + 2 * j], f1 = gain * (float)y[i + 2 * j + 1];
                    if constexpr (OUT == PVQ_F16) {
                        p[j] = (uint32_t)f32_to_f16_rne(f0) | ((uint32_t)f32_to_f16_rne(f1) << 16);
                    } else {
                        p[j] = f32_to_bf16_rne(f0) | (f32_to_bf16_rne(f1) << 16);
                    }
                }
                *reinterpret_cast<uint4 *>(o + i) = make_uint4(p[0], p[1], p[2], p[3]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// decode fused into y = W_hat x
// ---------------------------------------------------------------------------------------------

// One wave per row: lanes walk the row's groups with stride 64, each keeps NB float32 partial sums
// (one per activation vector), and a fixed xor butterfly adds the 64 partial sums at the end.
template <int D, int W, int NB>
__global__ __launch_bounds__(kThreads) void gemv_kernel(tables_t tb, pvq_decode_args a, int b0)
{
    using T = typename wide<W>::type;
    extern __shared__ __align__(16) unsigned char smem[];
    const int K = tb.K;
    T *tab_u = reinterpret_cast<T *>(smem);
    float *sqrtc = reinterpret_cast<float *>(tab_u + D * (K + 2));
    copy_to_lds(tab_u, reinterpret_cast<const T *>(tb.tab_u), D * (K + 2));
    if (tb.scale_bits > 0) copy_to_lds(sqrtc, tb.sqrtc, 1 << tb.scale_bits);
    __syncthreads();

    const int G = (int)a.groups;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const uint16_t *xb = reinterpret_cast<const uint16_t *>(a.x) + (int64_t)b0 * a.ldx;
    for (int64_t row = (int64_t)blockIdx.x * (kThreads / kWave) + wave; row < a.rows;
         row += (int64_t)gridDim.x * (kThreads / kWave)) {
        const uint32_t *irow = a.index + row * a.index_row_words;
        const float srn = tb.scale_bits > 0 ? sqrtf(a.rownorm[row]) : 0.0f;
        float acc[NB];
#pragma unroll
        for (int b = 0; b < NB; b++) acc[b] = 0.0f;
        for (int g = lane; g < G; g += kWave) {
            const T c = load_field<W>(irow, (uint32_t)g * (uint32_t)tb.index_bits, tb.index_bits);
            int y[D];
            const int n2 = unrank_point<D, W>(c, K, tab_u, y);
            const float amp = load_amplitude(tb, a, row, g, srn, sqrtc);
            const float gain = amp / sqrtf((float)n2);
#pragma unroll
            for (int b = 0; b < NB; b++) {
                const uint16_t *xp = xb + (int64_t)b * a.ldx + (int64_t)g * D;
                float s = 0.0f;
#pragma unroll
                for (int i = 0; i < D; i += 8) {
                    const uint4 q = *reinterpret_cast<const uint4 *>(xp + i);
                    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        s = fmaf((float)y[i + 2 * j], bf16_to_f32(u[j] & 0xFFFFu), s);
                        s = fmaf((float)y[i + 2 * j + 1], __uint_as_float(u[j] & 0xFFFF0000u), s);
                    }
                }
                acc[b] = fmaf(gain, s, acc[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < NB; b++) {
            float v = acc[b];
#pragma unroll
            for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
            if (lane == 0) a.y[(int64_t)(b0 + b) * a.ldy + row] = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

tables_t make_tables(const pvq_ctx *c)
{
    tables_t t;
    t.tab_n = c->tab_n; t.tab_u = c->tab_u; t.edges = c->edges; t.sqrtc = c->sqrtc;
    t.K = c->K; t.index_bits = c->index_bits; t.scale_bits = c->scale_bits;
    return t;
}

constexpr size_t kMaxLds = 64 * 1024;

template <int D, int W>
hipError_t launch_encode_dw(const pvq_ctx *c, const pvq_encode_args &a, int dtype, hipStream_t s)
{
    const size_t G = (size_t)a.groups;
    size_t lds = (size_t)D * (c->K + 2) * W * 4 + (size_t)8 * c->index_bits * 4 + 64 * 4 + 256 * 4;
    if (c->scale_bits > 0) lds += (G + (G + 1) / 2 + (G + 3) / 4 + 4) * 4;
    if (lds > kMaxLds) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)std::min<int64_t>(a.rows, 1 << 20);
    if (dtype == PVQ_F32)
        hipLaunchKernelGGL((encode_kernel<D, W, float>), dim3(grid), dim3(kThreads), lds, s, make_tables(c), a);
    else
        hipLaunchKernelGGL((encode_kernel<D, W, uint16_t>), dim3(grid), dim3(kThreads), lds, s, make_tables(c), a);
    return hipGetLastError();
}

template <int D, int W>
hipError_t launch_decode_dw(const pvq_ctx *c, const pvq_decode_args &a, int out_dtype, hipStream_t s)
{
    const size_t lds = (size_t)D * (c->K + 2) * W * 4 + 256 * 4;
    if (lds > kMaxLds) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((a.groups + kThreads - 1) / kThreads), (unsigned)std::min<int64_t>(a.rows, 65535));
    const tables_t t = make_tables(c);
    switch (out_dtype) {
    case PVQ_F32: hipLaunchKernelGGL((decode_kernel<D, W, PVQ_F32>), grid, dim3(kThreads), lds, s, t, a); break;
    case PVQ_F16: hipLaunchKernelGGL((decode_kernel<D, W, PVQ_F16>), grid, dim3(kThreads), lds, s, t, a); break;
    default: hipLaunchKernelGGL((decode_kernel<D, W, PVQ_BF16>), grid, dim3(kThreads), lds, s, t, a); break;
    }
    return hipGetLastError();
}

template <int D, int W>
hipError_t launch_gemv_dw(const pvq_ctx *c, const pvq_decode_args &a, hipStream_t s)
{
    const size_t lds = (size_t)D * (c->K + 2) * W * 4 + 256 * 4;
    if (lds > kMaxLds) return hipErrorInvalidValue;
    const int rows_per_block = kThreads / kWave;
    const dim3 grid((unsigned)std::min<int64_t>((a.rows + rows_per_block - 1) / rows_per_block, 1 << 20));
    const tables_t t = make_tables(c);
    // the batch is cut into chunks of 4, 2 and 1 activation vectors per pass over the codes
    int b0 = 0;
    while (b0 < a.batch) {
        const int left = a.batch - b0;
        if (left >= 4) { hipLaunchKernelGGL((gemv_kernel<D, W, 4>), grid, dim3(kThreads), lds, s, t, a, b0); b0 += 4; }
        else if (left >= 2) { hipLaunchKernelGGL((gemv_kernel<D, W, 2>), grid, dim3(kThreads), lds, s, t, a, b0); b0 += 2; }
        else { hipLaunchKernelGGL((gemv_kernel<D, W, 1>), grid, dim3(kThreads), lds, s, t, a, b0); b0 += 1; }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

hipError_t pvq_launch_encode(const pvq_ctx *c, const pvq_encode_args &a, int dtype, hipStream_t s)
{
    if (c->D == 8) {
        if (c->words == 1) return launch_encode_dw<8, 1>(c, a, dtype, s);
        return launch_encode_dw<8, 2>(c, a, dtype, s);
    }
    if (c->D == 16) {
        if (c->words == 1) return launch_encode_dw<16, 1>(c, a, dtype, s);
        if (c->words == 2) return launch_encode_dw<16, 2>(c, a, dtype, s);
        return launch_encode_dw<16, 4>(c, a, dtype, s);
    }
    if (c->words == 1) return launch_encode_dw<32, 1>(c, a, dtype, s);
    if (c->words == 2) return launch_encode_dw<32, 2>(c, a, dtype, s);
    return launch_encode_dw<32, 4>(c, a, dtype, s);
}

hipError_t pvq_launch_decode(const pvq_ctx *c, const pvq_decode_args &a, int out_dtype, hipStream_t s)
{
    if (c->D == 8) {
        if (c->words == 1) return launch_decode_dw<8, 1>(c, a, out_dtype, s);
        return launch_decode_dw<8, 2>(c, a, out_dtype, s);
    }
    if (c->D == 16) {
        if (c->words == 1) return launch_decode_dw<16, 1>(c, a, out_dtype, s);
        if (c->words == 2) return launch_decode_dw<16, 2>(c, a, out_dtype, s);
        return launch_decode_dw<16, 4>(c, a, out_dtype, s);
    }
    if (c->words == 1) return launch_decode_dw<32, 1>(c, a, out_dtype, s);
    if (c->words == 2) return launch_decode_dw<32, 2>(c, a, out_dtype, s);
    return launch_decode_dw<32, 4>(c, a, out_dtype, s);
}

hipError_t pvq_launch_decode_gemv(const pvq_ctx *c, const pvq_decode_args &a, hipStream_t s)
{
    if (c->D == 8) {
        if (c->words == 1) return launch_gemv_dw<8, 1>(c, a, s);
        return launch_gemv_dw<8, 2>(c, a, s);
    }
    if (c->D == 16) {
        if (c->words == 1) return launch_gemv_dw<16, 1>(c, a, s);
        if (c->words == 2) return launch_gemv_dw<16, 2>(c, a, s);
        return launch_gemv_dw<16, 4>(c, a, s);
    }
    if (c->words == 1) return launch_gemv_dw<32, 1>(c, a, s);
    if (c->words == 2) return launch_gemv_dw<32, 2>(c, a, s);
    return launch_gemv_dw<32, 4>(c, a, s);
}

// ---------------------------------------------------------------------------------------------
// y = 0 for a product over zero columns (a kernel rather than a memset, so that a caller may
// capture the call into a graph)
// ---------------------------------------------------------------------------------------------

namespace {
__global__ void fill_zero_kernel(float *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}
}  // namespace

hipError_t pvq_launch_fill_zero(float *p, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
    return hipGetLastError();
}
