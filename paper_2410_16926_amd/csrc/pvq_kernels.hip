// gfx950 kernels of libpvq: the generic encoder (every group size and index width that has no kernel of its
// own); the matching decoders are in pvq_walk.hip.
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
// tab_u rows are shifted by one entry so that U(-1) is stored.  With k' = k - m that is
// [U(k) + U(k-1)] - [U(k') + U(k'-[x<0])], and the form of a negative coordinate is also right for a zero (k' = k:
// nothing is added), so the coordinate's value need not be branched on: with four-word entries the straight form
// is the faster one (D = 32, K = 60: 0.47 against 0.51 ms on 28672 x 8192), with one- and two-word entries the
// branch (D = 16, K = 33: 0.31 against 0.33 ms; a second table of U(k) + U(k-1), two reads per coordinate: 0.34 ms).
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
        if constexpr (W == 4) {
            const int kp = k - m;
            c += (u[k] + u[k - 1]) - (u[kp] + u[kp - (y[i] > 0 ? 0 : 1)]);
            k = kp;
        } else if (m > 0) {
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
                float ss;
                if constexpr (D == 8) ss = quantize_group8(w, K, y);
                else ss = quantize_group_select<D>(w, K, y);
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

// LDS of encode_kernel for a row of G groups: the size table's rows, the row's index words being assembled,
// and with amplitude codes the row's amplitudes
size_t encode_lds_bytes(const pvq_ctx *c, size_t G)
{
    size_t lds = (size_t)c->D * (c->K + 2) * c->words * 4 + (size_t)8 * c->index_bits * 4 + 64 * 4 + 256 * 4;
    if (c->scale_bits > 0) lds += (G + (G + 1) / 2 + (G + 3) / 4 + 4) * 4;
    return lds;
}

template <int D, int W>
hipError_t launch_encode_dw(const pvq_ctx *c, const pvq_encode_args &a, int dtype, hipStream_t s)
{
    const size_t lds = encode_lds_bytes(c, (size_t)a.groups);
    if (lds > kMaxLds) return hipErrorInvalidValue;      // (the caller has asked pvq_encode_fits)
    const unsigned grid = (unsigned)std::min<int64_t>(a.rows, 1 << 20);
    if (dtype == PVQ_F32)
        hipLaunchKernelGGL((encode_kernel<D, W, float>), dim3(grid), dim3(kThreads), lds, s, make_tables(c), a);
    else
        hipLaunchKernelGGL((encode_kernel<D, W, uint16_t>), dim3(grid), dim3(kThreads), lds, s, make_tables(c), a);
    return hipGetLastError();
}

}  // namespace

bool pvq_encode_fits(const pvq_ctx *c, const pvq_encode_args &a) { return encode_lds_bytes(c, (size_t)a.groups) <= kMaxLds; }

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
