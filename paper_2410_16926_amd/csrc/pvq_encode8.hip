// Encoder specialised for D = 8 with 24-bit indices (the 3 bits/weight setting).
//
// Same arithmetic, in the same order, as the generic encoder (pvq_kernels.hip) — results are bit for
// bit the same — but organised for throughput:
//   * one lane per group, workgroups of 256 lanes that take whole rows, 256 groups at a time (several
//     workgroups share a compute unit, so one's loads and barriers hide behind the others' arithmetic;
//     1024-lane workgroups measured twice as slow);
//   * the pulse-count repair (Sec. 2.5) adjusts the coordinates that hold the |sum - K| first places in the
//     order of deviations, found in one short round per place (first_places8).  This equals the
//     one-at-a-time repair because no coordinate is ever adjusted twice (for finite input the
//     |sum - K| largest deviations are all positive, an adjusted coordinate drops below -1/2);
//   * the index (App. B.2) is a sum of seven table entries, one per coordinate, from a table of
//     per-coordinate offsets indexed by (coordinate, pulses left, magnitude, sign);
//   * four neighbouring lanes assemble their 24-bit indices into three dwords with DPP moves and write
//     them straight to global memory; amplitude codes are OR-reduced across lanes the same way;
//   * the row normaliser's pairwise sum is a wave butterfly followed by a small tree over wave sums
//     (adding +0.0 for absent groups is exact, so padding a row to a power of two does not change
//     the pair-level sum).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "pvq_hadamard_dev.h"
#include "pvq_internal.h"
#include "pvq_quantize_dev.h"

namespace {


constexpr int kWave = 64;
constexpr int D = 8;

struct enc8_launch {
    const uint32_t *offs;   // [7][K+1][K+1][2]
    const float *edges;     // 2^scale_bits entries, last = +inf (or nullptr)
    int K, scale_bits;
};

// v + (v moved across lanes by one data-parallel-primitive pattern); lanes outside ROWS add zero
template <int CTRL, int ROWS = 0xF>
__device__ inline float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xF, false);
    return v + __builtin_bit_cast(float, moved);
}

// Sum of the 64 lanes' values over adjacent pairs, level by level (lanes 2i and 2i+1, then pairs of
// pairs, ...), valid in lane 63.  Each level adds the two halves' sums, in whichever operand order
// the lane pattern gives (addition commutes exactly), so the result is the pair-level sum bit for bit.
__device__ inline float wave_pair_sum(float v)
{
    v = dpp_add<0xB1>(v);          // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);          // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);         // row_half_mirror
    v = dpp_add<0x140>(v);         // row_mirror
    v = dpp_add<0x142, 0xA>(v);    // row_bcast15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);    // row_bcast31 into rows 2 and 3
    return v;
}

// OR of v over aligned runs of n lanes (n = 1, 2, 4, ... 32), in every lane of the run: the first four levels
// by lane patterns inside a row of 16 lanes (within a quad; then, the quads being uniform, the mirror images
// inside 8 and 16 lanes bring the other half), the fifth across rows.
template <int CTRL>
__device__ inline uint32_t dpp_or(uint32_t v)
{
    return v | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
__device__ inline uint32_t or_over_lanes(uint32_t v, int n)
{
    if (n > 1) v = dpp_or<0xB1>(v);            // quad_perm [1,0,3,2]
    if (n > 2) v = dpp_or<0x4E>(v);            // quad_perm [2,3,0,1]
    if (n > 4) v = dpp_or<0x141>(v);           // row_half_mirror
    if (n > 8) v = dpp_or<0x140>(v);           // row_mirror
    if (n > 16) v |= __shfl_xor(v, 16, kWave);
    return v;
}

// Sum over adjacent pairs, level by level (fixed order, float32).
__device__ inline float tree8(float (&v)[D])
{
#pragma unroll
    for (int s = 1; s < D; s *= 2)
#pragma unroll
        for (int i = 0; i < D; i += 2 * s) v[i] = v[i] + v[i + s];
    return v[0];
}

template <typename TIn>
__device__ inline void load8(const TIn *__restrict__ p, float (&w)[D])
{
    if constexpr (sizeof(TIn) == 4) {
        const float4 q0 = *reinterpret_cast<const float4 *>(p), q1 = *reinterpret_cast<const float4 *>(p + 4);
        w[0] = q0.x; w[1] = q0.y; w[2] = q0.z; w[3] = q0.w; w[4] = q1.x; w[5] = q1.y; w[6] = q1.z; w[7] = q1.w;
    } else {
        const uint4 q = *reinterpret_cast<const uint4 *>(p);
        const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int j = 0; j < 4; j++) {
            w[2 * j] = __uint_as_float(u[j] << 16);
            w[2 * j + 1] = __uint_as_float(u[j] & 0xFFFF0000u);
        }
    }
}

// One group: returns its 24-bit index, the sum of squares, and the signed point in y.
__device__ inline uint32_t encode_group8(const float (&w)[D], int K, const uint32_t *offs, float &ss_out,
                                         int (&y)[D])
{
    float a[D], tmp[D];
#pragma unroll
    for (int i = 0; i < D; i++) { a[i] = fabsf(w[i]); tmp[i] = a[i]; }
    const float l1 = tree8(tmp);
#pragma unroll
    for (int i = 0; i < D; i++) tmp[i] = w[i] * w[i];
    ss_out = tree8(tmp);

    const float g = (float)K / l1;
    // no direction: all zeros, a norm whose reciprocal overflows, or anything not finite
    const bool degenerate = !(l1 > 0.0f) || !(l1 < INFINITY) || !(g < INFINITY);
    // from here on every t is finite and within [0, K(1+eps)] unless `degenerate`
    float t[D], yf[D];
    float S = 0.0f;
#pragma unroll
    for (int i = 0; i < D; i++) {
        t[i] = a[i] * g;
        yf[i] = rintf(t[i]);
        S += yf[i];                       // small integers: exact in any order
    }
    const float m = (float)K - S;         // > 0: pulses to add, < 0: pulses to take away
    float key[D];
#pragma unroll
    for (int i = 0; i < D; i++) {
        const float d = t[i] - yf[i];     // how far below its projected value
        key[i] = m < 0.0f ? -d : d;
    }
    const int need = degenerate ? 0 : (int)fminf(fabsf(m), (float)D);   // coordinates to adjust; they hold the places 0 .. need-1
    bool adj[D];
    pvq_quantize_dev::first_places8(key, need, adj);
    const float unit = m < 0.0f ? -1.0f : 1.0f;
    uint32_t c = 0;
    int k = K;
#pragma unroll
    for (int i = 0; i < D; i++) {
        int mag = (int)(yf[i] + (adj[i] ? unit : 0.0f));
        // sign bit of the weight; a degenerate group takes +K.  (-0.0 never carries a pulse: a
        // coordinate whose projection is zero is not among the ones raised.)
        const uint32_t neg = __float_as_uint(w[i]) >> 31;
        if (degenerate) mag = (i == D - 1) ? K : 0;
        // the magnitudes of the adjusted point lie in [0, k] and sum to K (a degenerate group was
        // given its point just above); the last coordinate takes what is left
        if (i == D - 1) mag = k;
        y[i] = (neg && !degenerate) ? -mag : mag;
        if (i < D - 1) {
            // offs[i][k][mag][neg]: what coordinate i adds to the index with k pulses left (App. B.2);
            // with mag = 0 both signs hold 0
            // (24-bit multiplies: everything here is far below 2^24)
            c += offs[(__mul24(i * (K + 1) + k, K + 1) + mag) * 2 + neg];
            k -= mag;
        } else {
            c += (neg && !degenerate && k > 0) ? 1u : 0u;
        }
    }
    return c;
}

// TIn: float or uint16_t (bf16 bits).  A block of kBlock lanes takes whole rows, kBlock groups at a
// time; several blocks share a compute unit, so one block's loads and barriers hide behind the
// others' arithmetic.
constexpr int kBlock = 256;
constexpr int kMaxGroups = 4096;   // groups per row this kernel takes (their sums of squares sit in LDS)

// LS: least-squares amplitudes (Sec. 3.3 Step 4) instead of norms.
template <typename TIn, bool CODES, bool LS>
__global__ __launch_bounds__(kBlock) void encode8_kernel(enc8_launch f, pvq_encode_args a)
{
    extern __shared__ __align__(16) uint32_t smem[];
    const int K = f.K, sb = f.scale_bits;
    const int ntab = 7 * (K + 1) * (K + 1) * 2;
    uint32_t *offs = smem;
    float *edges = reinterpret_cast<float *>(smem + ntab);       // 256 floats
    float *wsum = edges + 256;                                    // 64 wave sums of the row (zero padded)
    float *ss_row = wsum + 64;                                    // the row's sums of squares (CODES)
    for (int i = threadIdx.x; i < ntab; i += kBlock) offs[i] = f.offs[i];
    if constexpr (CODES)
        for (int i = threadIdx.x; i < (1 << sb); i += kBlock) edges[i] = f.edges[i];
    if (threadIdx.x < 64) wsum[threadIdx.x] = 0.0f;
    __syncthreads();

    const int G = (int)a.groups;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int quad_pos = lane & 3;
    const int tiles = (G + kBlock - 1) / kBlock;

    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const TIn *wrow = reinterpret_cast<const TIn *>(a.W) + row * a.ldw;
        uint32_t *irow = a.index_out + row * a.index_row_words;
        for (int tix = 0; tix < tiles; tix++) {
            const int g = tix * kBlock + (int)threadIdx.x;
            uint32_t c = 0;
            float ss = 0.0f;
            if (g < G) {
                float w[D];
                int y[D];
                load8<TIn>(wrow + (int64_t)g * D, w);
                c = encode_group8(w, K, offs, ss, y);
                float amp;
                if constexpr (LS) { amp = pvq_ls_amplitude<D>(w, y); ss = amp * amp; }
                else amp = sqrtf(ss);
                if (a.pulses_out) {
                    uint32_t lo = 0, hi = 0;
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        lo |= ((uint32_t)y[j] & 0xFFu) << (8 * j);
                        hi |= ((uint32_t)y[4 + j] & 0xFFu) << (8 * j);
                    }
                    *reinterpret_cast<uint2 *>(a.pulses_out + row * a.cols + (int64_t)g * D) = make_uint2(lo, hi);
                }
                if constexpr (CODES) ss_row[g] = ss;
                else reinterpret_cast<float *>(a.scale_out)[row * G + g] = amp;
            }
            // four neighbouring 24-bit indices -> three dwords: lane j of a quad (j < 3) builds dword j
            // from its own index and the next lane's
            const uint32_t cn = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xF9, 0xF, 0xF, false);
            const uint32_t lo = c | (cn << 24), hi = cn >> 8;
            const uint32_t word = __builtin_amdgcn_alignbit(hi, lo, 8 * quad_pos);
            if (quad_pos < 3 && g < G) irow[3 * (g >> 2) + quad_pos] = word;
            if constexpr (CODES) {
                // pairwise sum over the wave's 64 groups (absent groups add +0.0, which is exact)
                const float v = wave_pair_sum(ss);
                if (lane == kWave - 1) wsum[tix * (kBlock / kWave) + wave] = v;
            }
        }
        if constexpr (CODES) {
            __syncthreads();
            // the pairwise tree continues over the (at most 64, zero padded) wave sums
            float rowss = wsum[lane];
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) rowss += __shfl_xor(rowss, off, kWave);
            if (threadIdx.x == 0) a.rownorm_out[row] = rowss;
            // Sec. 3.3 Step 5: code = number of quantile edges <= u, u = ss_g / rowss (bisection over
            // the ascending edges), packed 32/sb lanes to a dword by an OR butterfly
            uint32_t *srow = reinterpret_cast<uint32_t *>(a.scale_out) + row * a.scale_row_words;
            const int nedges = (1 << sb) - 1;
            const int lanes_per_word = 32 / sb;
            for (int tix = 0; tix < tiles; tix++) {
                const int g = tix * kBlock + (int)threadIdx.x;
                uint32_t v = 0;
                if (g < G) {
                    const float u = ss_row[g] / rowss;
                    int lo = 0, hi = nedges;
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if (edges[mid] <= u) lo = mid + 1; else hi = mid;
                    }
                    v = (uint32_t)lo << ((lane * sb) & 31);
                }
                v = or_over_lanes(v, lanes_per_word);
                if ((lane & (lanes_per_word - 1)) == 0 && g < G) srow[((uint32_t)g * (uint32_t)sb) >> 5] = v;
            }
            __syncthreads();   // ss_row and wsum are rewritten by the next row
        }
    }
}

// Rotation of the rows (Sec. 3.3 Step 1) and encoding of the rotated values in one kernel: the transform's
// stages (pvq_hadamard_dev.h) end with 8 consecutive rotated values per lane, which is one group, so the
// lane goes straight on into the encoder above and the rotated matrix is never written.  A workgroup of L
// lanes takes whole rows, a chunk of 8 L values (whole blocks of the rotation) at a time; everything
// after the rotation is encode8_kernel's (its lanes are groups in row order here too, so the row sum's
// pair levels, the quads that assemble index words and the code words come out the same).  The rotated
// values are float32 (scaled by float32(1 / sqrt(block))), exactly those of the rotation kernel with a
// float32 result.  LOG2N as in pvq_hadamard.hip: 9 for blocks of up to 512 values, 10 .. 13 for that block.
template <typename TIn, bool CODES, bool LS, int LOG2N>
__device__ inline void rotate_encode8_body(const enc8_launch &f, const pvq_encode_args &a, int log2n,
                                           const uint8_t *signs, float scale)
{
    using namespace pvq_hadamard_dev;
    extern __shared__ __align__(16) uint32_t smem[];
    const int K = f.K, sb = f.scale_bits;
    const int L = blockDim.x;
    const int ntab = 7 * (K + 1) * (K + 1) * 2;
    const int G = (int)a.groups;
    uint32_t *offs = smem;
    float *edges = reinterpret_cast<float *>(smem + ntab);       // 256 floats
    float *wsum = edges + 256;                                    // 64 wave sums of the row (zero padded)
    float *ss_row = wsum + 64;                                    // the row's sums of squares (CODES)
    float *hbuf = ss_row + (CODES ? ((G + 3) & ~3) : 0);          // the rotation's exchange buffers
    for (int i = threadIdx.x; i < ntab; i += L) offs[i] = f.offs[i];
    if constexpr (CODES)
        for (int i = threadIdx.x; i < (1 << sb); i += L) edges[i] = f.edges[i];
    if (threadIdx.x < 64) wsum[threadIdx.x] = 0.0f;
    __syncthreads();

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int quad_pos = lane & 3;
    const int chunks = G / L;                                    // whole chunks: every lane has a group
    const int waves = L / kWave;

    for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
        const TIn *xrow = reinterpret_cast<const TIn *>(a.W) + row * a.ldw;
        uint32_t *irow = a.index_out + row * a.index_row_words;
        for (int ch = 0; ch < chunks; ch++) {
            const int g = ch * L + tid;
            float v[D];
            load8<TIn>(xrow + (int64_t)g * D, v);
            if (signs) {
                const uint2 s8 = *reinterpret_cast<const uint2 *>(signs + (int64_t)g * D);
#pragma unroll
                for (int j = 0; j < D; j++) {
                    const uint32_t byte = ((j < 4 ? s8.x : s8.y) >> (8 * (j & 3))) & 0xFFu;
                    if (byte) v[j] = -v[j];
                }
            }
            // one exchange buffer (a barrier in front of every exchange, which also keeps a chunk's writes
            // behind the reads of the chunk before): two workgroups of 1024 lanes then fit a unit's LDS
            // (which cross-lane stages go through the LDS permute unit: all of them for blocks of up to 512 values,
            // where the encoder's arithmetic is what the kernel waits for and that unit is idle; only the one over
            // 4 lanes for 1024 and 2048; none from 4096 on, where the exchanges through LDS need it: measured)
            constexpr int kPermuted = LOG2N <= 9 ? 4 + 8 + 16 + 32 : LOG2N <= 11 ? 4 : 0;
            hadamard_stages<LOG2N, false, true, kPermuted>(v, tid, log2n, hbuf, L);
            float w[D];
#pragma unroll
            for (int j = 0; j < D; j++) w[j] = v[j] * scale;
            int y[D];
            float ss;
            const uint32_t c = encode_group8(w, K, offs, ss, y);
            float amp;
            if constexpr (LS) { amp = pvq_ls_amplitude<D>(w, y); ss = amp * amp; }
            else amp = sqrtf(ss);
            if constexpr (CODES) ss_row[g] = ss;
            else reinterpret_cast<float *>(a.scale_out)[row * G + g] = amp;
            const uint32_t cn = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xF9, 0xF, 0xF, false);
            const uint32_t lo = c | (cn << 24), hi = cn >> 8;
            const uint32_t word = __builtin_amdgcn_alignbit(hi, lo, 8 * quad_pos);
            if (quad_pos < 3) irow[3 * (g >> 2) + quad_pos] = word;
            if constexpr (CODES) {
                const float s64 = wave_pair_sum(ss);
                if (lane == kWave - 1) wsum[ch * waves + wave] = s64;
            }
        }
        if constexpr (CODES) {
            __syncthreads();
            float rowss = wsum[lane];
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) rowss += __shfl_xor(rowss, off, kWave);
            if (threadIdx.x == 0) a.rownorm_out[row] = rowss;
            uint32_t *srow = reinterpret_cast<uint32_t *>(a.scale_out) + row * a.scale_row_words;
            const int nedges = (1 << sb) - 1;
            const int lanes_per_word = 32 / sb;
            for (int ch = 0; ch < chunks; ch++) {
                const int g = ch * L + tid;
                const float u = ss_row[g] / rowss;
                int lo = 0, hi = nedges;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (edges[mid] <= u) lo = mid + 1; else hi = mid;
                }
                uint32_t code = (uint32_t)lo << ((lane * sb) & 31);
                code = or_over_lanes(code, lanes_per_word);
                if ((lane & (lanes_per_word - 1)) == 0) srow[((uint32_t)g * (uint32_t)sb) >> 5] = code;
            }
            __syncthreads();   // ss_row and wsum are rewritten by the next row
        }
    }
}

// Blocks of 8192 values need workgroups of 1024 lanes; two of them share a unit only within 64 registers a
// lane (the body needs 68: a few values go to scratch), which measured 0.60 against 0.73 ms on 28672 x 8192.
// The smaller workgroups of the other block sizes keep all their registers.
template <typename TIn, bool CODES, bool LS, int LOG2N>
__global__ __launch_bounds__(512) void rotate_encode8_kernel(enc8_launch f, pvq_encode_args a, int log2n,
                                                            const uint8_t *signs, float scale)
{
    rotate_encode8_body<TIn, CODES, LS, LOG2N>(f, a, log2n, signs, scale);
}

template <typename TIn, bool CODES, bool LS>
__global__ __launch_bounds__(1024, 8) void rotate_encode8_kernel_8192(enc8_launch f, pvq_encode_args a, int log2n,
                                                                      const uint8_t *signs, float scale)
{
    rotate_encode8_body<TIn, CODES, LS, 13>(f, a, log2n, signs, scale);
}

}  // namespace

// lanes of the fused kernel's workgroup for a rotation block: whole blocks, at least 256 lanes
static int rotate8_lanes(int block) { return std::min(1024, std::max(256, block / 8)); }

bool pvq_rotate_encode8_usable(const pvq_ctx *c, const pvq_encode_args &a, int block)
{
    // the encoder's own conditions, and rows of whole chunks (so that every lane of a workgroup has a group
    // in every chunk and the transform's barriers are reached by all)
    return pvq_encode8_usable(c, a) && a.pulses_out == nullptr && a.groups % rotate8_lanes(block) == 0;
}

hipError_t pvq_rotate_encode8_launch(const pvq_ctx *c, const pvq_encode_args &a, int dtype, int block,
                                     const uint8_t *signs, hipStream_t s)
{
    enc8_launch f;
    f.offs = c->enc8_offs; f.edges = c->edges; f.K = c->K; f.scale_bits = c->scale_bits;
    int log2n = 0;
    while ((1 << log2n) < block) log2n++;
    const int L = rotate8_lanes(block);
    const bool codes = c->scale_bits > 0, ls = a.ls_amplitude != 0;
    const float scale = (float)(1.0 / std::sqrt((double)block));
    const size_t hbuf = log2n > 9 ? (size_t)(8 * L + 8 * L / 32 + 1) : 0;
    const size_t lds = ((size_t)7 * (c->K + 1) * (c->K + 1) * 2 + 256 + 64 + (codes ? (size_t)((a.groups + 3) & ~3) : 0) + hbuf) * 4;
    const unsigned grid = (unsigned)std::min<int64_t>(a.rows, 8192);
#define PVQ_RE8_LAUNCH(KERNEL)                                                                                   \
    do {                                                                                                        \
        if (lds > 64 * 1024) {                                                                                  \
            const hipError_t e_ = hipFuncSetAttribute(reinterpret_cast<const void *>(KERNEL),                   \
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);    \
            if (e_ != hipSuccess) return e_;                                                                    \
        }                                                                                                       \
        hipLaunchKernelGGL(KERNEL, dim3(grid), dim3(L), lds, s, f, a, log2n, signs, scale);                     \
    } while (0)
#define PVQ_RE8_N(T, C, LS_)                                                        \
    switch (log2n) {                                                                \
    case 13: PVQ_RE8_LAUNCH((rotate_encode8_kernel_8192<T, C, LS_>)); break;        \
    case 12: PVQ_RE8_LAUNCH((rotate_encode8_kernel<T, C, LS_, 12>)); break;         \
    case 11: PVQ_RE8_LAUNCH((rotate_encode8_kernel<T, C, LS_, 11>)); break;         \
    case 10: PVQ_RE8_LAUNCH((rotate_encode8_kernel<T, C, LS_, 10>)); break;         \
    default: PVQ_RE8_LAUNCH((rotate_encode8_kernel<T, C, LS_, 9>)); break;          \
    }
    if (dtype == PVQ_F32) {
        if (codes) { if (ls) PVQ_RE8_N(float, true, true) else PVQ_RE8_N(float, true, false) }
        else { if (ls) PVQ_RE8_N(float, false, true) else PVQ_RE8_N(float, false, false) }
    } else {
        if (codes) { if (ls) PVQ_RE8_N(uint16_t, true, true) else PVQ_RE8_N(uint16_t, true, false) }
        else { if (ls) PVQ_RE8_N(uint16_t, false, true) else PVQ_RE8_N(uint16_t, false, false) }
    }
#undef PVQ_RE8_N
#undef PVQ_RE8_LAUNCH
    return hipGetLastError();
}

bool pvq_encode8_usable(const pvq_ctx *c, const pvq_encode_args &a)
{
    // quads of lanes write whole dword triples; a row's sums of squares must fit the LDS buffer
    return c->enc8_offs != nullptr && a.groups % 4 == 0 && a.groups <= kMaxGroups;
}

hipError_t pvq_encode8_launch(const pvq_ctx *c, const pvq_encode_args &a, int dtype, hipStream_t s)
{
    enc8_launch f;
    f.offs = c->enc8_offs; f.edges = c->edges; f.K = c->K; f.scale_bits = c->scale_bits;
    const dim3 block(kBlock);
    const bool with_codes = c->scale_bits > 0;
    const size_t lds = ((size_t)7 * (c->K + 1) * (c->K + 1) * 2 + 256 + 64 + (with_codes ? (size_t)a.groups : 0)) * 4;
    // rows are strided over the blocks; enough blocks to fill every unit several times over
    const unsigned grid = (unsigned)std::min<int64_t>(a.rows, 8192);
    const bool codes = c->scale_bits > 0;
#define PVQ_ENC8_CASE(T, C, L) hipLaunchKernelGGL((encode8_kernel<T, C, L>), dim3(grid), dim3(block), lds, s, f, a)
    const bool ls = a.ls_amplitude != 0;
    if (dtype == PVQ_F32) {
        if (codes) { if (ls) PVQ_ENC8_CASE(float, true, true); else PVQ_ENC8_CASE(float, true, false); }
        else { if (ls) PVQ_ENC8_CASE(float, false, true); else PVQ_ENC8_CASE(float, false, false); }
    } else {
        if (codes) { if (ls) PVQ_ENC8_CASE(uint16_t, true, true); else PVQ_ENC8_CASE(uint16_t, true, false); }
        else { if (ls) PVQ_ENC8_CASE(uint16_t, false, true); else PVQ_ENC8_CASE(uint16_t, false, false); }
    }
#undef PVQ_ENC8_CASE
    return hipGetLastError();
}
