// PVQ of long groups, D = 64 or 128 values with indices of up to 512 bits: the setting of on-the-fly
// quantisation of activations (Sec. 3.2, Sec. 4.3), e.g. D = 128, K = 187 for
// 3 bits per value (384-bit indices).  Amplitudes are float32 (Sec. 3.3 Step 5 quantises them only for
// small groups).  The size table no longer fits LDS (1.2 MB for (128,187)); it is read from device
// memory, where the L2 keeps it.
//
// Tables of W-word integers (W = 4, 8, 12 or 16; arithmetic is modulo 2^(32W), every true result
// fits):  N(d,k), and E(d,k) = 2 (N(d,0) + ... + N(d,k)).  With them the number of points of P(d,k)
// whose first coordinate has magnitude below m >= 1 is  A(m) = N(d,k) - E(d-1,k-m)  (all points minus
// those of magnitude m or more, two signs each), so that, in the order 0, +1, -1, +2, -2, ... of
// App. B.2, a first coordinate +m has A(m) points before it and -m has A(m) + N(d-1,k-m).
//
// Encoding (Sec. 2.5 for the point, App. B.2 for its index): one wave per group, lane l holds coordinates
// CP*l .. CP*l+CP-1 (CP = D/64).  The quantiser's sums run over adjacent pairs level by level (in the
// lane, then across lanes by data-parallel-primitive moves, no LDS traffic), the repair of the pulse
// count picks one coordinate per step by a wave-wide argmax (lowest coordinate on ties).  The index is a sum of per-coordinate terms that depend
// on the coordinate's magnitude, sign and the pulses left before it only; a prefix sum over the
// magnitudes gives the latter.  Because the pulses left after coordinate j-1 are those before
// coordinate j, the terms regroup by the cells (d_j, k_j) that the walk visits: cell j adds
// N(d_j,k_j) ([m_j > 0] + [coordinate j-1 negative]) - E(d_j,k_j) [m_{j-1} > 0].  A third table holds, per
// cell, the four forms this can take (N, -E, N-E, 2N-E), so a coordinate costs one table entry and one
// multi-word addition; six levels of multi-word additions across the lanes give the total.
//
// Decoding (App. B.3): one lane per group, coordinate by coordinate.  The lane keeps q = N(d,k) - 1 - r
// for the residual r; the coordinate's magnitude is the smallest m with E(d-1,k-1-m) <= q (E(.,-1) = 0),
// one table entry and one multi-word subtraction per step, and the difference of the last failed step
// gives the next q.  Points go to LDS as int16, and the waves then write whole groups with consecutive
// lanes on consecutive addresses.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <cmath>

#include "pvq_hadamard_dev.h"
#include "pvq_internal.h"

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

template <int W>
struct wint {
    uint32_t w[W];
};

template <int W>
__device__ inline wint<W> load_entry(const uint32_t *tab, int64_t entry)
{
    wint<W> r;
    const uint4 *p = reinterpret_cast<const uint4 *>(tab + entry * W);
#pragma unroll
    for (int i = 0; i < W / 4; i++) {
        const uint4 v = p[i];
        r.w[4 * i] = v.x; r.w[4 * i + 1] = v.y; r.w[4 * i + 2] = v.z; r.w[4 * i + 3] = v.w;
    }
    return r;
}

// a += b (modulo 2^(32W))
template <int W>
__device__ inline void add_to(wint<W> &a, const wint<W> &b)
{
    uint32_t carry = 0;
#pragma unroll
    for (int i = 0; i < W; i++) a.w[i] = __builtin_addc(a.w[i], b.w[i], carry, &carry);
}

// a - b (modulo 2^(32W)); *borrow = 1 when b > a
template <int W>
__device__ inline wint<W> subtract(const wint<W> &a, const wint<W> &b, uint32_t *borrow)
{
    wint<W> r;
    uint32_t br = 0;
#pragma unroll
    for (int i = 0; i < W; i++) r.w[i] = __builtin_subc(a.w[i], b.w[i], br, &br);
    *borrow = br;
    return r;
}

// a -= b (modulo 2^(32W)); *borrow = 1 when b > a
template <int W>
__device__ inline void subtract_from(wint<W> &a, const wint<W> &b, uint32_t *borrow)
{
    uint32_t br = 0;
#pragma unroll
    for (int i = 0; i < W; i++) a.w[i] = __builtin_subc(a.w[i], b.w[i], br, &br);
    *borrow = br;
}

// A lane's value moved by one data-parallel-primitive pattern; lanes whose row is not in ROWS, or whose
// source lies outside their row, get `idle`.
template <int CTRL, int ROWS = 0xF>
__device__ inline uint32_t dpp_move(uint32_t v, uint32_t idle = 0)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)idle, (int)v, CTRL, ROWS, 0xF, false);
}

// The six steps that bring a combination of all 64 lanes' values to lane 63: lane^1, lane^2 (quad
// permutations), the other quad of the half row and the other half of the row (mirror patterns: the
// partner holds the same value as every lane of its group by then), row 0 into 1 and 2 into 3, rows 0..1
// into 2..3.  For sums this is the adjacent-pair order, level by level.  No LDS traffic.
#define PVQ_WAVE_STEPS(STEP)                                       \
    STEP(0xB1, 0xF) STEP(0x4E, 0xF) STEP(0x141, 0xF) STEP(0x140, 0xF) STEP(0x142, 0xA) STEP(0x143, 0xC)

__device__ inline float wave_sum_pairs(float v)
{
#define PVQ_STEP(CTRL, ROWS) v = v + __uint_as_float(dpp_move<CTRL, ROWS>(__float_as_uint(v)));
    PVQ_WAVE_STEPS(PVQ_STEP)
#undef PVQ_STEP
    return __uint_as_float(__builtin_amdgcn_readlane((int)__float_as_uint(v), 63));
}
__device__ inline int wave_sum_int(int v)
{
#define PVQ_STEP(CTRL, ROWS) v += (int)dpp_move<CTRL, ROWS>((uint32_t)v);
    PVQ_WAVE_STEPS(PVQ_STEP)
#undef PVQ_STEP
    return __builtin_amdgcn_readlane(v, 63);
}

struct encode_wide_params {
    const void *X;
    int64_t ldx, groups, index_row_words;
    int K, bits, tile_groups, tiles_per_row, ls;
    const uint32_t *tab_c;   // per cell (d,k) the four forms N, -E, N-E, 2N-E
    uint32_t *index_out;
    float *scale_out;
    int8_t *pulses_out;
    int64_t cols;
};

// TIN: 0 = float32, 2 = bf16.  A workgroup takes tile_groups consecutive groups of one row, chosen so
// that their indices fill whole words; the words are put together in LDS and stored once.
template <int TIN, int CP, int W>
__global__ __launch_bounds__(512) void encode_wide_kernel(encode_wide_params p)
{
    extern __shared__ __align__(16) uint32_t stream[];
    constexpr int D = 64 * CP;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
    const int64_t row = blockIdx.x / p.tiles_per_row;
    const int tile = blockIdx.x - (int)(row * p.tiles_per_row);
    const int64_t g0 = (int64_t)tile * p.tile_groups;
    const int ng = (int)min((int64_t)p.tile_groups, p.groups - g0);
    const int tile_words = (int)(((int64_t)ng * p.bits + 31) / 32);
    const int64_t first_word = g0 * p.bits / 32;   // exact: tile_groups * bits is a multiple of 32
    const int K = p.K;

    for (int i = threadIdx.x; i < tile_words; i += blockDim.x) stream[i] = 0;
    __syncthreads();

    for (int gi = wave; gi < ng; gi += nwaves) {
        const int64_t g = g0 + gi;
        float w[CP];
        if constexpr (TIN == PVQ_F32) {
            const float *src = reinterpret_cast<const float *>(p.X) + row * p.ldx + g * D + CP * lane;
            if constexpr (CP == 2) {
                const float2 v = *reinterpret_cast<const float2 *>(src);
                w[0] = v.x; w[1] = v.y;
            } else {
                w[0] = src[0];
            }
        } else {
            const uint16_t *src = reinterpret_cast<const uint16_t *>(p.X) + row * p.ldx + g * D + CP * lane;
            if constexpr (CP == 2) {
                const uint32_t v = *reinterpret_cast<const uint32_t *>(src);
                w[0] = __uint_as_float(v << 16); w[1] = __uint_as_float(v & 0xFFFF0000u);
            } else {
                w[0] = __uint_as_float((uint32_t)src[0] << 16);
            }
        }

        // ---- the point (Sec. 2.5): project onto sum |t| = K, round, repair the pulse count
        float a[CP], l1p, ssp;
#pragma unroll
        for (int j = 0; j < CP; j++) a[j] = fabsf(w[j]);
        if constexpr (CP == 2) { l1p = a[0] + a[1]; ssp = w[0] * w[0] + w[1] * w[1]; }
        else { l1p = a[0]; ssp = w[0] * w[0]; }
        const float l1 = wave_sum_pairs(l1p), ss = wave_sum_pairs(ssp);
        const float gain = (float)K / l1;
        const bool degenerate = !(l1 > 0.0f) || !(l1 < INFINITY) || !(gain < INFINITY);
        float t[CP];
        int m[CP];
        int S = 0;
#pragma unroll
        for (int j = 0; j < CP; j++) {
            t[j] = a[j] * gain;
            m[j] = degenerate ? 0 : (int)rintf(t[j]);
            S += m[j];
        }
        S = wave_sum_int(S);
        if (degenerate) {
            if (lane == 63) m[CP - 1] = K;   // the point (0, ..., 0, +K): index 0
            S = K;
        }
        // one pulse per step: off the coordinate that lies furthest above its projected value (among
        // those that have one), or onto the one furthest below; ties go to the lowest coordinate.  A
        // valid group needs at most D/2 steps.
        for (int step = 0; step < D && S != K; step++) {
            const bool down = S > K;
            float be = -INFINITY;
            int bi = 0x7FFFFFFF;
#pragma unroll
            for (int j = 0; j < CP; j++) {
                const float e = down ? (float)m[j] - t[j] : t[j] - (float)m[j];
                const bool can = !down || m[j] > 0;
                if (can && (bi == 0x7FFFFFFF || e > be)) { be = e; bi = CP * lane + j; }
            }
#define PVQ_STEP(CTRL, ROWS)                                                                             \
    {                                                                                                    \
        const float oe = __uint_as_float(dpp_move<CTRL, ROWS>(__float_as_uint(be), 0xFF800000u));        \
        const int oi = (int)dpp_move<CTRL, ROWS>((uint32_t)bi, 0x7FFFFFFFu);                             \
        const bool take = oi != 0x7FFFFFFF && (bi == 0x7FFFFFFF || oe > be || (oe == be && oi < bi));    \
        if (take) { be = oe; bi = oi; }                                                                  \
    }
            PVQ_WAVE_STEPS(PVQ_STEP)
#undef PVQ_STEP
            bi = __builtin_amdgcn_readlane(bi, 63);
#pragma unroll
            for (int j = 0; j < CP; j++)
                if (bi == CP * lane + j) m[j] += down ? -1 : 1;
            S += down ? -1 : 1;
        }

        // ---- amplitude (Sec. 2.3, or Sec. 3.3 Step 4)
        float amp;
        if (p.ls) {
            float dp;
            int n2 = 0;
            float pr[CP];
#pragma unroll
            for (int j = 0; j < CP; j++) {
                const int ys = w[j] < 0.0f ? -m[j] : m[j];
                pr[j] = (float)ys * w[j];
                n2 += m[j] * m[j];
            }
            if constexpr (CP == 2) dp = pr[0] + pr[1]; else dp = pr[0];
            amp = wave_sum_pairs(dp) / sqrtf((float)wave_sum_int(n2));
        } else {
            amp = sqrtf(ss);
        }
        if (lane == 0) p.scale_out[row * p.groups + g] = amp;
        if (p.pulses_out) {
#pragma unroll
            for (int j = 0; j < CP; j++)
                p.pulses_out[row * p.cols + g * D + CP * lane + j] = (int8_t)(w[j] < 0.0f ? -m[j] : m[j]);
        }

        // ---- the index (App. B.2): pulses left before each coordinate, then the terms
        int mine = 0;
#pragma unroll
        for (int j = 0; j < CP; j++) mine += m[j];
        int incl = mine;   // inclusive prefix sum over the lanes: inside the rows of 16, then across them
        incl += (int)dpp_move<0x111>((uint32_t)incl);        // row_shr:1
        incl += (int)dpp_move<0x112>((uint32_t)incl);        // row_shr:2
        incl += (int)dpp_move<0x114>((uint32_t)incl);        // row_shr:4
        incl += (int)dpp_move<0x118>((uint32_t)incl);        // row_shr:8
        incl += (int)dpp_move<0x142, 0xA>((uint32_t)incl);   // lane 15 of rows 0, 2 into rows 1, 3
        incl += (int)dpp_move<0x143, 0xC>((uint32_t)incl);   // lane 31 into rows 2, 3
        int k = K - (incl - mine);   // pulses left before this lane's first coordinate
        // The walk visits the cells (d_j, k_j), j = 0..D, d_j = D - j, k_j = pulses left before coordinate
        // j.  Cell j adds  N(d_j,k_j) ([m_j > 0] + [coordinate j-1 negative]) - E(d_j,k_j) [m_{j-1} > 0]
        // (the -E(d-1,k-m) of coordinate j-1 and the N(d-1,k-m) of a negative one are values of the next
        // cell): one table entry, in the form that the two coordinates around the cell call for.
        int prev_state;              // of the coordinate before: bit 0 = magnitude > 0, bit 1 = negative
        {
            const int last = (m[CP - 1] > 0 ? 1 : 0) | ((m[CP - 1] > 0 && w[CP - 1] < 0.0f) ? 2 : 0);
            const int up = __shfl_up(last, 1, 64);
            prev_state = lane > 0 ? up : 0;
        }
        wint<W> acc;
#pragma unroll
        for (int i = 0; i < W; i++) acc.w[i] = 0;
#pragma unroll
        for (int j = 0; j < CP; j++) {
            const int d = D - (CP * lane + j);
            const int kk = min(max(k, 0), K), mm = min(max(m[j], 0), kk);   // in range whatever the input
            const int times = (mm > 0 ? 1 : 0) + (prev_state >> 1);         // how often N(d,k) counts
            const bool prev_pos = prev_state & 1;
            if (prev_pos || times) {
                const int form = prev_pos ? 1 + times : 0;
                add_to(acc, load_entry<W>(p.tab_c, ((int64_t)d * (K + 1) + kk) * 4 + form));
            }
            prev_state = (mm > 0 ? 1 : 0) | ((mm > 0 && w[j] < 0.0f) ? 2 : 0);
            k = kk - mm;
        }
        if (lane == 63) {
            // the last cell is (0, 0): N = 1, E = 2
            const int32_t last_cell = (prev_state >> 1) - 2 * (prev_state & 1);
            wint<W> small;
#pragma unroll
            for (int i = 0; i < W; i++) small.w[i] = last_cell < 0 ? 0xFFFFFFFFu : 0u;
            small.w[0] = (uint32_t)last_cell;
            add_to(acc, small);
        }
#define PVQ_STEP(CTRL, ROWS)                                                           \
    {                                                                                  \
        wint<W> other;                                                                 \
        _Pragma("unroll") for (int i = 0; i < W; i++) other.w[i] = dpp_move<CTRL, ROWS>(acc.w[i]); \
        add_to(acc, other);                                                            \
    }
        PVQ_WAVE_STEPS(PVQ_STEP)
#undef PVQ_STEP

        // ---- into the tile's bit stream: lane i takes word i of the index (lane 63 has it), shifted to
        // its place
        uint32_t word = 0;
#pragma unroll
        for (int i = 0; i < W; i++) {
            const uint32_t wi = (uint32_t)__builtin_amdgcn_readlane((int)acc.w[i], 63);
            word = lane == i ? wi : word;
        }
        const int off = gi * p.bits, sh = off & 31, w0 = off >> 5;
        const uint32_t below = __shfl_up(word, 1, 64);
        const uint32_t prev = lane > 0 ? below : 0u;
        const uint32_t out = sh ? (word << sh) | (prev >> (32 - sh)) : word;
        if (lane <= W && w0 + lane < tile_words && out) atomicOr(&stream[w0 + lane], out);
    }
    __syncthreads();
    uint32_t *dst = p.index_out + row * p.index_row_words + first_word;
    for (int i = threadIdx.x; i < tile_words; i += blockDim.x) dst[i] = stream[i];
}

// The same encoder with 16 lanes per group and four groups per wave (lane = 16 * group + sub, sub holds
// coordinates CP*sub .. CP*sub+CP-1, CP = D/16): the sums, the argmax, the prefix sum and the multi-word
// total then need four cross-lane levels instead of six, all of them permutations inside a row of 16
// lanes after which every lane of the row holds the result, and a lane's own coordinates (four or eight)
// are independent work in between.  That form remains for indices of more than 12 words, whose 17
// stream words do not fit 16 lanes.
#define PVQ_ROW_STEPS(STEP) STEP(0xB1) STEP(0x4E) STEP(0x141) STEP(0x140)

__device__ inline float row_sum_pairs(float v)
{
#define PVQ_STEP(CTRL) v = v + __uint_as_float(dpp_move<CTRL>(__float_as_uint(v)));
    PVQ_ROW_STEPS(PVQ_STEP)
#undef PVQ_STEP
    return v;
}
__device__ inline int row_sum_int(int v)
{
#define PVQ_STEP(CTRL) v += (int)dpp_move<CTRL>((uint32_t)v);
    PVQ_ROW_STEPS(PVQ_STEP)
#undef PVQ_STEP
    return v;
}

// sum of CP values over adjacent pairs, level by level
template <int CP>
__device__ inline float tree_sum(const float (&x)[CP])
{
    float t[CP];
#pragma unroll
    for (int j = 0; j < CP; j++) t[j] = x[j];
#pragma unroll
    for (int st = 1; st < CP; st *= 2)
#pragma unroll
        for (int j = 0; j < CP; j += 2 * st) t[j] = t[j] + t[j + st];
    return t[0];
}

// One group of 16 * CP values held by 16 lanes (lane `sub` of the group: coordinates CP*sub .. CP*sub+CP-1):
// the point, the amplitude, the index, and the index's words into the tile's bit stream in LDS at group
// position gl.  `on` = false: the lanes go through the motions (every cross-lane step needs them) and
// write nothing.  K and D = 16 * CP as in the context.
template <int CP, int W>
__device__ inline void encode_group16(const float (&w)[CP], int sub, bool on, int gl, int64_t row, int64_t g,
                                      const encode_wide_params &p, uint32_t *stream, int tile_words)
{
    constexpr int D = 16 * CP;
    const int K = p.K;
    // ---- the point (Sec. 2.5)
    float a[CP], sq[CP], t[CP];
#pragma unroll
    for (int j = 0; j < CP; j++) { a[j] = fabsf(w[j]); sq[j] = w[j] * w[j]; }
    const float l1 = row_sum_pairs(tree_sum<CP>(a)), ss = row_sum_pairs(tree_sum<CP>(sq));
    const float gain = (float)K / l1;
    const bool degenerate = !(l1 > 0.0f) || !(l1 < INFINITY) || !(gain < INFINITY);
    int m[CP];
    int S = 0;
#pragma unroll
    for (int j = 0; j < CP; j++) {
        t[j] = a[j] * gain;
        m[j] = degenerate ? 0 : (int)rintf(t[j]);
        S += m[j];
    }
    S = row_sum_int(S);
    if (degenerate) {
        if (sub == 15) m[CP - 1] = K;   // the point (0, ..., 0, +K): index 0
        S = K;
    }
    // one pulse per step and group, as in the wave-per-group form; the wave goes on while any of its
    // four groups is off the pyramid (a valid group needs at most D/2 steps)
    for (int step = 0; step < D; step++) {
        const bool need = S != K;           // the same in the 16 lanes of a group
        if (!__any(need)) break;
        const bool down = S > K;
        float be = -INFINITY;
        int bi = 0x7FFFFFFF;
#pragma unroll
        for (int j = 0; j < CP; j++) {
            const float e = down ? (float)m[j] - t[j] : t[j] - (float)m[j];
            const bool can = !down || m[j] > 0;
            if (can && (bi == 0x7FFFFFFF || e > be)) { be = e; bi = CP * sub + j; }
        }
#define PVQ_STEP(CTRL)                                                                                   \
{                                                                                                    \
    const float oe = __uint_as_float(dpp_move<CTRL>(__float_as_uint(be), 0xFF800000u));              \
    const int oi = (int)dpp_move<CTRL>((uint32_t)bi, 0x7FFFFFFFu);                                   \
    const bool take = oi != 0x7FFFFFFF && (bi == 0x7FFFFFFF || oe > be || (oe == be && oi < bi));    \
    if (take) { be = oe; bi = oi; }                                                                  \
}
        PVQ_ROW_STEPS(PVQ_STEP)
#undef PVQ_STEP
        if (need) {
#pragma unroll
            for (int j = 0; j < CP; j++)
                if (bi == CP * sub + j) m[j] += down ? -1 : 1;
            S += down ? -1 : 1;
        }
    }

    // ---- amplitude (Sec. 2.3, or Sec. 3.3 Step 4)
    float amp;
    if (p.ls) {
        float pr[CP];
        int n2 = 0;
#pragma unroll
        for (int j = 0; j < CP; j++) {
            const int ys = w[j] < 0.0f ? -m[j] : m[j];
            pr[j] = (float)ys * w[j];
            n2 += m[j] * m[j];
        }
        amp = row_sum_pairs(tree_sum<CP>(pr)) / sqrtf((float)row_sum_int(n2));
    } else {
        amp = sqrtf(ss);
    }
    if (on && sub == 0) p.scale_out[row * p.groups + g] = amp;
    if (on && p.pulses_out) {
#pragma unroll
        for (int j = 0; j < CP; j++)
            p.pulses_out[row * p.cols + g * D + CP * sub + j] = (int8_t)(w[j] < 0.0f ? -m[j] : m[j]);
    }

    // ---- the index (App. B.2)
    int mine = 0;
#pragma unroll
    for (int j = 0; j < CP; j++) mine += m[j];
    int incl = mine;   // inclusive prefix sum over the 16 lanes of the group
    incl += (int)dpp_move<0x111>((uint32_t)incl);        // row_shr:1
    incl += (int)dpp_move<0x112>((uint32_t)incl);        // row_shr:2
    incl += (int)dpp_move<0x114>((uint32_t)incl);        // row_shr:4
    incl += (int)dpp_move<0x118>((uint32_t)incl);        // row_shr:8
    int k = K - (incl - mine);
    // cell by cell as in the wave-per-group form: one table entry per cell, in the form that the two
    // coordinates around it call for
    const uint32_t last_state = (m[CP - 1] > 0 ? 1u : 0u) | ((m[CP - 1] > 0 && w[CP - 1] < 0.0f) ? 2u : 0u);
    int prev_state = (int)dpp_move<0x111>(last_state);   // the lane before in the row; none for sub = 0
    wint<W> acc;
#pragma unroll
    for (int i = 0; i < W; i++) acc.w[i] = 0;
#pragma unroll
    for (int j = 0; j < CP; j++) {
        const int d = D - (CP * sub + j);
        const int kk = min(max(k, 0), K), mm = min(max(m[j], 0), kk);   // in range whatever the input
        const int times = (mm > 0 ? 1 : 0) + (prev_state >> 1);
        const bool prev_pos = prev_state & 1;
        if (prev_pos || times) {
            const int form = prev_pos ? 1 + times : 0;
            add_to(acc, load_entry<W>(p.tab_c, ((int64_t)d * (K + 1) + kk) * 4 + form));
        }
        prev_state = (mm > 0 ? 1 : 0) | ((mm > 0 && w[j] < 0.0f) ? 2 : 0);
        k = kk - mm;
    }
    if (sub == 15) {
        // the last cell is (0, 0): N = 1, E = 2
        const int32_t last_cell = (prev_state >> 1) - 2 * (prev_state & 1);
        wint<W> small;
#pragma unroll
        for (int i = 0; i < W; i++) small.w[i] = last_cell < 0 ? 0xFFFFFFFFu : 0u;
        small.w[0] = (uint32_t)last_cell;
        add_to(acc, small);
    }
#define PVQ_STEP(CTRL)                                                                  \
{                                                                                   \
    wint<W> other;                                                                  \
    _Pragma("unroll") for (int i = 0; i < W; i++) other.w[i] = dpp_move<CTRL>(acc.w[i]); \
    add_to(acc, other);                                                             \
}
    PVQ_ROW_STEPS(PVQ_STEP)
#undef PVQ_STEP

    // ---- into the tile's bit stream: lane sub = i of the group takes word i of the index
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < W; i++) word = sub == i ? acc.w[i] : word;
    const int off = gl * p.bits, sh = off & 31, w0 = off >> 5;
    const uint32_t prev = dpp_move<0x111>(word);         // word sub-1, zero for sub = 0
    const uint32_t out = sh ? (word << sh) | (prev >> (32 - sh)) : word;
    if (on && sub <= W && w0 + sub < tile_words && out) atomicOr(&stream[w0 + sub], out);
}

template <int TIN, int CP, int W>
__global__ __launch_bounds__(512) void encode_wide16_kernel(encode_wide_params p)
{
    extern __shared__ __align__(16) uint32_t stream[];
    constexpr int D = 16 * CP;
    const int lane = threadIdx.x & 63, sub = lane & 15, quarter = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
    const int64_t row = blockIdx.x / p.tiles_per_row;
    const int tile = blockIdx.x - (int)(row * p.tiles_per_row);
    const int64_t g0 = (int64_t)tile * p.tile_groups;
    const int ng = (int)min((int64_t)p.tile_groups, p.groups - g0);
    const int tile_words = (int)(((int64_t)ng * p.bits + 31) / 32);
    const int64_t first_word = g0 * p.bits / 32;   // exact: tile_groups * bits is a multiple of 32

    for (int i = threadIdx.x; i < tile_words; i += blockDim.x) stream[i] = 0;
    __syncthreads();

    for (int gi = 4 * wave; gi < ng; gi += 4 * nwaves) {
        const int gl = gi + quarter;           // this quarter's group inside the tile
        const bool on = gl < ng;               // quarters beyond the tile work on its first group again, unused
        const int64_t g = g0 + (on ? gl : gi);
        float w[CP];
        if constexpr (TIN == PVQ_F32) {
            const float4 *src = reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(p.X) + row * p.ldx + g * D + CP * sub);
#pragma unroll
            for (int j = 0; j < CP / 4; j++) {
                const float4 v = src[j];
                w[4 * j] = v.x; w[4 * j + 1] = v.y; w[4 * j + 2] = v.z; w[4 * j + 3] = v.w;
            }
        } else {
            const uint2 *src = reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(p.X) + row * p.ldx + g * D + CP * sub);
#pragma unroll
            for (int j = 0; j < CP / 4; j++) {
                const uint2 v = src[j];
                w[4 * j] = __uint_as_float(v.x << 16); w[4 * j + 1] = __uint_as_float(v.x & 0xFFFF0000u);
                w[4 * j + 2] = __uint_as_float(v.y << 16); w[4 * j + 3] = __uint_as_float(v.y & 0xFFFF0000u);
            }
        }

        encode_group16<CP, W>(w, sub, on, gl, row, g, p, stream, tile_words);
    }
    __syncthreads();
    uint32_t *dst = p.index_out + row * p.index_row_words + first_word;
    for (int i = threadIdx.x; i < tile_words; i += blockDim.x) dst[i] = stream[i];
}

// Rotation and quantisation of activations in one kernel (Sec. 3.3 Step 1 in front of the encoder): a
// workgroup of L lanes takes 8L consecutive values of a row, 8 per lane, runs the block Walsh-Hadamard
// transform of the rotation kernel on them (same stages, same order, float32), and, since a lane ends with
// 8 consecutive rotated values, 16 neighbouring lanes hold one group of 128: the group encoder above
// takes them from the registers.  The rotated values are never written.
struct rotate_encode_params {
    const void *X;
    int64_t ldx, cols;
    int log2n, chunks_per_row;
    const uint8_t *signs;
    float scale;
    encode_wide_params e;
};

template <int TIN, int W, int LOG2N>
__global__ __launch_bounds__(1024) void rotate_encode16_kernel(rotate_encode_params p)
{
    extern __shared__ __align__(16) float smem[];
    const int L = blockDim.x;
    const int lane = threadIdx.x;
    const int64_t row = blockIdx.x / p.chunks_per_row;
    const int chunk = blockIdx.x - (int)(row * p.chunks_per_row);
    const int64_t col0 = (int64_t)chunk * 8 * L + 8 * lane;   // first of this lane's 8 columns
    const bool live = col0 < p.cols;                           // whole blocks and groups: a lane is in or out

    float v[8];
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = 0.0f;
    if (live) {
        if constexpr (TIN == PVQ_F32) {
            const float *src = reinterpret_cast<const float *>(p.X) + row * p.ldx + col0;
            const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        } else {
            const uint4 q = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(p.X) + row * p.ldx + col0);
            const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                v[2 * j] = __uint_as_float(u[j] << 16);
                v[2 * j + 1] = __uint_as_float(u[j] & 0xFFFF0000u);
            }
        }
        if (p.signs) {
            const uint2 s8 = *reinterpret_cast<const uint2 *>(p.signs + col0);
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const uint32_t byte = ((j < 4 ? s8.x : s8.y) >> (8 * (j & 3))) & 0xFFu;
                if (byte) v[j] = -v[j];
            }
        }
    }
    pvq_hadamard_dev::hadamard_stages<LOG2N, false>(v, lane, p.log2n, smem, L);
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = v[j] * p.scale;

    // the chunk's groups are a tile of the index plane (whole words: the host checks it)
    uint32_t *stream = reinterpret_cast<uint32_t *>(smem) + (LOG2N > 9 ? 2 * (pvq_hadamard_dev::pad(8u * (uint32_t)L) + 1u) : 0u);
    const int per_chunk = L / 16;
    const int64_t g0 = (int64_t)chunk * per_chunk;
    const int ng = (int)min((int64_t)per_chunk, p.e.groups - g0);
    const int tile_words = ng > 0 ? (int)(((int64_t)ng * p.e.bits + 31) / 32) : 0;
    const int64_t first_word = g0 * p.e.bits / 32;
    for (int i = threadIdx.x; i < tile_words; i += blockDim.x) stream[i] = 0;
    __syncthreads();
    const int sub = lane & 15, gl = lane >> 4;
    const bool on = gl < ng;
    encode_group16<8, W>(v, sub, on, gl, row, g0 + (on ? gl : 0), p.e, stream, tile_words);
    __syncthreads();
    uint32_t *dst = p.e.index_out + row * p.e.index_row_words + first_word;
    for (int i = threadIdx.x; i < tile_words; i += blockDim.x) dst[i] = stream[i];
}

struct decode_wide_params {
    const uint32_t *index;
    const float *scale;
    int64_t groups, total_groups, index_row_words, ldw;
    int K, bits;
    const uint32_t *tab_n, *tab_e, *tab_key;
    void *W_out;
};

constexpr int kDecodeLanes = 128;

// Bytes of LDS per lane for the decoded point of a group of D: magnitudes and signs.  With K <= 255 a magnitude is a
// byte and the signs are a bit each (D + D/8 bytes); else int16 values.  Rounded up to an odd number of words, so
// that the lanes' rows spread over the banks.
__host__ __device__ inline int decode_point_bytes(int D, int K)
{
    const int words = K <= 255 ? D / 4 + D / 32 : D / 2;
    return 4 * (words | 1);
}

// OUT: pvq_dtype of the result.  LDS: kDecodeLanes points (decode_point_bytes each), kDecodeLanes float32 gains;
// little per lane, so that many waves share a unit: a wave's walk is a chain of dependent steps, and what a unit
// gets done is the number of chains it holds.
// A coordinate's magnitude is the smallest m with E(d-1,k-1-m) <= q.  Tried one m after the other with the
// multi-word entries, that is a dependent trip to the tables and a multi-word subtraction per unit of magnitude,
// and a wave takes as many as its largest magnitude.  Here the search runs on 32-bit keys of the entries
// (pvq_wide_key), four at a time, against the key of q: keys that differ order the integers, and equal keys (about
// one comparison in a million) send the lane through the multi-word search.  The entries themselves are then read
// once per coordinate, together: E at the magnitude found, and N for the sign.
template <int OUT, int CP, int W>
__global__ __launch_bounds__(kDecodeLanes, 4) void decode_wide_kernel(decode_wide_params p)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    constexpr int D = 64 * CP;
    const int K = p.K;
    const bool bytes = K <= 255;
    const int LB = decode_point_bytes(D, K);
    float *gains = reinterpret_cast<float *>(lds_raw + (size_t)kDecodeLanes * LB);
    const int64_t gid = (int64_t)blockIdx.x * kDecodeLanes + threadIdx.x;
    unsigned char *mine = lds_raw + (size_t)threadIdx.x * LB;      // magnitudes [D], sign bytes [D/8]; or int16 [D]

    if (gid < p.total_groups) {
        const int64_t row = gid / p.groups, g = gid - row * p.groups;
        const uint32_t *src = p.index + row * p.index_row_words;
        // the group's index: bits [g*bits, (g+1)*bits) of the row's stream
        wint<W> r;
#pragma unroll
        for (int i = 0; i < W; i++) {
            const int left = p.bits - 32 * i;
            uint32_t v = 0;
            if (left > 0) {
                const int64_t at = g * p.bits + 32 * i;
                const int64_t wi = at >> 5;
                const int sh = (int)(at & 31);
                v = src[wi] >> sh;
                if (sh && wi + 1 < p.index_row_words) v |= src[wi + 1] << (32 - sh);
                if (left < 32) v &= (1u << left) - 1u;
            }
            r.w[i] = v;
        }
        // q = N(D,K) - 1 - r; an index that is no codeword decodes to zeros
        uint32_t br;
        wint<W> q = subtract(load_entry<W>(p.tab_n, (int64_t)D * (K + 1) + K), r, &br);
        bool valid = !br;
        {
            wint<W> one;
#pragma unroll
            for (int i = 0; i < W; i++) one.w[i] = 0;
            one.w[0] = 1;
            q = subtract(q, one, &br);
            valid = valid && !br;
        }
        int k = valid ? K : 0;
        int n2 = 0;
        uint32_t sign_byte = 0;
        for (int i = 0; i < D; i++) {
            const int d = D - i;
            int y = 0;
            if (k > 0) {
                if (d == 1) {
                    // the two points +k, -k of P(1,k): q = 1, 0
                    bool zero = true;
#pragma unroll
                    for (int x = 0; x < W; x++) zero = zero && q.w[x] == 0;
                    y = zero ? -k : k;
                    k = 0;
                } else {
                    const int rw = d - 1;                                   // the tables' row
                    const uint32_t *erow = p.tab_e + (int64_t)rw * (K + 1) * W;
                    const uint32_t *krow = p.tab_key + (int64_t)rw * (K + 1);
                    // the search on keys: m = the magnitude, or `unsure` at a pair of equal keys
                    const uint32_t kq = pvq_wide_key(q.w, W);
                    int m = k;
                    bool unsure = false;
                    for (int m0 = 0; m0 < k; m0 += 4) {
                        uint32_t ke[4];
#pragma unroll
                        for (int u = 0; u < 4; u++) ke[u] = krow[max(k - 1 - m0 - u, 0)];
                        bool done = false;
#pragma unroll
                        for (int u = 0; u < 4; u++) {
                            if (!done && m0 + u < k && ke[u] <= kq) {
                                done = true;
                                m = m0 + u;
                                unsure = ke[u] == kq;
                            }
                        }
                        if (done) break;
                    }
                    // q - E(d-1, k-1) for m = 0 (the next q); for m > 0, q - E(d-1, k-m), the entry of the last
                    // magnitude that failed.  In place: the walk's integers are not copied.
                    // (requested together with E; for m = 0 it is not used.  After the rare search below m is another,
                    // and it is read again)
                    wint<W> n = load_entry<W>(p.tab_n, (int64_t)rw * (K + 1) + (k - m));
                    if (unsure) {
                        // the multi-word search from the start
                        const wint<W> q0 = q;
                        for (m = 0; m < k; m++) {
                            uint32_t b;
                            const wint<W> t = subtract(q0, load_entry<W>(erow, k - 1 - m), &b);
                            if (!b) { if (m == 0) q = t; break; }   // E <= q: magnitude m
                            q = t;
                        }
                        n = load_entry<W>(p.tab_n, (int64_t)rw * (K + 1) + (k - m));
                    } else {
                        uint32_t b;
                        subtract_from(q, load_entry<W>(erow, m == 0 ? k - 1 : k - m), &b);
                    }
                    if (m > 0) {
                        // inside the block of magnitude m: v = q - E(d-1,k-m) + N(d-1,k-m); negative means
                        // the second half of the block (the coordinate is -m), whose q is v + N(d-1,k-m)
                        add_to(q, n);
                        const bool negative = q.w[W - 1] >> 31;
                        if (negative) add_to(q, n);
                        y = negative ? -m : m;
                        k -= m;
                    }
                }
            }
            if (bytes) {
                mine[i] = (unsigned char)(y < 0 ? -y : y);
                sign_byte = ((i & 7) ? sign_byte : 0u) | ((y < 0 ? 1u : 0u) << (i & 7));
                if ((i & 7) == 7) mine[D + (i >> 3)] = (unsigned char)sign_byte;
            } else {
                reinterpret_cast<int16_t *>(mine)[i] = (int16_t)y;
            }
            n2 += y * y;
        }
        gains[threadIdx.x] = valid ? p.scale[gid] / sqrtf((float)n2) : 0.0f;
    }
    __syncthreads();

    // whole groups out, a wave per group in turn
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int s = wave; s < kDecodeLanes; s += kDecodeLanes / 64) {
        const int64_t og = (int64_t)blockIdx.x * kDecodeLanes + s;
        if (og >= p.total_groups) break;
        const int64_t row = og / p.groups, g = og - row * p.groups;
        const float gain = gains[s];
        const unsigned char *pt = lds_raw + (size_t)s * LB;
        float v[CP];
#pragma unroll
        for (int j = 0; j < CP; j++) {
            const int c = CP * lane + j;
            int y;
            if (bytes) {
                const int mag = pt[c];
                y = (pt[D + (c >> 3)] >> (c & 7)) & 1 ? -mag : mag;
            } else {
                y = reinterpret_cast<const int16_t *>(pt)[c];
            }
            v[j] = gain * (float)y;
        }
        const int64_t at = row * p.ldw + g * D + CP * lane;
        if constexpr (OUT == PVQ_F32) {
            float *o = reinterpret_cast<float *>(p.W_out) + at;
            if constexpr (CP == 2) *reinterpret_cast<float2 *>(o) = make_float2(v[0], v[1]);
            else o[0] = v[0];
        } else if constexpr (OUT == PVQ_F16) {
            __half *o = reinterpret_cast<__half *>(p.W_out) + at;
            if constexpr (CP == 2) *reinterpret_cast<__half2 *>(o) = __halves2half2(__float2half_rn(v[0]), __float2half_rn(v[1]));
            else o[0] = __float2half_rn(v[0]);
        } else {
            uint16_t *o = reinterpret_cast<uint16_t *>(p.W_out) + at;
            if constexpr (CP == 2) {
                const f32x2_t pair = {v[0], v[1]};
                *reinterpret_cast<uint32_t *>(o) = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t));
            } else {
                const f32x2_t pair = {v[0], 0.0f};
                o[0] = (uint16_t)__builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t));
            }
        }
    }
}

int gcd_int(int a, int b) { return b ? gcd_int(b, a % b) : a; }

}  // namespace

hipError_t pvq_wide_launch_encode(const pvq_ctx *c, const pvq_encode_args &a, int dtype, hipStream_t s)
{
    encode_wide_params p;
    p.X = a.W; p.ldx = a.ldw; p.groups = a.groups; p.index_row_words = a.index_row_words;
    p.K = c->K; p.bits = c->index_bits; p.ls = a.ls_amplitude;
    p.tab_c = c->tab_c;
    p.index_out = a.index_out; p.scale_out = reinterpret_cast<float *>(a.scale_out); p.pulses_out = a.pulses_out;
    p.cols = a.cols;
    // 16 lanes per group, four groups per wave, when the index and the word it may spill into fit 16 lanes
    // and there are enough groups to fill the waves; else a wave per group (shorter chain per group)
    const bool rows16 = c->words <= 12 && a.rows * a.groups >= 16384;
    p.tile_groups = 32 / gcd_int(c->index_bits, 32);
    if (rows16 && p.tile_groups < 4) p.tile_groups = 4;
    p.tiles_per_row = (int)((a.groups + p.tile_groups - 1) / p.tile_groups);
    if (a.rows * p.tiles_per_row > 0x7FFFFFFF) return hipErrorInvalidValue;
    const int per_wave = rows16 ? 4 : 1;
    const int waves = std::min(p.tile_groups / per_wave, 8);
    const size_t lds = (size_t)(p.tile_groups * c->index_bits / 32) * 4;
    const dim3 grid((unsigned)(a.rows * p.tiles_per_row)), blk(64u * waves);
#define PVQ_WIDE_ENC(T, CP, W) hipLaunchKernelGGL((encode_wide_kernel<T, CP, W>), grid, blk, lds, s, p)
#define PVQ_WIDE_ENC16(T, CP, W) hipLaunchKernelGGL((encode_wide16_kernel<T, CP, W>), grid, blk, lds, s, p)
#define PVQ_WIDE_ENC_W(T, D64)                                                                                  \
    switch (c->words) {                                                                                         \
    case 4: if (rows16) { if (D64) PVQ_WIDE_ENC16(T, 4, 4); else PVQ_WIDE_ENC16(T, 8, 4); }                     \
            else { if (D64) PVQ_WIDE_ENC(T, 1, 4); else PVQ_WIDE_ENC(T, 2, 4); } break;                         \
    case 8: if (rows16) { if (D64) PVQ_WIDE_ENC16(T, 4, 8); else PVQ_WIDE_ENC16(T, 8, 8); }                     \
            else { if (D64) PVQ_WIDE_ENC(T, 1, 8); else PVQ_WIDE_ENC(T, 2, 8); } break;                         \
    case 12: if (rows16) { if (D64) PVQ_WIDE_ENC16(T, 4, 12); else PVQ_WIDE_ENC16(T, 8, 12); }                  \
             else { if (D64) PVQ_WIDE_ENC(T, 1, 12); else PVQ_WIDE_ENC(T, 2, 12); } break;                      \
    default: if (D64) PVQ_WIDE_ENC(T, 1, 16); else PVQ_WIDE_ENC(T, 2, 16); break;                               \
    }
    const bool d64 = c->D == 64;
    if (dtype == PVQ_F32) { PVQ_WIDE_ENC_W(PVQ_F32, d64) } else { PVQ_WIDE_ENC_W(PVQ_BF16, d64) }
#undef PVQ_WIDE_ENC_W
#undef PVQ_WIDE_ENC16
#undef PVQ_WIDE_ENC
    return hipGetLastError();
}

hipError_t pvq_wide_launch_rotate_encode(const pvq_ctx *c, const pvq_encode_args &a, int dtype, int block,
                                         const uint8_t *signs, hipStream_t s)
{
    rotate_encode_params p;
    int log2n = 0;
    while ((1 << log2n) < block) log2n++;
    const int L = std::min(1024, std::max(256, block / 8));
    const int chunk = 8 * L;
    p.X = a.W; p.ldx = a.ldw; p.cols = a.cols; p.log2n = log2n; p.signs = signs;
    p.chunks_per_row = (int)((a.cols + chunk - 1) / chunk);
    p.scale = (float)(1.0 / std::sqrt((double)block));
    p.e.X = nullptr; p.e.ldx = 0; p.e.groups = a.groups; p.e.index_row_words = a.index_row_words;
    p.e.K = c->K; p.e.bits = c->index_bits; p.e.ls = a.ls_amplitude;
    p.e.tile_groups = L / 16; p.e.tiles_per_row = p.chunks_per_row;
    p.e.tab_c = c->tab_c; p.e.index_out = a.index_out; p.e.scale_out = reinterpret_cast<float *>(a.scale_out);
    p.e.pulses_out = nullptr; p.e.cols = a.cols;
    if (a.rows * p.chunks_per_row > 0x7FFFFFFF) return hipErrorInvalidValue;
    size_t lds = (size_t)(L / 16) * c->index_bits / 8 + 16;
    if (log2n > 9) lds += 2 * (size_t)(chunk + chunk / 32 + 1) * sizeof(float);
    const dim3 grid((unsigned)(a.rows * p.chunks_per_row)), blk((unsigned)L);
#define PVQ_RE(T, W, N) hipLaunchKernelGGL((rotate_encode16_kernel<T, W, N>), grid, blk, lds, s, p)
#define PVQ_RE_N(T, W)                             \
    switch (log2n) {                               \
    case 13: PVQ_RE(T, W, 13); break;              \
    case 12: PVQ_RE(T, W, 12); break;              \
    case 11: PVQ_RE(T, W, 11); break;              \
    case 10: PVQ_RE(T, W, 10); break;              \
    default: PVQ_RE(T, W, 9); break;               \
    }
#define PVQ_RE_W(T)                                \
    switch (c->words) {                            \
    case 4: PVQ_RE_N(T, 4) break;                  \
    case 8: PVQ_RE_N(T, 8) break;                  \
    default: PVQ_RE_N(T, 12) break;                \
    }
    if (dtype == PVQ_F32) { PVQ_RE_W(PVQ_F32) } else { PVQ_RE_W(PVQ_BF16) }
#undef PVQ_RE_W
#undef PVQ_RE_N
#undef PVQ_RE
    return hipGetLastError();
}

hipError_t pvq_wide_launch_decode(const pvq_ctx *c, const pvq_decode_args &a, int out_dtype, hipStream_t s)
{
    decode_wide_params p;
    p.index = a.index; p.scale = reinterpret_cast<const float *>(a.scale);
    p.groups = a.groups; p.total_groups = a.rows * a.groups; p.index_row_words = a.index_row_words; p.ldw = a.ldw;
    p.K = c->K; p.bits = c->index_bits; p.tab_n = c->tab_n; p.tab_e = c->tab_u; p.tab_key = c->tab_key; p.W_out = a.W_out;
    if ((p.total_groups + kDecodeLanes - 1) / kDecodeLanes > 0x7FFFFFFF) return hipErrorInvalidValue;
    const size_t lds = (size_t)kDecodeLanes * decode_point_bytes(c->D, c->K) + (size_t)kDecodeLanes * 4;
    const dim3 grid((unsigned)((p.total_groups + kDecodeLanes - 1) / kDecodeLanes)), blk(kDecodeLanes);
#define PVQ_WIDE_DEC(O, CP, W) hipLaunchKernelGGL((decode_wide_kernel<O, CP, W>), grid, blk, lds, s, p)
#define PVQ_WIDE_DEC_W(O, CP)                                  \
    switch (c->words) {                                        \
    case 4: PVQ_WIDE_DEC(O, CP, 4); break;                     \
    case 8: PVQ_WIDE_DEC(O, CP, 8); break;                     \
    case 12: PVQ_WIDE_DEC(O, CP, 12); break;                   \
    default: PVQ_WIDE_DEC(O, CP, 16); break;                   \
    }
#define PVQ_WIDE_DEC_D(O) if (c->D == 128) { PVQ_WIDE_DEC_W(O, 2) } else { PVQ_WIDE_DEC_W(O, 1) }
    if (out_dtype == PVQ_F32) { PVQ_WIDE_DEC_D(PVQ_F32) }
    else if (out_dtype == PVQ_F16) { PVQ_WIDE_DEC_D(PVQ_F16) }
    else { PVQ_WIDE_DEC_D(PVQ_BF16) }
#undef PVQ_WIDE_DEC_D
#undef PVQ_WIDE_DEC_W
#undef PVQ_WIDE_DEC
    return hipGetLastError();
}
