// The coordinate-by-coordinate decoder with one table probe per coordinate: its step, shared by the kernels
// (pvq_walk.hip, which explains the method) and by a host replay that checks the tables.
#pragma once

#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <utility>

#include "pvq_fast8.h"      // PVQ_HD
#include "pvq_internal.h"   // pvq_walk_params

namespace pvq_walk {

PVQ_HD uint32_t pvq_float_bits(float f)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __float_as_uint(f);
#else
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
#endif
}

template <int W> struct wide;
template <> struct wide<1> { using type = uint32_t; };
template <> struct wide<2> { using type = uint64_t; };
template <> struct wide<4> { using type = unsigned __int128; };

// Keeps a 32-bit word of a wider integer a 32-bit value in the compiler's eyes: otherwise the conversion of a
// word known to be a shifted-down 64-bit value is widened back into a 64-bit-to-float conversion (five
// instructions instead of one).
#if defined(__HIP_DEVICE_COMPILE__)
#define PVQ_WALK_OPAQUE(x) asm volatile("" : "+v"(x))
#else
#define PVQ_WALK_OPAQUE(x) ((void)0)
#endif

// ---- layout of the blob (shared with the host builder) ---------------------------------------------------
// entry width class of row DP under the schedule (DA, DB): 0 full, 1 half, 2 quarter
constexpr int pvq_walk_class(int dp, int DA, int DB) { return dp >= DA ? 0 : dp >= DB ? 1 : 2; }
// fraction bits of guess row DP: the rows of the lowest dimensions grow slowly and get finer buckets
constexpr int pvq_walk_mb(int dp) { return dp == 2 ? 5 : dp == 3 ? 4 : 3; }
// entries of guess row DP: every value of the row's integer type (entry_bits wide) lands inside
constexpr uint32_t pvq_walk_guess_entries(int dp, int entry_bits) { return ((uint32_t)(entry_bits + 3) << pvq_walk_mb(dp)) + 1u; }
constexpr int pvq_walk_entry_bits(int dp, int W, int DA, int DB) { return (32 * W) >> pvq_walk_class(dp, DA, DB); }
// byte offset of guess row DP behind guess_base
constexpr uint32_t pvq_walk_guess_offset(int dp, int W, int DA, int DB)
{
    uint32_t off = 0;
    for (int j = 2; j < dp; j++) off += pvq_walk_guess_entries(j, pvq_walk_entry_bits(j, W, DA, DB));
    return off;
}
// rows 1 .. dp-1 lie in front of row dp: how many of each width class
constexpr int pvq_walk_rows_before(int dp, int cls, int DA, int DB)
{
    int n = 0;
    for (int j = 1; j < dp; j++) n += pvq_walk_class(j, DA, DB) == cls;
    return n;
}
// byte offset of U(DP, 0) (the row starts one entry earlier, with U(DP,-1) = 0)
template <int DP, int W, int DA, int DB>
PVQ_HD uint32_t pvq_walk_row(const pvq_walk_params &p)
{
    return p.row_bytes[0] * (uint32_t)pvq_walk_rows_before(DP, 0, DA, DB) + p.row_bytes[1] * (uint32_t)pvq_walk_rows_before(DP, 1, DA, DB) +
           p.row_bytes[2] * (uint32_t)pvq_walk_rows_before(DP, 2, DA, DB) + (uint32_t)(pvq_walk_entry_bits(DP, W, DA, DB) / 8);
}

// Place of h among the buckets of a guess row with MB fraction bits: 0 for h = 0, else 1 + (e << MB) + f for
// h in [2^e (1 + f / 2^MB), 2^e (1 + (f+1) / 2^MB)), or the bucket below when h lies within 2^-20 (relative)
// of the bucket's lower edge: conversions and sums round to nearest, the last factor takes back more than
// they can add, so the float is not above h.
template <int MB>
PVQ_HD uint32_t bucket_of_float(float f, uint32_t cap)
{
    f *= 1.0f - 0x1p-21f;
    constexpr uint32_t base = (127u << MB) - 1u;
    const uint32_t idx = std::max(pvq_float_bits(f) >> (23u - MB), base) - base;
    return std::min(idx, cap);
}

// Half of q as the integer h, and its bucket.  For two-word integers h is put together from the two words that
// the conversion to float uses, so that the shift is made once.
template <typename T, int MB>
PVQ_HD uint32_t half_and_bucket(T q, T &h)
{
    if constexpr (sizeof(T) == 4) {
        h = q >> 1;
        return bucket_of_float<MB>((float)h, 0xFFFFFFFFu);
    } else if constexpr (sizeof(T) == 8) {
        uint32_t hi = (uint32_t)(q >> 33);
        const uint32_t lo = (uint32_t)(q >> 1);
        PVQ_WALK_OPAQUE(hi);
        h = ((T)hi << 32) | lo;
        return bucket_of_float<MB>(fmaf((float)hi, 4294967296.0f, (float)lo), 0xFFFFFFFFu);
    } else {
        h = q >> 1;
        uint32_t w3 = (uint32_t)(h >> 96), w2 = (uint32_t)(h >> 64), w1 = (uint32_t)(h >> 32);
        PVQ_WALK_OPAQUE(w3); PVQ_WALK_OPAQUE(w2); PVQ_WALK_OPAQUE(w1);
        float f = fmaf((float)w3, 4294967296.0f, (float)w2);
        f = fmaf(f, 4294967296.0f, (float)w1);
        f = fmaf(f, 4294967296.0f, (float)(uint32_t)h);
        return bucket_of_float<MB>(f, 130u << MB);                            // 2^128 - 1 rounds to infinity
    }
}

// One coordinate with d = DP + 1 dimensions left (row DP of the cumulative table) under the schedule
// <W, DA, DB>.  q, k in and out; returns the coordinate's magnitude, sets `negative` and adds the square to n2.
template <typename T, int DP, int W, int DA, int DB>
PVQ_HD uint32_t walk_step(const unsigned char *lds, const pvq_walk_params &p, T &q, int &k, int &n2, bool &negative)
{
    T h;
    uint32_t C;
    T um, ux;
    if constexpr (DP == 1) {
        // U(1,x) = 2x + 1
        h = q >> 1;
        C = (uint32_t)std::min<T>((h + 1) >> 1, (T)(uint32_t)k);
        ux = (T)(2u * C + 1u);
        um = C ? (T)(2u * C - 1u) : (T)0;
    } else {
        const uint32_t idx = half_and_bucket<T, pvq_walk_mb(DP)>(q, h);
        C = lds[p.guess_base + pvq_walk_guess_offset(DP, W, DA, DB) + idx];
        const T *u = reinterpret_cast<const T *>(lds + pvq_walk_row<DP, W, DA, DB>(p));   // u[x] = U(DP, x), x = -1 .. K+1
        um = u[(int)C - 1];
        ux = u[C];
        const T up = u[C + 1];
        if (ux <= h) { C++; um = ux; ux = up; }
        while (ux <= h) { C++; um = ux; ux = u[C]; }                          // ends: u[K+1] is all ones
        C = std::min(C, (uint32_t)k);                                          // (a stored index >= N(D,K) only)
    }
    const uint32_t m = (uint32_t)k - C;
    const T t = q - um;
    negative = t < ux;
    q = negative ? t - um : t - ux;
    k = (int)C;
#if defined(__HIP_DEVICE_COMPILE__)
    n2 += __mul24((int)m, (int)m);                  // m <= K < 2^12
#else
    n2 += (int)(m * m);
#endif
    return m;
}

// The state of a walk: the residual in the three widths (one of them is live at a time), pulses left, sum of
// squares.  coordinate<I>() decodes coordinate I (dimensions left: D - I) in the width of its schedule.
template <int D, int W, int DA, int DB>
struct walk_state {
    using T0 = typename wide<W>::type;
    using T1 = typename wide<(W >= 2 ? W / 2 : 1)>::type;
    using T2 = typename wide<(W >= 4 ? W / 4 : 1)>::type;
    T0 q0;
    T1 q1;
    T2 q2;
    int k, n2;

    template <int I, typename Emit>
    PVQ_HD void coordinate(const unsigned char *lds, const pvq_walk_params &p, Emit &emit)
    {
        constexpr int d = D - I;                 // dimensions left, this coordinate included
        uint32_t v;
        bool negative;
        if constexpr (d > DA) {
            v = walk_step<T0, d - 1, W, DA, DB>(lds, p, q0, k, n2, negative);
            if constexpr (d - 1 == DA) q1 = (T1)q0;          // the next coordinate runs in the narrower type
            if constexpr (d - 1 == DA && DA == DB) q2 = (T2)q0;
        } else if constexpr (d > DB) {
            v = walk_step<T1, d - 1, W, DA, DB>(lds, p, q1, k, n2, negative);
            if constexpr (d - 1 == DB) q2 = (T2)q1;
        } else {
            v = walk_step<T2, d - 1, W, DA, DB>(lds, p, q2, k, n2, negative);
        }
        emit(I, v, negative);
    }
    template <typename Emit, int... Is>
    PVQ_HD void all(const unsigned char *lds, const pvq_walk_params &p, Emit &emit, std::integer_sequence<int, Is...>)
    {
        (coordinate<Is>(lds, p, emit), ...);
    }
};

// The whole point from its index c.  emit(i, |y_i|, y_i < 0) for i = 0 .. D-1 in order (a coordinate that is 0
// may come with either sign); returns sum y_i^2.
template <int D, int W, int DA, int DB, typename Emit>
PVQ_HD int unrank_walk(typename wide<W>::type c, const unsigned char *lds, const pvq_walk_params &p,
                                  Emit &&emit)
{
    using T0 = typename wide<W>::type;
    static_assert(DA < D && DB <= DA, "width schedule");
    const int K = p.K;
    const T0 *u0 = reinterpret_cast<const T0 *>(lds + pvq_walk_row<D - 1, W, DA, DB>(p));
    walk_state<D, W, DA, DB> st;
    st.q0 = u0[K] + u0[K - 1] - 1 - c;          // N(D,K) - 1 - c
    st.q1 = 0; st.q2 = 0; st.k = K; st.n2 = 0;
    st.all(lds, p, emit, std::make_integer_sequence<int, D - 1>{});
    // the two points +k, -k of P(1,k): q = 1, 0
    bool zero;
    if constexpr (DB >= 1) zero = st.q2 == 0;
    else if constexpr (DA >= 1) zero = st.q1 == 0;
    else zero = st.q0 == 0;
    emit(D - 1, (uint32_t)st.k, zero);
    return st.n2 + st.k * st.k;
}


}  // namespace pvq_walk

// Which width schedule a context gets: fit_half / fit_quarter = the largest number of dimensions d whose
// N(d,K) fits half / a quarter of the index's words.  Names only schedules listed in PVQ_WALK_DISPATCH.
inline void pvq_walk_schedule(int D, int words, int fit_half, int fit_quarter, int *dA, int *dB)
{
    *dA = 0; *dB = 0;
    if (D == 16 && words == 2 && fit_half >= 8) *dA = 8;
    if (D == 32 && words == 2 && fit_half >= 12) *dA = 12;
    if (D == 32 && words == 4 && fit_half >= 15 && fit_quarter >= 6) { *dA = 15; *dB = 6; }
}

// The instantiated width schedules <D, W, DA, DB>: CALL(D, W, DA, DB) for the schedule (dA, dB) chosen for a
// context of group size D with `words`-word indices.
#define PVQ_WALK_DISPATCH(CALL, D_, W_, dA_, dB_)                                                       \
    do {                                                                                                \
        if ((D_) == 8) {                                                                                \
            if ((W_) == 1) return CALL(8, 1, 0, 0);                                                     \
            return CALL(8, 2, 0, 0);                                                                    \
        }                                                                                               \
        if ((D_) == 16) {                                                                               \
            if ((W_) == 1) return CALL(16, 1, 0, 0);                                                    \
            if ((W_) == 2) { if ((dA_) == 8) return CALL(16, 2, 8, 0); return CALL(16, 2, 0, 0); }      \
            return CALL(16, 4, 0, 0);                                                                   \
        }                                                                                               \
        if ((W_) == 1) return CALL(32, 1, 0, 0);                                                        \
        if ((W_) == 2) { if ((dA_) == 12) return CALL(32, 2, 12, 0); return CALL(32, 2, 0, 0); }        \
        if ((dA_) == 15 && (dB_) == 6) return CALL(32, 4, 15, 6);                                       \
        return CALL(32, 4, 0, 0);                                                                       \
    } while (0)
