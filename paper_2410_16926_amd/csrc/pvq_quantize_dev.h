// Device code shared by the kernels that quantise a group onto the pyramid (Sec. 2.5): the encoders and
// the error correction of Sec. 3.3 Step 6.  float32, fixed evaluation order: the results are part of the
// format.  quantize_group<D> is the repair as a loop, for any D; quantize_group8 the same point without
// branches for D = 8, built on count_wins, which the D = 8 encoder uses as well.
#pragma once

#include <hip/hip_runtime.h>

namespace pvq_quantize_dev {

// Sum over adjacent pairs, level by level: ((v0+v1)+(v2+v3))+...  (fixed order, float32).
template <int D>
__device__ inline float tree_sum(float (&v)[D])
{
#pragma unroll
    for (int s = 1; s < D; s *= 2)
#pragma unroll
        for (int i = 0; i < D; i += 2 * s) v[i] = v[i] + v[i + s];
    return v[0];
}

// Sec. 2.5: project onto the l1 ball of radius K, round to nearest even, then move single pulses
// on the coordinates of largest deviation (lowest coordinate on ties) until the count is K.
// Returns the sum of squares; y gets the signed point.
template <int D>
__device__ inline float quantize_group(const float (&w)[D], int K, int (&y)[D])
{
    float a[D], t[D], tmp[D];
#pragma unroll
    for (int i = 0; i < D; i++) { a[i] = fabsf(w[i]); tmp[i] = a[i]; }
    const float l1 = tree_sum<D>(tmp);
#pragma unroll
    for (int i = 0; i < D; i++) tmp[i] = w[i] * w[i];
    const float ss = tree_sum<D>(tmp);

    const float g = (float)K / l1;
    if (!(l1 > 0.0f) || !(fabsf(g) < INFINITY)) {
#pragma unroll
        for (int i = 0; i < D; i++) y[i] = 0;
        y[D - 1] = K;
        return ss;
    }
    int S = 0;
#pragma unroll
    for (int i = 0; i < D; i++) {
        t[i] = a[i] * g;
        // a non-finite weight must not turn into an out-of-range pulse count
        float r = fminf(rintf(t[i]), (float)K);
        y[i] = r >= 0.0f ? (int)r : 0;
        S += y[i];
    }
    // At most D adjustments ever make sense (each coordinate moves at most once for finite
    // input); the bound also ends the loops for non-finite input.
    for (int it = 0; it < D && S > K; it++) {
        int best = -1;
        float dev = 0.0f;
#pragma unroll
        for (int i = 0; i < D; i++) {
            const float e = (float)y[i] - t[i];
            const bool take = y[i] > 0 && (best < 0 || e > dev);
            best = take ? i : best;
            dev = take ? e : dev;
        }
#pragma unroll
        for (int i = 0; i < D; i++) y[i] -= (i == best);
        S -= best >= 0;
    }
    for (int it = 0; it < D && S < K; it++) {
        int best = -1;
        float dev = 0.0f;
#pragma unroll
        for (int i = 0; i < D; i++) {
            const float e = t[i] - (float)y[i];
            const bool take = best < 0 || e > dev;
            best = take ? i : best;
            dev = take ? e : dev;
        }
#pragma unroll
        for (int i = 0; i < D; i++) y[i] += (i == best);
        S += 1;
    }
    if (S != K) {  // only reachable with non-finite input: fall back to a valid point
#pragma unroll
        for (int i = 0; i < D; i++) y[i] = 0;
        y[D - 1] = K;
        return ss;
    }
#pragma unroll
    for (int i = 0; i < D; i++) y[i] = w[i] < 0.0f ? -y[i] : y[i];
    return ss;
}

// Position of every coordinate in the order of keys (largest first, lower coordinate first on
// ties): wins[i] = number of coordinates that i comes before.  One comparison per pair feeds two
// counters through its carry: i's wins over later coordinates and j's losses against earlier ones.
__device__ inline void count_wins(const float (&key)[8], int (&wins)[8])
{
    constexpr int D = 8;
    int lose[D];
#pragma unroll
    for (int i = 0; i < D; i++) { wins[i] = 0; lose[i] = 0; }
#pragma unroll
    for (int i = 0; i < D; i++)
#pragma unroll
        for (int j = i + 1; j < D; j++) {
            const int first = key[i] >= key[j] ? 1 : 0;
            wins[i] += first;
            lose[j] += first;
        }
#pragma unroll
    for (int j = 0; j < D; j++) wins[j] += j - lose[j];   // j beat every earlier coordinate it did not lose to
}

// The quantiser above for groups of 8 without branches: the coordinates' places in the order of deviations
// are counted with 28 comparisons and the |sum - K| first places are adjusted, which equals the one-at-a-time
// repair because no coordinate is ever adjusted twice (for finite input the |sum - K| largest deviations are
// all positive, and an adjusted coordinate drops below -1/2).  Same results as quantize_group<8> for finite
// input; weights that are not finite give unspecified points.
__device__ inline float quantize_group8(const float (&w)[8], int K, int (&y)[8])
{
    constexpr int D = 8;
    float a[D], tmp[D];
#pragma unroll
    for (int i = 0; i < D; i++) { a[i] = fabsf(w[i]); tmp[i] = a[i]; }
    const float l1 = tree_sum<D>(tmp);
#pragma unroll
    for (int i = 0; i < D; i++) tmp[i] = w[i] * w[i];
    const float ss = tree_sum<D>(tmp);
    const float g = (float)K / l1;
    const bool degenerate = !(l1 > 0.0f) || !(l1 < INFINITY) || !(g < INFINITY);
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
        const float d = t[i] - yf[i];
        key[i] = m < 0.0f ? -d : d;
    }
    int wins[D];
    count_wins(key, wins);
    const int need = (int)fabsf(m);
    const float unit = m < 0.0f ? -1.0f : 1.0f;
    int k = K;
#pragma unroll
    for (int i = 0; i < D; i++) {
        const bool adjust = wins[i] + need >= D;      // place = D-1-wins < need
        int mag = (int)(yf[i] + (adjust ? unit : 0.0f));
        if (degenerate) mag = 0;
        if (i == D - 1) mag = k;                      // the last coordinate takes what is left
        y[i] = (w[i] < 0.0f && !degenerate) ? -mag : mag;
        k -= mag;
    }
    return ss;
}

}  // namespace pvq_quantize_dev
