// Device code shared by the kernels that quantise a group onto the pyramid (Sec. 2.5): the encoders and
// the error correction of Sec. 3.3 Step 6.  float32, fixed evaluation order: the results are part of the
// format.  The point: project onto the l1 ball of radius K, round to nearest even, then move single pulses on
// the coordinates of largest deviation (lowest coordinate on ties) until the count is K.  quantize_group8 finds
// it without branches for D = 8 (count_wins); the D = 8 encoder and quantize_group_select<D>, for any D, take one
// round per pulse to move (first_places8 for D = 8).
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

// adj[i] = coordinate i holds one of the `need` first places in the order of keys (largest first, lower coordinate
// first on ties).  A round takes the largest key left (three-operand maxima), marks the first coordinate that has
// it and takes its key out; a wave runs as many rounds as its lane with the largest `need`, two or three for
// groups of 8, at 20 instructions each, against a hundred for count_wins: the form for kernels that are short of
// vector instructions (the encoders).  Changes key.
__device__ inline void first_places8(float (&key)[8], int need, bool (&adj)[8])
{
#pragma unroll
    for (int i = 0; i < 8; i++) adj[i] = false;
    for (int round = 0; round < 8; round++) {
        if (!__any(round < need)) break;
        const float best = fmaxf(fmaxf(fmaxf(key[0], key[1]), fmaxf(key[2], key[3])),
                                 fmaxf(fmaxf(key[4], key[5]), fmaxf(key[6], key[7])));
        bool taken = !(round < need);             // a lane that needs no more takes nothing
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const bool hit = !taken && key[i] == best;
            adj[i] = adj[i] || hit;
            taken = taken || hit;
            key[i] = hit ? -INFINITY : key[i];
        }
    }
}

// Groups of 8 without branches (for the error correction, whose waves wait for one group after the other: rounds
// with a wave-wide vote measured 2 % slower there): the coordinates' places in the order of deviations are counted
// with 28 comparisons and the |sum - K| first places are adjusted, which equals the one-at-a-time repair because no
// coordinate is ever adjusted twice (for finite input the |sum - K| largest deviations are all positive, and an
// adjusted coordinate drops below -1/2).  Returns the sum of squares; y gets the signed point.  Weights that are
// not finite give (0, ..., 0, K).
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

// The same point for any D, without the two repair loops' re-evaluation of every deviation: the deviations are
// formed once (as keys, negated when pulses have to be taken away), and each of the |sum - K| rounds picks the
// largest key, lowest coordinate on ties, adjusts that coordinate and takes its key out.  This is the one-at-a-time
// repair itself, since an adjusted coordinate never comes up again (see quantize_group8); a wave runs as many rounds
// as its lane with the largest |sum - K| needs, two to five for D = 16 and 32 (re-evaluating all deviations in every
// round, in one loop for pulses to take away and one for pulses to add, took 2.5 times the instructions).
// Weights that are not finite give (0, ..., 0, K).
template <int D>
__device__ inline float quantize_group_select(const float (&w)[D], int K, int (&y)[D])
{
    float a[D], tmp[D];
#pragma unroll
    for (int i = 0; i < D; i++) { a[i] = fabsf(w[i]); tmp[i] = a[i]; }
    const float l1 = tree_sum<D>(tmp);
#pragma unroll
    for (int i = 0; i < D; i++) tmp[i] = w[i] * w[i];
    const float ss = tree_sum<D>(tmp);
    const float g = (float)K / l1;
    const bool degenerate = !(l1 > 0.0f) || !(l1 < INFINITY) || !(g < INFINITY);
    float key[D], yf[D];
    float S = 0.0f;
#pragma unroll
    for (int i = 0; i < D; i++) {
        const float t = a[i] * g;
        yf[i] = rintf(t);
        S += yf[i];                       // small integers: exact in any order
        key[i] = t - yf[i];
    }
    const float m = (float)K - S;         // > 0: pulses to add, < 0: pulses to take away
    const float unit = m < 0.0f ? -1.0f : 1.0f;
    if (m < 0.0f) {
#pragma unroll
        for (int i = 0; i < D; i++) key[i] = -key[i];
    }
    const int need = degenerate ? 0 : (int)fminf(fabsf(m), (float)D);
    for (int round = 0; round < D; round++) {
        if (!__any(round < need)) break;
        float best = key[0];
        int at = 0;
#pragma unroll
        for (int i = 1; i < D; i++) {
            const bool take = key[i] > best;
            best = take ? key[i] : best;
            at = take ? i : at;
        }
        if (round < need) {
#pragma unroll
            for (int i = 0; i < D; i++) {
                const bool hit = i == at;
                yf[i] += hit ? unit : 0.0f;
                key[i] = hit ? -INFINITY : key[i];
            }
        }
    }
    int k = K;
#pragma unroll
    for (int i = 0; i < D; i++) {
        int mag = degenerate ? 0 : (int)yf[i];
        if (i == D - 1) mag = k;                      // the last coordinate takes what is left
        y[i] = (w[i] < 0.0f && !degenerate) ? -mag : mag;
        k -= mag;
    }
    return ss;
}

}  // namespace pvq_quantize_dev
