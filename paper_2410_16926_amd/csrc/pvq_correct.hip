// Correcting the quantisation error group after group (Sec. 3.3 Step 6), rows of W in place.
//
// For every row, groups g = 0 .. G-1 in order: the group's current values w_g are quantised as in Steps 3
// and 4 (point y, amplitude s), q = (s / sqrt(sum y^2)) y, e = w_g - q, and the columns behind the group
// take up the error:  t U_gg = e by substitution, then w_c <- w_c - t_0 U[gD][c] - ... - t_{D-1} U[gD+D-1][c],
// with U the upper triangular factor of the inverse Hessian (U^T U = H^-1).  float32; every "- t_i U" is
// one fused multiply-add applied in the order i = 0, 1, ... to the running value, group after group: the
// order is part of the definition, because later roundings are decided from these values.  On return W
// holds, for every group, the values that were quantised: encoding it gives the corrected code.
//
// Rows are independent, groups of a row strictly sequential, and U is the same for every row.  Columns are
// taken in panels of 128.  Panel p takes two launches on the caller's stream:
//   correct_narrow_kernel  panel p - 1's 128 multiply-adds per element onto the columns of panel p, which is all that
//           panel p waits for: tiles of 16 rows x 128 columns, so that even a few rows spread over many compute units.
//   correct_step_kernel    workgroups with one of two roles:
//     panel   (the first ceil(rows / 64) workgroups) 64 rows of panel p, one lane per row, four waves that own the
//             panel's groups in turn: the owner of a group quantises it and publishes its t values, the other
//             waves meanwhile bring their own later groups up to date.  Leaves the panel's t values (rows x 128) in a
//             work buffer.  Bound by the latency of one wave's quantiser and substitution, 128 / D times in a row.
//     update  (all others) panel p - 1's 128 multiply-adds per element, in the same order, for the columns
//             behind panel p: tiles of 128 rows x 128 columns, 8 x 8 per lane, t and U tiles in LDS (32 rows
//             of U at a time), W read and written once per panel.  Bound: float32 vector ALU.
// The two roles touch different columns, and the update reads panel p - 1's t values while the panel role writes
// panel p's, which is why there are two work buffers used in turn.  The panel workgroups come first in the grid
// and raise their waves' priority, so they are placed before the flood of update tiles and run beside it: the
// chain of panels (each needs the one before) stays off the critical path as long as a launch has enough update
// tiles to outlast it; with few rows the chain is what remains.  Both roles need the same LDS (33 KB), four
// workgroups per compute unit.
// Not on the matrix cores: their accumulation order inside an instruction is not the one defined above.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>

#include "pvq_internal.h"
#include "pvq_quantize_dev.h"

namespace {

using namespace pvq_quantize_dev;

constexpr int kPanelCols = 128;   // columns per panel
constexpr int kPanelWaves = 4;    // waves of a workgroup: group g of the panel belongs to wave g % 4
constexpr int kThreads = 64 * kPanelWaves;
constexpr int kTile = 128;        // rows and columns of an update tile
constexpr int kStage = 32;        // rows of U (and t values per row) that an update tile holds in LDS at a time
// update tiles from which on a launch's panel workgroups do the narrow update themselves (one and a half rounds of
// four workgroups on each of 256 units); a test lowers it to reach that path with small matrices
std::atomic<int64_t> g_front_tiles{1536};
constexpr int kLdsFloats = kStage * (kTile + 4) + kStage * kTile;   // update: t tile and U tile; panel: 128 x 64 t values
static_assert(kLdsFloats >= kPanelCols * 64, "the panel role's t values fit");

struct correct_shape {
    int64_t ldw, rows, cols, ldu;
    int K, ls;
};

// Panel role.  Lane = row in each of the four waves; wave w holds the values of groups w, w + 4, ... of its rows
// in registers.
//   With `front` (a launch with enough update tiles to outlast it), first the panel before's 128 multiply-adds per
// element onto this panel's columns, which otherwise a launch of correct_narrow_kernel has done.
//   Step G (one barrier per step): the owner of group G applies to it the updates of group G - 1 (the only ones
// still missing: it caught up with the rest one step earlier), stores what is then quantised to W, runs
// quantiser, amplitude, error and substitution, and puts the t values into LDS and the work buffer; the other
// waves apply the t values published so far to all groups they still own.  Per element these are the same
// multiply-adds in the same order (rows of U ascending) as if every group had updated all later columns at
// once.  The owner's step is the chain's length: one group's quantiser plus D rows of updates.
//   U is the same for every lane.  No wave is ever more than two groups behind, so step G reads the rows of U of
// groups G - 2, G - 1 and G only (and the t values of G - 2 and G - 1).  D = 8: rings of four groups in LDS, rows
// of U ([slot][row][128 columns], the rows of group G + 1 are fetched during step G) and t values
// ([slot][column][lane]).  D = 16, 32: such rings would not leave LDS for four workgroups per compute unit; all
// t values of the panel are kept, and the rows of U come through scalar loads (the pointer is read-only for the
// kernel and the address is the same in all lanes), which costs the owner a few exposed load latencies per step.
template <int D>
__device__ inline void panel_role(float *__restrict__ W, const float *__restrict__ U, const float *__restrict__ Tprev,
                                  float *__restrict__ Tcur, const correct_shape &a, int64_t p0, int width, bool front,
                                  float *lds)
{
    constexpr int NG = kPanelCols / D, OWN = NG / kPanelWaves;
    constexpr bool kRing = D == 8;
    constexpr int R = 4;                                        // slots of the rings
    static_assert(!kRing || (D * kPanelCols / 4 == kThreads && R * D * (kPanelCols + 64) <= kLdsFloats), "a float4 per lane fills a slot");
    float *uring = lds;                                         // [slot][row of the group][column of the panel]
    float *ts = kRing ? lds + R * D * kPanelCols : lds;         // ring: [slot][column of the group][lane]; else [column][lane]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t r = (int64_t)blockIdx.x * 64 + lane;
    const bool in = r < a.rows;
    // lanes beyond the rows work on the last row again (no lane waits for another); they store nothing
    const int64_t row = in ? r : a.rows - 1;
    float *wrow = W + row * a.ldw + p0;
    const int ngroups = width / D;
    const float *Up = U + p0 * a.ldu + p0;                      // row p0 + k, column p0 + c of the factor

    float w[OWN][D];
#pragma unroll
    for (int o = 0; o < OWN; o++) {
        const int g = wave + kPanelWaves * o;
#pragma unroll
        for (int i = 0; i < D; i += 4) {
            const float4 q = *reinterpret_cast<const float4 *>(wrow + (g < ngroups ? g : 0) * D + i);
            w[o][i] = q.x; w[o][i + 1] = q.y; w[o][i + 2] = q.z; w[o][i + 3] = q.w;
        }
    }

    if (front) {
        // w <- w - t'[0] U[p0 - 128][c] - ... - t'[127] U[p0 - 1][c] for the wave's 32 columns c, t' = the panel before's
        // t values of the row: 32 rows of U and 32 t values per row go through LDS at a time, fetched into
        // registers while the 32 before are worked on
        constexpr int kChunk = 32, kTPitch = 65;                // t values transposed: [k][row], rows 65 words apart
        float *uc = lds, *tc = lds + kChunk * kPanelCols;
        static_assert((kChunk + 1) * kPanelCols + (kChunk + 1) * kTPitch <= kLdsFloats, "a chunk fits, and a row more may be read");
        const float *Ub = U + (p0 - kPanelCols) * a.ldu + p0;   // row p0 - 128 + k, column p0 + c
        const int64_t row0 = (int64_t)blockIdx.x * 64;
        float4 uq[4], tq[2];
        auto fetch = [&](int chunk) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int e = threadIdx.x + i * kThreads, k = e / (kPanelCols / 4), c = (e % (kPanelCols / 4)) * 4;
                uq[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (c < width) uq[i] = *reinterpret_cast<const float4 *>(Ub + (int64_t)(chunk * kChunk + k) * a.ldu + c);
            }
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int e = threadIdx.x + i * kThreads, rr = e / (kChunk / 4), k4 = (e % (kChunk / 4)) * 4;
                const int64_t rsrc = std::min<int64_t>(row0 + rr, a.rows - 1);
                tq[i] = *reinterpret_cast<const float4 *>(Tprev + rsrc * kPanelCols + chunk * kChunk + k4);
            }
        };
        fetch(0);
        for (int chunk = 0; chunk < kPanelCols / kChunk; chunk++) {
            if (chunk) __syncthreads();                         // the chunk before is no longer read
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const int e = threadIdx.x + i * kThreads, k = e / (kPanelCols / 4), c = (e % (kPanelCols / 4)) * 4;
                *reinterpret_cast<float4 *>(uc + k * kPanelCols + c) = uq[i];
            }
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int e = threadIdx.x + i * kThreads, rr = e / (kChunk / 4), k4 = (e % (kChunk / 4)) * 4;
                tc[k4 * kTPitch + rr] = tq[i].x; tc[(k4 + 1) * kTPitch + rr] = tq[i].y;
                tc[(k4 + 2) * kTPitch + rr] = tq[i].z; tc[(k4 + 3) * kTPitch + rr] = tq[i].w;
            }
            __syncthreads();
            if (chunk + 1 < kPanelCols / kChunk) fetch(chunk + 1);
            // the wave's 32 values of a row of U: one half on its way while the other is worked on (past the last
            // row of a chunk the words behind it are read and not used)
            auto half_row = [&](int k, int h, float4 (&q)[OWN * D / 8]) {
                const float *urow = uc + k * kPanelCols;
#pragma unroll
                for (int i = 0; i < OWN * D / 8; i++) {
                    const int col = h * (OWN * D / 2) + 4 * i;          // of the wave's values: group col / D, value col % D
                    q[i] = *reinterpret_cast<const float4 *>(urow + (wave + kPanelWaves * (col / D)) * D + col % D);
                }
            };
            auto half_fma = [&](float tk, int h, const float4 (&q)[OWN * D / 8]) {
#pragma unroll
                for (int i = 0; i < OWN * D / 8; i++) {
                    const int col = h * (OWN * D / 2) + 4 * i, o = col / D, j = col % D;
                    w[o][j] = __builtin_fmaf(-tk, q[i].x, w[o][j]);
                    w[o][j + 1] = __builtin_fmaf(-tk, q[i].y, w[o][j + 1]);
                    w[o][j + 2] = __builtin_fmaf(-tk, q[i].z, w[o][j + 2]);
                    w[o][j + 3] = __builtin_fmaf(-tk, q[i].w, w[o][j + 3]);
                }
            };
            float4 qa[OWN * D / 8], qb[OWN * D / 8];
            half_row(0, 0, qa);
            float tk = tc[lane];
#pragma unroll 2
            for (int k = 0; k < kChunk; k++) {
                half_row(k, 1, qb);
                half_fma(tk, 0, qa);
                half_row(k + 1, 0, qa);
                const float tn = tc[(k + 1) * kTPitch + lane];
                half_fma(tk, 1, qb);
                tk = tn;
            }
        }
        __syncthreads();                                        // LDS now takes this panel's rows of U and t values
    }

    // the rows of U of group g, from device memory to the ring: a float4 per lane
    const int ring_k = threadIdx.x / (kPanelCols / 4), ring_c = (threadIdx.x % (kPanelCols / 4)) * 4;
    auto ring_fetch = [&](int g) {
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (g < ngroups && ring_c < width) v = *reinterpret_cast<const float4 *>(Up + (int64_t)(g * D + ring_k) * a.ldu + ring_c);
        return v;
    };
    auto ring_store = [&](int g, const float4 &v) {
        *reinterpret_cast<float4 *>(uring + ((g % R) * D + ring_k) * kPanelCols + ring_c) = v;
    };
    if constexpr (kRing) {
        ring_store(0, ring_fetch(0));
        __syncthreads();
    }
    // row k of the panel's part of U from column c on, and the t values of column k
    auto u_at = [&](int k, int c) -> const float * {
        if constexpr (kRing) return uring + (((k / D) % R) * D + k % D) * kPanelCols + c;
        else return Up + (int64_t)k * a.ldu + c;
    };
    auto t_at = [&](int k) -> float * {
        if constexpr (kRing) return ts + (((k / D) % R) * D + k % D) * 64 + lane;
        else return ts + k * 64 + lane;
    };
    float *trow = Tcur + row * kPanelCols;
    // rows k0 .. k1 - 1 of the panel's part of U, times the t values of those columns, onto group g's values
    auto apply = [&](float (&v)[D], int g, int k0, int k1) {
        constexpr int kRowsAhead = 64 / D;    // rows of U on their way at a time
#pragma unroll kRowsAhead
        for (int k = k0; k < k1; k++) {
            const float tk = *t_at(k);
            const float *u = u_at(k, g * D);
            float uv[D];
#pragma unroll
            for (int j = 0; j < D; j += 4) {
                const float4 q = *reinterpret_cast<const float4 *>(u + j);
                uv[j] = q.x; uv[j + 1] = q.y; uv[j + 2] = q.z; uv[j + 3] = q.w;
            }
#pragma unroll
            for (int j = 0; j < D; j++) v[j] = __builtin_fmaf(-tk, uv[j], v[j]);
        }
    };

    int applied = 0;   // the wave's groups that are still to come hold the updates of groups 0 .. applied - 1
#pragma unroll
    for (int o = 0; o < OWN; o++) {
#pragma unroll 1
        for (int turn = 0; turn < kPanelWaves; turn++) {
            const int G = kPanelWaves * o + turn;
            if (G >= ngroups) break;                  // the same for every wave
            float4 ahead;
            if constexpr (kRing) ahead = ring_fetch(G + 1);
            if (wave == turn) {
                float (&wg)[D] = w[o];
                apply(wg, G, applied * D, G * D);
                // what is quantised, and stays in W
                if (in) {
#pragma unroll
                    for (int i = 0; i < D; i += 4) *reinterpret_cast<float4 *>(wrow + G * D + i) = make_float4(wg[i], wg[i + 1], wg[i + 2], wg[i + 3]);
                }
                int y[D];
                float ss;
                if constexpr (D == 8) ss = quantize_group8(wg, a.K, y);
                else ss = quantize_group_select<D>(wg, a.K, y);
                const float s = a.ls ? pvq_ls_amplitude<D>(wg, y) : sqrtf(ss);
                int n2 = 0;
#pragma unroll
                for (int i = 0; i < D; i++) n2 += y[i] * y[i];
                const float gain = s / sqrtf((float)n2);
                // t U_GG = e, row after row of the group's own D x D part: t_i is final once rows 0 .. i - 1 have been
                // taken off e_i (for every e_j the multiply-adds come in the order of the rows)
                float t[D];
#pragma unroll
                for (int j = 0; j < D; j++) t[j] = wg[j] - gain * (float)y[j];
#pragma unroll
                for (int i = 0; i < D; i++) {
                    const float *u = u_at(G * D + i, G * D);
                    float ui[D];
#pragma unroll
                    for (int j = 0; j < D; j += 4) {
                        const float4 q = *reinterpret_cast<const float4 *>(u + j);
                        ui[j] = q.x; ui[j + 1] = q.y; ui[j + 2] = q.z; ui[j + 3] = q.w;
                    }
                    t[i] = t[i] / ui[i];
#pragma unroll
                    for (int j = i + 1; j < D; j++) t[j] = __builtin_fmaf(-t[i], ui[j], t[j]);
                }
#pragma unroll
                for (int j = 0; j < D; j++) *t_at(G * D + j) = t[j];
                if (in) {
#pragma unroll
                    for (int i = 0; i < D; i += 4) *reinterpret_cast<float4 *>(trow + G * D + i) = make_float4(t[i], t[i + 1], t[i + 2], t[i + 3]);
                }
            } else {
#pragma unroll
                for (int oo = 0; oo < OWN; oo++) {
                    const int g = wave + kPanelWaves * oo;
                    if (g > G && g < ngroups) apply(w[oo], g, applied * D, G * D);
                }
                applied = G;
            }
            if constexpr (kRing) ring_store(G + 1, ahead);      // a slot that no wave reads during this step
            __syncthreads();      // the step's t values, and the next group's rows of U, are in LDS
        }
    }
}

// Update role.  Tile (row tile, column tile) of the columns [c1, cols): W[r][c] <- W[r][c] - t[r][0] U[c0][c] - ...
// - t[r][127] U[c0 + 127][c], one multiply-add after the other, t = the t values of the panel at column c0; the
// tile of W is read and written once for its 128 multiply-adds per element (with 64 per pass the update was
// bound by HBM as much as by the vector ALU).  A stage = 32 rows of U and 32 t values per row in LDS (with 64
// per stage, and two workgroups per compute unit, it ran at 57 instead of 66 TFLOP/s).
// Neighbouring workgroups share the tile of U.
__device__ inline void update_role(float *__restrict__ W, const float *__restrict__ U, const float *__restrict__ T,
                                   const correct_shape &a, int64_t c0, int64_t c1, int row_tile, int col_tile, float *lds)
{
    float (*Ts)[kTile + 4] = reinterpret_cast<float (*)[kTile + 4]>(lds);               // [k][row of the tile]
    float (*Us)[kTile] = reinterpret_cast<float (*)[kTile]>(lds + kStage * (kTile + 4)); // [k][column of the tile]
    const int64_t row0 = (int64_t)row_tile * kTile, col0 = c1 + (int64_t)col_tile * kTile;
    const int tid = threadIdx.x;
    const int ty = tid >> 4, tx = tid & 15;       // rows 8 ty .. 8 ty + 7, columns 8 tx .. 8 tx + 7 of the tile
    const bool cols_in = col0 + 8 * tx < a.cols;  // eight columns are in or out together
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int64_t r = row0 + 8 * ty + i;
        float4 v0 = make_float4(0.0f, 0.0f, 0.0f, 0.0f), v1 = v0;
        if (r < a.rows && cols_in) {
            const float *p = W + r * a.ldw + col0 + 8 * tx;
            v0 = *reinterpret_cast<const float4 *>(p); v1 = *reinterpret_cast<const float4 *>(p + 4);
        }
        acc[i][0] = v0.x; acc[i][1] = v0.y; acc[i][2] = v0.z; acc[i][3] = v0.w;
        acc[i][4] = v1.x; acc[i][5] = v1.y; acc[i][6] = v1.z; acc[i][7] = v1.w;
    }
    for (int st = 0; st < kPanelCols / kStage; st++) {
        if (st) __syncthreads();                  // the tiles of the stage before are no longer read
        // t tile: 128 rows x 32 values, a float4 per lane and pass, stored transposed
        for (int e = tid; e < kTile * (kStage / 4); e += kThreads) {
            const int rr = e / (kStage / 4), k4 = (e % (kStage / 4)) * 4;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (row0 + rr < a.rows) v = *reinterpret_cast<const float4 *>(T + (row0 + rr) * kPanelCols + st * kStage + k4);
            Ts[k4][rr] = v.x; Ts[k4 + 1][rr] = v.y; Ts[k4 + 2][rr] = v.z; Ts[k4 + 3][rr] = v.w;
        }
        // U tile: 32 rows x 128 columns (columns in whole fours: cols is a multiple of 64)
        for (int e = tid; e < kStage * (kTile / 4); e += kThreads) {
            const int k = e / (kTile / 4), cc = (e % (kTile / 4)) * 4;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (col0 + cc < a.cols) v = *reinterpret_cast<const float4 *>(U + (c0 + st * kStage + k) * a.ldu + col0 + cc);
            *reinterpret_cast<float4 *>(&Us[k][cc]) = v;
        }
        __syncthreads();
#pragma unroll 4
        for (int k = 0; k < kStage; k++) {
            const float4 a0 = *reinterpret_cast<const float4 *>(&Ts[k][8 * ty]), a1 = *reinterpret_cast<const float4 *>(&Ts[k][8 * ty + 4]);
            const float4 b0 = *reinterpret_cast<const float4 *>(&Us[k][8 * tx]), b1 = *reinterpret_cast<const float4 *>(&Us[k][8 * tx + 4]);
            const float tv[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const float uv[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int i = 0; i < 8; i++)
#pragma unroll
                for (int j = 0; j < 8; j++) acc[i][j] = __builtin_fmaf(-tv[i], uv[j], acc[i][j]);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int64_t r = row0 + 8 * ty + i;
        if (r < a.rows && cols_in) {
            float *p = W + r * a.ldw + col0 + 8 * tx;
            *reinterpret_cast<float4 *>(p) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
            *reinterpret_cast<float4 *>(p + 4) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
        }
    }
}

// Columns [c1, c1 + width) of all rows: W[r][c] <- W[r][c] - t[r][0] U[c0][c] - ... - t[r][127] U[c0 + 127][c], one
// multiply-add after the other, t = the t values of the panel at column c0 = c1 - 128.  16 rows x 128 columns per
// workgroup, 1 x 8 per lane; a stage = 32 rows of U and 32 t values per row in LDS.
__global__ __launch_bounds__(kThreads) void correct_narrow_kernel(float *__restrict__ W, const float *__restrict__ U,
                                                                   const float *__restrict__ T, correct_shape a, int64_t c1, int width)
{
    constexpr int RT = 16;
    __shared__ __align__(16) float Ts[kStage][RT + 4];      // [k][row of the tile]
    __shared__ __align__(16) float Us[kStage][kPanelCols];  // [k][column]
    const int64_t row0 = (int64_t)blockIdx.x * RT, c0 = c1 - kPanelCols;
    const int tid = threadIdx.x;
    const int ty = tid >> 4, tx = tid & 15;       // row ty, columns 8 tx .. 8 tx + 7 of the tile
    const int64_t r = row0 + ty;
    const bool mine = r < a.rows && 8 * tx < width;          // (width is 128 or 64: eight columns are in or out together)
    float acc[8];
    {
        float4 v0 = make_float4(0.0f, 0.0f, 0.0f, 0.0f), v1 = v0;
        if (mine) {
            const float *p = W + r * a.ldw + c1 + 8 * tx;
            v0 = *reinterpret_cast<const float4 *>(p); v1 = *reinterpret_cast<const float4 *>(p + 4);
        }
        acc[0] = v0.x; acc[1] = v0.y; acc[2] = v0.z; acc[3] = v0.w; acc[4] = v1.x; acc[5] = v1.y; acc[6] = v1.z; acc[7] = v1.w;
    }
    // t tile of a stage: 16 rows x 32 values = 128 float4 (lanes 0 .. 127), stored transposed; U tile: 32 rows x 128
    // columns = 4 float4 per lane.  All four stages are requested at once (80 registers): the workgroup's time is
    // one trip to memory plus its arithmetic, whatever the other workgroups of the compute unit do.
    constexpr int kStages = kPanelCols / kStage;
    const int t_rr = tid / (kStage / 4), t_k4 = (tid % (kStage / 4)) * 4;
    const bool t_lane = tid < RT * (kStage / 4);
    float4 tq[kStages], uq[kStages][4];
#pragma unroll
    for (int st = 0; st < kStages; st++) {
        tq[st] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (t_lane && row0 + t_rr < a.rows) tq[st] = *reinterpret_cast<const float4 *>(T + (row0 + t_rr) * kPanelCols + st * kStage + t_k4);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int e = tid + i * kThreads, k = e / (kPanelCols / 4), cc = (e % (kPanelCols / 4)) * 4;
            uq[st][i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (cc < width) uq[st][i] = *reinterpret_cast<const float4 *>(U + (c0 + st * kStage + k) * a.ldu + c1 + cc);
        }
    }
#pragma unroll
    for (int st = 0; st < kStages; st++) {
        if (st) __syncthreads();                  // the tiles of the stage before are no longer read
        if (t_lane) { Ts[t_k4][t_rr] = tq[st].x; Ts[t_k4 + 1][t_rr] = tq[st].y; Ts[t_k4 + 2][t_rr] = tq[st].z; Ts[t_k4 + 3][t_rr] = tq[st].w; }
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int e = tid + i * kThreads, k = e / (kPanelCols / 4), cc = (e % (kPanelCols / 4)) * 4;
            *reinterpret_cast<float4 *>(&Us[k][cc]) = uq[st][i];
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < kStage; k++) {
            const float tv = Ts[k][ty];
            const float4 b0 = *reinterpret_cast<const float4 *>(&Us[k][8 * tx]), b1 = *reinterpret_cast<const float4 *>(&Us[k][8 * tx + 4]);
            const float uv[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int j = 0; j < 8; j++) acc[j] = __builtin_fmaf(-tv, uv[j], acc[j]);
        }
    }
    if (mine) {
        float *p = W + r * a.ldw + c1 + 8 * tx;
        *reinterpret_cast<float4 *>(p) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4 *>(p + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

// The panel at column p0 (its own 128 or 64 columns, which have taken the panel before's update), and the
// panel before's update of the columns from p0 + 128 on.  Tprev: the t values of the panel before (unused for
// p0 = 0), Tcur: where this panel's go.  panel_wgs = ceil(rows / 64), row_tiles = ceil(rows / 128); the grid is
// panel_wgs + row_tiles * (column tiles behind the panel) workgroups, the latter none for p0 = 0.
// (at most 128 registers per lane, four workgroups per compute unit; 170 and three for groups of 32)
template <int D>
__global__ __launch_bounds__(kThreads, D == 32 ? 3 : 4) void correct_step_kernel(float *__restrict__ W, const float *__restrict__ U,
                                                                 const float *__restrict__ Tprev, float *__restrict__ Tcur,
                                                                 correct_shape a, int64_t p0, int width, int panel_wgs, int row_tiles,
                                                                 int front)
{
    __shared__ __align__(16) float lds[kLdsFloats];
    if ((int)blockIdx.x < panel_wgs) {
        // the chain's waves go first where they share a SIMD with update waves, which have plenty of others to fill in
        __builtin_amdgcn_s_setprio(2);
        panel_role<D>(W, U, Tprev, Tcur, a, p0, width, front != 0, lds);
    } else {
        const int tile = (int)blockIdx.x - panel_wgs;
        update_role(W, U, Tprev, a, p0 - kPanelCols, p0 + kPanelCols, tile % row_tiles, tile / row_tiles, lds);
    }
}

// W: rows x cols float32 (cols a multiple of 64), U: cols x cols, work: two buffers of rows x 128 floats.
hipError_t launch_correct(const pvq_ctx *c, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                          int64_t ldu, float *work, hipStream_t s)
{
    correct_shape a;
    a.ldw = ldw; a.rows = rows; a.cols = cols; a.ldu = ldu; a.K = c->K; a.ls = c->amplitude == PVQ_AMP_LS ? 1 : 0;
    const int panel_wgs = (int)((rows + 63) / 64), row_tiles = (int)((rows + kTile - 1) / kTile);
    int p = 0;
    for (int64_t p0 = 0; p0 < cols; p0 += kPanelCols, p++) {
        const int width = (int)std::min<int64_t>(kPanelCols, cols - p0);   // 128, or 64 at the end
        const int64_t behind = cols - (p0 + kPanelCols);
        const int col_tiles = p0 > 0 && behind > 0 ? (int)((behind + kTile - 1) / kTile) : 0;
        float *Tcur = work + (int64_t)(p & 1) * rows * kPanelCols, *Tprev = work + (int64_t)((p & 1) ^ 1) * rows * kPanelCols;
        // the panel before's update of this panel's columns: by the panel workgroups themselves (64 rows x 128 columns
        // x 128 terms on four waves: 25 us) where the launch's update tiles outlast that, else by a launch of its own
        // that spreads over the machine
        const int front = p0 > 0 && (int64_t)row_tiles * col_tiles >= g_front_tiles.load(std::memory_order_relaxed) ? 1 : 0;
        if (p0 > 0 && !front) hipLaunchKernelGGL(correct_narrow_kernel, dim3((unsigned)((rows + 15) / 16)), dim3(kThreads), 0, s, W, U, Tprev, a, p0, width);
        const dim3 grid((unsigned)(panel_wgs + row_tiles * col_tiles));
        switch (c->D) {
        case 8: hipLaunchKernelGGL((correct_step_kernel<8>), grid, dim3(kThreads), 0, s, W, U, Tprev, Tcur, a, p0, width, panel_wgs, row_tiles, front); break;
        case 16: hipLaunchKernelGGL((correct_step_kernel<16>), grid, dim3(kThreads), 0, s, W, U, Tprev, Tcur, a, p0, width, panel_wgs, row_tiles, front); break;
        default: hipLaunchKernelGGL((correct_step_kernel<32>), grid, dim3(kThreads), 0, s, W, U, Tprev, Tcur, a, p0, width, panel_wgs, row_tiles, front); break;
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Work buffers of the entry point that allocates nothing: the t values of two panels for up to kStaticRows rows
// (twice 128 floats per row), 8 MiB on every GPU that loads the library, until the process ends.
constexpr int64_t kStaticRows = 8192;
static __device__ __align__(256) float scratch[2 * kStaticRows * kPanelCols];

// The array's address on each device (in host code the array's name is only a stand-in for it), asked
// for once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
float *g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_on_current_device(float **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

hipError_t pvq_launch_correct(const pvq_ctx *c, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                              int64_t ldu, float *work, hipStream_t s)
{
    return launch_correct(c, W, rows, cols, ldw, U, ldu, work, s);
}

int64_t pvq_correct_static_max_rows(void) { return kStaticRows; }

int64_t pvq_correct_front_tiles(int64_t tiles) { return g_front_tiles.exchange(tiles); }

// The same launches with the library's own work buffers.
hipError_t pvq_launch_correct_static(const pvq_ctx *c, float *W, int64_t rows, int64_t cols, int64_t ldw,
                                     const float *U, int64_t ldu, hipStream_t s)
{
    if (rows > kStaticRows) return hipErrorInvalidValue;   // (the entry point has refused it already)
    float *work = nullptr;
    const hipError_t e = scratch_on_current_device(&work);
    if (e != hipSuccess) return e;
    return launch_correct(c, W, rows, cols, ldw, U, ldu, work, s);
}
