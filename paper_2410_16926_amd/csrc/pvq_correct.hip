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
// taken in blocks of 64:
//   correct_block_kernel   one lane per row holds the block's 64 values in registers, goes through the
//                          block's groups (pending updates from the block's earlier groups, quantise,
//                          substitution) and leaves the block's t values (rows x 64) in a work buffer.  U is
//                          the same in every lane: its entries are read through the scalar unit and
//                          enter the multiply-adds as scalar operands.
//   correct_trailing_kernel  applies a block's 64 multiply-adds per element, in the same order, to columns
//                          behind it: 128 x 128 tiles, 8 x 8 per lane, t and U tiles in LDS (32 rows of U at a
//                          time).  Two blocks
//                          make a panel: the first block's update goes to the second block's columns
//                          only, and after the second block one launch applies both blocks' 128
//                          multiply-adds to everything behind the panel, reading and writing W once
//                          (with 64 per pass the kernel was bound by HBM as much as by the vector ALU).
//                          Bound: float32 vector ALU.
// Not on the matrix cores: their accumulation order inside an instruction is not the one defined above.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <utility>

#include "pvq_internal.h"
#include "pvq_quantize_dev.h"

namespace {

using namespace pvq_quantize_dev;

constexpr int kBlockCols = 64;    // columns per block
constexpr int kPanelCols = 128;   // columns per panel: two blocks, whose updates of the columns behind the panel go together
constexpr int kTile = 128;        // rows and columns of a tile of the trailing update
constexpr int kTrailThreads = 256;
constexpr int kStage = 32;        // rows of U (and t values per row) that the trailing update holds in LDS at a time

struct correct_args {
    float *W; int64_t ldw, rows, cols;
    const float *U; int64_t ldu;
    float *T;            // [rows][128]: the t values of the two blocks of a panel
    int K, ls;
};

// Group G of the block (a template parameter, so that every register index below is a constant).  First the
// group's columns take the updates of the block's earlier groups, which are still pending (rows 0 .. G D - 1
// of the block's part of U, in that order: per element the same multiply-adds in the same order as if every
// group had updated all later columns at once, with the entries of U read right where they are used);
// then quantise and substitution.  U points at the block's first diagonal entry; its entries are the same in
// every lane and are read through the scalar unit.  The fences keep the compiler from fetching many rows
// ahead, which the scalar registers do not hold.
template <int D, int G>
__device__ inline void block_step(float (&w)[kBlockCols], float (&t)[kBlockCols], const float *__restrict__ U, int64_t ldu,
                                  int K, int ls)
{
    float wg[D];
    int y[D];
#pragma unroll
    for (int i = 0; i < D; i++) wg[i] = w[G * D + i];
    // rows in batches of R, the next batch's entries of U requested before the current batch's
    // multiply-adds (a fence per batch: no more than two batches are ever in the scalar registers)
    constexpr int R = D >= 16 ? 2 : 4;
    float cur[R][D], nxt[R][D];
    if constexpr (G > 0) {
#pragma unroll
        for (int r = 0; r < R; r++)
#pragma unroll
            for (int j = 0; j < D; j++) cur[r][j] = U[(int64_t)r * ldu + G * D + j];
    }
#pragma unroll
    for (int k0 = 0; k0 < G * D; k0 += R) {
        __builtin_amdgcn_sched_barrier(0);
        if (k0 + R < G * D) {
#pragma unroll
            for (int r = 0; r < R; r++)
#pragma unroll
                for (int j = 0; j < D; j++) nxt[r][j] = U[(int64_t)(k0 + R + r) * ldu + G * D + j];
        }
#pragma unroll
        for (int r = 0; r < R; r++)
#pragma unroll
            for (int j = 0; j < D; j++) wg[j] = __builtin_fmaf(-t[k0 + r], cur[r][j], wg[j]);
#pragma unroll
        for (int r = 0; r < R; r++)
#pragma unroll
            for (int j = 0; j < D; j++) cur[r][j] = nxt[r][j];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < D; i++) w[G * D + i] = wg[i];   // what is quantised, and stays in W
    const float ss = quantize_group<D>(wg, K, y);
    const float s = ls ? pvq_ls_amplitude<D>(wg, y) : sqrtf(ss);
    int n2 = 0;
#pragma unroll
    for (int i = 0; i < D; i++) n2 += y[i] * y[i];
    const float gain = s / sqrtf((float)n2);
    const float *__restrict__ Ug = U + (int64_t)(G * D) * ldu + G * D;   // the group's D x D part
#pragma unroll
    for (int j = 0; j < D; j++) {
        float acc = wg[j] - gain * (float)y[j];
#pragma unroll
        for (int i = 0; i < j; i++) acc = __builtin_fmaf(-t[G * D + i], Ug[(int64_t)i * ldu + j], acc);
        t[G * D + j] = acc / Ug[(int64_t)j * ldu + j];
    }
}

template <int D, int... Gs>
__device__ inline void block_steps(float (&w)[kBlockCols], float (&t)[kBlockCols], const float *__restrict__ U, int64_t ldu,
                                   int K, int ls, std::integer_sequence<int, Gs...>)
{
    (block_step<D, Gs>(w, t, U, ldu, K, ls), ...);
}

template <int D>
__global__ __launch_bounds__(64) void correct_block_kernel(correct_args a, int64_t c0)
{
    const int64_t r = (int64_t)blockIdx.x * 64 + threadIdx.x;
    if (r >= a.rows) return;
    float *wrow = a.W + r * a.ldw + c0;
    const float *__restrict__ U = a.U + c0 * a.ldu + c0;   // row c0 + i, column c0 + c of the factor
    float w[kBlockCols], t[kBlockCols];
#pragma unroll
    for (int c = 0; c < kBlockCols; c += 4) {
        const float4 v = *reinterpret_cast<const float4 *>(wrow + c);
        w[c] = v.x; w[c + 1] = v.y; w[c + 2] = v.z; w[c + 3] = v.w;
    }
    block_steps<D>(w, t, U, a.ldu, a.K, a.ls, std::make_integer_sequence<int, kBlockCols / D>{});
    float *trow = a.T + r * kPanelCols + (c0 % kPanelCols);
#pragma unroll
    for (int c = 0; c < kBlockCols; c += 4) {
        *reinterpret_cast<float4 *>(wrow + c) = make_float4(w[c], w[c + 1], w[c + 2], w[c + 3]);
        *reinterpret_cast<float4 *>(trow + c) = make_float4(t[c], t[c + 1], t[c + 2], t[c + 3]);
    }
}

// Columns [c1, cend): W[r][c] <- W[r][c] - t[r][0] U[c0][c] - ... - t[r][n - 1] U[c0 + n - 1][c], n = 32 stages,
// one multiply-add after the other; t[r][k] = T[r][t0 + k].  n = 64: one block's update (of the second block
// of its panel); n = 128: a panel's update of everything behind it, with the tile of W read and written once
// for 128 multiply-adds per element.  A stage = 32 rows of U and 32 t values per row in LDS (33 KB, four
// workgroups per compute unit; with 64 per stage, two workgroups, the update ran at 57 instead of 66 TFLOP/s).
// blockIdx.x = row tile (neighbouring workgroups share the tile of U), blockIdx.y = column tile.
__global__ __launch_bounds__(kTrailThreads) void correct_trailing_kernel(correct_args a, int64_t c0, int t0, int stages,
                                                                          int64_t c1, int64_t cend)
{
    __shared__ __align__(16) float Ts[kStage][kTile + 4];   // [k][row of the tile]
    __shared__ __align__(16) float Us[kStage][kTile];       // [k][column of the tile]
    const int64_t row0 = (int64_t)blockIdx.x * kTile, col0 = c1 + (int64_t)blockIdx.y * kTile;
    const int tid = threadIdx.x;
    const int ty = tid >> 4, tx = tid & 15;       // rows 8 ty .. 8 ty + 7, columns 8 tx .. 8 tx + 7 of the tile
    const bool cols_in = col0 + 8 * tx < cend;    // eight columns are in or out together
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int64_t r = row0 + 8 * ty + i;
        float4 v0 = make_float4(0.0f, 0.0f, 0.0f, 0.0f), v1 = v0;
        if (r < a.rows && cols_in) {
            const float *p = a.W + r * a.ldw + col0 + 8 * tx;
            v0 = *reinterpret_cast<const float4 *>(p); v1 = *reinterpret_cast<const float4 *>(p + 4);
        }
        acc[i][0] = v0.x; acc[i][1] = v0.y; acc[i][2] = v0.z; acc[i][3] = v0.w;
        acc[i][4] = v1.x; acc[i][5] = v1.y; acc[i][6] = v1.z; acc[i][7] = v1.w;
    }
    for (int st = 0; st < stages; st++) {
        if (st) __syncthreads();                  // the tiles of the stage before are no longer read
        // t tile: 128 rows x 32 values, a float4 per lane and pass, stored transposed
        for (int e = tid; e < kTile * (kStage / 4); e += kTrailThreads) {
            const int rr = e / (kStage / 4), k4 = (e % (kStage / 4)) * 4;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (row0 + rr < a.rows) v = *reinterpret_cast<const float4 *>(a.T + (row0 + rr) * kPanelCols + t0 + st * kStage + k4);
            Ts[k4][rr] = v.x; Ts[k4 + 1][rr] = v.y; Ts[k4 + 2][rr] = v.z; Ts[k4 + 3][rr] = v.w;
        }
        // U tile: 32 rows x 128 columns (columns in whole fours: cend is a multiple of 64)
        for (int e = tid; e < kStage * (kTile / 4); e += kTrailThreads) {
            const int k = e / (kTile / 4), cc = (e % (kTile / 4)) * 4;
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (col0 + cc < cend) v = *reinterpret_cast<const float4 *>(a.U + (c0 + st * kStage + k) * a.ldu + col0 + cc);
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
            float *p = a.W + r * a.ldw + col0 + 8 * tx;
            *reinterpret_cast<float4 *>(p) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
            *reinterpret_cast<float4 *>(p + 4) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
        }
    }
}

hipError_t make_side_streams(pvq_ctx *c)
{
    if (c->side_ready) return hipSuccess;
    hipError_t e = hipEventCreateWithFlags(&c->side_fork, hipEventDisableTiming);
    for (int i = 0; i < pvq_ctx::kSideStreams && e == hipSuccess; i++) {
        e = hipStreamCreateWithFlags(&c->side[i], hipStreamNonBlocking);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->side_join[i], hipEventDisableTiming);
    }
    c->side_ready = true;   // whatever was made is released with the context
    return e;
}

}  // namespace

// W: rows x cols float32 (cols a multiple of 64), U: cols x cols, work: rows x 128 floats.
// Rows are independent, and within a chunk of rows the launches form a chain in which every second one (the
// block kernel) is a single wave per 64 rows bound by its own latency: up to four chunks of rows run side by
// side, the first on the caller's stream and the others on streams of the context that fork from and
// join the caller's stream through events, so that one chunk's block kernel runs beside another
// chunk's trailing update.
hipError_t pvq_launch_correct(const pvq_ctx *cc, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                              int64_t ldu, float *work, hipStream_t s)
{
    pvq_ctx *c = const_cast<pvq_ctx *>(cc);
    const int64_t nch = std::max<int64_t>(1, std::min<int64_t>(1 + pvq_ctx::kSideStreams, rows / 512));
    const int64_t chunk_rows = ((rows + nch - 1) / nch + kTile - 1) / kTile * kTile;
    std::lock_guard<std::mutex> hold(c->side_lock);   // the events below belong to one call at a time
    hipError_t e = hipSuccess;
    if (nch > 1) {
        if ((e = make_side_streams(c)) != hipSuccess) return e;
        if ((e = hipEventRecord(c->side_fork, s)) != hipSuccess) return e;
        for (int i = 0; i + 1 < nch; i++)
            if ((e = hipStreamWaitEvent(c->side[i], c->side_fork, 0)) != hipSuccess) return e;
    }
    for (int64_t c0 = 0; c0 < cols && e == hipSuccess; c0 += kBlockCols) {
        for (int64_t ch = 0; ch < nch; ch++) {
            const int64_t r0 = ch * chunk_rows, nr = std::min(chunk_rows, rows - r0);
            if (nr <= 0) continue;
            hipStream_t st = ch == 0 ? s : c->side[ch - 1];
            correct_args a;
            a.W = W + r0 * ldw; a.ldw = ldw; a.rows = nr; a.cols = cols; a.U = U; a.ldu = ldu; a.T = work + r0 * kPanelCols;
            a.K = c->K; a.ls = c->amplitude == PVQ_AMP_LS ? 1 : 0;
            const dim3 bgrid((unsigned)((nr + 63) / 64)), bblock(64);
            switch (c->D) {
            case 8: hipLaunchKernelGGL((correct_block_kernel<8>), bgrid, bblock, 0, st, a, c0); break;
            case 16: hipLaunchKernelGGL((correct_block_kernel<16>), bgrid, bblock, 0, st, a, c0); break;
            default: hipLaunchKernelGGL((correct_block_kernel<32>), bgrid, bblock, 0, st, a, c0); break;
            }
            // behind the first block of a panel: the panel's second block only; behind the second: everything
            // behind the panel, for both blocks at once
            const int64_t c1 = c0 + kBlockCols;
            const bool first = c0 % kPanelCols == 0;
            const int64_t cend = first ? std::min(c1 + kBlockCols, cols) : cols;
            if (c1 < cend) {
                const dim3 tgrid((unsigned)((nr + kTile - 1) / kTile), (unsigned)((cend - c1 + kTile - 1) / kTile));
                if (first) hipLaunchKernelGGL(correct_trailing_kernel, tgrid, dim3(kTrailThreads), 0, st, a, c0, 0, kBlockCols / kStage, c1, cend);
                else hipLaunchKernelGGL(correct_trailing_kernel, tgrid, dim3(kTrailThreads), 0, st, a, c0 - kBlockCols, 0, kPanelCols / kStage, c1, cend);
            }
        }
        e = hipGetLastError();
    }
    // join also after a failed launch, so that the caller's stream never runs ahead of the side streams
    for (int i = 0; i + 1 < nch; i++) {
        hipError_t j = hipEventRecord(c->side_join[i], c->side[i]);
        if (j == hipSuccess) j = hipStreamWaitEvent(s, c->side_join[i], 0);
        if (e == hipSuccess) e = j;
    }
    return e;
}
