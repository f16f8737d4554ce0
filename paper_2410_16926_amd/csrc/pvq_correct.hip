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
// taken in panels of 128:
//   correct_panel_kernel   one lane per row goes through the panel's groups (pending updates from the
//                          panel's earlier groups, quantise, substitution) and leaves the panel's t values
//                          (rows x 128) in a work buffer.  Bound by its own latency: one wave per 64 rows.
//   correct_trailing_kernel  applies the panel's 128 multiply-adds per element, in the same order, to all
//                          columns behind it: 128 x 128 tiles, 8 x 8 per lane, t and U tiles in LDS (32 rows
//                          of U at a time), W read and written once per panel.  Bound: float32 vector ALU.
// Not on the matrix cores: their accumulation order inside an instruction is not the one defined above.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pvq_internal.h"
#include "pvq_quantize_dev.h"

namespace {

using namespace pvq_quantize_dev;

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

// A panel of `width` columns (128, or 64 at the end of a matrix with an odd number of blocks) from column p0
// on, one lane per row.  Group after group: the group's D values come from W (requested while the group
// before is worked on); they take the updates of the panel's earlier groups, which are still pending (rows
// 0 .. G D - 1 of the panel's part of U, in that order: per element the same multiply-adds in the same order
// as if every group had updated all later columns at once); then quantiser, amplitude, error and
// substitution; the values go back to W, the group's t values to the work buffer and to LDS (a column per
// lane: the pending updates of the later groups read them there, so that nothing is indexed by the group
// number in registers and the groups are a real loop: the code stays small).  U is the same in every lane:
// the rows that a group needs (its D columns of the panel's rows above it, and its own D x D part) are
// fetched a group ahead, one or two rows per lane, parked in registers while the current group is worked
// on, and then laid out in LDS, where every lane reads the same address (a broadcast).
template <int D>
__global__ __launch_bounds__(64) void correct_panel_kernel(correct_args a, int64_t p0, int width)
{
    __shared__ float ts[kPanelCols][64];                        // t values of the panel so far, [column][lane]
    __shared__ __align__(16) float us[2][kPanelCols][D];        // the U rows of the current and the next group
    const int lane = threadIdx.x;
    const int64_t r = (int64_t)blockIdx.x * 64 + lane;
    const bool in = r < a.rows;
    // lanes beyond the rows work on the last row again (no lane waits for another); they store nothing
    float *wrow = a.W + (in ? r : a.rows - 1) * a.ldw + p0;
    float *trow = a.T + (in ? r : a.rows - 1) * kPanelCols;
    const float *U = a.U + p0 * a.ldu + p0;                     // row p0 + i, column p0 + c of the factor
    const int ngroups = width / D;

    auto load_group_values = [&](int G, float (&v)[D]) {
#pragma unroll
        for (int i = 0; i < D; i += 4) {
            const float4 q = *reinterpret_cast<const float4 *>(wrow + G * D + i);
            v[i] = q.x; v[i + 1] = q.y; v[i + 2] = q.z; v[i + 3] = q.w;
        }
    };
    // rows lane and lane + 64 of the panel, the D columns of group G (rows up to the group's last one are
    // needed: (G + 1) D of them; the others are fetched from a row that exists and not used)
    auto fetch_u = [&](int G, float (&v)[2][D]) {
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int k = lane + 64 * h;
            const float *src = U + (int64_t)(k < (G + 1) * D ? k : 0) * a.ldu + G * D;
#pragma unroll
            for (int i = 0; i < D; i += 4) {
                const float4 q = *reinterpret_cast<const float4 *>(src + i);
                v[h][i] = q.x; v[h][i + 1] = q.y; v[h][i + 2] = q.z; v[h][i + 3] = q.w;
            }
        }
    };
    auto park_u = [&](int buf, const float (&v)[2][D]) {
#pragma unroll
        for (int h = 0; h < 2; h++)
#pragma unroll
            for (int i = 0; i < D; i += 4)
                *reinterpret_cast<float4 *>(&us[buf][lane + 64 * h][i]) = make_float4(v[h][i], v[h][i + 1], v[h][i + 2], v[h][i + 3]);
    };
    float wg[D], wn[D], un[2][D];
    load_group_values(0, wg);
    fetch_u(0, un);
    park_u(0, un);
    __syncthreads();
    for (int G = 0; G < ngroups; G++) {
        const int Gn = G + 1 < ngroups ? G + 1 : G;
        load_group_values(Gn, wn);
        fetch_u(Gn, un);
        const float (*ug)[D] = us[G & 1];
        // pending updates: rows k = 0 .. G D - 1 of the panel, this group's columns
        const int pending = G * D;
#pragma unroll 8
        for (int k = 0; k < pending; k++) {
            const float tk = ts[k][lane];
            float u[D];
#pragma unroll
            for (int j = 0; j < D; j += 4) {
                const float4 q = *reinterpret_cast<const float4 *>(&ug[k][j]);
                u[j] = q.x; u[j + 1] = q.y; u[j + 2] = q.z; u[j + 3] = q.w;
            }
#pragma unroll
            for (int j = 0; j < D; j++) wg[j] = __builtin_fmaf(-tk, u[j], wg[j]);
        }
        // what is quantised, and stays in W
        if (in) {
#pragma unroll
            for (int i = 0; i < D; i += 4) *reinterpret_cast<float4 *>(wrow + G * D + i) = make_float4(wg[i], wg[i + 1], wg[i + 2], wg[i + 3]);
        }
        int y[D];
        float ss;
        if constexpr (D == 8) ss = quantize_group8(wg, a.K, y);
        else ss = quantize_group<D>(wg, a.K, y);
        const float s = a.ls ? pvq_ls_amplitude<D>(wg, y) : sqrtf(ss);
        int n2 = 0;
#pragma unroll
        for (int i = 0; i < D; i++) n2 += y[i] * y[i];
        const float gain = s / sqrtf((float)n2);
        float t[D];
#pragma unroll
        for (int j = 0; j < D; j++) {
            float acc = wg[j] - gain * (float)y[j];
#pragma unroll
            for (int i = 0; i < j; i++) acc = __builtin_fmaf(-t[i], ug[pending + i][j], acc);
            t[j] = acc / ug[pending + j][j];
        }
#pragma unroll
        for (int j = 0; j < D; j++) ts[pending + j][lane] = t[j];
        if (in) {
#pragma unroll
            for (int i = 0; i < D; i += 4) *reinterpret_cast<float4 *>(trow + G * D + i) = make_float4(t[i], t[i + 1], t[i + 2], t[i + 3]);
        }
        park_u((G + 1) & 1, un);
        __syncthreads();      // one wave: orders the LDS writes above before the next group's reads
#pragma unroll
        for (int i = 0; i < D; i++) wg[i] = wn[i];
    }
}

// Columns [c1, cend): W[r][c] <- W[r][c] - t[r][0] U[c0][c] - ... - t[r][n - 1] U[c0 + n - 1][c], n = 32 stages,
// one multiply-add after the other; t[r][k] = T[r][t0 + k].  n = 128: a panel's update of everything behind it,
// with the tile of W read and written once for 128 multiply-adds per element (with 64 per pass the kernel was
// bound by HBM as much as by the vector ALU).  A stage = 32 rows of U and 32 t values per row in LDS (33 KB, four
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
// panel kernel) is a single wave per 64 rows bound by its own latency: up to four chunks of rows run side by
// side, the first on the caller's stream and the others on streams of the context that fork from and
// join the caller's stream through events, so that one chunk's panel kernel runs beside another
// chunk's trailing update.
namespace {

hipError_t launch_correct(const pvq_ctx *cc, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                          int64_t ldu, float *work, hipStream_t s, int64_t max_chunks)
{
    pvq_ctx *c = const_cast<pvq_ctx *>(cc);
    const int64_t nch = std::max<int64_t>(1, std::min<int64_t>(max_chunks, rows / 512));
    const int64_t chunk_rows = ((rows + nch - 1) / nch + kTile - 1) / kTile * kTile;
    std::lock_guard<std::mutex> hold(c->side_lock);   // the events below belong to one call at a time
    hipError_t e = hipSuccess;
    if (nch > 1) {
        if ((e = make_side_streams(c)) != hipSuccess) return e;
        if ((e = hipEventRecord(c->side_fork, s)) != hipSuccess) return e;
        for (int i = 0; i + 1 < nch; i++)
            if ((e = hipStreamWaitEvent(c->side[i], c->side_fork, 0)) != hipSuccess) return e;
    }
    for (int64_t p0 = 0; p0 < cols && e == hipSuccess; p0 += kPanelCols) {
        const int width = (int)std::min<int64_t>(kPanelCols, cols - p0);   // 128, or 64 at the end
        for (int64_t ch = 0; ch < nch; ch++) {
            const int64_t r0 = ch * chunk_rows, nr = std::min(chunk_rows, rows - r0);
            if (nr <= 0) continue;
            hipStream_t st = ch == 0 ? s : c->side[ch - 1];
            correct_args a;
            a.W = W + r0 * ldw; a.ldw = ldw; a.rows = nr; a.cols = cols; a.U = U; a.ldu = ldu; a.T = work + r0 * kPanelCols;
            a.K = c->K; a.ls = c->amplitude == PVQ_AMP_LS ? 1 : 0;
            const dim3 pgrid((unsigned)((nr + 63) / 64)), pblock(64);
            switch (c->D) {
            case 8: hipLaunchKernelGGL((correct_panel_kernel<8>), pgrid, pblock, 0, st, a, p0, width); break;
            case 16: hipLaunchKernelGGL((correct_panel_kernel<16>), pgrid, pblock, 0, st, a, p0, width); break;
            default: hipLaunchKernelGGL((correct_panel_kernel<32>), pgrid, pblock, 0, st, a, p0, width); break;
            }
            // everything behind the panel takes the panel's 128 multiply-adds per element in one launch
            const int64_t c1 = p0 + kPanelCols;
            if (c1 < cols) {
                const dim3 tgrid((unsigned)((nr + kTile - 1) / kTile), (unsigned)((cols - c1 + kTile - 1) / kTile));
                hipLaunchKernelGGL(correct_trailing_kernel, tgrid, dim3(kTrailThreads), 0, st, a, p0, 0, kPanelCols / kStage, c1, cols);
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

// Work buffer of the entry point that allocates nothing: the t values of a panel for up to kStaticRows rows
// (128 floats per row), 4 MiB on every GPU that loads the library, until the process ends.
constexpr int64_t kStaticRows = 8192;
static __device__ __align__(256) float scratch[kStaticRows * kPanelCols];

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

hipError_t pvq_launch_correct(const pvq_ctx *cc, float *W, int64_t rows, int64_t cols, int64_t ldw, const float *U,
                              int64_t ldu, float *work, hipStream_t s)
{
    return launch_correct(cc, W, rows, cols, ldw, U, ldu, work, s, 1 + pvq_ctx::kSideStreams);
}

int64_t pvq_correct_static_max_rows(void) { return kStaticRows; }

// The same chain of kernels with the library's own work buffer and on the caller's stream alone: one chunk
// of rows, so no stream or event is made or used.
hipError_t pvq_launch_correct_static(const pvq_ctx *cc, float *W, int64_t rows, int64_t cols, int64_t ldw,
                                     const float *U, int64_t ldu, hipStream_t s)
{
    if (rows > kStaticRows) return hipErrorInvalidValue;   // (the entry point has refused it already)
    float *work = nullptr;
    const hipError_t e = scratch_on_current_device(&work);
    if (e != hipSuccess) return e;
    return launch_correct(cc, W, rows, cols, ldw, U, ldu, work, s, 1);
}
