// Decoding coordinate by coordinate (App. B.3) with one table probe per coordinate, for every configuration
// that has no table-driven block decoder: groups of 16 and 32 (the paper's 3.25 bits/weight row is D = 16,
// K = 33, 52-bit indices), and groups of 8 with multi-word indices.  One lane owns one group.
//
// With U(d,x) = N(d,0) + ... + N(d,x) (U(d,-1) = 0) and q = N(d,k) - 1 - r for the residual r in the
// sub-pyramid still open, the coordinate's magnitude is m = k - C with C = #{x >= 0 : U(d-1,x) <= q/2}
// (the points with magnitude below m number N(d,k) - 2 U(d-1,k-m); C <= k because q/2 < U(d-1,k)).
// U(d-1, .) grows geometrically, so the position of q/2 among its values follows from the magnitude of
// q/2: a guess table per row, indexed by the exponent and the leading fraction bits of q/2 as a float
// (rounded down), gives g = #{x : U(d-1,x) <= lower edge of that bucket} <= C, and nearly always C is g or
// g+1.  One read of the three entries U(d-1,g-1), U(d-1,g), U(d-1,g+1) settles it (a loop moves on in the
// rare bucket that holds two thresholds) and holds everything the step needs:
//     um = U(d-1,C-1), ux = U(d-1,C);  t = q - um;  the sign is negative iff t < ux;
//     next q = negative ? t - um : t - ux;  next k = C
// (for m = 0 the "negative" case applies and leaves q - 2 U(d-1,k-1), as it must).  App. B.3's search over
// magnitudes, and a binary search over the row (six dependent probes at K = 33), become two LDS reads.
//
// Widths: the integers of a step with d dimensions left are below N(d,K), so the later coordinates run in
// narrower arithmetic: dimensions above DA in W words, above DB in W/2 words, the rest in W/4 (for D = 16,
// K = 33: 64 bits down to nine dimensions, 32 bits from eight on, N(8,33) < 2^32).  The last two coordinates
// need no table: U(1,x) = 2x + 1, and P(1,k) = {+k, -k}.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <utility>

#include "pvq_internal.h"
#include "pvq_walk.h"

namespace {

constexpr int kMaxThreads = 1024;   // lanes of a workgroup: 256 while the tables are small, 1024 (one copy of the
                                    // tables for sixteen waves, two workgroups to a unit) when they are not
constexpr int kWave = 64;

struct walk_launch {
    pvq_walk_params p;
    const unsigned char *blob;
    const float *sqrtc;
    int index_bits, scale_bits;
};

using namespace pvq_walk;

// What a group needs from memory, as it comes: the W + 1 words its index may touch, its amplitude (the float, or the
// word that holds its code) and, with codes, the row's normaliser.  Fetching does no arithmetic on loaded data and has
// no load under a condition, so the loads stay in flight until the item is taken apart, one item later: a wait placed
// right behind a load also waits for every store issued before it (memory operations complete in order).
template <int W>
struct raw_group {
    uint32_t w[W + 1];
    uint32_t amp;
    float rownorm;
};

// row: the row's index words, last_word: index of the row's last word (words past the field's own are read
// inside the row and dropped); srow: the row of the scale plane
template <int W>
__device__ inline void fetch_group(const uint32_t *__restrict__ row, uint32_t last_word, const void *__restrict__ srow,
                                   const float *__restrict__ rownorm, int g, int index_bits, int scale_bits, raw_group<W> &r)
{
    const uint32_t w0 = __umul24((uint32_t)g, (uint32_t)index_bits) >> 5;     // (rows have at most 2^21 groups)
#pragma unroll
    for (int i = 0; i <= W; i++) r.w[i] = row[std::min(w0 + (uint32_t)i, last_word)];
    const uint32_t aw = scale_bits == 0 ? (uint32_t)g : __umul24((uint32_t)g, (uint32_t)scale_bits) >> 5;
    r.amp = reinterpret_cast<const uint32_t *>(srow)[aw];
    r.rownorm = scale_bits == 0 ? 0.0f : *rownorm;
}

template <int W>
__device__ inline typename wide<W>::type group_index(const raw_group<W> &r, int g, int bits)
{
    using T = typename wide<W>::type;
    const uint32_t sh = __umul24((uint32_t)g, (uint32_t)bits) & 31;
    const int span = (int)sh + bits;
    T v = (T)(r.w[0] >> sh);
#pragma unroll
    for (int i = 1; i <= W; i++) {
        const int off = 32 * i - (int)sh;
        if (32 * i < span && off < 32 * W) v |= (T)r.w[i] << off;
    }
    if (bits < 32 * W) v &= (((T)1) << bits) - 1;
    return v;
}

template <int W>
__device__ inline float group_amp(const raw_group<W> &r, int g, int scale_bits, const float *sqrtc)
{
    if (scale_bits == 0) return __uint_as_float(r.amp);
    const uint32_t pos = __umul24((uint32_t)g, (uint32_t)scale_bits);
    const uint32_t code = (r.amp >> (pos & 31)) & ((1u << scale_bits) - 1u);
    return sqrtc[code] * sqrtf(r.rownorm);
}


__device__ inline uint32_t f32_to_bf16_rne(float f)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    const f32x2_t pair = {f, 0.0f};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t)) & 0xFFFFu;
}

__device__ inline uint16_t f32_to_f16_rne(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

__device__ inline void tables_to_lds(unsigned char *lds, const walk_launch &wl, float *sqrtc)
{
    for (uint32_t i = threadIdx.x * 16u; i < wl.p.bytes; i += blockDim.x * 16u)
        *reinterpret_cast<uint4 *>(lds + i) = *reinterpret_cast<const uint4 *>(wl.blob + i);
    if (wl.scale_bits > 0)
        for (int i = threadIdx.x; i < (1 << wl.scale_bits); i += blockDim.x) sqrtc[i] = wl.sqrtc[i];
    __syncthreads();
}

// Decode to a matrix.  Workgroups stay for the whole launch (the tables are copied once each); after the copy
// every wave works alone and takes (row, 64 consecutive groups) items in turn.  A lane's group is D consecutive
// outputs, so the lanes of a wave would each store 16 bytes out of every D * size; with STAGE the wave lays
// its 64 groups out in LDS instead and every store instruction writes 1 KiB of consecutive addresses.
template <int D, int W, int DA, int DB, int OUT, bool STAGE>
__global__ __launch_bounds__(kMaxThreads) void decode_walk_kernel(walk_launch wl, pvq_decode_args a, int tiles)
{
    using T = typename wide<W>::type;
    constexpr int OSZ = OUT == PVQ_F32 ? 4 : 2;
    constexpr int NC = D * OSZ / 16;                 // 16-byte chunks of one group
    const int kWaves = (int)blockDim.x / kWave;
    extern __shared__ __align__(16) unsigned char lds[];
    float *sqrtc = reinterpret_cast<float *>(lds + wl.p.bytes);
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    uint4 *stage = reinterpret_cast<uint4 *>(lds + wl.p.bytes + 256 * sizeof(float)) + wave * (kWave * NC);
    tables_to_lds(lds, wl, sqrtc);
    const int G = (int)a.groups;
    const int64_t items = a.rows * tiles, stride = (int64_t)gridDim.x * kWaves;
    // What an item needs from memory is requested one item ahead, in front of the current item's stores: a
    // wait for a load also waits for every memory operation issued before it, so loads that follow stores
    // would make each item wait for the stores of the one before.  A wave past its last item, and lanes
    // past a row's last group, fetch a valid place again and drop it.
    raw_group<W> nx;
    int g_nx = 0;
    const uint32_t last_word = (uint32_t)a.index_row_words - 1u;
    const int64_t srow_bytes = wl.scale_bits == 0 ? a.groups * 4 : a.scale_row_words * 4;
    // (row, tile) of an item without a division per item: a wave moves on by `stride` items at a time
    const int64_t step_rows = stride / tiles;
    const int step_tiles = (int)(stride - step_rows * tiles);
    auto fetch = [&](int64_t row, int tile) {
        const int g = tile * kWave + lane;
        g_nx = g < G ? g : 0;
        fetch_group<W>(a.index + row * a.index_row_words, last_word,
                       reinterpret_cast<const unsigned char *>(a.scale) + row * srow_bytes,
                       wl.scale_bits == 0 ? nullptr : a.rownorm + row, g_nx,
                       wl.index_bits, wl.scale_bits, nx);
    };
    const int64_t first = (int64_t)blockIdx.x * kWaves + wave;
    int64_t row_n = first / tiles;                              // the item that is being fetched
    int tile_n = (int)(first - row_n * tiles);
    if (first < items) fetch(row_n, tile_n);
    // The first item has arrived before the loop is entered (vmcnt(0), the other counters left alone): the loop then
    // starts, on its first pass as on every other, with nothing but stores in flight behind the item it takes
    // apart, and its waits are counted from there; sized for the entry path they would wait for the stores too.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    for (int64_t item = first; item < items; item += stride) {
        const int64_t row = row_n;
        const int g0 = tile_n * kWave;                          // the wave's first group
        const int g_mine = g_nx;                                // the lane's group: g0 + lane, or 0 past the row's end
        const T c = group_index<W>(nx, g_mine, wl.index_bits);
        const float amp = group_amp<W>(nx, g_mine, wl.scale_bits, sqrtc);
        row_n += step_rows;
        tile_n += step_tiles;
        if (tile_n >= tiles) { tile_n -= tiles; row_n++; }
        if (row_n >= a.rows) { row_n = a.rows - 1; tile_n = tiles - 1; }   // past the last item: its place again, dropped
        fetch(row_n, tile_n);
        float y[D];
        const int n2 = unrank_walk<D, W, DA, DB>(c, lds, wl.p, [&](int i, uint32_t m, bool negative) {
            y[i] = negative ? -(float)m : (float)m;            // (a zero coordinate comes as -0)
        });
        // direction on the unit sphere times the amplitude (Sec. 2.4): w = amp * y / ||y||_2
        const float gain = amp / sqrtf((float)n2);
        // gain * y + 0: the product as it is, and +0 for a zero coordinate
        auto value = [&](int i) { return fmaf(gain, y[i], 0.0f); };
        const int valid = std::min(kWave, G - g0);             // groups of this item inside the row
        unsigned char *orow = reinterpret_cast<unsigned char *>(a.W_out) + row * a.ldw * OSZ;
        unsigned char *o = orow + (int64_t)g0 * D * OSZ;
#pragma unroll
        for (int j = 0; j < NC; j++) {
            uint4 chunk;
            if constexpr (OUT == PVQ_F32) {
                chunk = make_uint4(__float_as_uint(value(4 * j)), __float_as_uint(value(4 * j + 1)),
                                   __float_as_uint(value(4 * j + 2)), __float_as_uint(value(4 * j + 3)));
            } else {
                uint32_t pk[4];
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const float f0 = value(8 * j + 2 * e), f1 = value(8 * j + 2 * e + 1);
                    if constexpr (OUT == PVQ_F16) pk[e] = (uint32_t)f32_to_f16_rne(f0) | ((uint32_t)f32_to_f16_rne(f1) << 16);
                    else pk[e] = f32_to_bf16_rne(f0) | (f32_to_bf16_rne(f1) << 16);
                }
                chunk = make_uint4(pk[0], pk[1], pk[2], pk[3]);
            }
            // without staging every lane stores its own group; lanes past the row's end have decoded the row's first
            // group once more and store it where it belongs (the same bytes as its owner writes): no store is
            // under a condition, see below
            if constexpr (STAGE) stage[lane * NC + j] = chunk;
            else *reinterpret_cast<uint4 *>(orow + ((size_t)g_mine * NC + j) * 16) = chunk;
        }
        if constexpr (STAGE) {
            // the item's groups are NC * valid consecutive chunks of the output.  Every lane stores in every pass:
            // lanes past the item's end store its last chunk once more (the same bytes to the same place), so that
            // the number of stores in flight is known where the next item's words are waited for, and that wait
            // does not have to cover them
            const int last = valid * NC - 1;
#pragma unroll
            for (int j = 0; j < NC; j++) {
                const int ch = std::min(j * kWave + lane, last);
                const uint4 v = stage[ch];                     // written by this wave only: no barrier
                *reinterpret_cast<uint4 *>(o + (size_t)ch * 16) = v;
            }
        }
    }
}

// Decode fused into y = W_hat x for NB vectors.  A wave takes whole rows (lanes stride the groups; the next
// group's index, amplitude and activations are requested before the current group is decoded) and adds its
// 64 partial sums with a fixed xor butterfly.
template <int D, int W, int DA, int DB, int NB>
__global__ __launch_bounds__(kMaxThreads) void gemv_walk_kernel(walk_launch wl, pvq_decode_args a, int b0)
{
    using T = typename wide<W>::type;
    extern __shared__ __align__(16) unsigned char lds[];
    float *sqrtc = reinterpret_cast<float *>(lds + wl.p.bytes);
    tables_to_lds(lds, wl, sqrtc);
    const int G = (int)a.groups;
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const uint16_t *xb = reinterpret_cast<const uint16_t *>(a.x) + (int64_t)b0 * a.ldx;
    constexpr int XW = D / 8;                       // 16-byte words of one group's activations
    const int kWaves = (int)blockDim.x / kWave;
    for (int64_t row = (int64_t)blockIdx.x * kWaves + wave; row < a.rows; row += (int64_t)gridDim.x * kWaves) {
        const uint32_t *irow = a.index + row * a.index_row_words;
        const uint32_t last_word = (uint32_t)a.index_row_words - 1u;
        const unsigned char *srow = reinterpret_cast<const unsigned char *>(a.scale) +
                                    row * (wl.scale_bits == 0 ? a.groups * 4 : a.scale_row_words * 4);
        float acc[NB];
#pragma unroll
        for (int b = 0; b < NB; b++) acc[b] = 0.0f;
        // what a group needs from memory; lanes past the row's end fetch group 0 again and drop it
        raw_group<W> nx;
        int g_nx = 0;
        uint4 x_n[NB][XW];
        auto fetch = [&](int g) {
            const int gg = g < G ? g : 0;
            g_nx = gg;
            fetch_group<W>(irow, last_word, srow, wl.scale_bits == 0 ? nullptr : a.rownorm + row, gg, wl.index_bits, wl.scale_bits, nx);
#pragma unroll
            for (int b = 0; b < NB; b++)
#pragma unroll
                for (int w = 0; w < XW; w++)
                    x_n[b][w] = *reinterpret_cast<const uint4 *>(xb + (int64_t)b * a.ldx + (int64_t)gg * D + 8 * w);
        };
        fetch(lane);
        for (int g = lane; g < G; g += kWave) {
            const T c = group_index<W>(nx, g_nx, wl.index_bits);
            const float amp = group_amp<W>(nx, g_nx, wl.scale_bits, sqrtc);
            uint4 x[NB][XW];
#pragma unroll
            for (int b = 0; b < NB; b++)
#pragma unroll
                for (int w = 0; w < XW; w++) x[b][w] = x_n[b][w];
            fetch(g + kWave);
            float s[NB];
#pragma unroll
            for (int b = 0; b < NB; b++) s[b] = 0.0f;
            const int n2 = unrank_walk<D, W, DA, DB>(c, lds, wl.p, [&](int i, uint32_t m, bool negative) {
                const float yv = negative ? -(float)m : (float)m;
#pragma unroll
                for (int b = 0; b < NB; b++) {
                    const uint4 q = x[b][i / 8];
                    const uint32_t word = (i % 8) / 2 == 0 ? q.x : (i % 8) / 2 == 1 ? q.y : (i % 8) / 2 == 2 ? q.z : q.w;
                    const float xv = (i & 1) ? __uint_as_float(word & 0xFFFF0000u) : __uint_as_float(word << 16);
                    s[b] = fmaf(yv, xv, s[b]);
                }
            });
            const float gain = amp / sqrtf((float)n2);
#pragma unroll
            for (int b = 0; b < NB; b++) acc[b] = fmaf(gain, s[b], acc[b]);
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

int g_units = 0;

int units()
{
    if (g_units == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            g_units = n;
        else
            g_units = 256;
    }
    return g_units;
}

walk_launch make_launch(const pvq_ctx *c)
{
    walk_launch wl;
    wl.p = c->walk; wl.blob = c->walk_blob; wl.sqrtc = c->sqrtc;
    wl.index_bits = c->index_bits; wl.scale_bits = c->scale_bits;
    return wl;
}

// lanes of a workgroup for a context: small tables are copied by many small workgroups, large ones once per
// sixteen waves
int block_threads(const pvq_ctx *c) { return c->walk.bytes <= 16 * 1024 ? 256 : kMaxThreads; }

// tables, amplitude table, and (decode with staging) 64 groups of outputs per wave
size_t lds_bytes(const pvq_ctx *c, size_t group_out_bytes = 0)
{
    return (size_t)c->walk.bytes + 256 * sizeof(float) + (block_threads(c) / kWave) * kWave * group_out_bytes;
}

// kernels that need more LDS than a kernel gets without asking (64 KiB) say so once
template <typename Kernel>
hipError_t allow_lds(Kernel kernel, size_t bytes)
{
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// workgroups of a launch over `items` wave items: 32 waves per unit, fewer if the work is small
unsigned persistent_grid(const pvq_ctx *c, int64_t items)
{
    const int64_t per_block = block_threads(c) / kWave;
    return (unsigned)std::max<int64_t>(1, std::min<int64_t>((items + per_block - 1) / per_block, (int64_t)units() * 32 / per_block));
}

template <int D, int W, int DA, int DB, int OUT, bool STAGE>
hipError_t launch_decode_staged(const pvq_ctx *c, const pvq_decode_args &a, hipStream_t s)
{
    const int tiles = (int)((a.groups + kWave - 1) / kWave);
    const size_t lds = lds_bytes(c, STAGE ? (size_t)D * (OUT == PVQ_F32 ? 4 : 2) : 0);
    const hipError_t e = allow_lds(decode_walk_kernel<D, W, DA, DB, OUT, STAGE>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((decode_walk_kernel<D, W, DA, DB, OUT, STAGE>), dim3(persistent_grid(c, a.rows * tiles)), dim3(block_threads(c)), lds, s,
                       make_launch(c), a, tiles);
    return hipGetLastError();
}

template <int D, int W, int DA, int DB, int OUT>
hipError_t launch_decode_out(const pvq_ctx *c, const pvq_decode_args &a, hipStream_t s)
{
    // the staging buffer is used where the unit's 160 KiB still hold 32 waves with it
    if (lds_bytes(c, (size_t)D * (OUT == PVQ_F32 ? 4 : 2)) * (2048 / block_threads(c)) <= 160 * 1024) return launch_decode_staged<D, W, DA, DB, OUT, true>(c, a, s);
    return launch_decode_staged<D, W, DA, DB, OUT, false>(c, a, s);
}

template <int D, int W, int DA, int DB>
hipError_t launch_decode(const pvq_ctx *c, const pvq_decode_args &a, int out_dtype, hipStream_t s)
{
    switch (out_dtype) {
    case PVQ_F32: return launch_decode_out<D, W, DA, DB, PVQ_F32>(c, a, s);
    case PVQ_F16: return launch_decode_out<D, W, DA, DB, PVQ_F16>(c, a, s);
    default: return launch_decode_out<D, W, DA, DB, PVQ_BF16>(c, a, s);
    }
}

template <int D, int W, int DA, int DB>
hipError_t launch_gemv(const pvq_ctx *c, const pvq_decode_args &a, hipStream_t s)
{
    const unsigned grid = persistent_grid(c, a.rows);
    const dim3 block((unsigned)block_threads(c));
    const walk_launch wl = make_launch(c);
    const size_t lds = lds_bytes(c);
    // the batch is cut into passes of 4, 2 and 1 activation vectors over the codes
    int b0 = 0;
    while (b0 < a.batch) {
        const int left = a.batch - b0;
        hipError_t e;
        if (left >= 4) {
            if ((e = allow_lds(gemv_walk_kernel<D, W, DA, DB, 4>, lds)) != hipSuccess) return e;
            hipLaunchKernelGGL((gemv_walk_kernel<D, W, DA, DB, 4>), dim3(grid), block, lds, s, wl, a, b0); b0 += 4;
        } else if (left >= 2) {
            if ((e = allow_lds(gemv_walk_kernel<D, W, DA, DB, 2>, lds)) != hipSuccess) return e;
            hipLaunchKernelGGL((gemv_walk_kernel<D, W, DA, DB, 2>), dim3(grid), block, lds, s, wl, a, b0); b0 += 2;
        } else {
            if ((e = allow_lds(gemv_walk_kernel<D, W, DA, DB, 1>, lds)) != hipSuccess) return e;
            hipLaunchKernelGGL((gemv_walk_kernel<D, W, DA, DB, 1>), dim3(grid), block, lds, s, wl, a, b0); b0 += 1;
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

bool pvq_walk_usable(const pvq_ctx *c)
{
    // the tables and the amplitude table must fit LDS
    return c->walk_blob != nullptr && lds_bytes(c) <= 160 * 1024;
}

hipError_t pvq_walk_launch_decode(const pvq_ctx *c, const pvq_decode_args &a, int out_dtype, hipStream_t s)
{
#define PVQ_WALK_DECODE(D, W, DA, DB) launch_decode<D, W, DA, DB>(c, a, out_dtype, s)
    PVQ_WALK_DISPATCH(PVQ_WALK_DECODE, c->D, c->words, c->walk.dA, c->walk.dB);
#undef PVQ_WALK_DECODE
}

hipError_t pvq_walk_launch_gemv(const pvq_ctx *c, const pvq_decode_args &a, hipStream_t s)
{
#define PVQ_WALK_GEMV(D, W, DA, DB) launch_gemv<D, W, DA, DB>(c, a, s)
    PVQ_WALK_DISPATCH(PVQ_WALK_GEMV, c->D, c->words, c->walk.dA, c->walk.dB);
#undef PVQ_WALK_GEMV
}
