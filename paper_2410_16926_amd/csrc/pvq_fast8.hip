// gfx950 kernels built on the D = 8 table-driven decoder (pvq_fast8.h): decode to a matrix, and
// decode fused into y = W_hat x.
//
// One workgroup per compute unit keeps the whole table blob (up to 156 KiB) in LDS and walks many
// rows, so the copy is paid once per launch and unit.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pvq_internal.h"

namespace {

constexpr int kWave = 64;
constexpr int kMaxThreads = 1024;
constexpr int kGemvThreads = 1024;   // lanes of a fused-product workgroup (half as many with twice the
                                     // groups in flight per lane measured 30 % slower)
constexpr int kGroupsPerLane = 4;
constexpr int kTileGroups = kWave * kGroupsPerLane;   // groups one wave covers in a row: 256
constexpr int kLdsBytes = 160 * 1024;                 // the whole LDS of a compute unit

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

__device__ inline float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

struct fast8_launch {
    pvq_fast8_params p;
    const unsigned char *blob;
    const float *sqrtc;  // 2^scale_bits entries, or nullptr
    int index_bits, scale_bits;
};

// Copies the blob into LDS.  With FUSED (amplitude codes of at most 2 bits) the blob's last table,
// 1/sqrt(n2), is left out and its place taken by gain[n2][q] = (1/sqrt(n2)) * sqrt(center[q]),
// 2^scale_bits floats per n2, so that one lookup gives a group's whole gain; otherwise the
// 2^scale_bits values sqrt(center[q]) follow the blob.
template <bool FUSED>
__device__ inline void load_tables(unsigned char *lds, const fast8_launch &f, float *sqrtc_l)
{
    const int nthreads = blockDim.x;
    const uint32_t bytes = FUSED ? f.p.lds_bytes : f.p.tab_bytes;
    // Every workgroup starts at another place of the blob (with all units asking for the same lines in the same
    // order, one L2 channel at a time serves the whole machine), two 16-byte pieces per lane and trip.  (All ten
    // pieces of a lane requested before the first LDS write measured 13 us slower per launch, one at a time and no
    // rotation 1.7 us slower.)
    const uint32_t pieces = (bytes + 15u) / 16u;
    const uint32_t rot = (uint32_t)((blockIdx.x * 37u) % 64u) * (pieces / 64u);
    for (uint32_t c = threadIdx.x; c < pieces; c += 2 * nthreads) {
        uint32_t s0 = c + rot, s1 = c + nthreads + rot;
        s0 = s0 >= pieces ? s0 - pieces : s0;
        s1 = s1 >= pieces ? s1 - pieces : s1;
        const bool two = c + nthreads < pieces;
        s1 = two ? s1 : s0;
        const uint4 v0 = *reinterpret_cast<const uint4 *>(f.blob + s0 * 16u);
        const uint4 v1 = *reinterpret_cast<const uint4 *>(f.blob + s1 * 16u);
        *reinterpret_cast<uint4 *>(lds + s0 * 16u) = v0;
        *reinterpret_cast<uint4 *>(lds + s1 * 16u) = v1;
    }
    if constexpr (FUSED) {
        const int n = (int)f.p.k2max + 1;
        for (int i = threadIdx.x; i < (n << f.scale_bits); i += nthreads) {
            const int n2 = i >> f.scale_bits, q = i & ((1 << f.scale_bits) - 1);
            sqrtc_l[i] = reinterpret_cast<const float *>(f.blob + f.p.invs)[n2] * f.sqrtc[q];
        }
    } else if (f.scale_bits > 0) {
        for (int i = threadIdx.x; i < (1 << f.scale_bits); i += nthreads) sqrtc_l[i] = f.sqrtc[i];
    }
    __syncthreads();
}

// Work mapping.  A wave works on a tile of 256 consecutive groups of one row; lane l owns the groups
// tile*256 + 64*j + l, j = 0..3.  So for every j the 64 lanes touch 64 consecutive groups: the index
// reads of one j cover 192 contiguous bytes and, in the decode kernel, the stores of one j cover one
// contiguous KiB (a lane that kept four neighbouring groups would write 16 bytes out of every 64 per
// store instruction, which measured 2.5x slower).

// What a lane fetches for its four groups of one row.  Raw words only: no arithmetic touches loaded
// data until the item is consumed, so that the loads stay in flight behind the previous item's work.
struct item_t {
    uint32_t w[kGroupsPerLane];   // index: the dword at byte 3g-1 of the row (24-bit path) or the index itself
    uint32_t a[kGroupsPerLane];   // amplitude: the code word holding group g's code, or the float's bits
};

// Branch-free on purpose: every lane loads (lanes beyond the row re-read its first group, a wave
// past its last item re-reads a valid one).  With loads under conditions the compiler cannot count
// how many are in flight and makes every use of an item wait for ALL outstanding memory operations,
// the stores of the previous item included.
template <bool CODES, bool B24>
__device__ inline void fetch_item(const fast8_launch &f, const pvq_decode_args &a, int64_t row, int gbase,
                                  item_t &it)
{
    const int G = (int)a.groups;
    const uint32_t *irow = a.index + row * a.index_row_words;
#pragma unroll
    for (int j = 0; j < kGroupsPerLane; j++) {
        const int gj = gbase + kWave * j;
        const int g = gj < G ? gj : 0;
        if constexpr (B24) {
            // the 3 bytes of group g start at byte 3g; one dword load from byte 3g-1 (3g for g = 0)
            // holds them and stays inside the row
            const unsigned char *p = reinterpret_cast<const unsigned char *>(irow) + 3 * g - (g > 0 ? 1 : 0);
            uint32_t v;
            __builtin_memcpy(&v, p, 4);
            it.w[j] = v;
        } else {
            const uint32_t b = (uint32_t)f.index_bits;
            const uint32_t pos = (uint32_t)g * b, w0 = pos >> 5, sh = pos & 31;
            uint64_t v = irow[w0];
            if (sh + b > 32) v |= (uint64_t)irow[w0 + 1] << 32;
            it.w[j] = (uint32_t)(v >> sh) & (uint32_t)((1ull << b) - 1ull);
        }
        if constexpr (CODES) {
            const uint32_t *srow = reinterpret_cast<const uint32_t *>(a.scale) + row * a.scale_row_words;
            it.a[j] = srow[((uint32_t)g * (uint32_t)f.scale_bits) >> 5];
        } else {
            it.a[j] = __float_as_uint(reinterpret_cast<const float *>(a.scale)[row * a.groups + g]);
        }
    }
}

// the four indices of an item
template <bool B24>
__device__ inline void item_indices(const item_t &it, int gbase, uint32_t (&c)[kGroupsPerLane])
{
#pragma unroll
    for (int j = 0; j < kGroupsPerLane; j++) {
        if constexpr (B24) c[j] = (gbase + kWave * j > 0) ? it.w[j] >> 8 : it.w[j] & 0xFFFFFFu;
        else c[j] = it.w[j];
    }
}

// amplitude code of group j of an item
__device__ inline uint32_t item_code(const fast8_launch &f, const item_t &it, int gbase, int j)
{
    const uint32_t pos = (uint32_t)(gbase + kWave * j) * (uint32_t)f.scale_bits;
    return (it.a[j] >> (pos & 31u)) & ((1u << f.scale_bits) - 1u);
}

// The fused product writes nothing per group, so there a lane takes four NEIGHBOURING groups
// (4*lane .. 4*lane+3 of its wave's 256): their 24-bit indices are three aligned dwords and their
// amplitude codes sit in one word, two loads per row instead of eight.
template <bool CODES>
struct quad_item_t {
    uint32_t w[3];                       // 24-bit path: three dwords; generic path: unused
    uint32_t c[kGroupsPerLane];          // generic path: the four indices
    float amp[CODES ? 1 : kGroupsPerLane];
    uint32_t codes;                      // CODES: the word that holds the four codes
};

// Per-lane byte offsets into a row of the planes; rows differ only in a wave-uniform base, so the
// loads take a scalar base and these offsets.  Lanes beyond the row's last group read the row's
// first quad: what they decode meets activations of zero.
struct quad_offsets {
    uint32_t index, scale;
};

template <bool CODES, bool B24>
__device__ inline quad_offsets make_quad_offsets(const fast8_launch &f, int g0, bool in_row)
{
    const uint32_t g = in_row ? (uint32_t)g0 : 0u;
    quad_offsets o;
    o.index = B24 ? (g >> 2) * 12u : 0u;
    o.scale = CODES ? ((g * (uint32_t)f.scale_bits) >> 5) * 4u : g * 4u;  // 4 codes never straddle a word
    return o;
}

// `row` must be uniform in the wave.  No arithmetic on loaded data here, so that fetches stay in
// flight until the item is split.
template <bool CODES, bool B24>
__device__ inline void fetch_quad(const fast8_launch &f, const pvq_decode_args &a, int64_t row, int g0, bool in_row,
                                  const quad_offsets &o, quad_item_t<CODES> &it)
{
    const unsigned char *irow = reinterpret_cast<const unsigned char *>(a.index + row * a.index_row_words);
    if constexpr (B24) {
        const uint32_t *p = reinterpret_cast<const uint32_t *>(irow + o.index);
        it.w[0] = p[0]; it.w[1] = p[1]; it.w[2] = p[2];
    } else {
        const uint32_t b = (uint32_t)f.index_bits;
        const uint32_t g = in_row ? (uint32_t)g0 : 0u;
#pragma unroll
        for (int j = 0; j < kGroupsPerLane; j++) {
            const uint32_t pos = (g + j) * b, w0 = pos >> 5, sh = pos & 31;
            uint64_t v = reinterpret_cast<const uint32_t *>(irow)[w0];
            if (sh + b > 32) v |= (uint64_t)reinterpret_cast<const uint32_t *>(irow)[w0 + 1] << 32;
            it.c[j] = (uint32_t)(v >> sh) & (uint32_t)((1ull << b) - 1ull);
        }
    }
    if constexpr (CODES) {
        const unsigned char *srow = reinterpret_cast<const unsigned char *>(
            reinterpret_cast<const uint32_t *>(a.scale) + row * a.scale_row_words);
        it.codes = *reinterpret_cast<const uint32_t *>(srow + o.scale);
    } else {
        const unsigned char *srow = reinterpret_cast<const unsigned char *>(
            reinterpret_cast<const float *>(a.scale) + row * a.groups);
        const float4 v = *reinterpret_cast<const float4 *>(srow + o.scale);
        it.amp[0] = v.x; it.amp[1] = v.y; it.amp[2] = v.z; it.amp[3] = v.w;
    }
}

// What the decoder needs of an item, copied out so that the item's registers can take the next fetch.
template <bool CODES>
struct quad_split_t {
    uint32_t c[kGroupsPerLane];
    uint32_t codes;                      // the four codes, lowest group in the low bits
    float amp[CODES ? 1 : kGroupsPerLane];
};

template <bool CODES, bool B24>
__device__ inline void split_quad(const fast8_launch &f, int g0, const quad_item_t<CODES> &it, quad_split_t<CODES> &q)
{
    q.codes = 0;
    if constexpr (CODES) q.codes = it.codes >> (((uint32_t)g0 * (uint32_t)f.scale_bits) & 31u);
    else {
#pragma unroll
        for (int j = 0; j < kGroupsPerLane; j++) q.amp[j] = it.amp[j];
    }
    if constexpr (B24) {
        q.c[0] = it.w[0] & 0xFFFFFFu;
        q.c[1] = __builtin_amdgcn_alignbit(it.w[1], it.w[0], 24) & 0xFFFFFFu;
        q.c[2] = __builtin_amdgcn_alignbit(it.w[2], it.w[1], 16) & 0xFFFFFFu;
        q.c[3] = it.w[2] >> 8;
    } else {
#pragma unroll
        for (int j = 0; j < kGroupsPerLane; j++) q.c[j] = it.c[j];
    }
}

// amplitude factor of group j without the row normaliser: sqrt(center[q]) or the stored amplitude
template <bool CODES>
__device__ inline float amp_factor(const fast8_launch &f, const quad_split_t<CODES> &q, int j, const float *sqrtc_l)
{
    if constexpr (CODES) {
        const uint32_t code = (q.codes >> (j * f.scale_bits)) & ((1u << f.scale_bits) - 1u);
        return sqrtc_l[code];
    } else {
        return q.amp[j];
    }
}

// v + (v moved across lanes by one data-parallel-primitive pattern); lanes outside ROWS add zero
template <int CTRL, int ROWS = 0xF>
__device__ inline float dpp_add(float v)
{
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xF, false);
    return v + __builtin_bit_cast(float, moved);
}

// Sum over the 64 lanes in a fixed order, valid in lane 63: pairs, quads, eights, rows of 16 (mirror
// patterns), then row 0 into 1 and row 2 into 3, then rows 0..1 into 2..3.  Pure vector-ALU work:
// no LDS traffic, unlike a shuffle butterfly.
__device__ inline float wave_sum_lane63(float v)
{
    v = dpp_add<0xB1>(v);          // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);          // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);         // row_half_mirror
    v = dpp_add<0x140>(v);         // row_mirror
    v = dpp_add<0x142, 0xA>(v);    // row_bcast15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);    // row_bcast31 into rows 2 and 3
    return v;
}

// ---------------------------------------------------------------------------------------------
// y = W_hat x
// ---------------------------------------------------------------------------------------------

// rows a wave decodes per batch of rows (= how far ahead it fetches), with and without S0 running
// a row ahead (whose state takes the registers of two more fetched rows)
constexpr int kGemvRowsPerWave = 4, kGemvRowsPerWaveAhead = 2;
// partial sums of one batch of rows: 64 (row, slice) pairs x 4 vectors, two buffers
constexpr size_t kPartBytes = 2 * 64 * 4 * sizeof(float);

// Waves are arranged as nsl column slices (256 groups each) x rl row lanes.  Per batch of 4*rl rows
// every wave handles 4 rows of its slice; lanes keep their 32 activations per vector in registers.
// Row sums: fixed-order sum inside the wave, then the slices' partial sums meet in LDS in slice order.
// AMP: 0 = float32 amplitudes, 1 = amplitude codes, 2 = amplitude codes with the fused gain table.
// AHEAD: S0 of a wave's next row is started before the current row is decoded, with S0's block
// entries read from device memory (tables in the flavour that keeps that table outside LDS).
template <int NB, int AMP, bool B24, bool AHEAD>
__global__ __launch_bounds__(kGemvThreads) void gemv8_kernel(fast8_launch f, pvq_decode_args a, int b0,
                                                             int nsl, int rl, int rows_per_block)
{
    constexpr bool CODES = AMP != 0;
    constexpr int RI = AHEAD ? kGemvRowsPerWaveAhead : kGemvRowsPerWave;
    // static, so that table offsets fold into the LDS instructions' immediate fields
    __shared__ __align__(16) unsigned char lds[kLdsBytes];
    // the fused gain table replaces the 1/sqrt(n2) table at the end of the blob
    float *sqrtc_l = reinterpret_cast<float *>(lds + (AMP == 2 ? f.p.lds_bytes : f.p.tab_bytes));
    float *part = sqrtc_l + (AMP == 2 ? ((f.p.k2max + 1) << f.scale_bits) : 256);

    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r_end = std::min<int64_t>(a.rows, r_begin + rows_per_block);

    const int G = (int)a.groups;
    const int lane = threadIdx.x & (kWave - 1);
    // the wave's number as a scalar, so that row addresses are computed once per wave, not per lane
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int slice = wave % nsl, rowlane = wave / nsl;
    const int g0 = slice * kTileGroups + lane * kGroupsPerLane;
    const bool in_row = g0 < G;
    const int RB = RI * rl;            // rows per batch
    const quad_offsets qo = make_quad_offsets<CODES, B24>(f, g0, in_row);
    const int64_t r_last = r_end - 1;  // rows beyond the range re-read the last one; their sums are dropped

    // first fetches go out before the table copy
    quad_item_t<CODES> item[RI];
    if (r_begin < r_end) {
#pragma unroll
        for (int i = 0; i < RI; i++)
            fetch_quad<CODES, B24>(f, a, std::min<int64_t>(r_begin + i * rl + rowlane, r_last), g0, in_row, qo, item[i]);
    }
    load_tables<AMP == 2>(lds, f, sqrtc_l);
    if (r_begin >= r_end) return;

    uint32_t xr[NB][16];
#pragma unroll
    for (int b = 0; b < NB; b++) {
        const uint16_t *xp = reinterpret_cast<const uint16_t *>(a.x) + (int64_t)(b0 + b) * a.ldx + (int64_t)g0 * 8;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (in_row) v = *reinterpret_cast<const uint4 *>(xp + 8 * j);
            xr[b][4 * j] = v.x; xr[b][4 * j + 1] = v.y; xr[b][4 * j + 2] = v.z; xr[b][4 * j + 3] = v.w;
        }
    }

    // S0 runs one row ahead.  Its block entries come from the table's copy in device memory, through
    // the vector cache: that takes one 16-byte lookup per group off the LDS, which is the busiest
    // unit of this kernel, and the cache's latency passes while the row before is decoded.
    struct ahead_t {
        quad_split_t<CODES> q;
        uint32_t r[kGroupsPerLane];
        pvq_u32x4 b[kGroupsPerLane];
    };
    // takes the item in `slot`, refills the slot with `refill_row`, and starts S0 for the item taken
    auto start_row = [&](int slot, int64_t refill_row, ahead_t &n) {
        split_quad<CODES, B24>(f, g0, item[slot], n.q);
        fetch_quad<CODES, B24>(f, a, std::min<int64_t>(refill_row, r_last), g0, in_row, qo, item[slot]);
        uint32_t addr[kGroupsPerLane];
        pvq_fast8_s0_find<kGroupsPerLane, true>(lds, f.p, n.q.c, n.r, addr);
#pragma unroll
        for (int j = 0; j < kGroupsPerLane; j++) n.b[j] = *reinterpret_cast<const pvq_u32x4 *>(f.blob + addr[j]);
    };
    ahead_t nx;
    if constexpr (AHEAD) start_row(0, r_begin + RB + rowlane, nx);

    int parity = 0;
    for (int64_t batch = r_begin; batch < r_end; batch += RB) {
        float *pbuf = part + parity * (64 * NB);
#pragma unroll
        for (int i = 0; i < RI; i++) {
            ahead_t cu;
            if constexpr (AHEAD) {
                cu = nx;
                // the slot after this one holds the next row: of this batch, or (last slot) of the following one
                const int slot = (i + 1) % RI;
                const int64_t held = i + 1 < RI ? batch : batch + RB;
                start_row(slot, held + RB + slot * rl + rowlane, nx);
            } else {
                split_quad<CODES, B24>(f, g0, item[i], cu.q);
                // the same registers take this wave's row of the next batch while the current one is decoded
                fetch_quad<CODES, B24>(f, a, std::min<int64_t>(batch + RB + i * rl + rowlane, r_last), g0, in_row, qo, item[i]);
            }

            uint32_t n2x4[kGroupsPerLane];
            float dot[kGroupsPerLane][NB];
            // every pair goes into the groups' dot products the moment its stage has found it
            auto emit = [&](int j, int pair, uint32_t w) {
#pragma unroll
                for (int b = 0; b < NB; b++)
                    dot[j][b] = dot2_bf16(w, xr[b][4 * j + pair], pair == 0 ? 0.0f : dot[j][b]);
            };
            if constexpr (AHEAD) pvq_fast8_rest<kGroupsPerLane, true>(lds, f.blob, f.p, cu.r, cu.b, emit, n2x4);
            else pvq_fast8_decode_emit<kGroupsPerLane, false>(lds, f.blob, f.p, cu.q.c, emit, n2x4);
            float acc[NB];
#pragma unroll
            for (int b = 0; b < NB; b++) acc[b] = 0.0f;
            const uint32_t codes4 = cu.q.codes << 2;
#pragma unroll
            for (int j = 0; j < kGroupsPerLane; j++) {
                float gain;
                if constexpr (AMP == 2) {
                    // byte offset of gain[n2][q]: 4 * (n2 * 2^bits + q), from 4*n2 and the code word
                    // shifted left by two
                    const uint32_t code4 = (codes4 >> (j * f.scale_bits)) & (((1u << f.scale_bits) - 1u) << 2);
                    gain = *reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(sqrtc_l) +
                                                            ((n2x4[j] << f.scale_bits) + code4));
                } else {
                    gain = *reinterpret_cast<const float *>(lds + f.p.invs + n2x4[j]) *
                           amp_factor<CODES>(f, cu.q, j, sqrtc_l);
                }
#pragma unroll
                for (int b = 0; b < NB; b++) acc[b] = fmaf(gain, dot[j][b], acc[b]);
            }
#pragma unroll
            for (int b = 0; b < NB; b++) {
                const float v = wave_sum_lane63(acc[b]);
                if (lane == kWave - 1) pbuf[((i * rl + rowlane) * nsl + slice) * NB + b] = v;
            }
        }
        // one barrier per batch: the next batch writes the other buffer, and a buffer is written
        // again only after the barrier that follows its readers
        __syncthreads();
        if ((int)threadIdx.x < RB * NB) {
            const int rloc = threadIdx.x / NB, b = threadIdx.x % NB;
            const int64_t row = batch + rloc;
            if (row < r_end) {
                float v = 0.0f;
                for (int s = 0; s < nsl; s++) v += pbuf[(rloc * nsl + s) * NB + b];
                if constexpr (CODES) v *= sqrtf(a.rownorm[row]);
                a.y[(int64_t)(b0 + b) * a.ldy + row] = v;
            }
        }
        parity ^= 1;
    }
}

// One vector, no barriers: every wave works alone.  A wave owns the rows  wave, wave + 16, ...  of its
// workgroup's range and takes them slice by slice (a slice = 256 groups, lane l: groups 4l .. 4l+3): all
// its rows of slice 0, then all of slice 1, ...  So the activations in registers are those of one slice
// (16 registers, reloaded when the slice changes), a row's partial sums are added up by the one wave that
// owns the row (its lane 63 adds each slice's sum, formed inside the wave, to a float of its own in LDS, in
// slice order: deterministic), and after the table copy nothing makes the sixteen waves of a unit meet:
// they drift apart, and their table lookups come spread out instead of in bursts after every barrier.
// S0 runs one item ahead with its block entries through the vector cache, as in gemv8_kernel<1, ., ., true>
// (tables in the flavour that keeps S0's block table outside LDS).  Rows of whole slices; AMP as in
// gemv8_kernel.
constexpr int kRowMaxRowsPerWave = 32;   // partial sums in LDS: 16 waves x 32 rows

template <int AMP, bool B24>
__global__ __launch_bounds__(kGemvThreads) void gemv8_row_kernel(fast8_launch f, pvq_decode_args a, int b0,
                                                                 int rows_per_block, int nsl)
{
    constexpr bool CODES = AMP != 0;
    constexpr int kWaves = kGemvThreads / kWave;
    __shared__ __align__(16) unsigned char lds[kLdsBytes];
    float *sqrtc_l = reinterpret_cast<float *>(lds + (AMP == 2 ? f.p.lds_bytes : f.p.tab_bytes));
    float *part = sqrtc_l + (AMP == 2 ? ((f.p.k2max + 1) << f.scale_bits) : 256);

    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r_end = std::min<int64_t>(a.rows, r_begin + rows_per_block);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // this wave's rows: r_begin + wave + 16 i, i < nrows; its items: (slice, row) pairs, rows innermost
    const int nrows = r_begin + wave < r_end ? (int)((r_end - r_begin - wave + kWaves - 1) / kWaves) : 0;
    const int nitems = nrows * nsl;
    const int gl = lane * kGroupsPerLane;             // the lane's first group inside a slice
    float *mine = part + wave * kRowMaxRowsPerWave;

    // byte offsets of the lane's quad inside slice 0 of a row of the planes; a slice further on adds a constant
    const quad_offsets q0 = make_quad_offsets<CODES, B24>(f, gl, true);
    const uint32_t index_step = B24 ? (uint32_t)(kTileGroups / 4) * 12u : 0u;
    const uint32_t scale_step = CODES ? (uint32_t)(kTileGroups / 32) * 4u * (uint32_t)f.scale_bits : (uint32_t)kTileGroups * 4u;

    // the stream of fetches: item after item, (slice, row) kept as scalars; past the last item the last one is
    // read again (nothing of it is kept)
    int f_sl = 0, f_i = 0;
    auto fetch_next = [&](quad_item_t<CODES> &it) {
        quad_offsets o;
        o.index = q0.index + (uint32_t)f_sl * index_step;
        o.scale = q0.scale + (uint32_t)f_sl * scale_step;
        fetch_quad<CODES, B24>(f, a, r_begin + wave + (int64_t)kWaves * f_i, f_sl * kTileGroups + gl, true, o, it);
        if (f_i + 1 < nrows) f_i++;
        else if (f_sl + 1 < nsl) { f_i = 0; f_sl++; }
    };

    quad_item_t<CODES> raw[2];
    if (nitems > 0) { fetch_next(raw[0]); fetch_next(raw[1]); }
    if (lane < kRowMaxRowsPerWave) mine[lane] = 0.0f;
    load_tables<AMP == 2>(lds, f, sqrtc_l);          // ends with the kernel's only barrier before the last one

    if (nitems > 0) {
        struct ahead_t {
            quad_split_t<CODES> q;
            uint32_t r[kGroupsPerLane];
            pvq_u32x4 b[kGroupsPerLane];
        };
        // takes the raw item out of set `slot` (an item of slice `sl`), refills the set from the stream, and
        // starts S0 for the item taken
        auto start_item = [&](int slot, int sl, ahead_t &n) {
            split_quad<CODES, B24>(f, sl * kTileGroups + gl, raw[slot], n.q);
            fetch_next(raw[slot]);
            uint32_t addr[kGroupsPerLane];
            pvq_fast8_s0_find<kGroupsPerLane, true>(lds, f.p, n.q.c, n.r, addr);
#pragma unroll
            for (int j = 0; j < kGroupsPerLane; j++) n.b[j] = *reinterpret_cast<const pvq_u32x4 *>(f.blob + addr[j]);
        };
        // (slice, row) of the item being decoded and of the one after it
        int c_sl = 0, c_i = 0, n_sl = 0, n_i = 0;
        auto advance = [&](int &sl, int &i) {
            if (i + 1 < nrows) i++;
            else { i = 0; sl++; }
        };
        ahead_t nx;
        start_item(0, 0, nx);
        advance(n_sl, n_i);

        uint32_t xr[16];
        int x_sl = -1;
        for (int it = 0; it < nitems; it += 2) {
#pragma unroll
            for (int h = 0; h < 2; h++) {
                if (it + h < nitems) {
                    ahead_t cu = nx;
                    // (in front of the next item's requests: memory operations complete in order, so the wait for the
                    // activations, which the compiler places before their use whether or not this branch ran, would
                    // otherwise cover those requests too, in every item)
                    if (c_sl != x_sl) {
                        const uint16_t *xp = reinterpret_cast<const uint16_t *>(a.x) + (int64_t)b0 * a.ldx +
                                             (int64_t)(c_sl * kTileGroups + gl) * 8;
#pragma unroll
                        for (int j = 0; j < 4; j++) {
                            const uint4 v = *reinterpret_cast<const uint4 *>(xp + 8 * j);
                            xr[4 * j] = v.x; xr[4 * j + 1] = v.y; xr[4 * j + 2] = v.z; xr[4 * j + 3] = v.w;
                        }
                        x_sl = c_sl;
                    }
                    // item it + h + 1 sits in set (h + 1) % 2
                    start_item((h + 1) % 2, std::min(n_sl, nsl - 1), nx);
                    advance(n_sl, n_i);
                    uint32_t n2x4[kGroupsPerLane];
                    float dot[kGroupsPerLane];
                    auto emit = [&](int j, int pair, uint32_t w) {
                        dot[j] = dot2_bf16(w, xr[4 * j + pair], pair == 0 ? 0.0f : dot[j]);
                    };
                    pvq_fast8_rest<kGroupsPerLane, true>(lds, f.blob, f.p, cu.r, cu.b, emit, n2x4);
                    float acc = 0.0f;
                    const uint32_t codes4 = cu.q.codes << 2;
#pragma unroll
                    for (int j = 0; j < kGroupsPerLane; j++) {
                        float gain;
                        if constexpr (AMP == 2) {
                            const uint32_t code4 = (codes4 >> (j * f.scale_bits)) & (((1u << f.scale_bits) - 1u) << 2);
                            gain = *reinterpret_cast<const float *>(reinterpret_cast<const unsigned char *>(sqrtc_l) +
                                                                    ((n2x4[j] << f.scale_bits) + code4));
                        } else {
                            gain = *reinterpret_cast<const float *>(lds + f.p.invs + n2x4[j]) *
                                   amp_factor<CODES>(f, cu.q, j, sqrtc_l);
                        }
                        acc = fmaf(gain, dot[j], acc);
                    }
                    const float v = wave_sum_lane63(acc);
                    // one lane, one address per row, slices in order: a plain sum in a fixed order
                    if (lane == kWave - 1) atomicAdd(&mine[c_i], v);
                    advance(c_sl, c_i);
                }
            }
        }
    }
    __syncthreads();
    if (lane < nrows) {
        const int64_t row = r_begin + wave + (int64_t)kWaves * lane;
        const float v = mine[lane];
        a.y[(int64_t)b0 * a.ldy + row] = CODES ? v * sqrtf(a.rownorm[row]) : v;
    }
}

// Sums of 16 per-lane values over the 64 lanes, all 16 at once: at each of the first four steps a lane
// hands half of its values to the partner lane (lane ^ 1, 2, 4, 8) and adds the partner's other half
// to the ones it keeps, so the work halves every step (8 + 4 + 2 + 1 additions instead of 16 per
// step); two more steps add the four rows of 16 lanes.  Returns, in every lane, the total of vector
// number  8*(lane&1) + 4*((lane>>1)&1) + 2*((lane>>2)&1) + ((lane>>3)&1).  Fixed order.
__device__ inline float wave_sum16(const float (&a)[16], int lane)
{
    const bool b0 = lane & 1, b1 = lane & 2, b2 = lane & 4, b3 = lane & 8;
    float n8[8], n4[4], n2[2];
#pragma unroll
    for (int c = 0; c < 8; c++) {
        const float keep = b0 ? a[c + 8] : a[c], send = b0 ? a[c] : a[c + 8];
        n8[c] = keep + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, false));
    }
#pragma unroll
    for (int c = 0; c < 4; c++) {
        const float keep = b1 ? n8[c + 4] : n8[c], send = b1 ? n8[c] : n8[c + 4];
        n4[c] = keep + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0x4E, 0xF, 0xF, false));
    }
#pragma unroll
    for (int c = 0; c < 2; c++) {
        const float keep = b2 ? n4[c + 2] : n4[c], send = b2 ? n4[c] : n4[c + 2];
        n2[c] = keep + __shfl_xor(send, 4, kWave);
    }
    const float keep = b3 ? n2[1] : n2[0], send = b3 ? n2[0] : n2[1];
    float v = keep + __shfl_xor(send, 8, kWave);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// Sixteen activation vectors in one pass over the codes.  With four neighbouring groups per lane the
// activations of 16 vectors would need 256 registers, so here a lane owns ONE group column (a wave
// covers 64 consecutive groups of a row, 64 registers of activations) and keeps three ROWS in flight
// instead (a fourth spills registers and measured slower): the table walks overlap as in the other kernels, and every decoded group is used for
// 16 dot products.  Waves: nsl slices of 64 groups x rl row lanes.  Per row and vector the wave's
// sum goes to LDS, where the slices' partial sums meet in slice order (deterministic).
// AMP: 0 = float32 amplitudes, 1 = amplitude codes.
constexpr int kWide = 16;            // vectors per pass
constexpr int kWideRows = 3;         // rows a wave keeps in flight
constexpr size_t kWidePartBytes = 64 * kWide * sizeof(float);   // (row, slice) pairs of a batch x vectors

template <int AMP, bool B24>
__global__ __launch_bounds__(kGemvThreads) void gemv8_wide_kernel(fast8_launch f, pvq_decode_args a, int b0,
                                                                  int nvec, int nsl, int rl, int rows_per_block)
{
    constexpr bool CODES = AMP != 0;
    constexpr int RI = kWideRows, NB = kWide;
    __shared__ __align__(16) unsigned char lds[kLdsBytes];
    float *sqrtc_l = reinterpret_cast<float *>(lds + f.p.tab_bytes);
    float *part = sqrtc_l + 256;

    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r_end = std::min<int64_t>(a.rows, r_begin + rows_per_block);
    const int64_t r_last = r_end - 1;
    const int G = (int)a.groups;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int slice = wave % nsl, rowlane = wave / nsl;
    const int g = slice * kWave + lane;
    const bool in_row = g < G;
    const uint32_t gc = in_row ? (uint32_t)g : 0u;     // lanes beyond the row decode its first group against zeros
    const int RB = RI * rl;
    // the vector whose wave total wave_sum16 leaves in this lane
    const int my_vector = 8 * (lane & 1) + 4 * ((lane >> 1) & 1) + 2 * ((lane >> 2) & 1) + ((lane >> 3) & 1);

    // what a lane fetches per row: the dword that holds its index, and its amplitude (code word or float)
    struct item { uint32_t w, s; };
    auto fetch = [&](int64_t row, item &it) {
        row = std::min<int64_t>(row, r_last);
        const unsigned char *irow = reinterpret_cast<const unsigned char *>(a.index + row * a.index_row_words);
        if constexpr (B24) {
            // the 3 bytes of group g start at byte 3g; one dword load from byte 3g-1 (3g for g = 0)
            // holds them and stays inside the row
            uint32_t v;
            __builtin_memcpy(&v, irow + 3u * gc - (gc > 0 ? 1u : 0u), 4);
            it.w = v;
        } else {
            const uint32_t b = (uint32_t)f.index_bits;
            const uint32_t pos = gc * b, w0 = pos >> 5, sh = pos & 31;
            uint64_t v = reinterpret_cast<const uint32_t *>(irow)[w0];
            if (sh + b > 32) v |= (uint64_t)reinterpret_cast<const uint32_t *>(irow)[w0 + 1] << 32;
            it.w = (uint32_t)(v >> sh) & (uint32_t)((1ull << b) - 1ull);
        }
        if constexpr (CODES)
            it.s = (reinterpret_cast<const uint32_t *>(a.scale) + row * a.scale_row_words)[(gc * (uint32_t)f.scale_bits) >> 5];
        else
            it.s = __float_as_uint(reinterpret_cast<const float *>(a.scale)[row * a.groups + gc]);
    };

    item cur[RI];
    if (r_begin < r_end) {
#pragma unroll
        for (int i = 0; i < RI; i++) fetch(r_begin + i * rl + rowlane, cur[i]);
    }
    load_tables<false>(lds, f, sqrtc_l);
    if (r_begin >= r_end) return;

    uint32_t xr[NB][4];
#pragma unroll
    for (int b = 0; b < NB; b++) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (in_row && b < nvec)     // fewer than 16 vectors: the missing ones are zeros and are not written
            v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(a.x) + (int64_t)(b0 + b) * a.ldx + (int64_t)g * 8);
        xr[b][0] = v.x; xr[b][1] = v.y; xr[b][2] = v.z; xr[b][3] = v.w;
    }

    for (int64_t batch = r_begin; batch < r_end; batch += RB) {
        uint32_t c[RI], pr[RI][4], n2x4[RI];
        float amp[RI];
#pragma unroll
        for (int i = 0; i < RI; i++) {
            if constexpr (B24) c[i] = gc > 0 ? cur[i].w >> 8 : cur[i].w & 0xFFFFFFu;
            else c[i] = cur[i].w;
            if constexpr (CODES) {
                const uint32_t code = (cur[i].s >> ((gc * (uint32_t)f.scale_bits) & 31u)) & ((1u << f.scale_bits) - 1u);
                amp[i] = sqrtc_l[code];
            } else {
                amp[i] = __uint_as_float(cur[i].s);
            }
            // the registers of the consumed row take this wave's row of the next batch
            fetch(batch + RB + i * rl + rowlane, cur[i]);
        }
        pvq_fast8_decode<RI, false>(lds, f.blob, f.p, c, pr, n2x4);
#pragma unroll
        for (int i = 0; i < RI; i++) {
            const float gain = amp[i] * *reinterpret_cast<const float *>(lds + f.p.invs + n2x4[i]);
            float acc[NB];
#pragma unroll
            for (int b = 0; b < NB; b++) {
                float s = dot2_bf16(pr[i][0], xr[b][0], 0.0f);
                s = dot2_bf16(pr[i][1], xr[b][1], s);
                s = dot2_bf16(pr[i][2], xr[b][2], s);
                s = dot2_bf16(pr[i][3], xr[b][3], s);
                acc[b] = gain * s;
            }
            const float v = wave_sum16(acc, lane);
            if (lane < NB) part[((i * rl + rowlane) * nsl + slice) * NB + my_vector] = v;
        }
        __syncthreads();
        if ((int)threadIdx.x < RB * NB) {
            const int rloc = threadIdx.x / NB, b = threadIdx.x % NB;
            const int64_t row = batch + rloc;
            if (row < r_end && b < nvec) {
                float v = 0.0f;
                for (int s = 0; s < nsl; s++) v += part[(rloc * nsl + s) * NB + b];
                if constexpr (CODES) v *= sqrtf(a.rownorm[row]);
                a.y[(int64_t)(b0 + b) * a.ldy + row] = v;
            }
        }
        __syncthreads();   // `part` is rewritten by the next batch
    }
}

// ---------------------------------------------------------------------------------------------
// Many activation vectors: the dot products on the matrix cores
// ---------------------------------------------------------------------------------------------

// With 3..16 vectors the dot products (8 x 16 multiply-adds per group) outweigh the decoding, and they go
// to the matrix cores as small independent products: v_mfma_f32_4x4x4_16b_bf16 multiplies, in each of the
// 16 blocks of four lanes, a 4 x 4 matrix A (row = lane of the block, 4 values along k per lane) by a 4 x 4
// matrix B (column = lane of the block), and leaves column (lane of the block) of the 4 x 4 result in the
// lane's four result registers.  B is what the decoder hands out: the lane's own pulse vector, small integers
// and therefore exact in bf16, two instructions for its 8 coordinates.  A holds the activations of the same 8
// columns for four vectors; with the instruction's broadcast control (cbsz 2: the blocks of a row of 16 lanes
// all take the A of block `abid` of that row) one load per group, lane (m, kb) fetching vector m, serves all
// sixteen lanes of the row for the vectors 4 abid .. 4 abid + 3.  A lane therefore gets y . x of ITS group for
// four vectors per instruction pair, multiplies by the group's gain (float32, as in the single-vector kernels:
// gain * (y . x), every product y_i x_i exact) and keeps a running sum per vector: four multiply-adds per group
// and four vectors beside the decoding, nothing of the weights is converted or split.
// A wave takes 16 rows x 64 consecutive groups: lane (m, kb) = (lane % 16, lane / 16) decodes the groups
// slab + 16*q + 4*kb + j of row m, quad q = 0..3 after quad (j = 0..3 through the table decoder at once), so
// that the four k-blocks read 16 neighbouring groups (48 contiguous bytes of indices, one word of codes).
// The sums of the lanes and waves that share a row meet at the end of a round: the four k-blocks inside the
// wave, then four waves per phase in LDS, added in wave order (deterministic).
typedef __attribute__((ext_vector_type(4))) short bf16x4_bits_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// y . x for the lane's group and the vectors 4 S .. 4 S + 3 (xlo, xhi: this row of lanes' activations, columns
// 0..3 and 4..7 of the group; ylo, yhi: the lane's pulses)
template <int S>
__device__ inline f32x4_t group_dots(bf16x4_bits_t xlo, bf16x4_bits_t xhi, bf16x4_bits_t ylo, bf16x4_bits_t yhi)
{
    const f32x4_t zero = {0.0f, 0.0f, 0.0f, 0.0f};
    const f32x4_t d = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(xlo, ylo, zero, 2, S, 0);
    return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(xhi, yhi, d, 2, S, 0);
}

constexpr int kMfmaRows = 16;                 // rows of a tile
constexpr int kMfmaSlab = 64;                 // groups of a row that one wave takes
constexpr int kMfmaSlots = 4;                 // waves whose results meet in LDS at a time
constexpr size_t kMfmaPartBytes = kMfmaSlots * 256 * sizeof(float);

// AMP: 0 = float32 amplitudes, 1 = amplitude codes.  NS = vectors / 4, rounded up.  24-bit indices.
// nslabs = slabs per row.  A workgroup
// owns tiles_per_block consecutive row tiles and takes them in rounds: four tiles at a time while four are
// left (four waves per tile, every wave the slabs slice, slice + 4, ...), then two (eight waves each), then
// one (sixteen waves, or as many as the row has slabs, rounded up to four).  Few, long rounds keep the
// barriers of the reduction and the unhidden first loads of a tile rare.
template <int AMP, int NS>
__global__ __launch_bounds__(kGemvThreads) void gemv8_mfma_kernel(fast8_launch f, pvq_decode_args a, int b0,
                                                                  int nvec, int tiles_per_block, int nslabs)
{
    constexpr bool CODES = AMP != 0;
    constexpr int kWaves = kGemvThreads / kWave;
    __shared__ __align__(16) unsigned char lds[kLdsBytes];
    float *sqrtc_l = reinterpret_cast<float *>(lds + f.p.tab_bytes);
    float *part = sqrtc_l + 256;

    const int64_t r_begin = (int64_t)blockIdx.x * tiles_per_block * kMfmaRows;
    const int64_t r_end = std::min<int64_t>(a.rows, r_begin + (int64_t)tiles_per_block * kMfmaRows);
    const int64_t r_last = r_end - 1;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int m = lane & 15, kb = lane >> 4;
    const uint32_t sb = (uint32_t)f.scale_bits;
    const int nsl_cap = std::min(kWaves, (nslabs + kMfmaSlots - 1) / kMfmaSlots * kMfmaSlots);

    load_tables<false>(lds, f, sqrtc_l);
    if (r_begin >= r_end) return;

    // the other operand: vector m, the 8 columns of the lane's group.  Lanes beyond the vectors given read
    // the last vector again (no condition around the loads); their columns of the result are not stored.
    const uint16_t *xvec = reinterpret_cast<const uint16_t *>(a.x) + (int64_t)(b0 + std::min(m, nvec - 1)) * a.ldx;

    // what a lane reads per four groups: three index words, and the word with the four codes or four floats
    struct quad_t { uint32_t w[3]; uint32_t s[CODES ? 1 : 4]; };
    auto fetch = [&](int64_t row, uint32_t g, quad_t &it) {
        const uint3 iw = *reinterpret_cast<const uint3 *>(a.index + row * a.index_row_words + (g >> 2) * 3u);   // one 12-byte load
        it.w[0] = iw.x; it.w[1] = iw.y; it.w[2] = iw.z;
        if constexpr (CODES) {
            it.s[0] = (reinterpret_cast<const uint32_t *>(a.scale) + row * a.scale_row_words)[(g * sb) >> 5];
        } else {
            const float *sp = reinterpret_cast<const float *>(a.scale) + row * a.groups + g;
#pragma unroll
            for (int j = 0; j < 4; j++) it.s[j] = __float_as_uint(sp[j]);
        }
    };

    const int tiles = (int)((r_end - r_begin + kMfmaRows - 1) / kMfmaRows);
    // a round: rl tiles from t0 on, nsl waves each (uniform in the workgroup); this wave's part of it
    struct round_t { int rl, nsl, nwaves, nq; uint32_t gl0; int64_t row; bool live; };
    auto make_round = [&](int t0) {
        round_t R;
        const int left = tiles - t0;
        R.rl = left >= 4 ? 4 : left >= 2 ? 2 : 1;
        R.nsl = std::min(kWaves / R.rl, nsl_cap);
        R.nwaves = R.nsl * R.rl;
        const int slice = wave % R.nsl, tile = t0 + wave / R.nsl;     // uniform in the wave
        // the lane's groups: slab slice + nsl * pass, there 4 * kb + 16 * q + j; quad number qq = 4 * pass + q
        R.gl0 = (uint32_t)(slice * kMfmaSlab + 4 * kb);
        R.nq = slice < nslabs ? 4 * ((nslabs - slice + R.nsl - 1) / R.nsl) : 0;
        R.live = left > 0 && wave < R.nwaves && tile < tiles && R.nq > 0;
        R.row = std::min<int64_t>(r_begin + (int64_t)tile * kMfmaRows + m, r_last);
        return R;
    };
    round_t R = make_round(0);
    quad_t cur, nxt;
    if (R.live) fetch(R.row, R.gl0, cur);
    for (int t0 = 0; t0 < tiles;) {
        // the first quad of the next round is fetched during the last quad of this one, so that the
        // reduction's barriers do not stand between a wave and its next indices
        const round_t N = make_round(t0 + R.rl);
        const int nsl = R.nsl, nwaves = R.nwaves, nq = R.nq;
        const bool live = R.live;
        auto quad_group = [&](int qq) { return R.gl0 + (uint32_t)((qq >> 2) * nsl * kMfmaSlab + 16 * (qq & 3)); };
        // tot[s][r]: this lane's part of (row m) . (vector 4 s + r)
        f32x4_t tot[4];
#pragma unroll
        for (int v = 0; v < 4; v++) tot[v] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
        if (!live && N.live) fetch(N.row, N.gl0, cur);
        if (live) {
#pragma unroll 1
            for (int q = 0; q < nq; q++) {
                const uint32_t gq = quad_group(q);
                const bool last = q + 1 == nq;
                fetch(last && N.live ? N.row : R.row, last ? (N.live ? N.gl0 : gq) : quad_group(q + 1), nxt);
                // With many vectors the activations' loads are what the vector memory path is busy with.  A lane's own
                // four groups lie side by side, so a load for "group j of every k-block" takes 16 bytes out of every 64;
                // with kSwap the four k-blocks of a row trade decoded groups instead (lane kb gets group kb of lane t for
                // instruction t: a 4 x 4 transposition over the rows of 16 lanes by register pairs trading halves and
                // rows), and instruction t's activations are 64 bytes in a row per vector.
                constexpr bool kSwap = NS >= 3;
                uint4 bx[4];
#pragma unroll
                for (int j = 0; j < 4; j++)
                    bx[j] = *reinterpret_cast<const uint4 *>(xvec + (int64_t)(kSwap ? gq - 4 * kb + 4 * j + kb : gq + j) * 8);
                uint32_t c[4], pr[4][4], n2x4[4];
                c[0] = cur.w[0] & 0xFFFFFFu;
                c[1] = __builtin_amdgcn_alignbit(cur.w[1], cur.w[0], 24) & 0xFFFFFFu;
                c[2] = __builtin_amdgcn_alignbit(cur.w[2], cur.w[1], 16) & 0xFFFFFFu;
                c[3] = cur.w[2] >> 8;
                pvq_fast8_decode<4, false>(lds, f.blob, f.p, c, pr, n2x4);
                const uint32_t codes = CODES ? cur.s[0] >> ((gq * sb) & 31u) : 0u;
                float gains[4];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    float gain = *reinterpret_cast<const float *>(lds + f.p.invs + n2x4[j]);
                    if constexpr (CODES) gain *= sqrtc_l[(codes >> (j * sb)) & ((1u << sb) - 1u)];
                    else gain *= __uint_as_float(cur.s[j]);
                    gains[j] = gain;
                }
                if constexpr (kSwap) {
                    // value j of row kb <-> value kb of row j, for the pulses' four words and the gain
                    auto transpose = [](uint32_t &r0, uint32_t &r1, uint32_t &r2, uint32_t &r3) {
                        auto a = __builtin_amdgcn_permlane32_swap(r0, r2, false, false);
                        auto b = __builtin_amdgcn_permlane32_swap(r1, r3, false, false);
                        auto e = __builtin_amdgcn_permlane16_swap(a[0], b[0], false, false);
                        auto g = __builtin_amdgcn_permlane16_swap(a[1], b[1], false, false);
                        r0 = e[0]; r1 = e[1]; r2 = g[0]; r3 = g[1];
                    };
#pragma unroll
                    for (int w = 0; w < 4; w++) transpose(pr[0][w], pr[1][w], pr[2][w], pr[3][w]);
                    uint32_t g0 = __float_as_uint(gains[0]), g1 = __float_as_uint(gains[1]), g2 = __float_as_uint(gains[2]),
                             g3 = __float_as_uint(gains[3]);
                    transpose(g0, g1, g2, g3);
                    gains[0] = __uint_as_float(g0); gains[1] = __uint_as_float(g1); gains[2] = __uint_as_float(g2);
                    gains[3] = __uint_as_float(g3);
                }
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float gain = gains[j];
                    const bf16x4_bits_t xlo = __builtin_bit_cast(bf16x4_bits_t, make_uint2(bx[j].x, bx[j].y)),
                                        xhi = __builtin_bit_cast(bf16x4_bits_t, make_uint2(bx[j].z, bx[j].w)),
                                        ylo = __builtin_bit_cast(bf16x4_bits_t, make_uint2(pr[j][0], pr[j][1])),
                                        yhi = __builtin_bit_cast(bf16x4_bits_t, make_uint2(pr[j][2], pr[j][3]));
                    f32x4_t d[4];
                    d[0] = group_dots<0>(xlo, xhi, ylo, yhi);
                    if constexpr (NS > 1) d[1] = group_dots<1>(xlo, xhi, ylo, yhi);
                    if constexpr (NS > 2) d[2] = group_dots<2>(xlo, xhi, ylo, yhi);
                    if constexpr (NS > 3) d[3] = group_dots<3>(xlo, xhi, ylo, yhi);
#pragma unroll
                    for (int v = 0; v < NS; v++) {
#pragma unroll
                        for (int r = 0; r < 4; r++) tot[v][r] = fmaf(gain, d[v][r], tot[v][r]);
                    }
                }
                cur = nxt;
            }
        }
        // The four k-blocks of a row sit in lanes m, m + 16, m + 32, m + 48: two exchanges, in each of which a
        // lane gives away half of the vectors it still holds and adds the partner's part of the half it keeps.
        // Lane (m, kb) ends with the wave's sums of row m for the vectors 4 s .. 4 s + 3, s = 2 (kb & 1) + (kb >> 1).
        f32x4_t fin;
        {
            const bool odd = kb & 1, upper = kb & 2;
            f32x4_t k0, k1;
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const float keep0 = odd ? tot[2][r] : tot[0][r], keep1 = odd ? tot[3][r] : tot[1][r];
                const float send0 = odd ? tot[0][r] : tot[2][r], send1 = odd ? tot[1][r] : tot[3][r];
                k0[r] = keep0 + __shfl_xor(send0, 16, kWave);
                k1[r] = keep1 + __shfl_xor(send1, 16, kWave);
            }
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const float keep = upper ? k1[r] : k0[r], send = upper ? k0[r] : k1[r];
                fin[r] = keep + __shfl_xor(send, 32, kWave);
            }
        }
        const int fin_vec = 4 * (2 * (kb & 1) + (kb >> 1));
        // Phases of four waves (nsl is a multiple of four, so a phase lies within one row tile); thread
        // (tile row, vector) of the first 256 adds them in wave order.
        float sum = 0.0f;
        const int phases = nwaves / kMfmaSlots;
        for (int ph = 0; ph < phases; ph++) {
            if (wave / kMfmaSlots == ph) {
                float *slot = part + (wave % kMfmaSlots) * 256;
                *reinterpret_cast<f32x4_t *>(slot + m * 16 + fin_vec) = fin;
            }
            __syncthreads();
            if (threadIdx.x < 256) {
#pragma unroll
                for (int sidx = 0; sidx < kMfmaSlots; sidx++) sum += part[sidx * 256 + threadIdx.x];
                // the last slices of a row tile: its sums are complete
                if (((ph + 1) * kMfmaSlots) % nsl == 0) {
                    const int otile = t0 + (ph * kMfmaSlots) / nsl;
                    const int64_t orow = r_begin + (int64_t)otile * kMfmaRows + (threadIdx.x >> 4);
                    const int n = threadIdx.x & 15;
                    if (otile < tiles && orow < r_end && n < nvec) {
                        float v = sum;
                        if constexpr (CODES) v *= sqrtf(a.rownorm[orow]);
                        a.y[(int64_t)(b0 + n) * a.ldy + orow] = v;
                    }
                    sum = 0.0f;
                }
            }
            __syncthreads();
        }
        t0 += R.rl;
        R = N;
    }
}

// ---------------------------------------------------------------------------------------------
// decode to a matrix
// ---------------------------------------------------------------------------------------------

template <int OUT>
__device__ inline void store_group(void *W_out, int64_t elem, const uint32_t (&pr)[4], float gain)
{
    float v[8];
#pragma unroll
    for (int j = 0; j < 4; j++) {
        v[2 * j] = gain * __uint_as_float(pr[j] << 16);
        v[2 * j + 1] = gain * __uint_as_float(pr[j] & 0xFFFF0000u);
    }
    if constexpr (OUT == PVQ_F32) {
        float *o = reinterpret_cast<float *>(W_out) + elem;
        *reinterpret_cast<float4 *>(o) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4 *>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
        uint32_t q[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if constexpr (OUT == PVQ_F16) {
                q[j] = (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v[2 * j]) |
                       ((uint32_t)__builtin_bit_cast(uint16_t, (_Float16)v[2 * j + 1]) << 16);
            } else {
                // v_cvt_pk_bf16_f32: round to nearest even, two values per instruction
                const f32x2_t pair = {v[2 * j], v[2 * j + 1]};
                q[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t));
            }
        }
        *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(W_out) + elem) = make_uint4(q[0], q[1], q[2], q[3]);
    }
}

// Wave items = (row, tile of 256 groups).  Items go round robin over all waves of the grid, so that at
// any moment the grid writes one contiguous, advancing window of the output (a few MB) rather than one
// window per block: DRAM pages are then filled by neighbours in time.  A wave fetches one item ahead.
template <int OUT, bool CODES, bool B24>
__global__ __launch_bounds__(kMaxThreads) void decode8_kernel(fast8_launch f, pvq_decode_args a)
{
    // static, so that table offsets fold into the LDS instructions' immediate fields
    __shared__ __align__(16) unsigned char lds[kLdsBytes];
    float *sqrtc_l = reinterpret_cast<float *>(lds + f.p.tab_bytes);
    load_tables<false>(lds, f, sqrtc_l);

    const int G = (int)a.groups;
    const int lane = threadIdx.x & (kWave - 1);
    // the wave's number as a scalar, so that rows, tiles and row addresses are computed once per wave
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int nwaves = blockDim.x / kWave;
    const uint32_t T = (uint32_t)((a.groups + kTileGroups - 1) / kTileGroups);   // tiles per row
    const int64_t total = a.rows * (int64_t)T;
    const int64_t i_end = total;
    // (row, tile) of this wave's item, advanced by one item of every wave of the grid per step
    // without dividing again
    const int64_t stride = (int64_t)gridDim.x * nwaves;
    const int64_t step_rows = stride / T;
    const uint32_t step_tiles = (uint32_t)(stride % T);
    int64_t item = (int64_t)blockIdx.x * nwaves + wave;
    int64_t row = item / T;
    uint32_t tile = (uint32_t)(item - row * T);

    item_t cur, nxt;
    float cur_rn = 1.0f, nxt_rn = 1.0f;
    bool live = item < i_end;     // uniform in the wave
    if (!live) return;            // (after the table copy's barrier; no barrier follows)
    fetch_item<CODES, B24>(f, a, row, (int)tile * kTileGroups + lane, cur);
    if constexpr (CODES) cur_rn = a.rownorm[row];
    while (live) {
        int64_t nrow = row + step_rows;
        uint32_t ntile = tile + step_tiles;
        if (ntile >= T) { ntile -= T; nrow += 1; }
        const bool nlive = item + stride < i_end;
        if (!nlive) { nrow = row; ntile = tile; }     // nothing follows: fetch this item again, unused
        fetch_item<CODES, B24>(f, a, nrow, (int)ntile * kTileGroups + lane, nxt);
        if constexpr (CODES) nxt_rn = a.rownorm[nrow];

        const int gbase = (int)tile * kTileGroups + lane;
        const float srn = CODES ? sqrtf(cur_rn) : 1.0f;
        uint32_t c[kGroupsPerLane], prs[kGroupsPerLane][4], n2x4s[kGroupsPerLane];
        item_indices<B24>(cur, gbase, c);
        pvq_fast8_decode<kGroupsPerLane, false>(lds, f.blob, f.p, c, prs, n2x4s);
#pragma unroll
        for (int j = 0; j < kGroupsPerLane; j++) {
            const int g = gbase + kWave * j;
            if (g < G) {
                // amp / sqrt(n2): the amplitude first (sqrt(center) * sqrt(row normaliser), or the stored
                // float), then the tabulated 1/sqrt(n2)
                const float amp = CODES ? sqrtc_l[item_code(f, cur, gbase, j)] * srn : __uint_as_float(cur.a[j]);
                const float gain = amp * *reinterpret_cast<const float *>(lds + f.p.invs + n2x4s[j]);
                store_group<OUT>(a.W_out, row * a.ldw + (int64_t)g * 8, prs[j], gain);
            }
        }
        cur = nxt; cur_rn = nxt_rn; row = nrow; tile = ntile; live = nlive; item += stride;
    }
}

fast8_launch make_launch(const pvq_ctx *c, bool gemv)
{
    fast8_launch f;
    f.p = gemv ? c->fast8g : c->fast8; f.blob = gemv ? c->fast8g_blob : c->fast8_blob; f.sqrtc = c->sqrtc;
    f.index_bits = c->index_bits; f.scale_bits = c->scale_bits;
    return f;
}

int g_num_cus = 0;

template <int NB, bool AHEAD>
hipError_t launch_gemv_nb(const fast8_launch &f, const pvq_decode_args &a, int b0, int nsl, int rl,
                          int rows_per_block, dim3 grid, dim3 block, size_t lds, hipStream_t s)
{
    const bool b24 = f.index_bits == 24;
    // the fused gain table must fit behind the blob together with the partial-sum buffer
    const size_t fused_bytes = ((size_t)(f.p.k2max + 1) << f.scale_bits) * 4;
    const bool fused = f.scale_bits > 0 && f.scale_bits <= 2 &&
                       f.p.lds_bytes + fused_bytes + kPartBytes <= (size_t)kLdsBytes;
    const int amp = f.scale_bits == 0 ? 0 : (fused ? 2 : 1);
#define PVQ_GEMV_CASE(AMP, B24) \
    hipLaunchKernelGGL((gemv8_kernel<NB, AMP, B24, AHEAD>), grid, block, lds, s, f, a, b0, nsl, rl, rows_per_block)
    if (amp == 2) { if (b24) PVQ_GEMV_CASE(2, true); else PVQ_GEMV_CASE(2, false); }
    else if (amp == 1) { if (b24) PVQ_GEMV_CASE(1, true); else PVQ_GEMV_CASE(1, false); }
    else { if (b24) PVQ_GEMV_CASE(0, true); else PVQ_GEMV_CASE(0, false); }
#undef PVQ_GEMV_CASE
    return hipGetLastError();
}

template <int OUT>
hipError_t launch_decode_out(const fast8_launch &f, const pvq_decode_args &a, dim3 grid,
                             dim3 block, size_t lds, hipStream_t s)
{
    const bool codes = f.scale_bits > 0, b24 = f.index_bits == 24;
    if (codes && b24) hipLaunchKernelGGL((decode8_kernel<OUT, true, true>), grid, block, lds, s, f, a);
    else if (codes) hipLaunchKernelGGL((decode8_kernel<OUT, true, false>), grid, block, lds, s, f, a);
    else if (b24) hipLaunchKernelGGL((decode8_kernel<OUT, false, true>), grid, block, lds, s, f, a);
    else hipLaunchKernelGGL((decode8_kernel<OUT, false, false>), grid, block, lds, s, f, a);
    return hipGetLastError();
}

}  // namespace

hipError_t pvq_fast8_prepare(void)
{
    static hipError_t once = [] {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&g_num_cus, hipDeviceAttributeMultiprocessorCount, dev);
        return e;
    }();
    return once;
}

bool pvq_fast8_decode_usable(const pvq_ctx *c, const pvq_decode_args &a)
{
    (void)a;
    return c->fast8_blob != nullptr;
}

bool pvq_fast8_gemv_usable(const pvq_ctx *c, const pvq_decode_args &a)
{
    // a row must fit the waves of one workgroup: at most 16 slices of 256 groups
    // lanes take whole quads of groups
    return c->fast8_blob != nullptr && a.groups % kGroupsPerLane == 0 &&
           (a.groups + kTileGroups - 1) / kTileGroups <= kGemvThreads / kWave;
}

hipError_t pvq_fast8_launch_decode(const pvq_ctx *c, const pvq_decode_args &a, int out_dtype, hipStream_t s)
{
    const fast8_launch f = make_launch(c, false);
    const size_t lds = 0;  // the kernels own the whole LDS statically
    const int64_t total = a.rows * ((a.groups + kTileGroups - 1) / kTileGroups);   // wave items
    // every block pays the table copy, so blocks get at least 64 wave items (16K groups) each
    const int64_t want_blocks = std::min<int64_t>(g_num_cus > 0 ? g_num_cus : 256, (total + 63) / 64);
    const int64_t nblocks = std::max<int64_t>(1, want_blocks);
    const dim3 grid((unsigned)nblocks), block(kMaxThreads);
    switch (out_dtype) {
    case PVQ_F32: return launch_decode_out<PVQ_F32>(f, a, grid, block, lds, s);
    case PVQ_F16: return launch_decode_out<PVQ_F16>(f, a, grid, block, lds, s);
    default: return launch_decode_out<PVQ_BF16>(f, a, grid, block, lds, s);
    }
}

namespace {

// one launch of the fused product for vectors [b0, b0 + NB)
template <int NB, bool AHEAD>
hipError_t launch_gemv_pass(const pvq_ctx *c, const pvq_decode_args &a, int b0, hipStream_t s)
{
    const fast8_launch f = make_launch(c, AHEAD);
    const int nsl = (int)((a.groups + kTileGroups - 1) / kTileGroups);
    const int rl = std::max(1, (kGemvThreads / kWave) / nsl);
    const int RB = (AHEAD ? kGemvRowsPerWaveAhead : kGemvRowsPerWave) * rl;
    const size_t lds = 0;  // the kernels own the whole LDS statically
    const int64_t batches = (a.rows + RB - 1) / RB;
    const int64_t nblocks = std::max<int64_t>(1, std::min<int64_t>(g_num_cus > 0 ? g_num_cus : 256, batches));
    const int rows_per_block = (int)(((batches + nblocks - 1) / nblocks) * RB);
    const dim3 grid((unsigned)((a.rows + rows_per_block - 1) / rows_per_block)), block((unsigned)(kWave * nsl * rl));
    return launch_gemv_nb<NB, AHEAD>(f, a, b0, nsl, rl, rows_per_block, grid, block, lds, s);
}

constexpr size_t kRowPartBytes = (kGemvThreads / kWave) * kRowMaxRowsPerWave * sizeof(float);

// the fused gain table (amplitude codes of at most 2 bits) must fit behind the tables with the partial sums
bool row_fused(const fast8_launch &f)
{
    const size_t fused_bytes = ((size_t)(f.p.k2max + 1) << f.scale_bits) * 4;
    return f.scale_bits > 0 && f.scale_bits <= 2 && f.p.lds_bytes + fused_bytes + kRowPartBytes <= (size_t)kLdsBytes;
}

// one launch of the barrier-free single-vector kernel for vector b0
hipError_t launch_gemv_row(const pvq_ctx *c, const pvq_decode_args &a, int b0, hipStream_t s)
{
    const fast8_launch f = make_launch(c, true);
    constexpr int kWaves = kGemvThreads / kWave;
    const int64_t units = g_num_cus > 0 ? g_num_cus : 256;
    // whole rounds of sixteen rows per workgroup, at most 32 rounds (the partial sums' place in LDS)
    const int64_t rounds = (a.rows + kWaves - 1) / kWaves;
    const int64_t nblocks = std::max<int64_t>(std::min<int64_t>(units, rounds), (rounds + kRowMaxRowsPerWave - 1) / kRowMaxRowsPerWave);
    const int rows_per_block = (int)(((rounds + nblocks - 1) / nblocks) * kWaves);
    const dim3 grid((unsigned)((a.rows + rows_per_block - 1) / rows_per_block)), block((unsigned)kGemvThreads);
    const int nsl = (int)(a.groups / kTileGroups);
    const bool b24 = f.index_bits == 24;
    const int amp = f.scale_bits == 0 ? 0 : (row_fused(f) ? 2 : 1);
#define PVQ_ROW_CASE(AMP, B24) \
    hipLaunchKernelGGL((gemv8_row_kernel<AMP, B24>), grid, block, 0, s, f, a, b0, rows_per_block, nsl)
    if (amp == 2) { if (b24) PVQ_ROW_CASE(2, true); else PVQ_ROW_CASE(2, false); }
    else if (amp == 1) { if (b24) PVQ_ROW_CASE(1, true); else PVQ_ROW_CASE(1, false); }
    else { if (b24) PVQ_ROW_CASE(0, true); else PVQ_ROW_CASE(0, false); }
#undef PVQ_ROW_CASE
    return hipGetLastError();
}

}  // namespace

namespace {

// one launch of the 16-vector kernel for vectors [b0, b0 + nvec), nvec <= 16
hipError_t launch_gemv_wide(const pvq_ctx *c, const pvq_decode_args &a, int b0, int nvec, hipStream_t s)
{
    const fast8_launch f = make_launch(c, false);
    const int nsl = (int)((a.groups + kWave - 1) / kWave);
    const int rl = std::max(1, (kGemvThreads / kWave) / nsl);
    const int RB = kWideRows * rl;
    const int64_t batches = (a.rows + RB - 1) / RB;
    const int64_t nblocks = std::max<int64_t>(1, std::min<int64_t>(g_num_cus > 0 ? g_num_cus : 256, batches));
    const int rows_per_block = (int)(((batches + nblocks - 1) / nblocks) * RB);
    const dim3 grid((unsigned)((a.rows + rows_per_block - 1) / rows_per_block)), block((unsigned)(kWave * nsl * rl));
    const bool b24 = f.index_bits == 24, codes = f.scale_bits > 0;
#define PVQ_WIDE_CASE(AMP, B24) \
    hipLaunchKernelGGL((gemv8_wide_kernel<AMP, B24>), grid, block, 0, s, f, a, b0, nvec, nsl, rl, rows_per_block)
    if (codes) { if (b24) PVQ_WIDE_CASE(1, true); else PVQ_WIDE_CASE(1, false); }
    else { if (b24) PVQ_WIDE_CASE(0, true); else PVQ_WIDE_CASE(0, false); }
#undef PVQ_WIDE_CASE
    return hipGetLastError();
}

// one launch of the matrix-core kernel for vectors [b0, b0 + nvec), nvec <= 16
hipError_t launch_gemv_mfma(const pvq_ctx *c, const pvq_decode_args &a, int b0, int nvec, hipStream_t s)
{
    const fast8_launch f = make_launch(c, false);
    const int nslabs = (int)(a.groups / kMfmaSlab);
    const int64_t tiles = (a.rows + kMfmaRows - 1) / kMfmaRows;
    const int64_t nblocks = std::max<int64_t>(1, std::min<int64_t>(g_num_cus > 0 ? g_num_cus : 256, tiles));
    const int tiles_per_block = (int)((tiles + nblocks - 1) / nblocks);
    const dim3 grid((unsigned)((tiles + tiles_per_block - 1) / tiles_per_block)), block((unsigned)kGemvThreads);
#define PVQ_MFMA_CASE(AMP, NS) \
    hipLaunchKernelGGL((gemv8_mfma_kernel<AMP, NS>), grid, block, 0, s, f, a, b0, nvec, tiles_per_block, nslabs)
    const int ns = (nvec + 3) / 4;
    if (f.scale_bits > 0) {
        if (ns == 1) PVQ_MFMA_CASE(1, 1); else if (ns == 2) PVQ_MFMA_CASE(1, 2); else if (ns == 3) PVQ_MFMA_CASE(1, 3); else PVQ_MFMA_CASE(1, 4);
    } else {
        if (ns == 1) PVQ_MFMA_CASE(0, 1); else if (ns == 2) PVQ_MFMA_CASE(0, 2); else if (ns == 3) PVQ_MFMA_CASE(0, 3); else PVQ_MFMA_CASE(0, 4);
    }
#undef PVQ_MFMA_CASE
    return hipGetLastError();
}

// the matrix-core kernel takes 24-bit indices and rows of four or more whole slabs of 64 groups, and needs
// room in LDS for the tables, the amplitude table and four waves' results
bool mfma_usable(const pvq_ctx *c, const pvq_decode_args &a)
{
    return c->index_bits == 24 && a.groups % kMfmaSlab == 0 && a.groups >= 4 * kMfmaSlab && a.groups <= (1 << 20) &&
           a.rows <= ((int64_t)1 << 30) &&
           (size_t)c->fast8.tab_bytes + 256 * sizeof(float) + kMfmaPartBytes <= (size_t)kLdsBytes;
}

// the 16-vector kernel takes rows of at most 16 slices of 64 groups whose tables, amplitude table and
// partial sums fit LDS together
bool wide_usable(const pvq_ctx *c, const pvq_decode_args &a)
{
    return (a.groups + kWave - 1) / kWave <= kGemvThreads / kWave &&
           (size_t)c->fast8.tab_bytes + 256 * sizeof(float) + kWidePartBytes <= (size_t)kLdsBytes;
}

// the barrier-free kernel takes rows of whole slices of 256 groups, and pays off when every wave of every
// unit gets a few rows
bool row_usable(const pvq_ctx *c, const pvq_decode_args &a)
{
    const int64_t units = g_num_cus > 0 ? g_num_cus : 256;
    return a.groups % kTileGroups == 0 && a.groups / kTileGroups <= 4096 && a.rows >= units * 16 * 2 &&
           (size_t)c->fast8g.tab_bytes + 256 * sizeof(float) + kRowPartBytes <= (size_t)kLdsBytes;
}

}  // namespace

// The passes that a product of a.batch vectors is made of, in order: which kernel takes how many vectors.
int pvq_fast8_plan_gemv(const pvq_ctx *c, const pvq_decode_args &a, pvq_gemv_pass *out)
{
    // a single vector runs S0 a row ahead (if the tables exist in that flavour); with more vectors
    // the registers go to the activations instead
    const bool ahead = c->fast8g_blob != nullptr;
    int n = 0, b0 = 0;
    while (b0 < a.batch) {
        const int left = a.batch - b0;
        // measured on the benchmark shape: 1 vector 78 us on the barrier-free kernel (84 us with row batches and
        // partial sums through LDS, which remains for short matrices and rows that are not whole slices),
        // 2 vectors 91 us and 4 vectors 111..125 us on the vector-ALU kernels; the matrix-core pass takes
        // 105..117 us whatever the count, so it takes three vectors and more.  Where it cannot run, one
        // 16-vector pass (about 215 us) beats two or more 4-vector passes from eight vectors on.
        pvq_gemv_pass p;
        if (left >= 3 && mfma_usable(c, a)) p = {PVQ_PASS_MFMA, std::min(left, 16)};
        else if (left >= 8 && wide_usable(c, a)) p = {PVQ_PASS_VALU16, std::min(left, kWide)};
        else if (left >= 4) p = {PVQ_PASS_VALU, 4};
        else if (left >= 2) p = {PVQ_PASS_VALU, 2};
        else if (ahead && row_usable(c, a)) p = {PVQ_PASS_VALU_ROWS, 1};
        else p = {PVQ_PASS_VALU, 1};
        out[n++] = p;
        b0 += p.nvec;
    }
    return n;
}

hipError_t pvq_fast8_launch_gemv(const pvq_ctx *c, const pvq_decode_args &a, hipStream_t s)
{
    const bool ahead = c->fast8g_blob != nullptr;
    pvq_gemv_pass plan[16];
    const int n = pvq_fast8_plan_gemv(c, a, plan);
    int b0 = 0;
    for (int i = 0; i < n; i++) {
        const int nvec = plan[i].nvec;
        hipError_t e;
        switch (plan[i].kind) {
        case PVQ_PASS_MFMA: e = launch_gemv_mfma(c, a, b0, nvec, s); break;
        case PVQ_PASS_VALU16: e = launch_gemv_wide(c, a, b0, nvec, s); break;
        case PVQ_PASS_VALU_ROWS: e = launch_gemv_row(c, a, b0, s); break;
        default:
            e = nvec == 4 ? launch_gemv_pass<4, false>(c, a, b0, s)
                : nvec == 2 ? launch_gemv_pass<2, false>(c, a, b0, s)
                : ahead ? launch_gemv_pass<1, true>(c, a, b0, s) : launch_gemv_pass<1, false>(c, a, b0, s);
        }
        if (e != hipSuccess) return e;
        b0 += nvec;
    }
    return hipSuccess;
}
