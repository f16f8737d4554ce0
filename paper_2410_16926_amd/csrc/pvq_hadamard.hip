// Randomised Hadamard rotation along the rows (Sec. 2.3, Sec. 3.3 Step 1): every block of n
// consecutive values of a row becomes H (s . x) / sqrt(n), or, for the inverse, s . (H x) / sqrt(n).
//
// float32 butterflies a,b -> a+b, a-b over strides 1, 2, 4, ..., n/2 in that order, then one
// multiplication by float32(1/sqrt(n)): every value of a stage is one rounded sum or difference of two
// values of the stage before, so the result is the same bit for bit however a stage is scheduled.
//
// A workgroup of L lanes takes 8L consecutive values of a row (whole blocks), 8 per lane.  Strides 1, 2, 4
// run inside a lane's registers; strides 8 .. 256 pair lanes of one wave (lane ^ 1 .. lane ^ 32) and run
// on cross-lane moves, without LDS traffic or barriers; for strides from 512 on the values go through LDS
// so that a lane then owns the 8 values that differ in the next (up to three) index bits.  Blocks of up
// to 512 values therefore never touch LDS.  Loads and stores are 16 or 32 bytes per lane, consecutive
// lanes consecutive addresses.  Bound: HBM (one read, one write of the matrix).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "pvq_internal.h"

namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

// one word of padding per 32: neighbouring groups of lanes that are 64 or 512 words apart fall into
// different banks
__device__ inline uint32_t pad(uint32_t a) { return a + (a >> 5); }

// butterflies over register distance 1, 2, 4 for the first `bits` of them
__device__ inline void stages_in_registers(float (&v)[8], int bits)
{
#pragma unroll
    for (int t = 0; t < 3; t++) {
        if (t < bits) {
            const int h = 1 << t;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                if ((j & h) == 0) {
                    const float a = v[j], b = v[j + h];
                    v[j] = a + b;
                    v[j + h] = a - b;
                }
            }
        }
    }
}

// One butterfly stage between lanes `mask` apart: the lane whose bit is clear holds a and gets a + b, the
// other holds b and gets a - b.
template <int MASK>
__device__ inline void stage_across_lanes(float (&v)[8], int lane)
{
    const bool upper = lane & MASK;
#pragma unroll
    for (int j = 0; j < 8; j++) {
        float partner;
        if constexpr (MASK == 1)
            partner = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[j]), 0xB1, 0xF, 0xF, false));
        else if constexpr (MASK == 2)
            partner = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[j]), 0x4E, 0xF, 0xF, false));
        else
            partner = __shfl_xor(v[j], MASK, 64);
        v[j] = upper ? partner - v[j] : v[j] + partner;
    }
}

// Ownership (P, R): the lane holds the 8 values of its chunk whose index differs in bits 3P .. 3P+R-1 (the
// R low bits of the register number) and, for R < 3, in bits 0 .. 2-R (the other bits of the register
// number); the lane number fills the remaining index bits in order.  (0, 3) is 8 consecutive values.
// The index of register q is own_base(lane) | own_offset(q): the two never share a bit, so the padded
// address splits the same way and the register's part is a compile-time constant.
template <int P, int R>
__device__ inline uint32_t own_base(uint32_t lane)
{
    const uint32_t rest = lane << (3 - R);
    return (rest & ((1u << (3 * P)) - 1u)) | ((rest >> (3 * P)) << (3 * P + R));
}
template <int P, int R>
__device__ constexpr uint32_t own_offset(int q)
{
    return ((uint32_t)q >> R) + (((uint32_t)q & ((1u << R) - 1u)) << (3 * P));
}

// Through LDS from ownership (P0, R0) to (P1, R1); the caller alternates two buffers, so that one barrier
// per exchange is enough (a buffer is written again only after a barrier that every wave reaches after
// its reads of it).
template <int P0, int R0, int P1, int R1>
__device__ inline void exchange(float (&v)[8], float *buf, uint32_t lane)
{
    float *w = buf + pad(own_base<P0, R0>(lane));
#pragma unroll
    for (int q = 0; q < 8; q++) w[pad(own_offset<P0, R0>(q))] = v[q];
    __syncthreads();
    const float *r = buf + pad(own_base<P1, R1>(lane));
#pragma unroll
    for (int q = 0; q < 8; q++) v[q] = r[pad(own_offset<P1, R1>(q))];
}

// IN / OUT: 0 = float32, 2 = bf16 (pvq_dtype values).  LOG2N: 9 stands for every block of up to 512 values
// (log2n says which), 10 .. 13 for that block size.
template <int IN, int OUT, int LOG2N>
__global__ __launch_bounds__(1024) void hadamard_kernel(const void *X, int64_t ldx, void *Y, int64_t ldy,
                                                        int64_t cols, int log2n, const uint8_t *signs,
                                                        int signs_after, float scale, int chunks_per_row)
{
    extern __shared__ __align__(16) float smem[];
    const int L = blockDim.x;
    const int lane = threadIdx.x;
    const int64_t row = blockIdx.x / chunks_per_row;
    const int chunk = blockIdx.x - (int)(row * chunks_per_row);
    const int64_t col0 = (int64_t)chunk * 8 * L + 8 * lane;   // first of this lane's 8 columns
    const bool live = col0 < cols;                             // whole blocks: a lane is in or out

    float v[8];
#pragma unroll
    for (int j = 0; j < 8; j++) v[j] = 0.0f;
    if (live) {
        if constexpr (IN == PVQ_F32) {
            const float *p = reinterpret_cast<const float *>(X) + row * ldx + col0;
            const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
            v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        } else {
            const uint4 q = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(X) + row * ldx + col0);
            const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < 4; j++) {
                v[2 * j] = __uint_as_float(u[j] << 16);
                v[2 * j + 1] = __uint_as_float(u[j] & 0xFFFF0000u);
            }
        }
    }
    uint32_t flip[8];   // sign bit where the column's sign is -1
#pragma unroll
    for (int j = 0; j < 8; j++) flip[j] = 0;
    if (signs && live) {
        const uint2 s8 = *reinterpret_cast<const uint2 *>(signs + col0);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const uint32_t byte = ((j < 4 ? s8.x : s8.y) >> (8 * (j & 3))) & 0xFFu;
            flip[j] = byte ? 0x80000000u : 0u;
        }
    }
    if (!signs_after) {
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = __uint_as_float(__float_as_uint(v[j]) ^ flip[j]);
    }

    // index bits 0..2 are the register number, bits 3..8 the lane number inside the wave
    if constexpr (LOG2N > 9) log2n = LOG2N;
    stages_in_registers(v, min(3, log2n));
    if (log2n > 3) stage_across_lanes<1>(v, lane);
    if (log2n > 4) stage_across_lanes<2>(v, lane);
    if (log2n > 5) stage_across_lanes<4>(v, lane);
    if (log2n > 6) stage_across_lanes<8>(v, lane);
    if (log2n > 7) stage_across_lanes<16>(v, lane);
    if (log2n > 8) stage_across_lanes<32>(v, lane);
    // from bit 9 on the partners sit in other waves
    // Blocks of 1024 and 8192 values end with a single stage (index bit 9, or 12): its ownership (P, 1)
    // still has runs of four consecutive values per lane, so the results are stored from there, as two
    // runs 8^P apart, instead of going through LDS once more.
    constexpr bool kSplitStore = LOG2N == 10 || LOG2N == 13;
    constexpr int kSplitP = LOG2N == 13 ? 4 : 3;
    if constexpr (LOG2N > 9) {
        constexpr int R3 = LOG2N - 9 < 3 ? LOG2N - 9 : 3;
        float *buf0 = smem, *buf1 = smem + pad(8u * (uint32_t)L) + 1u;
        exchange<0, 3, 3, R3>(v, buf0, lane);
        stages_in_registers(v, R3);
        if constexpr (LOG2N > 12) {
            exchange<3, R3, 4, LOG2N - 12>(v, buf1, lane);
            stages_in_registers(v, LOG2N - 12);
        } else if constexpr (!kSplitStore) {
            exchange<3, R3, 0, 3>(v, buf1, lane);
        }
    }

    if constexpr (kSplitStore) {
        // register q holds column  own_base(lane) + (q >> 1) + (q & 1) * 8^P  of the chunk
        const int64_t cbase = (int64_t)chunk * 8 * L + own_base<kSplitP, 1>((uint32_t)lane);
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int64_t col = cbase + ((int64_t)h << (3 * kSplitP));
            if (col >= cols) continue;            // whole blocks: a run is in or out
            uint32_t sg = 0;
            if (signs && signs_after) sg = *reinterpret_cast<const uint32_t *>(signs + col);
            float w[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                w[i] = v[2 * i + h] * scale;
                if ((sg >> (8 * i)) & 0xFFu) w[i] = -w[i];
            }
            if constexpr (OUT == PVQ_F32) {
                *reinterpret_cast<float4 *>(reinterpret_cast<float *>(Y) + row * ldy + col) = make_float4(w[0], w[1], w[2], w[3]);
            } else {
                const f32x2_t p0 = {w[0], w[1]}, p1 = {w[2], w[3]};
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(Y) + row * ldy + col) =
                    make_uint2(__builtin_bit_cast(uint32_t, __builtin_convertvector(p0, bf16x2_t)),
                               __builtin_bit_cast(uint32_t, __builtin_convertvector(p1, bf16x2_t)));
            }
        }
        return;
    }

#pragma unroll
    for (int j = 0; j < 8; j++) {
        v[j] = v[j] * scale;
        if (signs_after) v[j] = __uint_as_float(__float_as_uint(v[j]) ^ flip[j]);
    }
    if (!live) return;
    if constexpr (OUT == PVQ_F32) {
        float *o = reinterpret_cast<float *>(Y) + row * ldy + col0;
        *reinterpret_cast<float4 *>(o) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4 *>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
        uint32_t q[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const f32x2_t pair = {v[2 * j], v[2 * j + 1]};
            q[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pair, bf16x2_t));   // round to nearest even
        }
        *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(Y) + row * ldy + col0) = make_uint4(q[0], q[1], q[2], q[3]);
    }
}

}  // namespace

hipError_t pvq_launch_hadamard(const void *X, int in_dtype, int64_t rows, int64_t cols, int64_t ldx, int block,
                               const uint8_t *signs, int signs_after, void *Y, int out_dtype, int64_t ldy,
                               hipStream_t s)
{
    int log2n = 0;
    while ((1 << log2n) < block) log2n++;
    const int L = std::min(1024, std::max(256, block / 8));   // whole blocks per workgroup either way
    const int chunk = 8 * L;
    const int chunks_per_row = (int)((cols + chunk - 1) / chunk);
    const float scale = (float)(1.0 / std::sqrt((double)block));
    // two buffers for the exchanges between waves (none for blocks that fit a wave's 512 values)
    const size_t lds = log2n > 9 ? 2 * (size_t)(chunk + chunk / 32 + 1) * sizeof(float) : 0;
    const dim3 grid((unsigned)(rows * chunks_per_row)), blk((unsigned)L);
#define PVQ_HAD_LAUNCH(I, O, N) \
    hipLaunchKernelGGL((hadamard_kernel<I, O, N>), grid, blk, lds, s, X, ldx, Y, ldy, cols, log2n, signs, signs_after, scale, chunks_per_row)
#define PVQ_HAD_CASE(I, O)                                   \
    switch (log2n) {                                         \
    case 13: PVQ_HAD_LAUNCH(I, O, 13); break;                \
    case 12: PVQ_HAD_LAUNCH(I, O, 12); break;                \
    case 11: PVQ_HAD_LAUNCH(I, O, 11); break;                \
    case 10: PVQ_HAD_LAUNCH(I, O, 10); break;                \
    default: PVQ_HAD_LAUNCH(I, O, 9); break;                 \
    }
    if (in_dtype == PVQ_F32) { if (out_dtype == PVQ_F32) PVQ_HAD_CASE(PVQ_F32, PVQ_F32) else PVQ_HAD_CASE(PVQ_F32, PVQ_BF16) }
    else { if (out_dtype == PVQ_F32) PVQ_HAD_CASE(PVQ_BF16, PVQ_F32) else PVQ_HAD_CASE(PVQ_BF16, PVQ_BF16) }
#undef PVQ_HAD_LAUNCH
#undef PVQ_HAD_CASE
    return hipGetLastError();
}
