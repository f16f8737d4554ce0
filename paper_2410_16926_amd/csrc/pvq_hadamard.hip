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

#include "pvq_hadamard_dev.h"
#include "pvq_internal.h"

namespace {

using namespace pvq_hadamard_dev;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;

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

    // Blocks of 1024 and 8192 values end with a single stage (index bit 9, or 12): its ownership (P, 1)
    // still has runs of four consecutive values per lane, so the results are stored from there, as two
    // runs 8^P apart, instead of going through LDS once more.
    constexpr bool kSplitStore = LOG2N == 10 || LOG2N == 13;
    constexpr int kSplitP = LOG2N == 13 ? 4 : 3;
    hadamard_stages<LOG2N, true, false, LOG2N <= 9 ? 4 : 0>(v, lane, log2n, smem, L);

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
