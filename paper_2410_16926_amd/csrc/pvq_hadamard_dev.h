// Device side of the block Walsh-Hadamard transform (Sec. 3.3 Step 1), shared by the rotation kernel and
// by the kernel that quantises activations right after rotating them.  A workgroup of L lanes holds 8L
// consecutive values of a row, 8 per lane; hadamard_stages runs the butterflies a,b -> a+b, a-b over
// strides 1, 2, 4, ..., n/2 in that order (every value of a stage is one rounded sum or difference of two
// values of the stage before, so the schedule does not change the bits).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pvq_hadamard_dev {

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

// One butterfly stage between lanes MASK apart: the lane whose bit is clear holds a and gets a + b, the
// other holds b and gets a - b.  No stage goes through LDS.
// MASK 1, 2, 4, 8: the partner's value comes by a lane pattern inside the row of 16 lanes (a quad
// permutation; for 4 a rotation by 12 into the lanes whose bit is clear and by 4 into the others; for 8 a
// rotation by 8).
// MASK 16, 32: two registers at a time trade places instead.  v_permlane16_swap exchanges the odd rows of one
// register with the even rows of another (v_permlane32_swap: the upper half of one with the lower half of the
// other), after which every lane holds both partners of a butterfly, one in each register: rows 0 and 2 (the
// lower half) those of the first register, the others those of the second.  One addition and one subtraction
// later the same exchange puts sums and differences where they belong.
template <int MASK, bool PERMUTE = false>
__device__ inline void stage_across_lanes(float (&v)[8], int lane)
{
    if constexpr (PERMUTE && MASK > 2) {
        const bool upper = lane & MASK;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const float partner = __shfl_xor(v[j], MASK, 64);
            v[j] = upper ? partner - v[j] : v[j] + partner;
        }
    } else if constexpr (MASK == 16 || MASK == 32) {
#pragma unroll
        for (int j = 0; j < 8; j += 2) {
            uint32_t lo, hi;
            if constexpr (MASK == 16) {
                const auto t = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[j]), __float_as_uint(v[j + 1]), false, false);
                lo = t[0]; hi = t[1];
            } else {
                const auto t = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[j]), __float_as_uint(v[j + 1]), false, false);
                lo = t[0]; hi = t[1];
            }
            const float a = __uint_as_float(lo), b = __uint_as_float(hi);
            const float sum = a + b, diff = a - b;
            if constexpr (MASK == 16) {
                const auto t = __builtin_amdgcn_permlane16_swap(__float_as_uint(sum), __float_as_uint(diff), false, false);
                v[j] = __uint_as_float(t[0]); v[j + 1] = __uint_as_float(t[1]);
            } else {
                const auto t = __builtin_amdgcn_permlane32_swap(__float_as_uint(sum), __float_as_uint(diff), false, false);
                v[j] = __uint_as_float(t[0]); v[j + 1] = __uint_as_float(t[1]);
            }
        }
    } else {
        const bool upper = lane & MASK;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int x = __builtin_bit_cast(int, v[j]);
            int moved;
            if constexpr (MASK == 1) {
                moved = __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false);          // quad_perm [1,0,3,2]
            } else if constexpr (MASK == 2) {
                moved = __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false);          // quad_perm [2,3,0,1]
            } else if constexpr (MASK == 4) {
                moved = __builtin_amdgcn_update_dpp(0, x, 0x12C, 0xF, 0x5, false);         // row_ror:12 into lanes 0-3, 8-11
                moved = __builtin_amdgcn_update_dpp(moved, x, 0x124, 0xF, 0xA, false);     // row_ror:4 into lanes 4-7, 12-15
            } else {
                static_assert(MASK == 8, "lane distances 1 .. 32");
                moved = __builtin_amdgcn_update_dpp(0, x, 0x128, 0xF, 0xF, false);         // row_ror:8
            }
            const float partner = __builtin_bit_cast(float, moved);
            v[j] = upper ? partner - v[j] : v[j] + partner;
        }
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
template <int P0, int R0, int P1, int R1, bool SYNC_BEFORE = false>
__device__ inline void exchange(float (&v)[8], float *buf, uint32_t lane)
{
    if constexpr (SYNC_BEFORE) __syncthreads();   // a single buffer: its readers of the exchange before are done
    float *w = buf + pad(own_base<P0, R0>(lane));
#pragma unroll
    for (int q = 0; q < 8; q++) w[pad(own_offset<P0, R0>(q))] = v[q];
    __syncthreads();
    const float *r = buf + pad(own_base<P1, R1>(lane));
#pragma unroll
    for (int q = 0; q < 8; q++) v[q] = r[pad(own_offset<P1, R1>(q))];
}

// All stages of blocks of 2^log2n values (LOG2N = 9: any block of up to 512 values, log2n says which;
// 10 .. 13: that block size).  smem: two buffers of pad(8 L) + 1 floats when LOG2N > 9.
// STAY: blocks of 1024 and 8192 values end with a single stage, whose ownership (P, 1), P = 3 or 4, still
// has runs of four consecutive values per lane; with STAY the values are left there (register q holds
// column own_base<P,1>(lane) + (q >> 1) + (q & 1) * 8^P of the chunk) instead of going through LDS once
// more.  Otherwise the lane ends with its 8 consecutive values.
// ONEBUF: one buffer of pad(8 L) + 1 floats instead of two, with a barrier in front of every exchange as
// well (for a kernel that would rather have the LDS than save the barriers).
template <int LOG2N, bool STAY, bool ONEBUF = false, int PERMUTED = 0>
__device__ inline void hadamard_stages(float (&v)[8], int lane, int log2n, float *smem, int L)
{
    if constexpr (LOG2N > 9) log2n = LOG2N;
    // index bits 0..2 are the register number, bits 3..8 the lane number inside the wave
    stages_in_registers(v, log2n < 3 ? log2n : 3);
    if (log2n > 3) stage_across_lanes<1>(v, lane);
    if (log2n > 4) stage_across_lanes<2>(v, lane);
    if (log2n > 5) stage_across_lanes<4, (PERMUTED & 4) != 0>(v, lane);
    if (log2n > 6) stage_across_lanes<8, (PERMUTED & 8) != 0>(v, lane);
    if (log2n > 7) stage_across_lanes<16, (PERMUTED & 16) != 0>(v, lane);
    if (log2n > 8) stage_across_lanes<32, (PERMUTED & 32) != 0>(v, lane);
    // from bit 9 on the partners sit in other waves
    if constexpr (LOG2N > 9) {
        constexpr int R3 = LOG2N - 9 < 3 ? LOG2N - 9 : 3;
        constexpr bool kSingleLast = LOG2N == 10 || LOG2N == 13;
        float *buf0 = smem, *buf1 = ONEBUF ? smem : smem + pad(8u * (uint32_t)L) + 1u;
        exchange<0, 3, 3, R3, ONEBUF>(v, buf0, lane);
        stages_in_registers(v, R3);
        if constexpr (LOG2N > 12) {
            exchange<3, R3, 4, LOG2N - 12, ONEBUF>(v, buf1, lane);
            stages_in_registers(v, LOG2N - 12);
            if constexpr (!(STAY && kSingleLast)) exchange<4, LOG2N - 12, 0, 3, ONEBUF>(v, buf0, lane);
        } else if constexpr (!(STAY && kSingleLast)) {
            exchange<3, R3, 0, 3, ONEBUF>(v, buf1, lane);
        }
    }
}

}  // namespace pvq_hadamard_dev
