// The size table N(d,k) on the GPU (App. C.2, the parallel size-table computation).
//
// Row d follows from row d-1 by a prefix sum over k: with N(d,0) = 1,
//     N(d,k) = N(d,k-1) + N(d-1,k) + N(d-1,k-1)   =>   N(d,k) = 1 + sum_{i=1..k} (N(d-1,i) + N(d-1,i-1)).
// One workgroup, one lane per k.  A lane keeps its entry of the current row in registers as W 32-bit
// words; per row it adds its left neighbour's entry (the diagonal term) and the lanes then run an
// inclusive scan of those sums through LDS (log2(K) steps of multi-word additions with carry).
// Rows are written to device memory as they are made; nothing is read back except through LDS.
// An entry that does not fit its words sets the overflow flag (a carry out of the top word, or
// non-zero words above the ones the caller asked for).
#include <hip/hip_runtime.h>

#include "pvq_internal.h"

namespace {

constexpr int kMaxLanes = 1024;

template <int W>
struct big {
    uint32_t w[W];
};

// a += b, returns the carry out of the top word
template <int W>
__device__ inline uint32_t add_into(big<W> &a, const big<W> &b)
{
    uint32_t carry = 0;
#pragma unroll
    for (int i = 0; i < W; i++) {
        const uint64_t s = (uint64_t)a.w[i] + b.w[i] + carry;
        a.w[i] = (uint32_t)s;
        carry = (uint32_t)(s >> 32);
    }
    return carry;
}

// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS operations, not
// for its global stores (__syncthreads would also wait for every row written so far to reach memory,
// a microsecond per row).
__device__ inline void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0); vmcnt and expcnt left alone
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// W: words kept per entry; `words` <= W of them are stored per entry.
template <int W>
__global__ __launch_bounds__(kMaxLanes) void size_table_kernel(int D, int K, int words, uint32_t *table,
                                                               uint32_t *overflow)
{
    // blockDim.x entries of W words, word-major (word i of lane k at smem[i * lanes + k]): neighbouring
    // lanes touch neighbouring banks
    extern __shared__ __align__(16) uint32_t smem[];
    const int lanes = blockDim.x;
    auto put = [&](int at, const big<W> &x) {
#pragma unroll
        for (int i = 0; i < W; i++) smem[i * lanes + at] = x.w[i];
    };
    auto get = [&](int at) {
        big<W> x;
#pragma unroll
        for (int i = 0; i < W; i++) x.w[i] = smem[i * lanes + at];
        return x;
    };
    const int k = threadIdx.x;
    const bool live = k <= K;
    uint32_t lost = 0;
    // the flag starts at zero (cleared here rather than by a memset, so that the call can be captured)
    if (k == 0) *overflow = 0;
    __syncthreads();

    // row 0: N(0,0) = 1, N(0,k) = 0
    big<W> v;
#pragma unroll
    for (int i = 0; i < W; i++) v.w[i] = 0;
    if (k == 0) v.w[0] = 1;

    for (int d = 0; d <= D; d++) {
        if (d > 0) {
            // diagonal term: own entry of row d-1 plus the left neighbour's; lane 0 contributes nothing
            put(k, v);
            lds_barrier();
            big<W> s = v;
            if (k >= 1) lost |= add_into(s, get(k - 1));
            else {
#pragma unroll
                for (int i = 0; i < W; i++) s.w[i] = 0;
            }
            lds_barrier();
            // inclusive scan of s over the lanes (lane 0 holds zero, so the sum runs over i = 1..k)
            for (int off = 1; off <= K; off <<= 1) {
                put(k, s);
                lds_barrier();
                if (k >= off) lost |= add_into(s, get(k - off));
                lds_barrier();
            }
            // N(d,k) = 1 + the scan
            big<W> one;
#pragma unroll
            for (int i = 0; i < W; i++) one.w[i] = 0;
            one.w[0] = 1;
            lost |= add_into(s, one);
            v = s;
        }
        if (live) {
            uint32_t *out = table + ((size_t)d * (K + 1) + k) * words;
#pragma unroll
            for (int i = 0; i < W; i++) {
                if (i < words) out[i] = v.w[i];
                else lost |= v.w[i];
            }
        }
    }
    __syncthreads();   // the flag's clearing store and every row are out before the flag is raised
    if (live && lost) atomicOr(overflow, 1u);
}

template <int W>
hipError_t launch(int D, int K, int words, uint32_t *table, uint32_t *overflow, hipStream_t s)
{
    const int lanes = ((K + 1 + 63) / 64) * 64;
    const size_t lds = (size_t)lanes * W * 4;
    hipLaunchKernelGGL((size_table_kernel<W>), dim3(1), dim3(lanes), lds, s, D, K, words, table, overflow);
    return hipGetLastError();
}

}  // namespace

hipError_t pvq_launch_size_table(int D, int K, int words, uint32_t *table, uint32_t *overflow, hipStream_t s)
{
    if (words <= 1) return launch<1>(D, K, words, table, overflow, s);
    if (words <= 2) return launch<2>(D, K, words, table, overflow, s);
    if (words <= 4) return launch<4>(D, K, words, table, overflow, s);
    if (words <= 8) return launch<8>(D, K, words, table, overflow, s);
    return launch<16>(D, K, words, table, overflow, s);
}
