// Ranking of the blocks of a layer by a per-block score and the split into two pools (step 2 of the
// per-layer pair search): the score tau of the block of rank n_top (ranks count from the best score)
// is found exactly, every block at least as good as tau stays in the first pool, the others form the
// fitting pool of the second codebook.
//
// The score is mapped to a 32-bit key whose unsigned order is the ranking order (+0 and -0 share a
// key; for "lower is better" the key is complemented, so the best score always has the largest key).
// Three counting passes over the keys fix tau's key from the top: 11 bits, 11 bits, 10 bits.  A pass
// counts, in a 2048-bin histogram, the digit of every key that agrees with the digits fixed so far;
// the next kernel finds, from that histogram, the digit in which the wanted rank falls.  A last
// kernel writes the pool mask, tau and the size of the first pool.  Counts are integers added with
// atomics, so every result is exact and reproducible.  The histograms live in the context and are
// left at zero by the last kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

__device__ __forceinline__ uint32_t rank_key(float v, bool higher)
{
    uint32_t u = __float_as_uint(v);
    if (u == 0x80000000u) u = 0u;                                  // -0 ranks with +0
    const uint32_t k = (u & 0x80000000u) ? ~u : (u | 0x80000000u); // ascending with the value
    return higher ? k : ~k;
}
__device__ __forceinline__ float key_score(uint32_t k, bool higher)
{
    if (!higher) k = ~k;
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
    return __uint_as_float(u);
}

struct Found { int digit; unsigned long long rank_in, above; };

// Wave 0 of the workgroup walks a histogram from its top bin down and finds the bin in which the
// key of rank `rank` (1-based from the top) falls: `above` keys lie in higher bins and the wanted
// key has rank `rank_in` inside the bin.  The result reaches every thread through LDS.
__device__ Found find_digit(const unsigned int* hist, int nb, unsigned long long rank, Found* s_found)
{
    if (threadIdx.x == 0) { s_found->digit = 0; s_found->rank_in = 1; s_found->above = 0; }   // histogram shorter than rank: stay in bounds
    __syncthreads();
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const int per = nb / 64;
        const int top = nb - 1 - lane * per;
        unsigned long long sum = 0;
        for (int i = 0; i < per; ++i) sum += hist[top - i];
        unsigned long long inc = sum;
#pragma unroll
        for (int st = 1; st < 64; st <<= 1) {
            const unsigned long long t = __shfl_up(inc, st, 64);
            if (lane >= st) inc += t;
        }
        const unsigned long long exc = inc - sum;
        if (exc < rank && rank <= inc) {                            // exactly one lane
            unsigned long long c = exc;
            int d = top;
            for (int i = 0; i < per; ++i) {
                const unsigned long long h = hist[top - i];
                if (c + h >= rank) { d = top - i; break; }
                c += h;
            }
            s_found->digit = d; s_found->rank_in = rank - c; s_found->above = c;
        }
    }
    __syncthreads();
    const Found f = *s_found;
    __syncthreads();
    return f;
}

// digits of a key: pass 0 bits 31..21, pass 1 bits 20..10, pass 2 bits 9..0
__device__ __forceinline__ int digit_of(uint32_t k, int pass) { return pass == 0 ? (int)(k >> 21) : pass == 1 ? (int)((k >> 10) & 0x7FFu) : (int)(k & 0x3FFu); }

template <int PASS>
__global__ __launch_bounds__(SOP_K_SEL_THREADS) void rank_count_kernel(const SelParams p)
{
    __shared__ unsigned int s_hist[SOP_K_SEL_BINS];
    __shared__ Found s_found;
    for (int i = threadIdx.x; i < SOP_K_SEL_BINS; i += SOP_K_SEL_THREADS) s_hist[i] = 0u;
    // the digits fixed by the earlier passes
    uint32_t prefix = 0, pmask = 0;
    if (PASS >= 1) {
        const Found f0 = find_digit(p.hist, SOP_K_SEL_BINS, (unsigned long long)p.n_top, &s_found);
        prefix = (uint32_t)f0.digit << 21; pmask = 0xFFE00000u;
        if (PASS >= 2) {
            const Found f1 = find_digit(p.hist + SOP_K_SEL_BINS, SOP_K_SEL_BINS, f0.rank_in, &s_found);
            prefix |= (uint32_t)f1.digit << 10; pmask = 0xFFFFFC00u;
        }
    }
    __syncthreads();
    const bool higher = p.higher != 0;
    const long long n4 = p.n >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(p.score);
    for (long long i = (long long)blockIdx.x * SOP_K_SEL_THREADS + threadIdx.x; i < n4; i += (long long)gridDim.x * SOP_K_SEL_THREADS) {
        const float4 v = s4[i];
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t k = rank_key(e[j], higher);
            if ((k & pmask) == prefix) atomicAdd(&s_hist[digit_of(k, PASS)], 1u);
        }
    }
    if (blockIdx.x == 0 && (long long)threadIdx.x < (p.n & 3)) {     // ragged tail
        const uint32_t k = rank_key(p.score[(n4 << 2) + threadIdx.x], higher);
        if ((k & pmask) == prefix) atomicAdd(&s_hist[digit_of(k, PASS)], 1u);
    }
    __syncthreads();
    unsigned int* out = p.hist + PASS * SOP_K_SEL_BINS;
    for (int i = threadIdx.x; i < SOP_K_SEL_BINS; i += SOP_K_SEL_THREADS) {
        const unsigned int v = s_hist[i];
        if (v) atomicAdd(out + i, v);
    }
}

__global__ __launch_bounds__(SOP_K_SEL_THREADS) void rank_split_kernel(const SelParams p)
{
    __shared__ Found s_found;
    __shared__ unsigned int s_flag;
    const bool higher = p.higher != 0;
    uint32_t tkey = 0xFFFFFFFFu;
    unsigned long long n_a = 0;
    float tau = higher ? __uint_as_float(0x7F800000u) : __uint_as_float(0xFF800000u);
    if (!p.all_b) {
        const Found f0 = find_digit(p.hist, SOP_K_SEL_BINS, (unsigned long long)p.n_top, &s_found);
        const Found f1 = find_digit(p.hist + SOP_K_SEL_BINS, SOP_K_SEL_BINS, f0.rank_in, &s_found);
        const Found f2 = find_digit(p.hist + 2 * SOP_K_SEL_BINS, SOP_K_SEL_BINS, f1.rank_in, &s_found);
        tkey = ((uint32_t)f0.digit << 21) | ((uint32_t)f1.digit << 10) | (uint32_t)f2.digit;
        tau = key_score(tkey, higher);
        // keys above tau's, plus every key equal to it
        n_a = f0.above + f1.above + f2.above + p.hist[2 * SOP_K_SEL_BINS + f2.digit];
    }
    const long long n4 = p.n >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(p.score);
    uint32_t* m4 = reinterpret_cast<uint32_t*>(p.pool_b);
    for (long long i = (long long)blockIdx.x * SOP_K_SEL_THREADS + threadIdx.x; i < n4; i += (long long)gridDim.x * SOP_K_SEL_THREADS) {
        uint32_t w = 0x01010101u;
        if (!p.all_b) {
            const float4 v = s4[i];
            const float e[4] = {v.x, v.y, v.z, v.w};
            w = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) w |= (rank_key(e[j], higher) < tkey ? 1u : 0u) << (8 * j);
        }
        m4[i] = w;
    }
    if (blockIdx.x == 0 && (long long)threadIdx.x < (p.n & 3)) {
        const long long i = (n4 << 2) + threadIdx.x;
        p.pool_b[i] = p.all_b ? 1 : (rank_key(p.score[i], higher) < tkey ? 1 : 0);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) { *p.tau = tau; *p.n_a = (long long)n_a; }
    // the workgroup that finishes last clears the histograms (every workgroup has read them by then)
    __syncthreads();
    if (threadIdx.x == 0) s_flag = atomicAdd(p.done, 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (s_flag) {
        for (int i = threadIdx.x; i < 3 * SOP_K_SEL_BINS; i += SOP_K_SEL_THREADS) atomicExch(p.hist + i, 0u);
        if (threadIdx.x == 0) atomicExch(p.done, 0u);
    }
}

}  // namespace sopk

extern "C" hipError_t sopk_sel_launch(const SelParams* pp, int n_wg, void* stream)
{
    const SelParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)n_wg), block(SOP_K_SEL_THREADS);
    if (!p.all_b) {
        hipLaunchKernelGGL((sopk::rank_count_kernel<0>), grid, block, 0, st, p);
        hipLaunchKernelGGL((sopk::rank_count_kernel<1>), grid, block, 0, st, p);
        hipLaunchKernelGGL((sopk::rank_count_kernel<2>), grid, block, 0, st, p);
    }
    hipLaunchKernelGGL(sopk::rank_split_kernel, grid, block, 0, st, p);
    return hipGetLastError();
}
