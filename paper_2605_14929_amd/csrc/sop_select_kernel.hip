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
// atomics, so every result is exact and reproducible.  The context holds two sets of histograms:
// a call counts into one and clears the other, which the next call then counts into.
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

struct Found { int digit; unsigned int rank_in, above; };

// The workgroup (at least 256 threads) walks a 2048-bin histogram from its top bin down and finds the bin in
// which the key of rank `rank` (1-based from the top) falls: `above` keys lie in higher bins and the
// wanted key has rank `rank_in` inside the bin.  Thread t holds the eight bins 2047-8t .. 2040-8t in
// registers; a scan over the threads' sums names the one thread whose bins contain the rank.
__device__ Found find_digit(const unsigned int* hist, unsigned int rank, Found* s_found, unsigned int* s_wave)
{
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const bool on = t < SOP_K_SEL_BINS / 8;                         // the first 256 threads hold the bins
    const int base = on ? SOP_K_SEL_BINS - 8 * (t + 1) : 0;
    uint4 lo = make_uint4(0, 0, 0, 0), hi = lo;
    if (on) { lo = *reinterpret_cast<const uint4*>(hist + base); hi = *reinterpret_cast<const uint4*>(hist + base + 4); }
    const unsigned int h[8] = {hi.w, hi.z, hi.y, hi.x, lo.w, lo.z, lo.y, lo.x};     // from the top bin down
    const unsigned int sum = ((h[0] + h[1]) + (h[2] + h[3])) + ((h[4] + h[5]) + (h[6] + h[7]));
    unsigned int inc = sum;
#pragma unroll
    for (int st = 1; st < 64; st <<= 1) {
        const unsigned int v = __shfl_up(inc, st, 64);
        if (lane >= st) inc += v;
    }
    if (t == 0) { s_found->digit = 0; s_found->rank_in = 1; s_found->above = 0; }   // histogram shorter than rank: stay in bounds
    if (on && lane == 63) s_wave[wv] = inc;
    __syncthreads();
    if (on) {
        for (int i = 0; i < wv; ++i) inc += s_wave[i];
        const unsigned int exc = inc - sum;
        if (exc < rank && rank <= inc) {                            // exactly one thread
            unsigned int c = exc;
            int d = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {                           // ci: keys above bin i of this thread
                const unsigned int ci = exc + (i > 0 ? h[0] : 0u) + (i > 1 ? h[1] : 0u) + (i > 2 ? h[2] : 0u) + (i > 3 ? h[3] : 0u)
                                      + (i > 4 ? h[4] : 0u) + (i > 5 ? h[5] : 0u) + (i > 6 ? h[6] : 0u);
                if (ci < rank && rank <= ci + h[i]) { d = i; c = ci; }
            }
            s_found->digit = base + 7 - d; s_found->rank_in = rank - c; s_found->above = c;
        }
    }
    __syncthreads();
    const Found f = *s_found;
    __syncthreads();
    return f;
}

// one count into an LDS histogram for every active lane; lanes that share the first active lane's
// digit are counted with one atomic (block cosines crowd into very few digits in the first pass)
__device__ __forceinline__ void count_digit(unsigned int* s_hist, bool active, int digit)
{
    const unsigned long long act = __builtin_amdgcn_ballot_w64(active);
    if (act == 0ull) return;
    const int first = __builtin_ctzll(act);
    const int lead = __builtin_amdgcn_readlane(digit, first);
    const bool same = active && digit == lead;
    const unsigned long long m = __builtin_amdgcn_ballot_w64(same);
    if ((int)(threadIdx.x & 63) == first) atomicAdd(&s_hist[lead], (unsigned int)__builtin_popcountll(m));
    if (active && !same) atomicAdd(&s_hist[digit], 1u);
}

// digits of a key: pass 0 bits 31..21, pass 1 bits 20..10, pass 2 bits 9..0
__device__ __forceinline__ int digit_of(uint32_t k, int pass) { return pass == 0 ? (int)(k >> 21) : pass == 1 ? (int)((k >> 10) & 0x7FFu) : (int)(k & 0x3FFu); }

template <int PASS>
__global__ __launch_bounds__(SOP_K_CNT_THREADS) void rank_count_kernel(const SelParams p)
{
    __shared__ unsigned int s_hist[SOP_K_SEL_BINS];
    __shared__ Found s_found;
    __shared__ unsigned int s_wave[SOP_K_SEL_BINS / 8 / 64];
    for (int i = threadIdx.x; i < SOP_K_SEL_BINS; i += SOP_K_CNT_THREADS) s_hist[i] = 0u;
    // the digits fixed by the earlier passes
    uint32_t prefix = 0, pmask = 0;
    if (PASS >= 1) {
        const Found f0 = find_digit(p.hist, (unsigned int)p.n_top, &s_found, s_wave);
        prefix = (uint32_t)f0.digit << 21; pmask = 0xFFE00000u;
        if (PASS >= 2) {
            const Found f1 = find_digit(p.hist + SOP_K_SEL_BINS, f0.rank_in, &s_found, s_wave);
            prefix |= (uint32_t)f1.digit << 10; pmask = 0xFFFFFC00u;
        }
    }
    __syncthreads();
    const bool higher = p.higher != 0;
    const long long n4 = p.n >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(p.score);
    for (long long i = (long long)blockIdx.x * SOP_K_CNT_THREADS + threadIdx.x; i < n4; i += (long long)gridDim.x * SOP_K_CNT_THREADS) {
        const float4 v = s4[i];
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t k = rank_key(e[j], higher);
            count_digit(s_hist, (k & pmask) == prefix, digit_of(k, PASS));
        }
    }
    if (blockIdx.x == 0 && (long long)threadIdx.x < (p.n & 3)) {     // ragged tail
        const uint32_t k = rank_key(p.score[(n4 << 2) + threadIdx.x], higher);
        if ((k & pmask) == prefix) atomicAdd(&s_hist[digit_of(k, PASS)], 1u);
    }
    __syncthreads();
    unsigned int* out = p.hist + PASS * SOP_K_SEL_BINS;
    for (int i = threadIdx.x; i < SOP_K_SEL_BINS; i += SOP_K_CNT_THREADS) {
        const unsigned int v = s_hist[i];
        if (v) atomicAdd(out + i, v);
    }
}

__global__ __launch_bounds__(SOP_K_SEL_THREADS) void rank_split_kernel(const SelParams p)
{
    __shared__ Found s_found;
    __shared__ unsigned int s_wave[SOP_K_SEL_THREADS / 64];
    const bool higher = p.higher != 0;
    uint32_t tkey = 0xFFFFFFFFu;
    unsigned int n_a = 0;
    float tau = higher ? __uint_as_float(0x7F800000u) : __uint_as_float(0xFF800000u);
    if (!p.all_b) {
        const Found f0 = find_digit(p.hist, (unsigned int)p.n_top, &s_found, s_wave);
        const Found f1 = find_digit(p.hist + SOP_K_SEL_BINS, f0.rank_in, &s_found, s_wave);
        const Found f2 = find_digit(p.hist + 2 * SOP_K_SEL_BINS, f1.rank_in, &s_found, s_wave);
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
    // clear the other set of histograms (the one the previous call counted into; nothing reads it
    // now) for the next call: no workgroup has to wait for the others
    for (long long gi = (long long)blockIdx.x * SOP_K_SEL_THREADS + threadIdx.x; gi < 3 * SOP_K_SEL_BINS; gi += (long long)gridDim.x * SOP_K_SEL_THREADS)
        p.hist_other[gi] = 0u;
}

// ---- several thresholds at once (the sweep over the partition parameter: nested pools) ----
// The first counting pass is shared by all thresholds; in the second and third pass every threshold counts
// the keys that agree with its own digits so far, in a histogram of its own.  Thresholds whose digits so
// far coincide share one histogram (the one of the first of them).  After each counting pass a kernel of one
// workgroup per plane walks the histograms and hands the digits on (were every counting workgroup to walk
// them itself, the walk's chain of loads and barriers would cost more than the counting).  A last kernel
// writes, per block, the number of thresholds it ranks strictly worse than: the pools are nested, pool j
// holds the blocks of level > j.
// After counting pass PASS a single workgroup per plane finds, for every threshold, the digit of that pass in
// which the wanted rank falls, and hands the digits so far on to the next pass (or, after the last pass, the
// thresholds' keys, scores and first-pool sizes to the level kernel and the caller).
template <int PASS>
__global__ __launch_bounds__(SOP_K_SEL_THREADS) void rank_find_kernel(const SelMParams pp);

// the parameters of one plane of a launch over several score planes
__device__ __forceinline__ SelMParams plane_of(SelMParams p, unsigned int q)
{
    p.score += (size_t)q * (size_t)p.n;
    p.hist += (size_t)q * SOP_K_SELM_WORDS;
    p.hist_other += (size_t)q * SOP_K_SELM_WORDS;
    p.level += (size_t)q * (size_t)p.n;
    p.tau += q * SOP_K_SEL_MAXLEV;
    p.n_a += q * SOP_K_SEL_MAXLEV;
    p.state += q;
    return p;
}

template <int PASS>
__global__ __launch_bounds__(SOP_K_CNT_THREADS) void rank_count_multi_kernel(const SelMParams pp)
{
    const SelMParams p = plane_of(pp, blockIdx.y);
    extern __shared__ unsigned int s_mh[];                          // pass 0: [BINS]; else [n_levels][BINS]
    const int L = PASS == 0 ? 1 : p.n_levels;
    for (int i = threadIdx.x; i < L * SOP_K_SEL_BINS; i += SOP_K_CNT_THREADS) s_mh[i] = 0u;
    const uint32_t pmask = PASS == 0 ? 0u : PASS == 1 ? 0xFFE00000u : 0xFFFFFC00u;
    SelMState mp;                                                    // (same values in every lane: scalar loads)
    if (PASS >= 1) mp = *p.state;
    __syncthreads();
    const bool higher = p.higher != 0;
    const long long n4 = p.n >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(p.score);
    for (long long i = (long long)blockIdx.x * SOP_K_CNT_THREADS + threadIdx.x; i < n4; i += (long long)gridDim.x * SOP_K_CNT_THREADS) {
        const float4 v = s4[i];
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t k = rank_key(e[j], higher);
            if (PASS == 0) count_digit(s_mh, true, digit_of(k, 0));
            else
                _Pragma("unroll") for (int t = 0; t < SOP_K_SEL_MAXLEV; ++t)
                    if (t < p.n_levels && p.n_top[t] != 0 && mp.alias[t] == t) count_digit(s_mh + t * SOP_K_SEL_BINS, (k & pmask) == mp.prefix[t], digit_of(k, PASS));
        }
    }
    if (blockIdx.x == 0 && (long long)threadIdx.x < (p.n & 3)) {     // ragged tail
        const uint32_t k = rank_key(p.score[(n4 << 2) + threadIdx.x], higher);
        if (PASS == 0) atomicAdd(&s_mh[digit_of(k, 0)], 1u);
        else
            _Pragma("unroll") for (int t = 0; t < SOP_K_SEL_MAXLEV; ++t)
                if (t < p.n_levels && p.n_top[t] != 0 && mp.alias[t] == t && (k & pmask) == mp.prefix[t]) atomicAdd(&s_mh[t * SOP_K_SEL_BINS + digit_of(k, PASS)], 1u);
    }
    __syncthreads();
    unsigned int* out = p.hist + (PASS == 0 ? 0 : PASS == 1 ? SOP_K_SEL_BINS : (1 + SOP_K_SEL_MAXLEV) * SOP_K_SEL_BINS);
    for (int i = threadIdx.x; i < L * SOP_K_SEL_BINS; i += SOP_K_CNT_THREADS) {
        const unsigned int v = s_mh[i];
        if (v) atomicAdd(out + i, v);
    }
}

__global__ __launch_bounds__(SOP_K_SEL_THREADS) void rank_level_kernel(const SelMParams pp)
{
    const SelMParams p = plane_of(pp, blockIdx.y);
    const bool higher = p.higher != 0;
    unsigned long long tkey[SOP_K_SEL_MAXLEV];
    _Pragma("unroll") for (int j = 0; j < SOP_K_SEL_MAXLEV; ++j) tkey[j] = j < p.n_levels ? p.state->tkey[j] : 0ull;   // (beyond n_levels: no block ranks worse)
    const long long n4 = p.n >> 2;
    const float4* s4 = reinterpret_cast<const float4*>(p.score);
    uint32_t* m4 = reinterpret_cast<uint32_t*>(p.level);
    for (long long i = (long long)blockIdx.x * SOP_K_SEL_THREADS + threadIdx.x; i < n4; i += (long long)gridDim.x * SOP_K_SEL_THREADS) {
        const float4 v = s4[i];
        const float e[4] = {v.x, v.y, v.z, v.w};
        uint32_t w = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned long long k = rank_key(e[j], higher);
            uint32_t lv = 0u;
            _Pragma("unroll") for (int t = 0; t < SOP_K_SEL_MAXLEV; ++t) lv += k < tkey[t] ? 1u : 0u;
            w |= lv << (8 * j);
        }
        m4[i] = w;
    }
    if (blockIdx.x == 0 && (long long)threadIdx.x < (p.n & 3)) {
        const long long i = (n4 << 2) + threadIdx.x;
        const unsigned long long k = rank_key(p.score[i], higher);
        unsigned int lv = 0u;
        _Pragma("unroll") for (int t = 0; t < SOP_K_SEL_MAXLEV; ++t) lv += k < tkey[t] ? 1u : 0u;
        p.level[i] = (unsigned char)lv;
    }
    // the other set of digit counts is cleared for the next call: every plane that holds counts, which can be more
    // planes than this launch has (a launch over fewer planes follows one over more)
    for (unsigned int cq = blockIdx.y; cq < (unsigned int)pp.n_clear; cq += gridDim.y) {
        unsigned int* dst = pp.hist_other + (size_t)cq * SOP_K_SELM_WORDS;
        for (long long gi = (long long)blockIdx.x * SOP_K_SEL_THREADS + threadIdx.x; gi < SOP_K_SELM_WORDS; gi += (long long)gridDim.x * SOP_K_SEL_THREADS)
            dst[gi] = 0u;
    }
}

template <int PASS>
__global__ __launch_bounds__(SOP_K_SEL_THREADS) void rank_find_kernel(const SelMParams pp)
{
    const SelMParams p = plane_of(pp, blockIdx.y);
    __shared__ Found s_found;
    __shared__ unsigned int s_wave[SOP_K_SEL_THREADS / 64];
    const bool higher = p.higher != 0;
    SelMState st;
    if (PASS >= 1) st = *p.state;
    _Pragma("unroll") for (int j = 0; j < SOP_K_SEL_MAXLEV; ++j) {
        if (PASS == 0) { st.prefix[j] = 0u; st.rank_in[j] = 1u; st.above[j] = 0u; st.alias[j] = j; }
        st.tkey[j] = 1ull << 32;
        if (j >= p.n_levels || p.n_top[j] == 0) continue;
        const unsigned int* h = PASS == 0 ? p.hist : p.hist + ((PASS == 1 ? 1 : 1 + SOP_K_SEL_MAXLEV) + st.alias[j]) * SOP_K_SEL_BINS;
        const Found f = find_digit(h, PASS == 0 ? (unsigned int)p.n_top[j] : st.rank_in[j], &s_found, s_wave);
        st.prefix[j] |= (uint32_t)f.digit << (PASS == 0 ? 21 : PASS == 1 ? 10 : 0);
        st.rank_in[j] = f.rank_in;
        if (PASS == 2) {
            st.tkey[j] = st.prefix[j];
            if (threadIdx.x == 0) { p.tau[j] = key_score(st.prefix[j], higher); p.n_a[j] = (long long)(st.above[j] + f.above + h[f.digit]); }   // keys above tau's, plus every key equal to it
        }
        st.above[j] += f.above;
    }
    if (PASS == 2) {
        _Pragma("unroll") for (int j = 0; j < SOP_K_SEL_MAXLEV; ++j)
            if (j < p.n_levels && p.n_top[j] == 0 && threadIdx.x == 0) {
                p.tau[j] = higher ? __uint_as_float(0x7F800000u) : __uint_as_float(0xFF800000u);
                p.n_a[j] = 0;
            }
    }
    // thresholds whose digits so far coincide share the histogram of the first of them in the next pass
    _Pragma("unroll") for (int j = 0; j < SOP_K_SEL_MAXLEV; ++j) {
        st.alias[j] = j;
        _Pragma("unroll") for (int i = j - 1; i >= 0; --i)
            if (j < p.n_levels && p.n_top[i] != 0 && p.n_top[j] != 0 && st.prefix[i] == st.prefix[j]) st.alias[j] = st.alias[i];
    }
    if (threadIdx.x == 0) *p.state = st;
}

}  // namespace sopk

extern "C" hipError_t sopk_selm_launch(const SelMParams* pp, int n_wg_count, int n_wg, void* stream)
{
    const SelMParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const unsigned planes = (unsigned)(p.n_planes > 0 ? p.n_planes : 1);
    const dim3 grid((unsigned)n_wg, planes), block(SOP_K_SEL_THREADS), cgrid((unsigned)n_wg_count, planes), cblock(SOP_K_CNT_THREADS);
    bool any = false;
    for (int j = 0; j < p.n_levels; ++j) any = any || p.n_top[j] != 0;
    const dim3 fgrid(1, planes);
    if (any) {
        const size_t lds0 = SOP_K_SEL_BINS * sizeof(unsigned int), ldsL = (size_t)p.n_levels * lds0;
        if (ldsL > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sopk::rank_count_multi_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsL);
            if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sopk::rank_count_multi_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldsL);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL((sopk::rank_count_multi_kernel<0>), cgrid, cblock, lds0, st, p);
        hipLaunchKernelGGL((sopk::rank_find_kernel<0>), fgrid, block, 0, st, p);
        hipLaunchKernelGGL((sopk::rank_count_multi_kernel<1>), cgrid, cblock, ldsL, st, p);
        hipLaunchKernelGGL((sopk::rank_find_kernel<1>), fgrid, block, 0, st, p);
        hipLaunchKernelGGL((sopk::rank_count_multi_kernel<2>), cgrid, cblock, ldsL, st, p);
    }
    hipLaunchKernelGGL((sopk::rank_find_kernel<2>), fgrid, block, 0, st, p);      // (with every first pool empty it only writes the defaults)
    hipLaunchKernelGGL(sopk::rank_level_kernel, grid, block, 0, st, p);
    return hipGetLastError();
}

extern "C" hipError_t sopk_sel_launch(const SelParams* pp, int n_wg_count, int n_wg, void* stream)
{
    const SelParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)n_wg), block(SOP_K_SEL_THREADS);
    if (!p.all_b) {
        // few, large workgroups: every workgroup adds its whole histogram to the layer's with
        // same-address atomics, which serialise
        const dim3 cgrid((unsigned)n_wg_count), cblock(SOP_K_CNT_THREADS);
        hipLaunchKernelGGL((sopk::rank_count_kernel<0>), cgrid, cblock, 0, st, p);
        hipLaunchKernelGGL((sopk::rank_count_kernel<1>), cgrid, cblock, 0, st, p);
        hipLaunchKernelGGL((sopk::rank_count_kernel<2>), cgrid, cblock, 0, st, p);
    }
    hipLaunchKernelGGL(sopk::rank_split_kernel, grid, block, 0, st, p);
    return hipGetLastError();
}
