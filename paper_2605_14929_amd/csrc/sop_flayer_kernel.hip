// Statistics pass of the per-layer scale shift: a histogram of the binary exponents of the ideal
// block scales of one layer.
//
// Definition: per block of g weights, sc = max(pmax / t+, nmax / -t-) with pmax = max(0, max w),
// nmax = max(0, max -w), each quotient one IEEE binary32 division; blocks with sc = 0 (or an
// overflowed quotient) are not counted.  With sc = m * 2^e, 1/2 <= m < 1:  hist[e + 160] += 1, and hist[320 + e + 160] += 1 when
// m exceeds `m_top` (the m of the scale format's largest value).  Counts are integers, so the result
// does not depend on the order of addition.
//
// Work mapping as in the search kernel; one counter update per block (not per weight), so the pass
// streams the layer at memory speed.  Workgroups count in LDS, add to the context's running
// histogram with integer atomics, and the workgroup that finishes last moves the result to the
// caller's buffer and leaves zeros behind.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

template <bool BF16, int EPL, int LPB>
__global__ __launch_bounds__(SOP_K_FL_THREADS) void scale_hist_kernel(const FlParams p)
{
    __shared__ unsigned int s_hist[2 * SOP_K_FL_BINS];
    __shared__ unsigned int s_flag;
    for (int i = threadIdx.x; i < 2 * SOP_K_FL_BINS; i += SOP_K_FL_THREADS) s_hist[i] = 0u;
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long wave = (long long)blockIdx.x * (SOP_K_FL_THREADS / 64) + wv;
    const long long u0 = p.total_units * wave / p.n_waves;
    const long long u1 = p.total_units * (wave + 1) / p.n_waves;
    long long strip = u0 / p.M;
    long long m = u0 - strip * p.M;

    // two rows in flight per wavefront: the next row is requested before the current one is used
    auto load = [&](long long st, long long row, uint4 (&raw)[BF16 ? EPL / 8 : EPL / 4]) {
        const long long col0 = (st * 64 + lane) * EPL;
        const bool valid = col0 < p.K;
        const char* src = reinterpret_cast<const char*>(p.W) + (row * p.ldw + col0) * (BF16 ? 2 : 4);
#pragma unroll
        for (int i = 0; i < (BF16 ? EPL / 8 : EPL / 4); ++i)
            raw[i] = valid ? reinterpret_cast<const uint4*>(src)[i] : make_uint4(0, 0, 0, 0);
    };
    uint4 nxt[BF16 ? EPL / 8 : EPL / 4];
    if (u0 < u1) load(strip, m, nxt);

    for (long long u = u0; u < u1; ++u) {
        const bool valid = (strip * 64 + lane) * EPL < p.K;
        float w[EPL];
        if (BF16) {
#pragma unroll
            for (int i = 0; i < EPL / 8; ++i) {
                const uint32_t v[4] = {nxt[i].x, nxt[i].y, nxt[i].z, nxt[i].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    w[8 * i + 2 * j] = __uint_as_float(v[j] << 16);
                    w[8 * i + 2 * j + 1] = __uint_as_float(v[j] & 0xFFFF0000u);
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < EPL / 4; ++i) {
                w[4 * i] = __uint_as_float(nxt[i].x); w[4 * i + 1] = __uint_as_float(nxt[i].y);
                w[4 * i + 2] = __uint_as_float(nxt[i].z); w[4 * i + 3] = __uint_as_float(nxt[i].w);
            }
        }
        if (++m == p.M) { m = 0; ++strip; }
        if (u + 1 < u1) load(strip, m, nxt);

        float pmax = 0.0f, nmin = 0.0f;
#pragma unroll
        for (int i = 0; i < EPL; i += 2) {
            pmax = fmaxf(fmaxf(pmax, w[i]), w[i + 1]);
            nmin = fminf(fminf(nmin, w[i]), w[i + 1]);
        }
        float nmax = -nmin;
        if (LPB >= 2) { pmax = fmaxf(pmax, __shfl_xor(pmax, 1, 64)); nmax = fmaxf(nmax, __shfl_xor(nmax, 1, 64)); }
        if (LPB >= 4) { pmax = fmaxf(pmax, __shfl_xor(pmax, 2, 64)); nmax = fmaxf(nmax, __shfl_xor(nmax, 2, 64)); }
        const float sc = fmaxf(pmax / p.t_pos, nmax / p.t_neg);
        if (valid && (lane % LPB == 0) && sc > 0.0f && sc <= 3.4028235e38f) {   // an overflowed quotient is not counted
            int e;
            const float mant = frexpf(sc, &e);              // sc = mant * 2^e, 1/2 <= mant < 1 (subnormals included)
            atomicAdd(&s_hist[e + 160], 1u);
            if (mant > p.m_top) atomicAdd(&s_hist[SOP_K_FL_BINS + e + 160], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * SOP_K_FL_BINS; i += SOP_K_FL_THREADS) {
        const unsigned int v = s_hist[i];
        if (v) {
            const unsigned long long before = atomicAdd(p.acc + i, (unsigned long long)v);
            asm volatile("" :: "v"(before) : "memory");     // completed before the ticket below
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) s_flag = atomicAdd(p.done, 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (s_flag) {
        for (int i = threadIdx.x; i < 2 * SOP_K_FL_BINS; i += SOP_K_FL_THREADS) p.hist[i] = (long long)atomicExch(p.acc + i, 0ull);
        if (threadIdx.x == 0) atomicExch(p.done, 0u);
    }
}

}  // namespace sopk

extern "C" hipError_t sopk_fl_launch(const FlParams* pp, int is_bf16, int g, void* stream)
{
    FlParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)(p.n_waves / (SOP_K_FL_THREADS / 64))), block(SOP_K_FL_THREADS);
#define SOPK_FL(B, E, L) hipLaunchKernelGGL((sopk::scale_hist_kernel<B, E, L>), grid, block, 0, st, p)
    if (is_bf16) {
        if (g == 8) SOPK_FL(true, 8, 1); else if (g == 16) SOPK_FL(true, 16, 1); else if (g == 32) SOPK_FL(true, 16, 2); else SOPK_FL(true, 16, 4);
    } else {
        if (g == 8) SOPK_FL(false, 8, 1); else if (g == 16) SOPK_FL(false, 16, 1); else if (g == 32) SOPK_FL(false, 16, 2); else SOPK_FL(false, 16, 4);
    }
#undef SOPK_FL
    return hipGetLastError();
}
