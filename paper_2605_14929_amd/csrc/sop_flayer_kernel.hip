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
    // row-major order: a wavefront's steps and neighbouring wavefronts cover consecutive memory.
    // Steps are taken four at a time and the next four are requested before the current four are
    // used, so that a wavefront keeps up to 8 KiB in flight (one load in flight per wavefront leaves
    // the memory system three quarters idle).
    constexpr int NV = BF16 ? EPL / 8 : EPL / 4;     // 16-byte pieces per lane and step
    constexpr int UNR = 4;
    auto load = [&](long long u, uint4 (&raw)[NV], bool& valid) {
        const long long row = u / p.strips, st = u - row * p.strips;
        const long long col0 = (st * 64 + lane) * EPL;
        valid = u < u1 && col0 < p.K;
        const char* src = reinterpret_cast<const char*>(p.W) + (row * p.ldw + col0) * (BF16 ? 2 : 4);
#pragma unroll
        for (int i = 0; i < NV; ++i) raw[i] = valid ? reinterpret_cast<const uint4*>(src)[i] : make_uint4(0, 0, 0, 0);
    };
    const bool unit_ends = p.t_pos == 1.0f && p.t_neg == 1.0f;      // uniform: a scalar branch
    uint4 nxt[UNR][NV];
    bool nxt_valid[UNR];
#pragma unroll
    for (int j = 0; j < UNR; ++j) load(u0 + j, nxt[j], nxt_valid[j]);

    for (long long ub = u0; ub < u1; ub += UNR) {
        uint4 cur[UNR][NV];
        bool cur_valid[UNR];
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            cur_valid[j] = nxt_valid[j];
#pragma unroll
            for (int i = 0; i < NV; ++i) cur[j][i] = nxt[j][i];
        }
#pragma unroll
        for (int j = 0; j < UNR; ++j) load(ub + UNR + j, nxt[j], nxt_valid[j]);
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            const bool valid = cur_valid[j];
            float w[EPL];
            if (BF16) {
#pragma unroll
                for (int i = 0; i < EPL / 8; ++i) {
                    const uint32_t v[4] = {cur[j][i].x, cur[j][i].y, cur[j][i].z, cur[j][i].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        w[8 * i + 2 * q] = __uint_as_float(v[q] << 16);
                        w[8 * i + 2 * q + 1] = __uint_as_float(v[q] & 0xFFFF0000u);
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < EPL / 4; ++i) {
                    w[4 * i] = __uint_as_float(cur[j][i].x); w[4 * i + 1] = __uint_as_float(cur[j][i].y);
                    w[4 * i + 2] = __uint_as_float(cur[j][i].z); w[4 * i + 3] = __uint_as_float(cur[j][i].w);
                }
            }
            float pmax = 0.0f, nmin = 0.0f;
#pragma unroll
            for (int i = 0; i < EPL; i += 2) {
                pmax = fmaxf(fmaxf(pmax, w[i]), w[i + 1]);
                nmin = fminf(fminf(nmin, w[i]), w[i + 1]);
            }
            float nmax = -nmin;
#pragma unroll
            for (int st = 1; st < LPB; st <<= 1) { pmax = fmaxf(pmax, __shfl_xor(pmax, st, 64)); nmax = fmaxf(nmax, __shfl_xor(nmax, st, 64)); }
            float sc;
            if (unit_ends) sc = fmaxf(pmax, nmax);        // x / 1 = x exactly: the divisions are skipped
            else sc = fmaxf(pmax / p.t_pos, nmax / p.t_neg);
            const bool counted = valid && (lane % LPB == 0) && sc > 0.0f && sc <= 3.4028235e38f;   // an overflowed quotient is not counted
            int e = 0;
            const float mant = frexpf(counted ? sc : 1.0f, &e);   // sc = mant * 2^e, 1/2 <= mant < 1 (subnormals included)
            const bool above = counted && mant > p.m_top;
            // the scales of a layer share a handful of exponents: the wavefront counts its lanes per
            // distinct exponent with ballots and one lane adds the count (64 lanes adding to one LDS
            // word would be served one after the other)
            unsigned long long todo = __ballot(counted);
            while (todo) {
                const int first = __builtin_ctzll(todo);
                const int e0 = __builtin_amdgcn_readlane(e, first);
                const unsigned long long same = __ballot(counted && e == e0);
                const unsigned long long same_above = __ballot(above && e == e0);
                if (lane == first) {
                    atomicAdd(&s_hist[e0 + 160], (unsigned int)__builtin_popcountll(same));
                    if (same_above) atomicAdd(&s_hist[SOP_K_FL_BINS + e0 + 160], (unsigned int)__builtin_popcountll(same_above));
                }
                todo &= ~same;
            }
        }
    }
    __syncthreads();
    // (all of a thread's atomics are issued before the first returned value is looked at: one round
    // trip; the values are consumed so that the adds have completed before the ticket below)
    constexpr int PER = (2 * SOP_K_FL_BINS + SOP_K_FL_THREADS - 1) / SOP_K_FL_THREADS;
    {
        unsigned long long before[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = threadIdx.x + j * SOP_K_FL_THREADS;
            before[j] = 0ull;
            if (i < 2 * SOP_K_FL_BINS) {
                const unsigned int v = s_hist[i];
                if (v) before[j] = atomicAdd(p.acc + i, (unsigned long long)v);
            }
        }
#pragma unroll
        for (int j = 0; j < PER; ++j) asm volatile("" :: "v"(before[j]) : "memory");
    }
    __syncthreads();
    if (threadIdx.x == 0) s_flag = atomicAdd(p.done, 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (s_flag) {
        unsigned long long got[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = threadIdx.x + j * SOP_K_FL_THREADS;
            got[j] = i < 2 * SOP_K_FL_BINS ? atomicExch(p.acc + i, 0ull) : 0ull;
        }
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = threadIdx.x + j * SOP_K_FL_THREADS;
            if (i < 2 * SOP_K_FL_BINS) p.hist[i] = (long long)got[j];
        }
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
    // a lane reads 16 bytes per step (8 bf16 or 4 fp32 weights): every load instruction of a wavefront
    // covers 1 KiB of consecutive memory; g / (weights per lane) lanes share a block
    if (is_bf16) {
        if (g == 8) SOPK_FL(true, 8, 1); else if (g == 16) SOPK_FL(true, 8, 2); else if (g == 32) SOPK_FL(true, 8, 4); else SOPK_FL(true, 8, 8);
    } else {
        if (g == 8) SOPK_FL(false, 4, 2); else if (g == 16) SOPK_FL(false, 4, 4); else if (g == 32) SOPK_FL(false, 4, 8); else SOPK_FL(false, 4, 16);
    }
#undef SOPK_FL
    return hipGetLastError();
}
