// Statistics pass of the per-layer scale shift: a histogram of the binary exponents of the ideal
// block scales of one layer.
//
// Definition: per block of g weights, sc = max(pmax / t+, nmax / -t-) with pmax = max(0, max w),
// nmax = max(0, max -w), each quotient one IEEE binary32 division; blocks with sc = 0 (or an
// overflowed quotient) are not counted.  With sc = m * 2^e, 1/2 <= m < 1:  hist[e + 160] += 1, and hist[320 + e + 160] += 1 when
// m exceeds `m_top` (the m of the scale format's largest value).  Counts are integers, so the result
// does not depend on the order of addition.
//
// Work mapping as in the search kernel; the lanes count in registers and a wavefront adds its counts to
// the workgroup's histogram in LDS a few times per launch.  Workgroups add to the context's running
// histogram with integer atomics, and the workgroup that finishes last moves the result to the
// caller's buffer and leaves zeros behind.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

// Sum of x over every row of 16 lanes with data-parallel-primitive moves on the vector ALU (quads, half
// rows, rows): every lane of a row then holds the row's sum.
__device__ __forceinline__ unsigned int row_total(unsigned int v)
{
    int x = (int)v;
    x += __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false);      // quad_perm [1,0,3,2]
    x += __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false);      // quad_perm [2,3,0,1]
    x += __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false);     // row_half_mirror
    x += __builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, false);     // row_mirror
    return (unsigned int)x;
}

template <bool BF16, int EPL, int LPB>
__global__ __launch_bounds__(SOP_K_FL_THREADS) void scale_hist_kernel(const FlParams p)
{
    __shared__ unsigned int s_hist[2 * SOP_K_FL_BINS];
    __shared__ unsigned int s_flag;
    for (int i = threadIdx.x; i < 2 * SOP_K_FL_BINS; i += SOP_K_FL_THREADS) s_hist[i] = 0u;
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // A workgroup takes a contiguous range of the layer's units (row-major: consecutive memory) and its
    // wavefronts take the units of the range in turn, so that at any moment the workgroup reads one
    // stretch of a few tens of KiB.  The (row, strip) of the next unit to load is kept on the scalar unit
    // and advanced per load (one division per wavefront, none per step).  A lane reads 16 or 32 bytes per
    // step; steps are taken UNR at a time and the next UNR are requested before the current ones are used:
    // 64 bytes per lane, 4 KiB per wavefront in flight.
    constexpr int WPG = SOP_K_FL_THREADS / 64;
    // (the host gives total_units / workgroups and the remainder, and total_units is below 2^31: no 64-bit
    // division here)
    const unsigned int bq = (unsigned int)p.units_per_wg, br = (unsigned int)p.units_rem;
    const unsigned int g0 = blockIdx.x * bq + (blockIdx.x < br ? blockIdx.x : br), g1 = g0 + bq + (blockIdx.x < br ? 1u : 0u);
    const unsigned int u0 = g0 + (unsigned int)wv;
    const int n_units = __builtin_amdgcn_readfirstlane(u0 < g1 ? (int)((g1 - u0 + WPG - 1) / WPG) : 0);
    constexpr int NV = BF16 ? EPL / 8 : EPL / 4;     // 16-byte pieces per lane and step
    constexpr int UNR = 4 / NV;
    const int strips = __builtin_amdgcn_readfirstlane((int)p.strips);
    long long lrow = u0 / (unsigned int)strips;
    int lst = __builtin_amdgcn_readfirstlane((int)(u0 - (unsigned int)lrow * (unsigned int)strips));
    int loaded = 0;                                   // units requested so far
    auto load = [&](uint4 (&raw)[NV], bool& valid) {
        const long long col0 = ((long long)lst * 64 + lane) * EPL;
        valid = loaded < n_units && col0 < p.K;
        const char* src = reinterpret_cast<const char*>(p.W) + (lrow * p.ldw + col0) * (BF16 ? 2 : 4);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            raw[i] = make_uint4(0, 0, 0, 0);
            if (valid) {                               // every weight is read once: the loads bypass-hint the caches
                const unsigned int* q = reinterpret_cast<const unsigned int*>(src) + 4 * i;
                raw[i].x = __builtin_nontemporal_load(q); raw[i].y = __builtin_nontemporal_load(q + 1);
                raw[i].z = __builtin_nontemporal_load(q + 2); raw[i].w = __builtin_nontemporal_load(q + 3);
            }
        }
        ++loaded;
        lst += WPG;
        while (lst >= strips) { lst -= strips; ++lrow; }
    };
    const bool unit_ends = p.t_pos == 1.0f && p.t_neg == 1.0f;      // uniform: a scalar branch
    // Counting.  The block scales of a layer share a handful of binary exponents, so 64 lanes adding to
    // LDS words would queue up on two or three addresses.  Instead every lane counts for itself, in
    // registers: 16 eight-bit counters for the exponents [wbase, wbase + 16) and 16 more for the blocks
    // above the top mantissa, wbase set by the first block the wavefront counts.  Every 255 steps and at
    // the end the wavefront adds its lanes' counters over every row of 16 lanes (widened to 16 bits, two to a
    // register, summed with data-parallel-primitive moves) and the first lane of each row adds the row's totals
    // to the workgroup's histogram in LDS (compiled with the compiler's atomic optimizer off, which would wrap
    // each of these adds in a scan over the active lanes).  An
    // exponent outside the window (rare) is added to LDS directly.
    unsigned long long c_lo = 0ull, c_hi = 0ull, a_lo = 0ull, a_hi = 0ull;
    int wbase = 0, pending = 0;
    bool have_base = false;
    auto flush = [&]() {
        const unsigned long long regs[4] = {c_lo, c_hi, a_lo, a_hi};
        const bool row_lead = (lane & 15) == 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const unsigned long long ev = regs[r] & 0x00FF00FF00FF00FFull, od = (regs[r] >> 8) & 0x00FF00FF00FF00FFull;
            // fields 0,2 | 4,6 | 1,3 | 5,7 of this register, 16 bits each (a row's total is at most 16 * 255)
            const unsigned int part[4] = {(unsigned int)ev, (unsigned int)(ev >> 32), (unsigned int)od, (unsigned int)(od >> 32)};
            const int first_field[4] = {0, 4, 1, 5};
            unsigned int t[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) t[q] = row_total(part[q]);      // four independent chains
            if (row_lead) {                                               // four lanes add their rows' totals
                const int bin = (r >> 1) * SOP_K_FL_BINS + wbase + 160 + (r & 1) * 8;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int f0 = first_field[q];                        // field of the low half; the high half is f0 + 2
                    if (t[q] & 0xFFFFu) atomicAdd(&s_hist[bin + f0], t[q] & 0xFFFFu);
                    if (t[q] >> 16) atomicAdd(&s_hist[bin + f0 + 2], t[q] >> 16);
                }
            }
        }
        c_lo = c_hi = a_lo = a_hi = 0ull;
        pending = 0;
    };

    uint4 nxt[UNR][NV];
    bool nxt_valid[UNR];
#pragma unroll
    for (int j = 0; j < UNR; ++j) load(nxt[j], nxt_valid[j]);

    for (int ub = 0; ub < n_units; ub += UNR) {
        uint4 cur[UNR][NV];
        bool cur_valid[UNR];
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            cur_valid[j] = nxt_valid[j];
#pragma unroll
            for (int i = 0; i < NV; ++i) cur[j][i] = nxt[j][i];
        }
#pragma unroll
        for (int j = 0; j < UNR; ++j) load(nxt[j], nxt_valid[j]);
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
            if (!have_base) {
                const unsigned long long any = __ballot(counted);
                if (any) {
                    // the first block's exponent, nine counters below it and six above (later blocks of a
                    // strip of heavy-tailed weights are more often smaller than larger)
                    wbase = __builtin_amdgcn_readlane(e, __builtin_ctzll(any)) - 9;
                    have_base = true;
                }
            }
            const unsigned int idx = (unsigned int)(e - wbase);
            const bool inw = counted && idx < 16u;
            const unsigned long long one = 1ull << ((idx & 7u) * 8u);
            const unsigned long long add_lo = inw && idx < 8u ? one : 0ull, add_hi = inw && idx >= 8u ? one : 0ull;
            c_lo += add_lo; c_hi += add_hi;
            a_lo += above ? add_lo : 0ull; a_hi += above ? add_hi : 0ull;
            if (__builtin_expect(__any(counted && !inw) != 0, 0)) {
                if (counted && !inw) {
                    atomicAdd(&s_hist[e + 160], 1u);
                    if (above) atomicAdd(&s_hist[SOP_K_FL_BINS + e + 160], 1u);
                }
            }
            if (++pending == 255) flush();
        }
    }
    if (pending) flush();
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

extern "C" int sopk_fl_weights_per_lane(int is_bf16, int g) { return is_bf16 ? (g < 16 ? g : 16) : 8; }

extern "C" hipError_t sopk_fl_launch(const FlParams* pp, int is_bf16, int g, void* stream)
{
    FlParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)(p.n_waves / (SOP_K_FL_THREADS / 64))), block(SOP_K_FL_THREADS);
#define SOPK_FL(B, E, L) hipLaunchKernelGGL((sopk::scale_hist_kernel<B, E, L>), grid, block, 0, st, p)
    // a lane reads 16 or 32 bytes per step (8 or 16 bf16 weights, 8 fp32 weights): every load instruction of
    // a wavefront covers 1 KiB of consecutive memory; g / (weights per lane) lanes share a block.
    // The host's strips are counted in these steps: sopk_fl_weights_per_lane().
    if (is_bf16) {
        if (g == 8) SOPK_FL(true, 8, 1); else if (g == 16) SOPK_FL(true, 16, 1); else if (g == 32) SOPK_FL(true, 16, 2); else SOPK_FL(true, 16, 4);
    } else {
        if (g == 8) SOPK_FL(false, 8, 1); else if (g == 16) SOPK_FL(false, 8, 2); else if (g == 32) SOPK_FL(false, 8, 4); else SOPK_FL(false, 8, 8);
    }
#undef SOPK_FL
    return hipGetLastError();
}
