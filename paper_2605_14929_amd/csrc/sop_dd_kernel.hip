// Statistics pass of the data-derived codebook (DD atom): a channel-norm-weighted histogram of the
// block-normalised weights of one layer, in exact integer arithmetic.
//
// Definition (every operation one IEEE binary32 rounding unless it is exact):
//   cmax   = max_k c_k                       cs = fl(2^20 / cmax)          (c == NULL: c_k = 1)
//   block  a = max_i |w_i|; blocks with a == 0 contribute nothing;  r = fl(1 / a)
//   weight x = fl(w_i * r)   in [-1, 1]      mass = rint(fl(c_i * cs))   (units of 2^-20 cmax, half to even)
//          bin    = clamp(floor(fl(fl(x * H/2) + H/2)), 0, H-1)         H bins over [-1, 1]
//   hist[bin] += mass                                                   (64-bit integers)
// Integer sums do not depend on the order of addition, so the histogram is reproducible bit for bit.
// Only rows 0, row_step, 2*row_step, ... enter (row_step = 1: the whole layer), and, when a block
// mask is given, only blocks whose mask byte is non-zero.  With levels (the sweep over the partition
// parameter of the per-layer search: nested fitting pools) the mask byte names one of L histograms, and
// the result holds the L pool histograms: one pass over the weights serves every pool of the sweep.  With several
// level planes (one per codebook of the search: each ranks the blocks its own way) the same pass fills every
// plane's histograms: the weights are read, normalised and binned once.
//
// Work mapping as in the search kernel: a lane owns min(g,16) consecutive elements of a row, a
// wavefront walks down the rows of a 64-lane strip.  Each workgroup (16 wavefronts, one per compute
// unit) finds cmax itself, accumulates into its own LDS histogram with 64-bit LDS atomics and adds
// that to the layer's running histogram (kept in the context, zero between calls) with 64-bit global
// atomics; the workgroup that finishes last moves the result to the caller's buffer and leaves
// zeros behind.  One kernel per call.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

template <bool BF16, int EPL, int LPB>
__global__ __launch_bounds__(SOP_K_DD_THREADS) void dd_hist_kernel(const DdParams p)
{
    extern __shared__ __align__(16) unsigned long long s_hist[];      // [H]
    __shared__ float s_max[SOP_K_DD_THREADS / 64];
    __shared__ unsigned int s_flag;
    const int HB = p.n_bins;                                          // bins of one histogram
    const int NP = p.n_levels > 0 ? p.n_planes : 1;                   // level planes
    const int H = p.n_bins * (p.n_levels > 0 ? p.n_levels : 1) * NP;  // words of all the histograms of the call
    for (int i = threadIdx.x; i < H; i += SOP_K_DD_THREADS) s_hist[i] = 0ull;
    // cmax = max_k c_k (order-independent), found by every workgroup for itself
    float cmax = 1.0f;
    if (p.c) {
        // 16 bytes per lane and four loads in flight (a loop of single dependent loads would spend a round
        // trip to L2 per element); K is a multiple of 8 and c is 16-byte aligned
        float v = 0.0f;
        const long long k4 = p.K >> 2;
        const float4* c4 = reinterpret_cast<const float4*>(p.c);
        for (long long k0 = threadIdx.x; k0 < k4; k0 += 4 * SOP_K_DD_THREADS) {
            float4 t[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] = k0 + j * SOP_K_DD_THREADS < k4 ? c4[k0 + j * SOP_K_DD_THREADS] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int j = 0; j < 4; ++j) v = fmaxf(fmaxf(fmaxf(v, t[j].x), fmaxf(t[j].y, t[j].z)), t[j].w);
        }
#pragma unroll
        for (int st = 1; st < 64; st <<= 1) v = fmaxf(v, __shfl_xor(v, st, 64));
        if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = v;
    }
    __syncthreads();
    if (p.c) {
        cmax = s_max[0];
#pragma unroll
        for (int i = 1; i < SOP_K_DD_THREADS / 64; ++i) cmax = fmaxf(cmax, s_max[i]);
    }

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long wave = (long long)blockIdx.x * (SOP_K_DD_THREADS / 64) + wv;
    const long long u0 = p.total_units * wave / p.n_waves;
    const long long u1 = p.total_units * (wave + 1) / p.n_waves;
    const float cs = cmax > 0.0f ? 1048576.0f / cmax : 0.0f;      // all-zero channel norms: an empty histogram
    const float half = 0.5f * (float)HB;

    long long strip = u0 / p.Ms;
    long long m = u0 - strip * p.Ms;              // index among the sampled rows
    long long cur_strip = -1;
    unsigned int mass[EPL]; // rint(fl(c*cs)) of the owned columns
#pragma unroll
    for (int i = 0; i < EPL; ++i) mass[i] = 0u;

    for (long long u = u0; u < u1; ++u) {
        const long long col0 = (strip * 64 + lane) * EPL;
        const bool valid = col0 < p.K;
        if (strip != cur_strip) {
            cur_strip = strip;
#pragma unroll
            for (int i = 0; i < EPL; i += 4) {
                float4 t = make_float4(1.f, 1.f, 1.f, 1.f);
                if (p.c) t = valid ? *reinterpret_cast<const float4*>(p.c + col0 + i) : make_float4(0.f, 0.f, 0.f, 0.f);
                const float cv[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    mass[i + j] = (unsigned int)__float2int_rn(cv[j] * cs);
                }
            }
        }
        float w[EPL];
        if (BF16) {
            const uint16_t* src = reinterpret_cast<const uint16_t*>(p.W) + m * p.row_step * p.ldw + col0;
#pragma unroll
            for (int i = 0; i < EPL; i += 8) {
                uint4 t = valid ? *reinterpret_cast<const uint4*>(src + i) : make_uint4(0, 0, 0, 0);
                const uint32_t v[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    w[i + 2 * j] = __uint_as_float(v[j] << 16);
                    w[i + 2 * j + 1] = __uint_as_float(v[j] & 0xFFFF0000u);
                }
            }
        } else {
            const float* src = reinterpret_cast<const float*>(p.W) + m * p.row_step * p.ldw + col0;
#pragma unroll
            for (int i = 0; i < EPL; i += 4) {
                float4 t = valid ? *reinterpret_cast<const float4*>(src + i) : make_float4(0.f, 0.f, 0.f, 0.f);
                w[i] = t.x; w[i + 1] = t.y; w[i + 2] = t.z; w[i + 3] = t.w;
            }
        }
        float a = 0.0f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) a = fmaxf(a, fabsf(w[i]));
        if (LPB >= 2) a = fmaxf(a, __shfl_xor(a, 1, 64));
        if (LPB >= 4) a = fmaxf(a, __shfl_xor(a, 2, 64));
        bool take = valid && a > 0.0f;
        if (NP > 1) {
            // several level planes: the bins are found once, every plane adds the block to the histogram of its level
            if (take) {
                const float r = 1.0f / a;
                int bin[EPL];
#pragma unroll
                for (int i = 0; i < EPL; ++i) {
                    const float x = w[i] * r;
                    const int b = (int)floorf(x * half + half);
                    bin[i] = b < 0 ? 0 : (b > HB - 1 ? HB - 1 : b);
                }
                const long long blk = m * p.row_step * p.Bk + (strip * 64 + lane) / LPB;
                for (int pl = 0; pl < NP; ++pl) {
                    const int lv = p.block_mask[(long long)pl * p.plane_stride + blk];
                    if (lv != 0) {
                        const int hb = (pl * p.n_levels + min(lv, p.n_levels) - 1) * HB;
#pragma unroll
                        for (int i = 0; i < EPL; ++i) atomicAdd(&s_hist[hb + bin[i]], (unsigned long long)mass[i]);
                    }
                }
            }
            if (++m == p.Ms) { m = 0; ++strip; }
            continue;
        }
        int hbase = 0;                              // first word of the block's histogram
        if (p.block_mask && take) {                 // only the blocks of the pool enter
            const long long blk = m * p.row_step * p.Bk + (strip * 64 + lane) / LPB;
            const int lv = p.block_mask[blk];
            take = lv != 0;
            if (p.n_levels > 0) hbase = (min(lv, p.n_levels) - 1) * HB;
        }
        if (take) {
            const float r = 1.0f / a;
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                const float x = w[i] * r;
                int bin = (int)floorf(x * half + half);          // x*half is exact: the sum rounds once
                bin = bin < 0 ? 0 : (bin > HB - 1 ? HB - 1 : bin);
                atomicAdd(&s_hist[hbase + bin], (unsigned long long)mass[i]);
            }
        }
        if (++m == p.Ms) { m = 0; ++strip; }
    }
    __syncthreads();
    // the workgroup's histogram joins the layer's through 64-bit integer atomics; their returned
    // values are consumed so that they have completed before the workgroup takes its ticket
    // (all of a thread's atomics are issued before the first returned value is looked at: one round trip)
    {
        unsigned long long before[SOP_K_DD_MAXBINS / SOP_K_DD_THREADS];
#pragma unroll
        for (int j = 0; j < SOP_K_DD_MAXBINS / SOP_K_DD_THREADS; ++j) {
            const int i = threadIdx.x + j * SOP_K_DD_THREADS;
            before[j] = 0ull;
            if (i < H) {
                const unsigned long long v = s_hist[i];
                if (v) before[j] = atomicAdd(p.acc + i, v);
            }
        }
#pragma unroll
        for (int j = 0; j < SOP_K_DD_MAXBINS / SOP_K_DD_THREADS; ++j) asm volatile("" :: "v"(before[j]) : "memory");
    }
    __syncthreads();
    if (threadIdx.x == 0) s_flag = atomicAdd(p.done, 1u) == gridDim.x - 1 ? 1u : 0u;
    __syncthreads();
    if (s_flag) {
        unsigned long long got[SOP_K_DD_MAXBINS / SOP_K_DD_THREADS];
#pragma unroll
        for (int j = 0; j < SOP_K_DD_MAXBINS / SOP_K_DD_THREADS; ++j) {
            const int i = threadIdx.x + j * SOP_K_DD_THREADS;
            got[j] = i < H ? atomicExch(p.acc + i, 0ull) : 0ull;
        }
        if (p.n_levels > 1 || NP > 1) {
            // nested pools: histogram j of the result is the sum of the level histograms j .. L-1
            __syncthreads();
#pragma unroll
            for (int j = 0; j < SOP_K_DD_MAXBINS / SOP_K_DD_THREADS; ++j) {
                const int i = threadIdx.x + j * SOP_K_DD_THREADS;
                if (i < H) s_hist[i] = got[j];
            }
            __syncthreads();
            for (int b = threadIdx.x; b < HB * NP; b += SOP_K_DD_THREADS) {
                const int pl = b / HB, bb = b - pl * HB;
                const int base = pl * p.n_levels * HB + bb;
                unsigned long long run = 0ull;
                for (int l = p.n_levels - 1; l >= 0; --l) { run += s_hist[base + l * HB]; p.hist[base + l * HB] = (long long)run; }
            }
        } else {
#pragma unroll
            for (int j = 0; j < SOP_K_DD_MAXBINS / SOP_K_DD_THREADS; ++j) {
                const int i = threadIdx.x + j * SOP_K_DD_THREADS;
                if (i < H) p.hist[i] = (long long)got[j];
            }
        }
        if (threadIdx.x == 0) atomicExch(p.done, 0u);
    }
}

}  // namespace sopk

extern "C" hipError_t sopk_dd_launch(const DdParams* pp, int is_bf16, int g, void* stream)
{
    DdParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const size_t lds = (size_t)p.n_bins * (size_t)(p.n_levels > 0 ? p.n_levels * p.n_planes : 1) * sizeof(unsigned long long);
    const dim3 grid((unsigned)(p.n_waves / (SOP_K_DD_THREADS / 64))), block(SOP_K_DD_THREADS);
#define SOPK_DD(B, E, L) hipLaunchKernelGGL((sopk::dd_hist_kernel<B, E, L>), grid, block, lds, st, p)
    if (is_bf16) {
        if (g == 8) SOPK_DD(true, 8, 1); else if (g == 16) SOPK_DD(true, 16, 1); else if (g == 32) SOPK_DD(true, 16, 2); else SOPK_DD(true, 16, 4);
    } else {
        if (g == 8) SOPK_DD(false, 8, 1); else if (g == 16) SOPK_DD(false, 16, 1); else if (g == 32) SOPK_DD(false, 16, 2); else SOPK_DD(false, 16, 4);
    }
#undef SOPK_DD
    return hipGetLastError();
}
