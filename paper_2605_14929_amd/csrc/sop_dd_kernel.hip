// Statistics pass of the data-derived codebook (DD atom): a channel-norm-weighted histogram of the
// block-normalised weights of one layer, in exact integer arithmetic.
//
// Definition (every operation one IEEE binary32 rounding unless it is exact):
//   cmax   = max_k c_k                       cs = fl(2^20 / cmax)          (c == NULL: c_k = 1)
//   block  a = max_i |w_i|; blocks with a == 0 contribute nothing;  r = fl(1 / a)
//   weight x = fl(w_i * r)   in [-1, 1]      u = fl(c_i * cs)
//          mass   = rint(u)                  (units of 2^-20 cmax, round half to even)
//          moment = rint(fl(fl(u * 1024) * x))   (units of 2^-30 cmax)
//          bin    = clamp(floor(fl(fl(x * H/2) + H/2)), 0, H-1)         H bins over [-1, 1]
//   hist[0][bin] += mass,  hist[1][bin] += moment                       (64-bit integers)
// Integer sums do not depend on the order of addition, so the histogram is reproducible bit for bit.
//
// Work mapping as in the search kernel: a lane owns min(g,16) consecutive elements of a row, a
// wavefront walks down the rows of a 64-lane strip.  Each workgroup (16 wavefronts, one per compute
// unit) accumulates into its own LDS histogram with 64-bit LDS atomics and writes it out once; a
// second kernel adds the workgroups' histograms entry by entry.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

template <bool BF16, int EPL, int LPB>
__global__ __launch_bounds__(SOP_K_DD_THREADS) void dd_hist_kernel(const DdParams p)
{
    extern __shared__ __align__(16) unsigned long long s_hist[];      // [2][H]
    const int H = p.n_bins;
    for (int i = threadIdx.x; i < 2 * H; i += SOP_K_DD_THREADS) s_hist[i] = 0ull;
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long wave = (long long)blockIdx.x * (SOP_K_DD_THREADS / 64) + wv;
    const long long u0 = p.total_units * wave / p.n_waves;
    const long long u1 = p.total_units * (wave + 1) / p.n_waves;
    const float cmax = p.c ? *p.cmax : 1.0f;
    const float cs = cmax > 0.0f ? 1048576.0f / cmax : 0.0f;      // all-zero channel norms: an empty histogram
    const float half = 0.5f * (float)H;

    long long strip = u0 / p.M;
    long long m = u0 - strip * p.M;
    long long cur_strip = -1;
    float uw[EPL];          // fl(c*cs)*1024 (exact scaling) per owned column
    unsigned int mass[EPL]; // rint(fl(c*cs))
#pragma unroll
    for (int i = 0; i < EPL; ++i) { uw[i] = 0.0f; mass[i] = 0u; }

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
                    const float uu = cv[j] * cs;
                    mass[i + j] = (unsigned int)__float2int_rn(uu);
                    uw[i + j] = uu * 1024.0f;
                }
            }
        }
        float w[EPL];
        if (BF16) {
            const uint16_t* src = reinterpret_cast<const uint16_t*>(p.W) + m * p.ldw + col0;
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
            const float* src = reinterpret_cast<const float*>(p.W) + m * p.ldw + col0;
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
        if (valid && a > 0.0f) {
            const float r = 1.0f / a;
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                const float x = w[i] * r;
                const int mom = __float2int_rn(uw[i] * x);
                int bin = (int)floorf(x * half + half);          // x*half is exact: the sum rounds once
                bin = bin < 0 ? 0 : (bin > H - 1 ? H - 1 : bin);
                atomicAdd(&s_hist[bin], (unsigned long long)mass[i]);
                atomicAdd(&s_hist[H + bin], (unsigned long long)(long long)mom);
            }
        }
        if (++m == p.M) { m = 0; ++strip; }
    }
    __syncthreads();
    unsigned long long* dst = p.partial + (long long)blockIdx.x * 2 * H;
    for (int i = threadIdx.x; i < 2 * H; i += SOP_K_DD_THREADS) dst[i] = s_hist[i];
}

// cmax = max_k c_k (order-independent); one workgroup
__global__ __launch_bounds__(256) void dd_cmax_kernel(const DdParams p)
{
    __shared__ float s[256];
    float v = 0.0f;
    for (long long k = threadIdx.x; k < p.K; k += 256) v = fmaxf(v, p.c[k]);
    s[threadIdx.x] = v;
    __syncthreads();
    for (int h = 128; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) s[threadIdx.x] = fmaxf(s[threadIdx.x], s[threadIdx.x + h]);
        __syncthreads();
    }
    if (threadIdx.x == 0) *p.cmax = s[0];
}

// hist[i] = sum over workgroups of partial[wg][i], one thread per entry, workgroups in order
__global__ __launch_bounds__(256) void dd_merge_kernel(const DdParams p)
{
    const int n = 2 * p.n_bins;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    unsigned long long t = 0ull;
    const long long n_wg = p.n_waves / (SOP_K_DD_THREADS / 64);
    for (long long g = 0; g < n_wg; ++g) t += p.partial[g * n + i];
    p.hist[i] = (long long)t;
}

}  // namespace sopk

extern "C" hipError_t sopk_dd_launch(const DdParams* pp, int is_bf16, int g, void* stream)
{
    DdParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    if (p.c) hipLaunchKernelGGL(sopk::dd_cmax_kernel, dim3(1), dim3(256), 0, st, p);
    const size_t lds = (size_t)2 * p.n_bins * sizeof(unsigned long long);
    const dim3 grid((unsigned)(p.n_waves / (SOP_K_DD_THREADS / 64))), block(SOP_K_DD_THREADS);
#define SOPK_DD(B, E, L) hipLaunchKernelGGL((sopk::dd_hist_kernel<B, E, L>), grid, block, lds, st, p)
    if (is_bf16) {
        if (g == 8) SOPK_DD(true, 8, 1); else if (g == 16) SOPK_DD(true, 16, 1); else if (g == 32) SOPK_DD(true, 16, 2); else SOPK_DD(true, 16, 4);
    } else {
        if (g == 8) SOPK_DD(false, 8, 1); else if (g == 16) SOPK_DD(false, 16, 1); else if (g == 32) SOPK_DD(false, 16, 2); else SOPK_DD(false, 16, 4);
    }
#undef SOPK_DD
    hipLaunchKernelGGL(sopk::dd_merge_kernel, dim3((unsigned)((2 * p.n_bins + 255) / 256)), dim3(256), 0, st, p);
    return hipGetLastError();
}
