// Second stage of the layer reduction, the kernel table over all compiled parts, and the launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

// One workgroup per output, fixed order, binary64.  Column sums hold deficits 1 - cos; lanes whose
// block had zero weighted norm (and the lanes past the end of a row) added exactly 1 to every
// column and are taken out again through the count column.
__global__ __launch_bounds__(256) void reduce_kernel(const KParams p)
{
    __shared__ double s[256], z[256];
    const int o = blockIdx.x;                      // 0..A-1 atoms (internal order), then pairs by output index
    int col;
    double* dst;
    if (o < p.A) { col = o; dst = p.acos_atom ? p.acos_atom + p.uidx[o] : nullptr; }
    else { col = SOP_K_MAXA + p.pair_pi[o - p.A]; dst = p.acos_pair ? p.acos_pair + (o - p.A) : nullptr; }
    const long long n_wg = p.n_waves / 4;
    double t = 0.0, tz = 0.0;
    for (long long g = threadIdx.x; g < n_wg; g += 256) {
        t += (double)p.partial[(long long)col * n_wg + g];
        tz += (double)p.partial[(long long)SOP_K_ZCOL * n_wg + g];
    }
    s[threadIdx.x] = t;
    z[threadIdx.x] = tz;
    __syncthreads();
    for (int h = 128; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) { s[threadIdx.x] += s[threadIdx.x + h]; z[threadIdx.x] += z[threadIdx.x + h]; }
        __syncthreads();
    }
    if (threadIdx.x == 0 && dst) *dst = 1.0 - (s[0] - z[0]) / ((double)p.Nb * (double)p.lpb);
}

}  // namespace sopk

#define SOPK_DECL(B, M) extern "C" const void* sopk_part_##B##_##M(int g, int is_signed, int emit, int na8);
SOPK_DECL(0, 0) SOPK_DECL(0, 1) SOPK_DECL(0, 2) SOPK_DECL(1, 0) SOPK_DECL(1, 1) SOPK_DECL(1, 2)
#undef SOPK_DECL

extern "C" const void* sopk_search_kernel(int is_bf16, int g, int is_signed, int metric, int emit, int na8)
{
    if (is_bf16) {
        if (metric == 0) return sopk_part_1_0(g, is_signed, emit, na8);
        if (metric == 1) return sopk_part_1_1(g, is_signed, emit, na8);
        return sopk_part_1_2(g, is_signed, emit, na8);
    }
    if (metric == 0) return sopk_part_0_0(g, is_signed, emit, na8);
    if (metric == 1) return sopk_part_0_1(g, is_signed, emit, na8);
    return sopk_part_0_2(g, is_signed, emit, na8);
}

extern "C" int sopk_variant_index(int is_bf16, int g, int is_signed, int metric, int emit, int na8)
{
    const int gi = g == 8 ? 0 : g == 16 ? 1 : g == 32 ? 2 : 3;
    return (((((is_bf16 ? 1 : 0) * 4 + gi) * 2 + (is_signed ? 1 : 0)) * 3 + metric) * 2 + (emit ? 1 : 0)) * 2 + (na8 ? 1 : 0);
}

extern "C" hipError_t sopk_launch(const void* fn, const KParams* pp, size_t dyn_lds, void* stream)
{
    KParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    void* args[] = {&p};
    hipError_t e = hipLaunchKernel(fn, dim3((unsigned)(p.n_waves / 4)), dim3(256), args, dyn_lds, st);
    if (e != hipSuccess) return e;
    if (p.acos_atom || p.acos_pair) {
        hipLaunchKernelGGL(sopk::reduce_kernel, dim3((unsigned)(p.A + p.P)), dim3(256), 0, st, p);
        e = hipGetLastError();
    }
    return e;
}
