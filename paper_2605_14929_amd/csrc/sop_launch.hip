// Kernel table over all compiled parts, and the launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

#define SOPK_DECL(B, M) extern "C" const void* sopk_part_##B##_##M(int g, int sign_mode, int emit, int na_class, int* occ);
SOPK_DECL(0, 0) SOPK_DECL(0, 1) SOPK_DECL(0, 2) SOPK_DECL(1, 0) SOPK_DECL(1, 1) SOPK_DECL(1, 2)
#undef SOPK_DECL

extern "C" const void* sopk_search_kernel(int is_bf16, int g, int sign_mode, int metric, int emit, int na_class, int* occ)
{
    if (is_bf16) {
        if (metric == 0) return sopk_part_1_0(g, sign_mode, emit, na_class, occ);
        if (metric == 1) return sopk_part_1_1(g, sign_mode, emit, na_class, occ);
        return sopk_part_1_2(g, sign_mode, emit, na_class, occ);
    }
    if (metric == 0) return sopk_part_0_0(g, sign_mode, emit, na_class, occ);
    if (metric == 1) return sopk_part_0_1(g, sign_mode, emit, na_class, occ);
    return sopk_part_0_2(g, sign_mode, emit, na_class, occ);
}

extern "C" int sopk_variant_index(int is_bf16, int g, int sign_mode, int metric, int emit, int na_class)
{
    const int gi = g == 8 ? 0 : g == 16 ? 1 : g == 32 ? 2 : 3;
    return (((((is_bf16 ? 1 : 0) * 4 + gi) * 3 + sign_mode) * 3 + metric) * 2 + (emit ? 1 : 0)) * 3 + na_class;
}

// n_wg workgroups of 256 * occ threads
extern "C" hipError_t sopk_launch(const void* fn, const KParams* pp, int n_wg, int occ, size_t dyn_lds, void* stream)
{
    KParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    void* args[] = {&p};
    return hipLaunchKernel(fn, dim3((unsigned)n_wg), dim3(256u * (unsigned)occ), args, dyn_lds, st);
}
