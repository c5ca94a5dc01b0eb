// Kernel table over all compiled parts, and the launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

#define SOPK_DECL(B, M) extern "C" const void* sopk_part_##B##_##M(int g, int sign_mode, int emit, int na_class, int mode, int* occ, int* mode_out);
SOPK_DECL(0, 0) SOPK_DECL(0, 1) SOPK_DECL(0, 2) SOPK_DECL(1, 0) SOPK_DECL(1, 1) SOPK_DECL(1, 2)
#undef SOPK_DECL

// mode: 0 one layer, 2 a list of layers; *mode_out tells which was given (0 where the one asked for does not exist)
extern "C" const void* sopk_search_kernel(int is_bf16, int g, int sign_mode, int metric, int emit, int na_class, int mode, int* occ, int* mode_out)
{
    if (is_bf16) {
        if (metric == 0) return sopk_part_1_0(g, sign_mode, emit, na_class, mode, occ, mode_out);
        if (metric == 1) return sopk_part_1_1(g, sign_mode, emit, na_class, mode, occ, mode_out);
        return sopk_part_1_2(g, sign_mode, emit, na_class, mode, occ, mode_out);
    }
    if (metric == 0) return sopk_part_0_0(g, sign_mode, emit, na_class, mode, occ, mode_out);
    if (metric == 1) return sopk_part_0_1(g, sign_mode, emit, na_class, mode, occ, mode_out);
    return sopk_part_0_2(g, sign_mode, emit, na_class, mode, occ, mode_out);
}

extern "C" int sopk_variant_index(int is_bf16, int g, int sign_mode, int metric, int emit, int na_class, int mode)
{
    const int gi = g == 8 ? 0 : g == 16 ? 1 : g == 32 ? 2 : 3;
    return ((((((is_bf16 ? 1 : 0) * 4 + gi) * 3 + sign_mode) * 3 + metric) * 2 + (emit ? 1 : 0)) * 3 + na_class) * 2 + (mode ? 1 : 0);
}

// n_wg workgroups of 256 * occ threads
extern "C" hipError_t sopk_launch(const void* fn, const KParams* pp, int n_wg, int occ, size_t dyn_lds, void* stream)
{
    KParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    void* args[] = {&p};
    return hipLaunchKernel(fn, dim3((unsigned)n_wg), dim3(256u * (unsigned)occ), args, dyn_lds, st);
}
