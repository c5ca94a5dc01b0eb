// Materialisation of a searched layer: per block, the scale word in its b-bit container (sign bit,
// magnitude code, codebook selector in the first metabit) and the block's codes as a dense string
// of n-bit fields.
//
// Bit positions (scale word SwExMy, m = b - w - x - y metabits): sign at bit b-1 when w = 1; the
// magnitude code (exponent, then mantissa) sits above the metabits of the low end; the selector is
// the first metabit: bit b-1 when w = 0, bit m-1 when w = 1.  Payload: code i of the block occupies
// bits i*n .. i*n+n-1 of a little-endian bit string of g*n/8 bytes (n = 4: two codes per byte, the
// first in the low half, which is also the layout of the search's code planes).
//
// One lane per block; a block's input codes and output bytes are contiguous, so neighbouring lanes
// touch neighbouring addresses.  Pure data movement: the kernel is bound by HBM.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

// COPY: both planes hold two codes per byte and n = 4, so the payload is a copy of the chosen plane
template <bool COPY>
__global__ __launch_bounds__(256) void pack_kernel(const PackParams p)
{
    const long long blk = (long long)blockIdx.x * 256 + threadIdx.x;
    if (blk >= p.Nb) return;
    unsigned int sel = 0;
    if (p.sel_words) {
        const unsigned int wsel = p.sel_u32 ? reinterpret_cast<const uint32_t*>(p.sel_words)[blk]
                                            : (unsigned int)reinterpret_cast<const uint16_t*>(p.sel_words)[blk];
        sel = (wsel >> p.pair_q) & 1u;
    }
    const unsigned int sc = sel ? p.scale_b[blk] : p.scale_a[blk];
    unsigned int word = (sc & 0x7FFFu) << p.mag_shift;
    if (p.sign_pos >= 0) word |= (sc >> 15) << p.sign_pos;
    if (p.sel_pos >= 0) word |= sel << p.sel_pos;
    p.words[blk] = (uint16_t)word;

    const unsigned char* src = sel ? p.codes_b : p.codes_a;
    const int wide = sel ? p.wide_b : p.wide_a;
    const int g = p.g, n = p.n_bits;
    unsigned char* dst = p.payload + blk * (long long)(g * n / 8);
    if (COPY) {
        const unsigned char* s = src + blk * (long long)(g / 2);
        if (g == 8) {
            *reinterpret_cast<uint32_t*>(dst) = *reinterpret_cast<const uint32_t*>(s);
        } else {
            for (int i = 0; i < g / 2; i += 8) *reinterpret_cast<uint2*>(dst + i) = *reinterpret_cast<const uint2*>(s + i);
        }
        return;
    }
    // eight codes at a time: 8*n bits = n bytes
    for (int i = 0; i < g; i += 8) {
        unsigned long long v = 0;
        if (wide) {
            const uint2 t = *reinterpret_cast<const uint2*>(src + blk * (long long)g + i);
            const unsigned long long b8 = ((unsigned long long)t.y << 32) | t.x;
            for (int j = 0; j < 8; ++j) v |= ((b8 >> (8 * j)) & 0xFFull) << (j * n);
        } else {
            const uint32_t t = *reinterpret_cast<const uint32_t*>(src + blk * (long long)(g / 2) + i / 2);
            for (int j = 0; j < 8; ++j) v |= (unsigned long long)((t >> (4 * j)) & 0xFu) << (j * n);
        }
        unsigned char* d = dst + (i / 8) * n;
        for (int j = 0; j < n; ++j) d[j] = (unsigned char)(v >> (8 * j));
    }
}

}  // namespace sopk

extern "C" hipError_t sopk_pack_launch(const PackParams* pp, void* stream)
{
    const PackParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)((p.Nb + 255) / 256)), block(256);
    const bool copy = p.n_bits == 4 && !p.wide_a && !(p.scale_b && p.wide_b);
    if (copy) hipLaunchKernelGGL((sopk::pack_kernel<true>), grid, block, 0, st, p);
    else hipLaunchKernelGGL((sopk::pack_kernel<false>), grid, block, 0, st, p);
    return hipGetLastError();
}
