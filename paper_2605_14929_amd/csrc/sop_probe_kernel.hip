// Calibration kernel: what a plain read of a buffer costs on this GPU.  Every statistics pass of the
// library reads a layer once; this kernel does only that (16-byte loads with a grid stride, nothing
// kept but an exclusive-or of the words), so its time is the floor those passes are measured against.
// The published HBM peak is a pin rate; the rate a kernel can reach depends on the size of the buffer.
//
// Result: out[b] = exclusive-or of all 32-bit words read by workgroup b (the caller combines the
// SOP_K_PROBE_WG values; an order-independent checksum, so the kernel can be tested).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

__global__ __launch_bounds__(256) void read_probe_kernel(const uint4* __restrict__ x, long long n16, unsigned int* __restrict__ out)
{
    const long long stride = (long long)gridDim.x * 256;
    unsigned int acc = 0u;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const uint4 v = x[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) acc ^= (unsigned int)__shfl_xor((int)acc, s, 64);
    __shared__ unsigned int s_part[4];
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = s_part[0] ^ s_part[1] ^ s_part[2] ^ s_part[3];
}

// Calibration kernel: the rate at which the vector ALUs take instructions of one kind.  The search kernel
// is bound by vector-ALU work, and what that work can cost depends on the kind of instruction and on how many
// wavefronts a SIMD holds: a wavefront issues at most one instruction about every four cycles, a SIMD takes
// plain two-operand arithmetic on registers (fma, multiply, add, logic, integer add) from its wavefronts at
// up to one per two cycles, and compares, selects, minima and maxima, conversions, left shifts, three-operand
// integer instructions and anything with a scalar-register operand at one per four cycles.  This kernel
// measures exactly that: every lane runs `iters` times 64 instructions of the chosen kind on eight
// independent chains (inline assembly, so that the instruction is the one named), no memory traffic in the
// loop; out[thread] = sum of the eight chain values, which a host loop reproduces for the arithmetic kinds.
//   kind 0  v_fmac_f32  x, a, b          (registers only)
//   kind 1  v_max_f32   x, x, a
//   kind 2  v_fma_f32   x, x, s, b       (one scalar-register operand)
//   kind 3  v_cmp_lt_f32 + v_cndmask_b32 (the nearest-entry decision of the search: compare and select)
//   kind 4  v_mul_f32   x, x, a
//   kind 5  v_mad_u32_u24 x, x, a, b
//   kind 6  v_fma_f32 then v_max_f32 on the same chain (one of each class, alternating)
//   kinds 7..14  v_add_f32, v_and_b32, v_add_u32, v_lshrrev_b32, v_lshlrev_b32, v_cvt_i32_f32, v_med3_f32, v_rcp_f32
//           (which class an instruction belongs to; their chain values are not meant to be checked)
// One statement holds the sixteen instructions of a round over the eight chains (the compiler separates inline-assembly
// statements by a no-op, which takes an issue slot of the wavefront: one per sixteen instructions measured here).
// I1, I2: the two instructions applied to a chain, with X for the chain's register and %8, %9, %10 for a, b, sa.
#define SOPK_R8(I) I("%0") "\n" I("%1") "\n" I("%2") "\n" I("%3") "\n" I("%4") "\n" I("%5") "\n" I("%6") "\n" I("%7") "\n"
#define SOPK_P(I1, I2, X) I1(X) "\n" I2(X) "\n"
#define SOPK_OPS : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3), "+v"(x4), "+v"(x5), "+v"(x6), "+v"(x7) : "v"(a), "v"(b), "s"(sa) : "vcc"
// the first instruction on every chain, then the second on every chain: neighbours in the stream are independent
#define SOPK_ISSUE16(I1, I2) asm volatile(SOPK_R8(I1) SOPK_R8(I2) SOPK_OPS);
// compare and select stay together (the select reads the mask the compare before it wrote)
#define SOPK_ISSUE16P(I1, I2) \
    asm volatile(SOPK_P(I1, I2, "%0") SOPK_P(I1, I2, "%1") SOPK_P(I1, I2, "%2") SOPK_P(I1, I2, "%3") \
                 SOPK_P(I1, I2, "%4") SOPK_P(I1, I2, "%5") SOPK_P(I1, I2, "%6") SOPK_P(I1, I2, "%7") SOPK_OPS);
#define SOPK_ISSUE_BODY(I1, I2) for (int it = 0; it < iters; ++it) { SOPK_ISSUE16(I1, I2) SOPK_ISSUE16(I1, I2) SOPK_ISSUE16(I1, I2) SOPK_ISSUE16(I1, I2) }
#define SOPK_ISSUE_BODYP(I1, I2) for (int it = 0; it < iters; ++it) { SOPK_ISSUE16P(I1, I2) SOPK_ISSUE16P(I1, I2) SOPK_ISSUE16P(I1, I2) SOPK_ISSUE16P(I1, I2) }

#define SOPK_K0A(X) "v_fmac_f32 " X ", %8, %9"
#define SOPK_K0B(X) "v_fmac_f32 " X ", %8, %9"
#define SOPK_K1A(X) "v_max_f32 " X ", " X ", %8"
#define SOPK_K1B(X) "v_max_f32 " X ", " X ", %9"
#define SOPK_K2A(X) "v_fma_f32 " X ", " X ", %10, %9"
#define SOPK_K2B(X) "v_fma_f32 " X ", " X ", %10, %9"
#define SOPK_K3A(X) "v_cmp_lt_f32 vcc, " X ", %8"
#define SOPK_K3B(X) "v_cndmask_b32 " X ", " X ", %9, vcc"
#define SOPK_K4A(X) "v_mul_f32 " X ", " X ", %8"
#define SOPK_K4B(X) "v_mul_f32 " X ", " X ", %8"
#define SOPK_K5A(X) "v_mad_u32_u24 " X ", " X ", %8, %9"
#define SOPK_K5B(X) "v_mad_u32_u24 " X ", " X ", %8, %9"
#define SOPK_K6A(X) "v_fma_f32 " X ", " X ", %8, %9"
#define SOPK_K6B(X) "v_max_f32 " X ", " X ", %9"
#define SOPK_K7A(X) "v_add_f32 " X ", " X ", %8"
#define SOPK_K7B(X) "v_add_f32 " X ", " X ", %9"
#define SOPK_K8A(X) "v_and_b32 " X ", " X ", %8"
#define SOPK_K8B(X) "v_and_b32 " X ", " X ", %9"
#define SOPK_K9A(X) "v_add_u32 " X ", " X ", %8"
#define SOPK_K9B(X) "v_add_u32 " X ", " X ", %9"
#define SOPK_K10A(X) "v_lshrrev_b32 " X ", 1, " X
#define SOPK_K10B(X) "v_lshrrev_b32 " X ", 1, " X
#define SOPK_K11A(X) "v_lshlrev_b32 " X ", 1, " X
#define SOPK_K11B(X) "v_lshlrev_b32 " X ", 1, " X
#define SOPK_K12A(X) "v_cvt_i32_f32 " X ", " X
#define SOPK_K12B(X) "v_cvt_i32_f32 " X ", " X
#define SOPK_K13A(X) "v_med3_f32 " X ", " X ", %8, %9"
#define SOPK_K13B(X) "v_med3_f32 " X ", " X ", %8, %9"
#define SOPK_K14A(X) "v_rcp_f32 " X ", " X
#define SOPK_K14B(X) "v_rcp_f32 " X ", " X

template <int KIND>
__global__ __launch_bounds__(1024) void issue_probe_kernel(float* __restrict__ out, int iters, float fa, float fb)
{
    float x0 = (float)(threadIdx.x & 7) * 0.125f, x1 = x0 + 1.0f, x2 = x0 + 2.0f, x3 = x0 + 3.0f, x4 = x0 + 4.0f, x5 = x0 + 5.0f, x6 = x0 + 6.0f, x7 = x0 + 7.0f;
    float a = fa, b = fb;
    const float sa = fa;
    // the operands must sit in vector registers for the kinds that name registers only
    asm volatile("" : "+v"(a), "+v"(b));
    if (KIND == 0) { SOPK_ISSUE_BODY(SOPK_K0A, SOPK_K0B) }
    else if (KIND == 1) { SOPK_ISSUE_BODY(SOPK_K1A, SOPK_K1B) }
    else if (KIND == 2) { SOPK_ISSUE_BODY(SOPK_K2A, SOPK_K2B) }
    else if (KIND == 3) { SOPK_ISSUE_BODYP(SOPK_K3A, SOPK_K3B) }
    else if (KIND == 4) { SOPK_ISSUE_BODY(SOPK_K4A, SOPK_K4B) }
    else if (KIND == 5) { SOPK_ISSUE_BODY(SOPK_K5A, SOPK_K5B) }
    else if (KIND == 6) { SOPK_ISSUE_BODY(SOPK_K6A, SOPK_K6B) }
    else if (KIND == 7) { SOPK_ISSUE_BODY(SOPK_K7A, SOPK_K7B) }
    else if (KIND == 8) { SOPK_ISSUE_BODY(SOPK_K8A, SOPK_K8B) }
    else if (KIND == 9) { SOPK_ISSUE_BODY(SOPK_K9A, SOPK_K9B) }
    else if (KIND == 10) { SOPK_ISSUE_BODY(SOPK_K10A, SOPK_K10B) }
    else if (KIND == 11) { SOPK_ISSUE_BODY(SOPK_K11A, SOPK_K11B) }
    else if (KIND == 12) { SOPK_ISSUE_BODY(SOPK_K12A, SOPK_K12B) }
    else if (KIND == 13) { SOPK_ISSUE_BODY(SOPK_K13A, SOPK_K13B) }
    else { SOPK_ISSUE_BODY(SOPK_K14A, SOPK_K14B) }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = ((x0 + x1) + (x2 + x3)) + ((x4 + x5) + (x6 + x7));
}


// Calibration kernel: the element pass of the search kernel on its own (kinds 15..18 of the issue probe).  Per
// iteration a lane runs six passes ("atoms") over 16 elements held in registers: a table look-up in LDS at a bin that
// differs from lane to lane (records of 33 words as in the search kernel, 256 bins), the choice between the two values
// read, residual fma, c*d, error fma, cosine-sum fma.  It tells what the look-ups cost beside the arithmetic: LDS serves
// 128 bytes a clock to the four SIMDs of a compute unit.
//   MODE 0  12-byte look-up: boundary, value below, value above            (6 vector instructions per element)
//   MODE 1   8-byte look-up: the two values, boundary = their sum          (7; what the search kernel does)
//   MODE 2  no look-up, the arithmetic of MODE 1 on register values        (7)
//   MODE 3  no look-up, the arithmetic of MODE 0 on register values        (6)
// out[thread] = the three running sums added up (not meant to be checked: the table holds a pattern, not a codebook).
#define SOPK_EP_BINS 256
#define SOPK_EP_WORDS 33
template <int MODE>
__global__ __launch_bounds__(1024) void elem_probe_kernel(float* __restrict__ out, int iters, float fa, float fb)
{
    extern __shared__ float s_ep[];
    for (int i = threadIdx.x; i < SOPK_EP_BINS * SOPK_EP_WORDS; i += blockDim.x) s_ep[i] = 0.25f + 0.001f * (float)(i % 97);
    __syncthreads();
    typedef __attribute__((address_space(3))) const float lds_cf;
    const int lane = threadIdx.x & 63;
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)s_ep + 4u * SOPK_EP_WORDS * (uint32_t)((lane * 7) & 127);
    float x[16], w[16], c[16];
    uint32_t addr[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        x[i] = fa + 0.001f * (float)lane + 0.01f * (float)i; w[i] = x[i] + 0.5f; c[i] = fb;
        addr[i] = base + 4u * SOPK_EP_WORDS * (uint32_t)((i * 37) & 63);          // bins (lane*7 & 127) + (i*37 & 63) < 256
    }
    const float ss = -fb;
    float e0 = 0.0f, e1 = 0.0f, wd = 0.0f;
    for (int it = 0; it < iters; ++it) {
        // (nothing below may be moved out of the loop: the compiler is told that the operands have changed)
#pragma unroll
        for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(x[i]), "+v"(w[i]), "+v"(addr[i]));
#pragma unroll
        for (int a = 0; a < 6; ++a) {
#pragma unroll
            for (int i0 = 0; i0 < 16; i0 += 4) {
                float thr[4], ylo[4], yhi[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = i0 + j;
                    if (MODE <= 1) {
                        lds_cf* rp = (lds_cf*)(size_t)addr[i];
                        if (MODE == 0) thr[j] = rp[a];
                        ylo[j] = rp[8 + a]; yhi[j] = rp[16 + a];
                        if (MODE == 1) thr[j] = ylo[j] + yhi[j];
                    } else {
                        ylo[j] = c[i]; yhi[j] = w[(i + a + 1) & 15];
                        thr[j] = MODE == 2 ? ylo[j] + yhi[j] : x[(i + a + 5) & 15];
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = i0 + j;
                    const float yv = x[i] > thr[j] ? yhi[j] : ylo[j];
                    const float d = __fmaf_rn(ss, yv, w[i]);
                    const float cd = c[i] * d;
                    if (i < 8) e0 = __fmaf_rn(cd, d, e0); else e1 = __fmaf_rn(cd, d, e1);
                    wd = __fmaf_rn(cd, w[i], wd);
                }
            }
        }
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = (e0 + e1) + wd;
}

}  // namespace sopk

extern "C" hipError_t sopk_issue_probe_launch(int kind, int n_wg, int n_threads, int iters, float a, float b, float* out, void* stream)
{
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)n_wg), block((unsigned)n_threads);
#define SOPK_IP(K) hipLaunchKernelGGL(sopk::issue_probe_kernel<K>, grid, block, 0, st, out, iters, a, b)
    if (kind >= 15) {
        const size_t lds = (size_t)SOPK_EP_BINS * SOPK_EP_WORDS * sizeof(float);
        switch (kind) {
        case 15: hipLaunchKernelGGL(sopk::elem_probe_kernel<0>, grid, block, lds, st, out, iters, a, b); break;
        case 16: hipLaunchKernelGGL(sopk::elem_probe_kernel<1>, grid, block, lds, st, out, iters, a, b); break;
        case 17: hipLaunchKernelGGL(sopk::elem_probe_kernel<2>, grid, block, lds, st, out, iters, a, b); break;
        default: hipLaunchKernelGGL(sopk::elem_probe_kernel<3>, grid, block, lds, st, out, iters, a, b); break;
        }
        return hipGetLastError();
    }
    switch (kind) {
    case 0: SOPK_IP(0); break;
    case 1: SOPK_IP(1); break;
    case 2: SOPK_IP(2); break;
    case 3: SOPK_IP(3); break;
    case 4: SOPK_IP(4); break;
    case 5: SOPK_IP(5); break;
    case 6: SOPK_IP(6); break;
    case 7: SOPK_IP(7); break;
    case 8: SOPK_IP(8); break;
    case 9: SOPK_IP(9); break;
    case 10: SOPK_IP(10); break;
    case 11: SOPK_IP(11); break;
    case 12: SOPK_IP(12); break;
    case 13: SOPK_IP(13); break;
    default: SOPK_IP(14); break;
    }
#undef SOPK_IP
    return hipGetLastError();
}

extern "C" hipError_t sopk_probe_launch(const void* x, long long n16, unsigned int* out, void* stream)
{
    hipLaunchKernelGGL(sopk::read_probe_kernel, dim3(SOP_K_PROBE_WG), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<const uint4*>(x), n16, out);
    return hipGetLastError();
}
