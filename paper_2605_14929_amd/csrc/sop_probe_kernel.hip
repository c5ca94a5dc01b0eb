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

}  // namespace sopk

extern "C" hipError_t sopk_probe_launch(const void* x, long long n16, unsigned int* out, void* stream)
{
    hipLaunchKernelGGL(sopk::read_probe_kernel, dim3(SOP_K_PROBE_WG), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<const uint4*>(x), n16, out);
    return hipGetLastError();
}
