// Layer-scope floating-point weight formats: one scale for the whole layer, weights rounded to an
// ExMy grid, reconstruction error out.  Three kernels:
//   layer_max_kernel    largest positive and largest negative weight of the layer (integer atomic
//                       max on the bit patterns: order-independent)
//   layer_scope_kernel  scale from those maxima exactly as for a block (absmax rule against the grid's
//                       end values, times 2^k, nearest scale-word value with ties to the lower code),
//                       then per weight x = fl(w*r), nearest grid value with ties to the lower value by
//                       arithmetic on the bit pattern, d = fma(-s, y, w), sums of c*d^2, d^2 and c*w^2
//   sum_kernel          sum of a binary32 array in binary64 (used for the per-block error plane of a
//                       block-scaled format)
// Sums: per lane binary32 within a step, binary64 across steps, lanes and wavefronts; every
// workgroup hands its binary64 partial over through an atomic exchange and the workgroup that
// finishes last adds the partials in workgroup order: the result is reproducible for a given GPU.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

// nearest code of a non-negative binary32 in an ExMy grid (every code finite, subnormals kept);
// ties go to the lower code, or to the upper one when tie_up; saturating at max_code
__device__ __forceinline__ int exmy_encode(float a, int y, int bias, int max_code, bool tie_up)
{
    const uint32_t u = __float_as_uint(a);
    const int E = (int)(u >> 23);
    const uint32_t dn = tie_up ? 0u : 1u;
    const uint32_t ut = u - ((uint32_t)(127 - bias) << 23);
    uint32_t q = (ut + ((1u << (22 - y)) - dn)) >> (23 - y);
    if (E < 128 - bias) {                              // below the smallest normal value: quantum 2^(1-bias-y)
        const int Ee = E > 0 ? E : 1;
        const uint32_t m = (u & 0x7FFFFFu) | (E > 0 ? 0x800000u : 0u);
        int S = 151 - bias - y - Ee;
        S = S > 31 ? 31 : S;
        q = (m + ((1u << (S - 1)) - dn)) >> S;
    }
    return (int)(q > (uint32_t)max_code ? (uint32_t)max_code : q);
}

// value(q) * 2^-k
__device__ __forceinline__ float exmy_decode(int q, int y, int bias, int k)
{
    const int e = q >> y, f = q & ((1 << y) - 1);
    const float nrm = __uint_as_float(((uint32_t)(e - bias - k + 127) << 23) | ((uint32_t)f << (23 - y)));
    const float sub = (float)f * __uint_as_float((uint32_t)(1 - bias - y - k + 127) << 23);
    return e > 0 ? nrm : sub;
}

// value of the nearest ExMy grid point of a non-negative binary32 (same rounding as exmy_encode
// followed by exmy_decode, without forming the code).  At and above the grid's smallest normal value
// the grid point is the binary32 pattern rounded to y mantissa bits: add just under (or exactly) half
// of the dropped field, clear it; a carry out of the mantissa lands on the next binade by itself.
// Below it the grid is uniform with step 2^(1-bias-y); that branch is taken by few lanes.
struct ExmyGrid {
    int y, bias;
    uint32_t half_m1;      // (1 << (22 - y)) - 1
    uint32_t keep;         // ~((1 << (23 - y)) - 1)
    float min_normal;      // 2^(1-bias)
    float quantum;         // 2^(1-bias-y)
    float vmax;            // value of max_code
};
__device__ __forceinline__ float exmy_round_value(float a, bool tie_up, const ExmyGrid& gd)
{
    const uint32_t u = __float_as_uint(a);
    float v = __uint_as_float((u + gd.half_m1 + (tie_up ? 1u : 0u)) & gd.keep);
    if (a < gd.min_normal) {
        asm volatile("");                              // a real branch: skipped when no lane is this small
        const int E = (int)(u >> 23);
        const int Ee = E > 0 ? E : 1;
        const uint32_t m = (u & 0x7FFFFFu) | (E > 0 ? 0x800000u : 0u);
        int S = 151 - gd.bias - gd.y - Ee;
        S = S > 31 ? 31 : S;
        const uint32_t q = (m + ((1u << (S - 1)) - (tie_up ? 0u : 1u))) >> S;
        v = (float)q * gd.quantum;
    }
    return fminf(v, gd.vmax);
}

// the same grid point for a signed x, sign included: ties go to the lower value, which for a negative x is
// the larger magnitude, so the sign bit itself is the tie increment; the sign bit rides through the
// rounding untouched (a finite value never carries out of the exponent), and the clamp to +-vmax is one
// median-of-three.
__device__ __forceinline__ float exmy_round_signed(float x, const ExmyGrid& gd)
{
    const uint32_t xb = __float_as_uint(x);
    float v = __uint_as_float((xb + gd.half_m1 + (xb >> 31)) & gd.keep);
    if (fabsf(x) < gd.min_normal) {
        asm volatile("");                              // a real branch: skipped when no lane is this small
        const uint32_t u = xb & 0x7FFFFFFFu;
        const int E = (int)(u >> 23);
        const int Ee = E > 0 ? E : 1;
        const uint32_t m = (u & 0x7FFFFFu) | (E > 0 ? 0x800000u : 0u);
        int S = 151 - gd.bias - gd.y - Ee;
        S = S > 31 ? 31 : S;
        const uint32_t q = (m + ((1u << (S - 1)) - 1u + (xb >> 31))) >> S;
        v = __uint_as_float(__float_as_uint((float)q * gd.quantum) | (xb & 0x80000000u));
    }
    return __builtin_amdgcn_fmed3f(v, -gd.vmax, gd.vmax);
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int st = 1; st < 64; st <<= 1) v += __shfl_xor(v, st, 64);
    return v;
}

// hands NV binary64 partials of this workgroup over and, in the last workgroup, adds all workgroups'
// partials in order into out[0..NV).  Returns true in the last workgroup.  s_buf: LDS, >= 4*NV + 1 doubles.
template <int NV>
__device__ __forceinline__ bool finish_sums(const double (&v)[NV], unsigned long long* part, unsigned int* done, double* out, double* s_buf)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const double t = wave_sum_f64(v[i]);
        if (lane == 0) s_buf[wv * NV + i] = t;
    }
    __syncthreads();
    if ((int)threadIdx.x < NV) {
        const int i = threadIdx.x;
        const double t = (s_buf[i] + s_buf[NV + i]) + (s_buf[2 * NV + i] + s_buf[3 * NV + i]);
        // an atomic exchange (not a plain store): it completes at the memory side, where the last
        // workgroup's atomic reads find it
        const unsigned long long before = atomicExch(part + (long long)blockIdx.x * NV + i, (unsigned long long)__double_as_longlong(t));
        asm volatile("" :: "v"(before) : "memory");
    }
    __syncthreads();
    unsigned int* s_flag = reinterpret_cast<unsigned int*>(s_buf + 4 * NV);
    // tickets in two levels (16 groups by workgroup number, then over the groups): atomics to one address
    // are served one after the other, and a thousand workgroups finish within a few microseconds
    if (threadIdx.x == 0) {
        const unsigned int r = blockIdx.x % 16u;
        const unsigned int in_group = (gridDim.x - r + 15u) / 16u;
        const unsigned int groups = gridDim.x < 16u ? gridDim.x : 16u;
        unsigned int last = 0u;
        if (atomicAdd(done + 1 + r, 1u) == in_group - 1) {
            atomicExch(done + 1 + r, 0u);
            if (atomicAdd(done, 1u) == groups - 1) last = 1u;
        }
        *s_flag = last;
    }
    __syncthreads();
    if (!*s_flag) return false;
    // last workgroup: every thread adds the partials of workgroups t, t+256, ... in that order, then a
    // fixed tree over the 256 threads (s_tree: 256 doubles of LDS)
    __shared__ double s_tree[256];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        double t = 0.0;
        for (unsigned int g = threadIdx.x; g < gridDim.x; g += 256)
            t += __longlong_as_double((long long)__hip_atomic_load(part + (long long)g * NV + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        s_tree[threadIdx.x] = t;
        __syncthreads();
        for (int h = 128; h >= 1; h >>= 1) {
            if ((int)threadIdx.x < h) s_tree[threadIdx.x] += s_tree[threadIdx.x + h];
            __syncthreads();
        }
        if (threadIdx.x == 0) out[i] = s_tree[0];
        __syncthreads();
    }
    if (threadIdx.x == 255) atomicExch(done, 0u);
    return true;
}

template <bool BF16>
__global__ __launch_bounds__(256) void layer_max_kernel(const LsParams p)
{
    constexpr int EPL = BF16 ? 8 : 4;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long wave = (long long)blockIdx.x * 4 + wv;
    const long long u0 = p.total_units * wave / p.n_waves, u1 = p.total_units * (wave + 1) / p.n_waves;
    float pmax = 0.0f, nmin = 0.0f;
    // the (row, strip) of the next unit is kept on the scalar unit and advanced per load: one division per
    // wavefront, none per step
    const int strips = __builtin_amdgcn_readfirstlane((int)p.strips);
    long long row = u0 / p.strips;
    int st = __builtin_amdgcn_readfirstlane((int)(u0 - row * p.strips));
    // four steps in flight: the loads of a group are issued before any of them is used
    for (long long ub = u0; ub < u1; ub += 4) {
        uint4 t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const long long u = ub + i;
            const long long col0 = ((long long)st * 64 + lane) * EPL;
            t[i] = make_uint4(0, 0, 0, 0);
            if (u < u1 && col0 < p.K)
                t[i] = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(p.W) + (row * p.ldw + col0) * (BF16 ? 2 : 4));
            if (++st == strips) { st = 0; ++row; }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t v[4] = {t[i].x, t[i].y, t[i].z, t[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float a = BF16 ? __uint_as_float(v[j] << 16) : __uint_as_float(v[j]);
                const float b = BF16 ? __uint_as_float(v[j] & 0xFFFF0000u) : a;
                pmax = fmaxf(fmaxf(pmax, a), b);
                nmin = fminf(fminf(nmin, a), b);
            }
        }
    }
    // (0 - nmin, not -nmin: a wavefront without negative weights, or without work, must hand on +0; the bit pattern of -0
    // would rank above every positive value in the unsigned maximum below and erase the copy's running value)
    float nmax = 0.0f - nmin;
#pragma unroll
    for (int st = 1; st < 64; st <<= 1) { pmax = fmaxf(pmax, __shfl_xor(pmax, st, 64)); nmax = fmaxf(nmax, __shfl_xor(nmax, st, 64)); }
    // workgroup maximum in LDS, then at most one atomic per workgroup and value, and only when it
    // would raise the running maximum (atomics to one address are served one after the other, about
    // 25 ns each: thousands of them would cost more than the pass over the layer)
    __shared__ float s_m[2][4];
    if (lane == 0) { s_m[0][wv] = pmax; s_m[1][wv] = nmax; }
    __syncthreads();
    if (threadIdx.x < 2) {
        const float v = fmaxf(fmaxf(s_m[threadIdx.x][0], s_m[threadIdx.x][1]), fmaxf(s_m[threadIdx.x][2], s_m[threadIdx.x][3]));
        const unsigned int bits = __float_as_uint(v) & 0x7FFFFFFFu;   // non-negative floats order like their bit patterns
        // (the running maxima have SOP_K_LS_MAXREP copies, chosen by workgroup number: the first workgroups
        // all finish at once and all find the running value still low)
        unsigned int* mb = p.maxbits + 32 * (blockIdx.x & (SOP_K_LS_MAXREP - 1)) + threadIdx.x;   // copies 128 bytes apart
        if (bits > __hip_atomic_load(mb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(mb, bits);
    }
}

template <bool BF16, bool CODES>
__global__ __launch_bounds__(256) void layer_scope_kernel(const LsParams p)
{
    __shared__ double s_buf[4 * 3 + 1];
    constexpr int EPL = BF16 ? 8 : 4;
    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long wave = (long long)blockIdx.x * 4 + wv;
    const long long u0 = p.total_units * wave / p.n_waves, u1 = p.total_units * (wave + 1) / p.n_waves;

    // ---- the layer's scale: the block rule with the whole layer as the block ----
    // (the copies of the running maxima sit in 64 lines: one wavefront of the workgroup reads them, the
    // others take the result from LDS; every wavefront reading them cost the pass 3 us)
    static_assert(SOP_K_LS_MAXREP == 64, "one copy of the running maxima per lane");
    __shared__ float s_mx[2];
    if (wv == 0) {
        float a = __uint_as_float(__hip_atomic_load(p.maxbits + 32 * lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        float b = __uint_as_float(__hip_atomic_load(p.maxbits + 32 * lane + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
#pragma unroll
        for (int sh = 1; sh < 64; sh <<= 1) { a = fmaxf(a, __shfl_xor(a, sh, 64)); b = fmaxf(b, __shfl_xor(b, sh, 64)); }
        if (lane == 0) { s_mx[0] = a; s_mx[1] = b; }
    }
    __syncthreads();
    const float pmax = s_mx[0], nmax = s_mx[1];
    const float tp = exmy_decode(p.w_max_code, p.w_man, p.w_bias, 0);            // the grid is symmetric: t+ = -t-
    const float sstar = fmaxf(pmax / tp, nmax / tp);
    const int q = exmy_encode(sstar * p.pow2k, p.s_man, p.s_bias, p.s_max_code, false);
    const float s = exmy_decode(q, p.s_man, p.s_bias, p.k);
    const float r = s > 0.0f ? 1.0f / s : 0.0f;
    ExmyGrid gd;
    gd.y = p.w_man; gd.bias = p.w_bias;
    gd.half_m1 = (1u << (22 - p.w_man)) - 1u;
    gd.keep = ~((1u << (23 - p.w_man)) - 1u);
    gd.min_normal = __uint_as_float((uint32_t)(1 - p.w_bias + 127) << 23);
    gd.quantum = __uint_as_float((uint32_t)(1 - p.w_bias - p.w_man + 127) << 23);
    gd.vmax = tp;

    double acc_w = 0.0, acc_u = 0.0, acc_n = 0.0;
    // A wavefront walks down the rows of a 64-lane strip, its channel norms in registers.  Its share of the
    // steps is cut at the strip boundaries into segments; within a segment the loads of four rows are in
    // flight at any time, in four buffers taken in turn.  No load of the inner loop sits under a branch (a
    // lane past the end of the row reads the row's last columns and uses nothing of them; past the last row
    // of the segment the last row is read again), so the count of loads in flight is known where a buffer is
    // waited for and the wait leaves the three younger loads in flight.
    const int esz = BF16 ? 2 : 4;
    long long u = u0;
    while (u < u1) {
        const long long st = u / p.M;
        const long long row0 = u - st * p.M;
        const long long seg_end = (st + 1) * p.M < u1 ? (st + 1) * p.M : u1;
        const long long n = seg_end - u;
        const long long col0 = (st * 64 + lane) * EPL;
        const bool valid = col0 < p.K;
        const long long colc = valid ? col0 : p.K - EPL;
        float c[EPL];
#pragma unroll
        for (int j = 0; j < EPL; j += 4) {
            float4 cc = make_float4(1.f, 1.f, 1.f, 1.f);
            if (p.c) cc = *reinterpret_cast<const float4*>(p.c + colc + j);
            c[j] = cc.x; c[j + 1] = cc.y; c[j + 2] = cc.z; c[j + 3] = cc.w;
        }
        const char* lp = reinterpret_cast<const char*>(p.W) + (row0 * p.ldw + colc) * esz;
        const long long row_bytes = p.ldw * esz;
        long long left = n;
        auto issue = [&]() {
            const uint4 t = *reinterpret_cast<const uint4*>(lp);
            if (--left > 0) lp += row_bytes;
            return t;
        };
        auto step = [&](const uint4 t, const long long my_row) {
            if (!valid) return;
            const uint32_t v[4] = {t.x, t.y, t.z, t.w};
            float w[EPL];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (BF16) { w[2 * j] = __uint_as_float(v[j] << 16); w[2 * j + 1] = __uint_as_float(v[j] & 0xFFFF0000u); }
                else w[j] = __uint_as_float(v[j]);
            }
            float ew = 0.0f, eu = 0.0f, wn = 0.0f;
            uint32_t packed[EPL / 2];
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                const float x = w[j] * r;
                // nearest grid value, ties to the lower value: for a negative x that is the larger magnitude
                float y;
                if (CODES) {
                    const bool negv = x < 0.0f;
                    const int m = exmy_encode(fabsf(x), p.w_man, p.w_bias, p.w_max_code, negv);
                    const float ym = exmy_decode(m, p.w_man, p.w_bias, 0);
                    y = negv ? -ym : ym;
                    const uint32_t idx = (uint32_t)(negv ? p.w_max_code - m : p.w_max_code + m);   // index in the ascending signed grid
                    if (j % 2 == 0) packed[j / 2] = idx; else packed[j / 2] |= idx << 16;
                } else {
                    y = exmy_round_signed(x, gd);
                }
                const float d = __fmaf_rn(-s, y, w[j]);
                const float cd = c[j] * d;
                ew = __fmaf_rn(cd, d, ew);
                eu = __fmaf_rn(d, d, eu);
                wn = __fmaf_rn(c[j] * w[j], w[j], wn);
            }
            acc_w += (double)ew; acc_u += (double)eu; acc_n += (double)wn;
            if (CODES) {
                uint32_t* dst = reinterpret_cast<uint32_t*>(p.codes + my_row * p.K + col0);
#pragma unroll
                for (int j = 0; j < EPL / 2; ++j) dst[j] = packed[j];
            }
        };
        // (issued in the order the loop takes them: the waits count the loads issued after the one waited for)
        uint4 q0 = issue();
        __builtin_amdgcn_sched_barrier(0);
        uint4 q1 = issue();
        __builtin_amdgcn_sched_barrier(0);
        uint4 q2 = issue();
        __builtin_amdgcn_sched_barrier(0);
        uint4 q3 = issue();
        __builtin_amdgcn_sched_barrier(0);
        for (long long i = 0; i < n; i += 4) {
            step(q0, row0 + i);
            q0 = issue();
            if (i + 1 < n) step(q1, row0 + i + 1);
            q1 = issue();
            if (i + 2 < n) step(q2, row0 + i + 2);
            q2 = issue();
            if (i + 3 < n) step(q3, row0 + i + 3);
            q3 = issue();
        }
        u = seg_end;
    }
    const double v3[3] = {acc_w, acc_u, acc_n};
    if (finish_sums<3>(v3, p.part, p.done, p.out, s_buf)) {
        if (threadIdx.x == 0) p.out[3] = (double)q;
        if (threadIdx.x < 2 * SOP_K_LS_MAXREP) atomicExch(p.maxbits + 32 * (threadIdx.x >> 1) + (threadIdx.x & 1), 0u);   // zero for the next call
    }
}

__global__ __launch_bounds__(256) void sum_kernel(const LsParams p)
{
    __shared__ double s_buf[4 * 1 + 1];
    const float* x = reinterpret_cast<const float*>(p.W);
    const long long n = p.total_units;                 // elements
    const long long per = (n + gridDim.x - 1) / gridDim.x;
    const long long b0 = (long long)blockIdx.x * per, b1 = b0 + per < n ? b0 + per : n;
    double acc = 0.0;
    for (long long i = b0 + threadIdx.x; i < b1; i += 256) acc += (double)x[i];
    const double v1[1] = {acc};
    finish_sums<1>(v1, p.part, p.done, p.out, s_buf);
}

}  // namespace sopk

extern "C" hipError_t sopk_ls_launch(const LsParams* pp, int is_bf16, void* stream)
{
    LsParams p = *pp;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)(p.n_waves / 4)), block(256);
    // the maxima pass keeps nothing per workgroup, so it is cut four times finer: compute units that get
    // through their share early take further workgroups (17 us instead of 20 for a 90 MB layer)
    LsParams pm = p;
    pm.n_waves = 4 * p.n_waves;
    const dim3 grid_max((unsigned)(pm.n_waves / 4));
    if (is_bf16) hipLaunchKernelGGL(sopk::layer_max_kernel<true>, grid_max, block, 0, st, pm);
    else hipLaunchKernelGGL(sopk::layer_max_kernel<false>, grid_max, block, 0, st, pm);
    if (is_bf16) {
        if (p.codes) hipLaunchKernelGGL((sopk::layer_scope_kernel<true, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((sopk::layer_scope_kernel<true, false>), grid, block, 0, st, p);
    } else {
        if (p.codes) hipLaunchKernelGGL((sopk::layer_scope_kernel<false, true>), grid, block, 0, st, p);
        else hipLaunchKernelGGL((sopk::layer_scope_kernel<false, false>), grid, block, 0, st, p);
    }
    return hipGetLastError();
}

extern "C" hipError_t sopk_sum_launch(const LsParams* pp, void* stream)
{
    LsParams p = *pp;
    hipLaunchKernelGGL(sopk::sum_kernel, dim3((unsigned)(p.n_waves / 4)), dim3(256), 0, (hipStream_t)stream, p);
    return hipGetLastError();
}
