// Pair-search kernels for gfx950 (MI355X).
//
// Work mapping.  A lane owns EPL = min(g,16) consecutive elements of one row (one block when
// g <= 16, a half or a quarter of a block when g = 32 / 64: LPB = g/EPL lanes cooperate through
// cross-lane exchanges).  A wavefront covers a "strip" of 64*EPL consecutive columns of one row
// per step and walks down the rows of that strip, so the channel norms of the strip stay in
// registers.  The (strip,row) steps of the whole layer are cut into equal contiguous ranges, one
// per wavefront, so every SIMD gets the same amount of work whatever the shape.
//
// Every block is read from HBM exactly once.  Codebook values and midpoints sit in LDS (16- and
// 32-entry tables occupy distinct banks, so the binary search reads are conflict free).
//
// Arithmetic contract (what makes the integer outputs reproducible on any implementation):
//   scale      s* = max(pmax/t+, nmax/-t-)  (IEEE division), times 2^k, rounded to the scale word
//              (nearest, ties to the lower code, saturating), s = value(q) * 2^-k, r = 1/s (IEEE)
//   element    x = fl(w*r); code = number of midpoints strictly below x
//   error      d = fma(-s, L[code], w);  err = sum fma(fl(c*d), d, .) over chunks of 8 consecutive
//              elements, chunk partials added in a balanced tree in index order
//   selection  strictly smaller err wins (second atom of a pair, negative scale sign)
// The cosine values are not decisions; they are evaluated in fp32 in the scaled domain, where the
// block scale cancels:  cos = sign(s) * <w,y>_c / sqrt(||w||_c^2 * ||y||_c^2),  y_i = L[code_i],
// and accumulated per lane as the deficit 1 - cos, reduced in binary64.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sop_kparams.h"

namespace sopk {

__device__ __forceinline__ float xor_lanes(float v, int mask) { return __shfl_xor(v, mask, 64); }

template <int LPB> __device__ __forceinline__ float group_max(float v)
{
    if (LPB >= 2) v = fmaxf(v, xor_lanes(v, 1));
    if (LPB >= 4) v = fmaxf(v, xor_lanes(v, 2));
    return v;
}
// balanced tree over the lanes of a block, in lane (= index) order; both partners compute the
// same rounded sum because addition commutes
template <int LPB> __device__ __forceinline__ float group_sum(float v)
{
    if (LPB >= 2) v = v + xor_lanes(v, 1);
    if (LPB >= 4) v = v + xor_lanes(v, 2);
    return v;
}

// round a non-negative fp32 to the scale word: nearest, ties to the lower code, saturating
__device__ __forceinline__ int encode_scale(float sp, const KParams& p)
{
    const uint32_t u = __float_as_uint(sp);
    const int E = (int)(u >> 23);
    const int y = p.man_bits;
    // normal range of the target: rebias the exponent, round the 23-bit mantissa to y bits
    const uint32_t ut = u - ((uint32_t)(127 - p.bias) << 23);
    uint32_t qn = (ut + ((1u << (22 - y)) - 1u)) >> (23 - y);
    // subnormal range of the target: quantum 2^(1-bias-y)
    const int Ee = E > 0 ? E : 1;
    const uint32_t m = (u & 0x7FFFFFu) | (E > 0 ? 0x800000u : 0u);
    int S = 151 - p.bias - y - Ee;
    S = S > 31 ? 31 : S;
    uint32_t qs = S > 0 ? ((m + ((1u << (S - 1)) - 1u)) >> S) : 0u;
    uint32_t q = (E >= 128 - p.bias) ? qn : qs;
    return (int)(q > (uint32_t)p.max_code ? (uint32_t)p.max_code : q);
}

// value(q) * 2^-k, exact
__device__ __forceinline__ float decode_scale(int q, const KParams& p)
{
    const int y = p.man_bits;
    const int e = q >> y, f = q & ((1 << y) - 1);
    const float nrm = __uint_as_float(((uint32_t)(e - p.bias - p.k + 127) << 23) | ((uint32_t)f << (23 - y)));
    const float sub = (float)f * p.sub_quantum;
    return e > 0 ? nrm : sub;
}

struct Cand {
    float err;    // decision score
    float ny;     // c-weighted <w,y>, signed by the scale sign
    float dy;     // c-weighted ||y||^2 (0 when the scale is 0: the reconstruction vanishes)
    int   q;
};

// Evaluate one (atom, scale sign) candidate on the lane's EPL elements.
template <int EPL, int LPB, int METRIC, bool CODES>
__device__ __forceinline__ Cand eval_candidate(const float (&w)[EPL], const float (&cb)[EPL], const float (&cw)[EPL],
                                               float pmax, float nmax, bool negative, int a, const KParams& p,
                                               const float* __restrict__ s_mid, const float* __restrict__ s_val,
                                               const float* __restrict__ s_vsq, uint32_t (&codes)[EPL / 4])
{
    const float tp = p.tpos[a], tn = p.tneg[a];
    const float s1 = negative ? pmax / tn : pmax / tp;
    const float s2 = negative ? nmax / tp : nmax / tn;
    const float sp = fmaxf(s1, s2) * p.pow2k;
    Cand r;
    r.q = encode_scale(sp, p);
    const float s = decode_scale(r.q, p);
    const float rinv = s > 0.0f ? 1.0f / s : 0.0f;
    const float ss = negative ? -s : s;
    const float rr = negative ? -rinv : rinv;

    const float* mid = s_mid + a * SOP_K_TAB;
    const float* val = s_val + a * SOP_K_TAB;
    const float* vsq = s_vsq + a * SOP_K_TAB;
    int idx[EPL];
    float x[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) { x[i] = w[i] * rr; idx[i] = 0; }
    for (int h = p.half0[a]; h >= 1; h >>= 1) {          // binary search over the padded midpoint table
#pragma unroll
        for (int i = 0; i < EPL; ++i) idx[i] += (x[i] > mid[idx[i] + h - 1]) ? h : 0;
    }
    float e0 = 0.0f, e1 = 0.0f, ny = 0.0f, dy = 0.0f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const float yv = val[idx[i]];
        const float d = __fmaf_rn(-ss, yv, w[i]);
        const float cd = METRIC == 2 ? d : cb[i] * d;
        if (i < 8) e0 = __fmaf_rn(cd, d, e0); else e1 = __fmaf_rn(cd, d, e1);
        ny = __fmaf_rn(cw[i], yv, ny);
        dy = __fmaf_rn(cb[i], vsq[idx[i]], dy);
    }
    if (CODES) {
#pragma unroll
        for (int j = 0; j < EPL / 4; ++j) codes[j] = 0;
        if (p.nent[a] <= 16) {
#pragma unroll
            for (int i = 0; i < EPL; ++i) codes[i / 8] |= (uint32_t)idx[i] << (4 * (i % 8));
        } else {
#pragma unroll
            for (int i = 0; i < EPL; ++i) codes[i / 4] |= (uint32_t)idx[i] << (8 * (i % 4));
        }
    }
    float err = EPL == 16 ? e0 + e1 : e0;
    r.err = group_sum<LPB>(err);
    r.ny = group_sum<LPB>(negative ? -ny : ny);
    const float dsum = group_sum<LPB>(dy);
    r.dy = s > 0.0f ? dsum : 0.0f;
    return r;
}

template <bool BF16, int EPL, int LPB, bool SIGNED, int METRIC, bool EMIT>
__global__ __launch_bounds__(256) void search_kernel(const KParams p)
{
    __shared__ float s_mid[SOP_K_MAXA * SOP_K_TAB];
    __shared__ float s_val[SOP_K_MAXA * SOP_K_TAB];
    __shared__ float s_vsq[SOP_K_MAXA * SOP_K_TAB];
    for (int i = threadIdx.x; i < SOP_K_MAXA * SOP_K_TAB; i += 256) {
        s_mid[i] = p.tab_mid[i];
        const float v = p.tab_val[i];
        s_val[i] = v;
        s_vsq[i] = v * v;
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long u0 = p.total_units * wave / p.n_waves;
    const long long u1 = p.total_units * (wave + 1) / p.n_waves;

    float acc[SOP_K_MAXA + SOP_K_MAXP];
#pragma unroll
    for (int i = 0; i < SOP_K_MAXA + SOP_K_MAXP; ++i) acc[i] = 0.0f;

    long long strip = u0 / p.M;
    long long m = u0 - strip * p.M;
    long long cur_strip = -1;
    float cb[EPL];
    bool valid = false;
    long long col0 = 0;

    for (long long u = u0; u < u1; ++u) {
        if (strip != cur_strip) {
            cur_strip = strip;
            col0 = (strip * 64 + lane) * EPL;
            valid = col0 < p.K;
#pragma unroll
            for (int i = 0; i < EPL; i += 4) {
                float4 t = valid ? *reinterpret_cast<const float4*>(p.c + col0 + i) : make_float4(0.f, 0.f, 0.f, 0.f);
                cb[i] = t.x; cb[i + 1] = t.y; cb[i + 2] = t.z; cb[i + 3] = t.w;
            }
        }
        // ---- the block: one read from HBM ----
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
        // ---- block statistics ----
        float pmax = 0.0f, nmax = 0.0f, wn = 0.0f, cw[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            pmax = fmaxf(pmax, w[i]);
            nmax = fmaxf(nmax, -w[i]);
            cw[i] = cb[i] * w[i];
            wn = __fmaf_rn(cw[i], w[i], wn);
        }
        pmax = group_max<LPB>(pmax);
        nmax = group_max<LPB>(nmax);
        wn = group_sum<LPB>(wn);

        const long long blk_in_row = (strip * 64 + lane) / LPB;
        const long long blk = m * p.Bk + blk_in_row;
        const bool leader = valid && (lane % LPB == 0);

        float err[SOP_K_MAXA], dlt[SOP_K_MAXA];
#pragma unroll
        for (int a = 0; a < SOP_K_MAXA; ++a) {
            err[a] = 0.0f; dlt[a] = 0.0f;
            if (a < p.A) {
                uint32_t codes[EPL / 4];
                Cand best = eval_candidate<EPL, LPB, METRIC, EMIT>(w, cb, cw, pmax, nmax, false, a, p, s_mid, s_val, s_vsq, codes);
                bool neg = false;
                if (SIGNED) {
                    uint32_t codes2[EPL / 4];
                    Cand c2 = eval_candidate<EPL, LPB, METRIC, EMIT>(w, cb, cw, pmax, nmax, true, a, p, s_mid, s_val, s_vsq, codes2);
                    neg = c2.err < best.err;
                    best.err = neg ? c2.err : best.err;
                    best.ny = neg ? c2.ny : best.ny;
                    best.dy = neg ? c2.dy : best.dy;
                    best.q = neg ? c2.q : best.q;
                    if (EMIT) {
#pragma unroll
                        for (int j = 0; j < EPL / 4; ++j) codes[j] = neg ? codes2[j] : codes[j];
                    }
                }
                // cosine value; a vanishing reconstruction gives 0, a zero-norm block counts as 1
                const float prod = wn * best.dy;
                const float cosv = prod > 0.0f ? fminf(fmaxf(best.ny * __frsqrt_rn(prod), -1.0f), 1.0f) : 0.0f;
                err[a] = best.err;
                dlt[a] = wn > 0.0f ? 1.0f - cosv : 0.0f;
                acc[a] += dlt[a];
                if (EMIT) {
                    if (p.scale_code && leader) p.scale_code[(long long)a * p.Nb + blk] = (uint16_t)(best.q | (neg ? 0x8000 : 0));
                    if (p.blk_err && leader) p.blk_err[(long long)a * p.Nb + blk] = best.err;
                    if (p.blk_cos && leader) p.blk_cos[(long long)a * p.Nb + blk] = 1.0f - dlt[a];
                    if (p.codes && valid) {
                        if (p.nent[a] <= 16) {
                            uint8_t* dst = p.codes + p.code_off[a] + (m * p.K + col0) / 2;
#pragma unroll
                            for (int j = 0; j < EPL / 8; ++j) reinterpret_cast<uint32_t*>(dst)[j] = codes[j];
                        } else {
                            uint8_t* dst = p.codes + p.code_off[a] + m * p.K + col0;
#pragma unroll
                            for (int j = 0; j < EPL / 4; ++j) reinterpret_cast<uint32_t*>(dst)[j] = codes[j];
                        }
                    }
                }
            }
        }
        // ---- selector of every requested pair ----
#pragma unroll
        for (int a = 0; a < SOP_K_MAXA; ++a) {
#pragma unroll
            for (int b = a + 1; b < SOP_K_MAXA; ++b) {
                const int slot = p.pair_slot[a * SOP_K_MAXA + b];
                if (slot >= 0) {
                    const bool sel = err[b] < err[a];
                    acc[SOP_K_MAXA + pair_index(a, b)] += sel ? dlt[b] : dlt[a];
                    if (p.sel_bits) {
                        unsigned long long mask = __ballot(sel);
                        if (LPB == 2) {            // keep one bit per block: bits of even lanes
                            mask &= 0x5555555555555555ull;
                            mask = (mask | (mask >> 1)) & 0x3333333333333333ull;
                            mask = (mask | (mask >> 2)) & 0x0F0F0F0F0F0F0F0Full;
                            mask = (mask | (mask >> 4)) & 0x00FF00FF00FF00FFull;
                            mask = (mask | (mask >> 8)) & 0x0000FFFF0000FFFFull;
                            mask = (mask | (mask >> 16)) & 0x00000000FFFFFFFFull;
                        } else if (LPB == 4) {     // bits of lanes 0,4,8,...
                            mask &= 0x1111111111111111ull;
                            mask = (mask | (mask >> 3)) & 0x0303030303030303ull;
                            mask = (mask | (mask >> 6)) & 0x000F000F000F000Full;
                            mask = (mask | (mask >> 12)) & 0x000000FF000000FFull;
                            mask = (mask | (mask >> 24)) & 0x000000000000FFFFull;
                        }
                        // the strip owns U = 4/LPB 16-bit pieces of the row's bit plane; the last
                        // strip also clears the padding piece of the last word
                        const int U = 4 / LPB;
                        const long long first = strip * U;
                        const long long n16 = (strip == p.strips - 1) ? (2 * p.Wr - first) : U;
                        if (lane < n16) {
                            const uint16_t piece = lane < 4 ? (uint16_t)(mask >> (16 * lane)) : (uint16_t)0;
                            uint16_t* plane = reinterpret_cast<uint16_t*>(p.sel_bits) + ((long long)slot * p.M + m) * (2 * p.Wr);
                            plane[first + lane] = piece;
                        }
                    }
                }
            }
        }
        // next step of the range
        if (++m == p.M) { m = 0; ++strip; }
    }

    // ---- per-wavefront partial sums (deficits 1-cos), summed over lanes ----
#pragma unroll
    for (int i = 0; i < SOP_K_MAXA + SOP_K_MAXP; ++i) {
        float v = acc[i];
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) v += __shfl_xor(v, s, 64);
        acc[i] = v;
    }
    if (lane == 0) {
        float* dst = p.partial + wave * (SOP_K_MAXA + SOP_K_MAXP);
#pragma unroll
        for (int i = 0; i < SOP_K_MAXA + SOP_K_MAXP; ++i) dst[i] = acc[i];
    }
}

// Second stage of the layer reduction: one workgroup per output, fixed order, binary64.
__global__ __launch_bounds__(256) void reduce_kernel(const KParams p)
{
    __shared__ double s[256];
    const int o = blockIdx.x;                      // 0..A-1 atoms, A..A+P-1 pairs (output order)
    int col;
    double* dst;
    if (o < p.A) { col = o; dst = p.acos_atom ? p.acos_atom + o : nullptr; }
    else { col = SOP_K_MAXA + p.pair_col[o - p.A]; dst = p.acos_pair ? p.acos_pair + (o - p.A) : nullptr; }
    double t = 0.0;
    for (long long wv = threadIdx.x; wv < p.n_waves; wv += 256) t += (double)p.partial[wv * (SOP_K_MAXA + SOP_K_MAXP) + col];
    s[threadIdx.x] = t;
    __syncthreads();
    for (int h = 128; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) s[threadIdx.x] += s[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0 && dst) *dst = 1.0 - s[0] / ((double)p.Nb * (double)p.lpb);
}

}  // namespace sopk

// ---- launch table ----
template <bool BF16, int EPL, int LPB>
static hipError_t launch_geom(const KParams& p, bool is_signed, int metric, bool emit, dim3 grid, hipStream_t st)
{
#define SOPK_GO(S, MT, E) hipLaunchKernelGGL((sopk::search_kernel<BF16, EPL, LPB, S, MT, E>), grid, dim3(256), 0, st, p)
    if (metric == 0) {
        if (is_signed) { if (emit) SOPK_GO(true, 0, true); else SOPK_GO(true, 0, false); }
        else           { if (emit) SOPK_GO(false, 0, true); else SOPK_GO(false, 0, false); }
    } else {
        if (is_signed) { if (emit) SOPK_GO(true, 2, true); else SOPK_GO(true, 2, false); }
        else           { if (emit) SOPK_GO(false, 2, true); else SOPK_GO(false, 2, false); }
    }
#undef SOPK_GO
    return hipGetLastError();
}

extern "C" hipError_t sopk_launch(const KParams* pp, int is_bf16, int g, int is_signed, int metric, int emit, void* stream)
{
    const KParams& p = *pp;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid((unsigned)(p.n_waves / 4));
    hipError_t e;
    if (is_bf16) {
        switch (g) {
            case 8:  e = launch_geom<true, 8, 1>(p, is_signed, metric, emit, grid, st); break;
            case 16: e = launch_geom<true, 16, 1>(p, is_signed, metric, emit, grid, st); break;
            case 32: e = launch_geom<true, 16, 2>(p, is_signed, metric, emit, grid, st); break;
            default: e = launch_geom<true, 16, 4>(p, is_signed, metric, emit, grid, st); break;
        }
    } else {
        switch (g) {
            case 8:  e = launch_geom<false, 8, 1>(p, is_signed, metric, emit, grid, st); break;
            case 16: e = launch_geom<false, 16, 1>(p, is_signed, metric, emit, grid, st); break;
            case 32: e = launch_geom<false, 16, 2>(p, is_signed, metric, emit, grid, st); break;
            default: e = launch_geom<false, 16, 4>(p, is_signed, metric, emit, grid, st); break;
        }
    }
    if (e != hipSuccess) return e;
    if (p.acos_atom || p.acos_pair) {
        hipLaunchKernelGGL(sopk::reduce_kernel, dim3((unsigned)(p.A + p.P)), dim3(256), 0, st, p);
        e = hipGetLastError();
    }
    return e;
}
