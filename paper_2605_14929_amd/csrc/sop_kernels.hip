// Pair-search kernels for gfx950 (MI355X).
//
// Work mapping.  A lane owns EPL = min(g,16) consecutive elements of one row (one block when
// g <= 16, a half or a quarter of a block when g = 32 / 64: LPB = g/EPL lanes cooperate through
// cross-lane exchanges).  A wavefront covers a "strip" of 64*EPL consecutive columns of one row
// per step and walks down the rows of that strip, so the channel norms of the strip stay in
// registers.  The (strip,row) steps of the whole layer are cut into equal contiguous ranges, one
// per resident wavefront, so every SIMD gets the same amount of work whatever the shape.
//
// Every block is read from HBM exactly once.  LDS holds a table over uniform bins of the scaled
// weight x: for every atom each bin contains at most one code boundary, so the nearest entry is a
// table read and one compare.  A bin is a record of 33 words (boundary, lower value, upper value
// and lower code of each of the 8 atoms, one word of padding): the odd stride puts the same field
// of 64 consecutive bins into 64 different banks, so lanes reading different bins do not conflict.
// For scale words of up to 11 magnitude bits LDS also holds the (scale, reciprocal) pair of every
// scale code.
//
// Atoms with equal endpoints form a scale group: they share the ideal scale, the scale code and the
// scaled weights, which are computed once per group.
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

#ifndef SOP_K_SEARCH_OCC
#define SOP_K_SEARCH_OCC 4          /* resident workgroups per compute unit the search-mode kernels are built for */
#endif

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

// write a wave-uniform 32-bit value into lane LANE of a register (other lanes keep `old`).
// gfx950 needs two wait states between a vector instruction that writes a scalar register (the
// compare producing the ballot) and a vector instruction that reads it; the compiler inserts them
// for its own code but not inside inline assembly, hence the s_nop.
template <int LANE> __device__ __forceinline__ uint32_t put_lane(uint32_t value, uint32_t old)
{
    const uint32_t s = __builtin_amdgcn_readfirstlane(value);
    asm("s_nop 1\n\tv_writelane_b32 %0, %1, %2" : "+v"(old) : "s"(s), "n"(LANE));
    return old;
}

// wave-uniform switches of the row loop
struct Switches {
    int A;
    uint32_t pair_mask, flip_mask, grp_first, unit_tpos, unit_tneg, wide;
};

// per-lane running sum kept in LDS (each lane owns its address: plain read-add-write, no atomics,
// which on this chip serialise the lanes of the wavefront)
__device__ __forceinline__ void lds_accumulate(float* slot, float v)
{
    *slot = *slot + v;
}

// round a non-negative fp32 to the scale word: nearest, ties to the lower code, saturating
__device__ __forceinline__ int encode_scale(float sp, const KParams& p)
{
    const uint32_t u = __float_as_uint(sp);
    const int E = (int)(u >> 23);
    const int y = p.man_bits;
    // normal range of the target: rebias the exponent, round the 23-bit mantissa to y bits
    const uint32_t ut = u - ((uint32_t)(127 - p.bias) << 23);
    uint32_t q = (ut + ((1u << (22 - y)) - 1u)) >> (23 - y);
    const bool sub = E < 128 - p.bias;
    if (__any(sub)) {
        // subnormal range of the target (or zero): quantum 2^(1-bias-y)
        const int Ee = E > 0 ? E : 1;
        const uint32_t m = (u & 0x7FFFFFu) | (E > 0 ? 0x800000u : 0u);
        int S = 151 - p.bias - y - Ee;
        S = S > 31 ? 31 : S;
        const uint32_t qs = S > 0 ? ((m + ((1u << (S - 1)) - 1u)) >> S) : 0u;
        q = sub ? qs : q;
    }
    return (int)(q > (uint32_t)p.max_code ? (uint32_t)p.max_code : q);
}

// value(q) * 2^-k (exact) and its IEEE reciprocal (0 for the zero scale)
__device__ __forceinline__ void decode_scale(int q, const KParams& p, const float2* __restrict__ s_tab, float& s, float& rinv)
{
    if (p.n_tab_codes) {
        const float2 t = s_tab[q];
        s = t.x;
        rinv = t.y;
    } else {
        const int y = p.man_bits;
        const int e = q >> y, f = q & ((1 << y) - 1);
        const float nrm = __uint_as_float(((uint32_t)(e - p.bias - p.k + 127) << 23) | ((uint32_t)f << (23 - y)));
        const float sub = (float)f * p.sub_quantum;
        s = e > 0 ? nrm : sub;
        rinv = s > 0.0f ? 1.0f / s : 0.0f;
    }
}

// ideal scale of a block against endpoints (tp, -tn); a unit endpoint needs no division
__device__ __forceinline__ float ideal_scale(float pmax, float nmax, float tp, float tn, bool unit_p, bool unit_n)
{
    float s1 = pmax, s2 = nmax;
    if (!unit_p) s1 = pmax / tp;
    if (!unit_n) s2 = nmax / tn;
    return fmaxf(s1, s2);
}

// Scale of one (group, sign): code q, signed scale ss, scaled weights x and their bin offsets.
template <int EPL>
__device__ __forceinline__ void prepare_sign(const float (&w)[EPL], float pmax, float nmax, bool negative, int a,
                                             const KParams& p, const Switches& sw, const float2* __restrict__ s_tab,
                                             const float4* __restrict__ s_gpar,
                                             int& q, float& ss, bool& nonzero, float (&x)[EPL], uint32_t (&boff)[EPL])
{
    const float4 gp = s_gpar[a];                       // (t+, -t-, bin scale, bin offset): same address in every lane
    const float tp = gp.x, tn = gp.y;
    const bool unit_p = (sw.unit_tpos >> a) & 1u, unit_n = (sw.unit_tneg >> a) & 1u;
    const float sstar = negative ? ideal_scale(pmax, nmax, tn, tp, unit_n, unit_p) : ideal_scale(pmax, nmax, tp, tn, unit_p, unit_n);
    q = encode_scale(sstar * p.pow2k, p);
    float s, rinv;
    decode_scale(q, p, s_tab, s, rinv);
    ss = negative ? -s : s;
    nonzero = s > 0.0f;
    const float rr = negative ? -rinv : rinv;
    const float sc = gp.z, off = gp.w;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        x[i] = w[i] * rr;
        const float xc = __builtin_amdgcn_fmed3f(x[i], -tn, tp);
        // off carries 1.5*2^23, so the low mantissa bits of the sum are the bin number; one 24-bit
        // multiply-add turns them into the byte offset of the bin record
        boff[i] = __umul24(__float_as_uint(__fmaf_rn(xc, sc, off)), SOP_K_BIN_BYTES) + SOP_K_BIN_NEGC;
    }
}

struct Cand {
    float err;    // decision score
    float ny;     // numerator of the block cosine, up to a power of the scale that cancels
    float dy;     // squared c-norm of the reconstruction, same convention: cos = ny / sqrt(||w||^2 dy)
};

// Element pass of one (atom, sign) candidate on the lane's EPL elements.
// FAST: the cosine inputs come from the residual sums through
//   <w,w^> = ||w||^2 - <w,d>,   ||w^||^2 = ||w||^2 - 2<w,d> + ||d||^2      (all c-weighted),
// which saves two operations per element but cancels when the reconstruction is much smaller than
// the block (saturated or vanished scale); the caller checks dy against ||w||^2 and falls back to
// direct_cosine_sums() for the wavefront in that case.
template <int EPL, int LPB, int METRIC, bool CODES, bool FAST>
__device__ __forceinline__ Cand eval_elements(const float (&w)[EPL], const float (&cb)[EPL], const float (&cw)[EPL],
                                              const float (&x)[EPL], const uint32_t (&boff)[EPL], float ss, bool nonzero,
                                              bool negative, float wn, const char* __restrict__ bins_a, bool wide_codes,
                                              uint32_t (&codes)[EPL / 4])
{
    float e0 = 0.0f, e1 = 0.0f, ny = 0.0f, dy = 0.0f, ew = 0.0f;
    if (CODES) {
#pragma unroll
        for (int j = 0; j < EPL / 4; ++j) codes[j] = 0;
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const float* rp = reinterpret_cast<const float*>(bins_a + boff[i]);      // bins_a = table + 4*a
        const float thr = rp[0], ylo = rp[SOP_K_MAXA], yhi = rp[2 * SOP_K_MAXA];
        int clo = 0;
        if (CODES) clo = reinterpret_cast<const int*>(rp)[3 * SOP_K_MAXA];
        const bool up = x[i] > thr;
        const float yv = up ? yhi : ylo;
        const float d = __fmaf_rn(-ss, yv, w[i]);
        const float cd = (METRIC == 2 && !FAST) ? d : cb[i] * d;     // MSE+FAST also needs c*d for the cosine
        const float dd = METRIC == 2 ? d : cd;
        if (i < 8) e0 = __fmaf_rn(dd, d, e0); else e1 = __fmaf_rn(dd, d, e1);
        if (FAST) {
            ny = __fmaf_rn(cd, w[i], ny);                               // <w,d>, from c*d which is at hand
            if (METRIC == 2) ew = __fmaf_rn(cd, d, ew);                   // weighted ||d||^2 beside the unweighted score
        } else {
            ny = __fmaf_rn(cw[i], yv, ny);
            dy = __fmaf_rn(cb[i], yv * yv, dy);
        }
        if (CODES) {
            const uint32_t code = (uint32_t)clo + (up ? 1u : 0u);
            if (wide_codes) codes[i / 4] |= code << (8 * (i % 4));
            else codes[i / 8] |= code << (4 * (i % 8));
        }
    }
    Cand r;
    const float err = EPL == 16 ? e0 + e1 : e0;
    r.err = group_sum<LPB>(err);
    if (FAST) {
        const float wd = group_sum<LPB>(ny);
        const float errw = METRIC == 2 ? group_sum<LPB>(ew) : r.err;
        r.ny = wn - wd;
        r.dy = __fmaf_rn(-2.0f, wd, wn) + errw;
    } else {
        const float nsum = group_sum<LPB>(negative ? -ny : ny);
        const float dsum = group_sum<LPB>(dy);
        r.ny = nonzero ? nsum : 0.0f;                                  // a zero scale reconstructs nothing
        r.dy = nonzero ? dsum : 0.0f;
    }
    return r;
}

// Cosine inputs straight from the codebook values (positive scale sign), used when the residual
// form above would cancel.
template <int EPL, int LPB>
__device__ __forceinline__ void direct_cosine_sums(const float (&cb)[EPL], const float (&w)[EPL], const float (&x)[EPL],
                                                   const uint32_t (&boff)[EPL], bool nonzero,
                                                   const char* __restrict__ bins_a, float& ny_out, float& dy_out)
{
    float ny = 0.0f, dy = 0.0f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const float* rp = reinterpret_cast<const float*>(bins_a + boff[i]);
        const float yv = x[i] > rp[0] ? rp[2 * SOP_K_MAXA] : rp[SOP_K_MAXA];
        ny = __fmaf_rn(cb[i] * w[i], yv, ny);
        dy = __fmaf_rn(cb[i], yv * yv, dy);
    }
    const float nsum = group_sum<LPB>(ny), dsum = group_sum<LPB>(dy);
    ny_out = nonzero ? nsum : 0.0f;
    dy_out = nonzero ? dsum : 0.0f;
}

// first / second atom of the pair with lexicographic position pi among all pairs of SOP_K_MAXA atoms
__host__ __device__ constexpr int pair_first(int pi) { int i = 0; while (pi >= SOP_K_MAXA - 1 - i) { pi -= SOP_K_MAXA - 1 - i; ++i; } return i; }
__host__ __device__ constexpr int pair_second(int pi) { const int i = pair_first(pi); return pi - pair_index(i, i + 1) + i + 1; }

// Selector of pair PI and of all following pairs (i < j in internal order).  The pair's ballot (one
// bit per block) is dropped into fixed lanes of `piece`; the caller stores those lanes afterwards.
template <int PI, int LPB>
__device__ __forceinline__ void all_pairs(const KParams& p, const Switches& sw, const float (&err)[SOP_K_MAXA],
                                          const float (&dlt)[SOP_K_MAXA], float* __restrict__ acc_lane, uint32_t& piece)
{
    constexpr int i = pair_first(PI), j = pair_second(PI);
    static_assert(pair_index(i, j) == PI, "pair enumeration");
    if ((sw.pair_mask >> PI) & 1u) {
        // caller's pair (a,b): selector = "b strictly better than a"; when the internal order
        // swapped the two, b is internal i
        const float ei = err[i], ej = err[j], di = dlt[i], dj = dlt[j];
        bool sel;
        float chosen;
        // the empty asm statements keep this a real (scalar) branch: one compare per pair
        if ((sw.flip_mask >> PI) & 1u) { asm volatile(""); sel = ei < ej; chosen = sel ? di : dj; }
        else                           { asm volatile(""); sel = ej < ei; chosen = sel ? dj : di; }
        // column of this pair among the requested ones
        const int col = sw.A + __builtin_popcount(sw.pair_mask & ((1u << PI) - 1u));
        lds_accumulate(acc_lane + col * 256, chosen);
        if (p.sel_bits) {
            unsigned long long mask = __ballot(sel);
            if (LPB == 1) {
                piece = put_lane<2 * PI>((uint32_t)mask, piece);
                piece = put_lane<2 * PI + 1>((uint32_t)(mask >> 32), piece);
            } else if (LPB == 2) {     // keep one bit per block: bits of even lanes
                mask &= 0x5555555555555555ull;
                mask = (mask | (mask >> 1)) & 0x3333333333333333ull;
                mask = (mask | (mask >> 2)) & 0x0F0F0F0F0F0F0F0Full;
                mask = (mask | (mask >> 4)) & 0x00FF00FF00FF00FFull;
                mask = (mask | (mask >> 8)) & 0x0000FFFF0000FFFFull;
                mask = (mask | (mask >> 16)) & 0x00000000FFFFFFFFull;
                piece = put_lane<PI>((uint32_t)mask, piece);
            } else {                   // bits of lanes 0,4,8,...
                mask &= 0x1111111111111111ull;
                mask = (mask | (mask >> 3)) & 0x0303030303030303ull;
                mask = (mask | (mask >> 6)) & 0x000F000F000F000Full;
                mask = (mask | (mask >> 12)) & 0x000000FF000000FFull;
                mask = (mask | (mask >> 24)) & 0x000000000000FFFFull;
                piece = put_lane<PI>((uint32_t)mask, piece);
            }
        }
    }
    if constexpr (PI + 1 < SOP_K_MAXP) all_pairs<PI + 1, LPB>(p, sw, err, dlt, acc_lane, piece);
}

// The search-mode kernels are kept within 128 registers so that four workgroups (16 wavefronts)
// stay resident per compute unit; the variants with two scale signs or per-block outputs need more.
template <bool BF16, int EPL, int LPB, bool SIGNED, int METRIC, bool EMIT>
__global__ __launch_bounds__(256, (SIGNED || EMIT) ? 1 : SOP_K_SEARCH_OCC) void search_kernel(const KParams p)
{
    extern __shared__ __align__(16) char s_mem[];
    // LDS: bin table | (scale, reciprocal) table | group parameters | per-lane ACos accumulators
    char* s_bins = s_mem;                                                         // [n_bins] records of 33 words
    const size_t bins_bytes = ((size_t)p.n_bins * SOP_K_BIN_BYTES + 15) & ~(size_t)15;
    float2* s_tab = reinterpret_cast<float2*>(s_mem + bins_bytes);
    float4* s_gpar = reinterpret_cast<float4*>(s_mem + bins_bytes + (((size_t)p.n_tab_codes * sizeof(float2) + 15) & ~(size_t)15));
    float* s_acc = reinterpret_cast<float*>(s_gpar + SOP_K_MAXA);                  // [n_cols][256]
    __shared__ float s_red[4][SOP_K_NCOL];
    const int n_cols = p.A + p.P;
    {
        const int nw = p.n_bins * (SOP_K_BIN_BYTES / 4);
        const uint32_t* src = reinterpret_cast<const uint32_t*>(p.bins);
        uint32_t* dst = reinterpret_cast<uint32_t*>(s_bins);
        for (int i = threadIdx.x; i < nw; i += 256) dst[i] = src[i];
        for (int i = threadIdx.x; i < p.n_tab_codes; i += 256) s_tab[i] = p.stab[i];
        if (threadIdx.x < SOP_K_MAXA) s_gpar[threadIdx.x] = make_float4(p.tpos[threadIdx.x], p.tneg[threadIdx.x], p.bin_sc[threadIdx.x], p.bin_off[threadIdx.x]);
        for (int i = 0; i < n_cols; ++i) s_acc[i * 256 + threadIdx.x] = 0.0f;
    }
    __syncthreads();
    float* acc_lane = s_acc + threadIdx.x;

    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const long long wave = (long long)blockIdx.x * 4 + wv;
    const long long u0 = p.total_units * wave / p.n_waves;
    const long long u1 = p.total_units * (wave + 1) / p.n_waves;

    // selector output: which pair's bit plane this lane stores into (-1: none)
    int sel_slot = -1;
    {
        const int my_pi = LPB == 1 ? (lane >> 1) : (LPB == 2 ? lane : (lane & 31));
#pragma unroll
        for (int pi = 0; pi < SOP_K_MAXP; ++pi)
            if (my_pi == pi && ((p.pair_mask >> pi) & 1u)) sel_slot = p.pair_slot[pi];
        if (LPB == 1 && lane >= 2 * SOP_K_MAXP) sel_slot = -1;
        if (LPB == 2 && lane >= SOP_K_MAXP) sel_slot = -1;
        if (LPB == 4 && (lane & 31) >= SOP_K_MAXP) sel_slot = -1;
    }

    long long strip = u0 / p.M;
    long long m = u0 - strip * p.M;
    long long cur_strip = -1;
    float cb[EPL];
    bool valid = false;
    long long col0 = 0;

    for (long long u = u0; u < u1; ++u) {
        // The uniform switches below are re-read every row.  Left loop-invariant, each test would be
        // hoisted out of the loop as a 64-bit lane mask and the hundred-odd masks would spill.
        Switches sw = {p.A, p.pair_mask, p.flip_mask, p.grp_first_mask, p.unit_tpos, p.unit_tneg, p.wide_mask};
        asm volatile("" : "+s"(sw.A), "+s"(sw.pair_mask), "+s"(sw.flip_mask), "+s"(sw.grp_first), "+s"(sw.unit_tpos), "+s"(sw.unit_tneg), "+s"(sw.wide));
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
        // state of the current scale group (positive sign)
        int gq = 0;
        float gss = 0.0f;
        bool gnz = false;
        float gx[EPL];
        uint32_t gboff[EPL];
#pragma unroll
        for (int i = 0; i < EPL; ++i) { gx[i] = 0.0f; gboff[i] = 0; }

#pragma unroll
        for (int a = 0; a < SOP_K_MAXA; ++a) {
            err[a] = 0.0f; dlt[a] = 0.0f;
            if (a < sw.A) {
                if ((sw.grp_first >> a) & 1u) prepare_sign<EPL>(w, pmax, nmax, false, a, p, sw, s_tab, s_gpar, gq, gss, gnz, gx, gboff);
                const char* bins_a = s_bins + 4 * a;
                const bool wide = EMIT && ((sw.wide >> a) & 1u);
                uint32_t codes[EPL / 4];
                constexpr bool FAST = !SIGNED;      // with two scale signs per atom the direct sums are used
                Cand best = eval_elements<EPL, LPB, METRIC, EMIT, FAST>(w, cb, cw, gx, gboff, gss, gnz, false, wn, bins_a, wide, codes);
                if (FAST) {
                    // the residual form is accurate while the reconstruction carries a fair share of
                    // the block's norm; otherwise the whole wavefront recomputes this atom directly
                    const bool weak = !(best.dy >= 0.25f * wn);
                    if (__builtin_expect(__any(weak) != 0, 0)) direct_cosine_sums<EPL, LPB>(cb, w, gx, gboff, gnz, bins_a, best.ny, best.dy);
                }
                int q = gq;
                bool neg = false;
                if (SIGNED) {
                    int q2;
                    float ss2, x2[EPL];
                    bool nz2;
                    uint32_t boff2[EPL], codes2[EPL / 4];
                    prepare_sign<EPL>(w, pmax, nmax, true, a, p, sw, s_tab, s_gpar, q2, ss2, nz2, x2, boff2);
                    const Cand c2 = eval_elements<EPL, LPB, METRIC, EMIT, false>(w, cb, cw, x2, boff2, ss2, nz2, true, wn, bins_a, wide, codes2);
                    neg = c2.err < best.err;
                    best.err = neg ? c2.err : best.err;
                    best.ny = neg ? c2.ny : best.ny;
                    best.dy = neg ? c2.dy : best.dy;
                    q = neg ? q2 : q;
                    if (EMIT) {
#pragma unroll
                        for (int j = 0; j < EPL / 4; ++j) codes[j] = neg ? codes2[j] : codes[j];
                    }
                }
                // cosine value; a vanishing reconstruction has ny = 0 and gives 0, a zero-norm block counts as 1
                const float cosv = best.ny * __frsqrt_rn(fmaxf(wn * best.dy, 1.0e-37f));
                err[a] = best.err;
                dlt[a] = wn > 0.0f ? 1.0f - cosv : 0.0f;
                lds_accumulate(acc_lane + a * 256, dlt[a]);
                if (EMIT) {
                    const long long ua = p.uidx[a];
                    if (p.scale_code && leader) p.scale_code[ua * p.Nb + blk] = (uint16_t)(q | (neg ? 0x8000 : 0));
                    if (p.blk_err && leader) p.blk_err[ua * p.Nb + blk] = best.err;
                    if (p.blk_cos && leader) p.blk_cos[ua * p.Nb + blk] = 1.0f - dlt[a];
                    if (p.codes && valid) {
                        if (!wide) {
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
        // ---- selector of every requested pair; afterwards the lanes that received a ballot store
        //      their piece of the bit planes in a single instruction ----
        uint32_t piece = 0;
        all_pairs<0, LPB>(p, sw, err, dlt, acc_lane, piece);
        if (p.sel_bits && sel_slot >= 0) {
            if (LPB == 1) {                        // lane 2*pi+h holds word 2*strip+h of the row
                const long long widx = strip * 2 + (lane & 1);
                if (widx < p.Wr) p.sel_bits[((long long)sel_slot * p.M + m) * p.Wr + widx] = piece;
            } else if (LPB == 2) {                 // lane pi holds word `strip` of the row
                p.sel_bits[((long long)sel_slot * p.M + m) * p.Wr + strip] = piece;
            } else {                               // lane pi holds 16-bit piece `strip`; lanes 32+pi clear the padding piece
                uint16_t* plane = reinterpret_cast<uint16_t*>(p.sel_bits) + ((long long)sel_slot * p.M + m) * (2 * p.Wr);
                if (lane < 32) plane[strip] = (uint16_t)piece;
                else if (strip == p.strips - 1 && p.strips < 2 * p.Wr) plane[p.strips] = 0;
            }
        }
        // next step of the range
        if (++m == p.M) { m = 0; ++strip; }
    }

    // ---- per-workgroup partial sums (deficits 1-cos): lanes, then the four wavefronts in order ----
    for (int i = 0; i < n_cols; ++i) {
        float v = acc_lane[i * 256];
#pragma unroll
        for (int st = 1; st < 64; st <<= 1) v += __shfl_xor(v, st, 64);
        if (lane == 0) s_red[wv][i] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < n_cols) {
        const int i = threadIdx.x;
        const float v = (s_red[0][i] + s_red[1][i]) + (s_red[2][i] + s_red[3][i]);
        p.partial[(long long)i * (p.n_waves / 4) + blockIdx.x] = v;
    }
}

// Second stage of the layer reduction: one workgroup per output, fixed order, binary64.
__global__ __launch_bounds__(256) void reduce_kernel(const KParams p)
{
    __shared__ double s[256];
    const int o = blockIdx.x;                      // 0..A-1 atoms (internal order), then pairs by output index
    int col;
    double* dst;
    if (o < p.A) { col = o; dst = p.acos_atom ? p.acos_atom + p.uidx[o] : nullptr; }
    else { col = p.A + p.pair_col[o - p.A]; dst = p.acos_pair ? p.acos_pair + (o - p.A) : nullptr; }
    const long long n_wg = p.n_waves / 4;
    double t = 0.0;
    for (long long g = threadIdx.x; g < n_wg; g += 256) t += (double)p.partial[(long long)col * n_wg + g];
    s[threadIdx.x] = t;
    __syncthreads();
    for (int h = 128; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) s[threadIdx.x] += s[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0 && dst) *dst = 1.0 - s[0] / ((double)p.Nb * (double)p.lpb);
}

}  // namespace sopk

// ---- kernel table ----
template <bool BF16, int EPL, int LPB>
static const void* pick_geom(bool is_signed, int metric, bool emit)
{
#define SOPK_FN(S, MT, E) reinterpret_cast<const void*>(&sopk::search_kernel<BF16, EPL, LPB, S, MT, E>)
    if (metric == 0) {
        if (is_signed) return emit ? SOPK_FN(true, 0, true) : SOPK_FN(true, 0, false);
        return emit ? SOPK_FN(false, 0, true) : SOPK_FN(false, 0, false);
    }
    if (is_signed) return emit ? SOPK_FN(true, 2, true) : SOPK_FN(true, 2, false);
    return emit ? SOPK_FN(false, 2, true) : SOPK_FN(false, 2, false);
#undef SOPK_FN
}

extern "C" const void* sopk_search_kernel(int is_bf16, int g, int is_signed, int metric, int emit)
{
    if (is_bf16) {
        switch (g) {
            case 8:  return pick_geom<true, 8, 1>(is_signed, metric, emit);
            case 16: return pick_geom<true, 16, 1>(is_signed, metric, emit);
            case 32: return pick_geom<true, 16, 2>(is_signed, metric, emit);
            default: return pick_geom<true, 16, 4>(is_signed, metric, emit);
        }
    }
    switch (g) {
        case 8:  return pick_geom<false, 8, 1>(is_signed, metric, emit);
        case 16: return pick_geom<false, 16, 1>(is_signed, metric, emit);
        case 32: return pick_geom<false, 16, 2>(is_signed, metric, emit);
        default: return pick_geom<false, 16, 4>(is_signed, metric, emit);
    }
}

extern "C" int sopk_variant_index(int is_bf16, int g, int is_signed, int metric, int emit)
{
    const int gi = g == 8 ? 0 : g == 16 ? 1 : g == 32 ? 2 : 3;
    return (((is_bf16 ? 1 : 0) * 4 + gi) * 2 + (is_signed ? 1 : 0)) * 4 + (metric == 0 ? 0 : 2) + (emit ? 1 : 0);
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
