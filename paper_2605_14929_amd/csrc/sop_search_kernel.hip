// Pair-search kernel for gfx950 (MI355X).  This file is compiled once per (weight dtype, metric)
// part; SOPK_PART_BF16 and SOPK_PART_METRIC select which instantiations the object holds.
//
// Work mapping.  A lane owns EPL = min(g,16) consecutive elements of one row (one block when
// g <= 16, a half or a quarter of a block when g = 32 / 64: LPB = g/EPL lanes cooperate through
// cross-lane exchanges).  A wavefront covers a "strip" of 64*EPL consecutive columns of one row
// per step and walks down the rows of that strip, so the channel norms of the strip stay in
// registers.  The (strip,row) steps of the whole layer are cut into equal contiguous ranges, one
// per resident wavefront, so every SIMD gets the same amount of work whatever the shape.  The
// weights of the next step are requested before the current step is evaluated.
//
// Every block is read from HBM exactly once.  LDS holds a table over uniform bins of the scaled
// weight x: for every atom each bin contains at most one code boundary, so the nearest entry is a
// table read and one compare.  A bin is a record of 33 words (boundary, half the lower value, half the
// upper value and lower code of each of the 8 atoms, one word of padding; see read_rec for the halves):
// the odd stride puts the same field of 32 consecutive bins into 32 different banks.  For scale words of
// up to 11 magnitude bits LDS also holds (twice the scale, the scale's reciprocal) of every scale code.
//
// Atoms with equal endpoints form a scale group: they share the ideal scale, the scale code and the
// scaled weights, which are computed once per group.
//
// Arithmetic contract (what makes the integer outputs reproducible on any implementation):
//   scale      s* = max(pmax/t+, nmax/-t-)  (IEEE division), times 2^k, rounded to the scale word
//              (nearest, ties to the lower code, saturating), s = value(q) * 2^-k, r = 1/s (IEEE)
//   element    x = fl(w*r); code = number of midpoints strictly below x
//   error      d = fma(-s, L[code], w) (evaluated as fma(-2s, L[code]/2, w): the same product, both factors exact);
//              err = sum fma(fl(c*d), d, .) over chunks of 8 consecutive
//              elements, chunk partials added in a balanced tree in index order
//   cosine     (metric COS only) w^ = fl(s*L[code]); num = sum fma(fl(c*w), w^, .),
//              den = sum fma(fl(c*w^), w^, .), same chunks and tree
//   selection  metrics WSE / MSE: strictly smaller err wins (second atom of a pair, negative scale
//              sign); metric COS: b beats a when fl(q_b*den_a) > fl(q_a*den_b), q = fl(num*|num|),
//              a zero reconstruction counting as q = 0, den = 1
// The cosine values are not decisions; they are evaluated in fp32 and accumulated per lane as the
// deficit 1 - cos; workgroup sums enter the layer sums as 64-bit fixed-point integers.  A lane whose
// block has zero weighted norm adds exactly 1 to every column and 1 to a count column that is
// subtracted at the end.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "sop_kparams.h"

#ifndef SOPK_PART_BF16
#error "compile with -DSOPK_PART_BF16=0|1 -DSOPK_PART_METRIC=0|1|2"
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

// wave-uniform switches of the row loop
struct Switches {
    int A;
    uint32_t pair_mask, flip_mask, gid, unit_tpos, unit_tneg, wide, mirror, selfsym;
};

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

// TWICE value(q) * 2^-k (exact; the element passes multiply it with the halved codebook values of the table) and the
// IEEE reciprocal of value(q) * 2^-k (0 for the zero scale); the tabulated pair holds the doubled scale already
__device__ __forceinline__ void decode_scale(int q, const KParams& p, const float2* __restrict__ s_tab, float& s2, float& rinv)
{
    if (p.n_tab_codes) {
        const float2 t = s_tab[q];
        s2 = t.x;
        rinv = t.y;
    } else {
        const int y = p.man_bits;
        const int e = q >> y, f = q & ((1 << y) - 1);
        const float nrm = __uint_as_float(((uint32_t)(e - p.bias - p.k + 127) << 23) | ((uint32_t)f << (23 - y)));
        const float sub = (float)f * p.sub_quantum;
        const float s = e > 0 ? nrm : sub;
        s2 = s + s;
        rinv = s > 0.0f ? 1.0f / s : 0.0f;
    }
}

// ideal scale of a block against endpoints (tp, -tn); a unit endpoint needs no division
__device__ __forceinline__ float ideal_scale(float pmax, float nmax, float tp, float tn, bool unit_p, bool unit_n)
{
    float s1 = pmax, s2 = nmax;
    // the flags are wave-uniform; the empty asm statements keep these real branches (a division is a
    // dozen instructions, and the common codebooks have unit endpoints)
    if (!unit_p) { asm volatile(""); s1 = pmax / tp; }
    if (!unit_n) { asm volatile(""); s2 = nmax / tn; }
    return fmaxf(s1, s2);
}

// Scale of one (group, sign): code q, twice the signed scale in ss, scaled weights x and their bin offsets.
// boff receives the LDS byte address of each element's bin record (lds_neg = table address minus the
// product the 24-bit multiply adds for the constant's exponent bits).
// ARGMAX: the scale maps the block's largest-magnitude element onto the endpoint of larger magnitude
// and its sign follows from the two signs (per lane, returned in neg_out); otherwise the absmax rule
// for the sign given in `negative`.
// Scale of one (group, sign) without the scaled weights: code q, TWICE the signed scale in ss (the table holds half of
// every codebook value, see read_rec: 2s * L/2 is the product s * L), signed reciprocal rr, and whether the scaled
// weights may leave the bin table (see prepare_sign).
struct ScalePrep { int q; float ss, rr; bool nonzero, beyond; };
__device__ __forceinline__ ScalePrep prepare_scale(float pmax, float nmax, bool negative, int a, const KParams& p, const Switches& sw,
                                                   const float2* __restrict__ s_tab, const float4* __restrict__ s_gpar)
{
    const float4 gp = s_gpar[2 * a];                   // (t+, -t-, bin scale, bin offset): same address in every lane
    const float tp = gp.x, tn = gp.y;
    const bool unit_p = (sw.unit_tpos >> a) & 1u, unit_n = (sw.unit_tneg >> a) & 1u;
    const float sstar = negative ? ideal_scale(pmax, nmax, tn, tp, unit_n, unit_p) : ideal_scale(pmax, nmax, tp, tn, unit_p, unit_n);
    ScalePrep r;
    r.q = encode_scale(sstar * p.pow2k, p);
    float s2, rinv;
    decode_scale(r.q, p, s_tab, s2, rinv);
    r.ss = negative ? -s2 : s2;
    r.nonzero = s2 > 0.0f;
    r.rr = negative ? -rinv : rinv;
    r.beyond = !(sstar * rinv <= SOP_K_BIN_SAFE);
    return r;
}

template <int EPL, bool ARGMAX>
__device__ __forceinline__ void prepare_sign(const float (&w)[EPL], float pmax, float nmax, bool negative, int a,
                                             const KParams& p, const Switches& sw, const float2* __restrict__ s_tab,
                                             const float4* __restrict__ s_gpar, uint32_t lds_neg,
                                             int& q, float& ss, bool& nonzero, float (&x)[EPL], uint32_t (&boff)[EPL], bool& neg_out)
{
    const float4 gp = s_gpar[2 * a];                   // (t+, -t-, bin scale, bin offset): same address in every lane
    const float tp = gp.x, tn = gp.y;
    const bool unit_p = (sw.unit_tpos >> a) & 1u, unit_n = (sw.unit_tneg >> a) & 1u;
    float sstar;
    if constexpr (ARGMAX) {
        const bool x_pos = pmax >= nmax, t_pos = tp >= tn;          // ties: the positive element, the positive endpoint
        sstar = (x_pos ? pmax : nmax) / (t_pos ? tp : tn);
        negative = x_pos != t_pos;
    } else {
        sstar = negative ? ideal_scale(pmax, nmax, tn, tp, unit_n, unit_p) : ideal_scale(pmax, nmax, tp, tn, unit_p, unit_n);
    }
    neg_out = negative;
    q = encode_scale(sstar * p.pow2k, p);
    float s2, rinv;
    decode_scale(q, p, s_tab, s2, rinv);             // (twice the scale: the element passes multiply it with half of the codebook value)
    ss = negative ? -s2 : s2;
    nonzero = s2 > 0.0f;
    const float rr = negative ? -rinv : rinv;
    const float sc = gp.z, off = gp.w;
    // the table covers a scale rounded down by up to the factor SOP_K_BIN_SAFE; beyond it (the scale
    // word saturated) the whole wavefront clamps its scaled weights into the table's range
    // (the argmax rule lets elements pass the smaller endpoint by any factor: always clamp)
    const bool beyond = ARGMAX || !(sstar * rinv <= SOP_K_BIN_SAFE);
    if (__builtin_expect(ARGMAX || __any(beyond) != 0, ARGMAX ? 1 : 0)) {
        const float4 g2 = s_gpar[2 * a + 1];           // (table range low, high, -, -)
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            x[i] = w[i] * rr;
            const float xc = __builtin_amdgcn_fmed3f(x[i], g2.x, g2.y);
            boff[i] = __umul24(__float_as_uint(__fmaf_rn(xc, sc, off)), SOP_K_BIN_BYTES) + lds_neg;
        }
    } else {
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            x[i] = w[i] * rr;
            // off carries 1.5*2^23, so the low mantissa bits of the sum are the bin number; one 24-bit
            // multiply-add turns them into the byte offset of the bin record
            boff[i] = __umul24(__float_as_uint(__fmaf_rn(x[i], sc, off)), SOP_K_BIN_BYTES) + lds_neg;
        }
    }
}

// Where an element pass takes a scaled weight and the LDS address of its bin record from: arrays filled by
// prepare_sign (a scale group's atoms share them), or formed on the spot from the weight and the scale's reciprocal
// (signed scale words: the arrays of two signs would cost a wavefront per SIMD in registers, and with every atom
// evaluated under two scales there is little left to share).  Same arithmetic either way.
template <int EPL>
struct ArrSrc {
    const float (&x)[EPL];
    const uint32_t (&boff)[EPL];
    __device__ __forceinline__ void get(int i, float& xo, uint32_t& bo) const { xo = x[i]; bo = boff[i]; }
};
template <int EPL, bool CLAMP>
struct FlySrc {
    const float (&w)[EPL];
    float rr, sc, off, lo, hi;
    uint32_t lds_neg;
    __device__ __forceinline__ void get(int i, float& xo, uint32_t& bo) const
    {
        xo = w[i] * rr;
        const float xc = CLAMP ? __builtin_amdgcn_fmed3f(xo, lo, hi) : xo;
        bo = __umul24(__float_as_uint(__fmaf_rn(xc, sc, off)), SOP_K_BIN_BYTES) + lds_neg;
    }
};

// Sums of one (atom, sign) candidate over the lane's elements, before the cross-lane tree.
struct Sums {
    float err;    // decision score of metrics WSE / MSE (and the blk_err output)
    float wd;     // RESIDUAL form: <w,d>_c;  DIRECT form: numerator sum
    float ew;     // RESIDUAL form with metric MSE: c-weighted ||d||^2;  DIRECT form: denominator sum
};

// One bin record read: boundary, value below, value above (and the lower code when codes are wanted).
// `addr` is the LDS byte address of the record and A the atom's slot in it: all reads are register + immediate offset.
// The table holds HALF of each codebook value (exact: the host refuses entries whose half is not), and every
// element pass multiplies by twice the block scale, which is the same product.  What that buys: the boundary
// between two neighbouring entries, the binary64 mean rounded once to binary32, equals the binary32 sum of their
// halves (one rounding of the same real number; the host checks it entry by entry), so a pass that needs the
// boundary only to choose between the two values forms it with one addition instead of reading it.  LDS serves
// 128 bytes a clock to the four SIMDs of a compute unit: with 12 bytes per weight and codebook the element passes
// were bound by that, with 8 they are bound by the vector ALUs.  In a bin without a boundary both values are the
// same entry, so the choice does not matter there; passes that form codes or look for scaled weights exactly on a
// boundary (THR) read the stored boundary, which is +infinity in such bins.
typedef __attribute__((address_space(3))) const float lds_cfloat;
typedef __attribute__((address_space(3))) const int lds_cint;
struct Rec { float thr, ylo, yhi; int clo; };
template <bool THR, bool CODES>
__device__ __forceinline__ Rec read_rec(uint32_t addr, int a)
{
    lds_cfloat* rp = (lds_cfloat*)(size_t)addr;
    Rec r;
    if (THR) r.thr = rp[a];
    r.ylo = rp[SOP_K_MAXA + a]; r.yhi = rp[2 * SOP_K_MAXA + a];
    if (!THR) r.thr = r.ylo + r.yhi;
    r.clo = CODES ? ((lds_cint*)(size_t)addr)[3 * SOP_K_MAXA + a] : 0;
    return r;
}

template <int EPL, bool CODES>
__device__ __forceinline__ void put_code(uint32_t (&codes)[EPL / 4], int i, uint32_t code, bool wide_codes)
{
    if (CODES) {
        if (wide_codes) codes[i / 4] |= code << (8 * (i % 4));
        else codes[i / 8] |= code << (4 * (i % 8));
    }
}

// Element pass, RESIDUAL form (metrics WSE and MSE): the cosine inputs come from the residual sums
//   <w,w^> = ||w||^2 - <w,d>,   ||w^||^2 = ||w||^2 - 2<w,d> + ||d||^2      (all c-weighted),
// which shares c*d with the error sum.  The form cancels when the reconstruction is much smaller
// than the block (saturated or vanished scale); the caller checks that and falls back to
// direct_cosine_sums() for the wavefront.
// TIES: `tie` collects, as a lane mask, the lanes that hold a scaled weight exactly on a code boundary (the one place
// where a codebook under the negative scale sign and its sign-negated copy under the positive sign part ways).  The
// comparison writes a scalar lane mask and the masks are joined on the scalar unit: one vector instruction per
// element.  (-0 and +0 compare equal, so a boundary at zero is seen from either side.)
template <int EPL, int METRIC, bool CODES, bool TIES = false, class SRC>
__device__ __forceinline__ Sums eval_residual(const float (&w)[EPL], const float (&cb)[EPL], const SRC& src, float ss, int a,
                                              bool wide_codes, uint32_t (&codes)[EPL / 4], unsigned long long* tie = nullptr)
{
    float e0 = 0.0f, e1 = 0.0f, wd = 0.0f, ew = 0.0f;
    if (CODES) {
#pragma unroll
        for (int j = 0; j < EPL / 4; ++j) codes[j] = 0;
    }
#pragma unroll
    for (int i0 = 0; i0 < EPL; i0 += 4) {
        Rec r[4];
        float xe[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t bo;
            src.get(i0 + j, xe[j], bo);
            r[j] = read_rec<CODES || TIES, CODES>(bo, a);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = i0 + j;
            const bool up = xe[j] > r[j].thr;
            if constexpr (TIES) *tie |= __builtin_amdgcn_ballot_w64(xe[j] == r[j].thr);
            const float yv = up ? r[j].yhi : r[j].ylo;
            const float d = __fmaf_rn(-ss, yv, w[i]);
            const float cd = cb[i] * d;
            const float dd = METRIC == 2 ? d : cd;
            if (i < 8) e0 = __fmaf_rn(dd, d, e0); else e1 = __fmaf_rn(dd, d, e1);
            wd = __fmaf_rn(cd, w[i], wd);
            if (METRIC == 2) ew = __fmaf_rn(cd, d, ew);
            put_code<EPL, CODES>(codes, i, (uint32_t)r[j].clo + (up ? 1u : 0u), wide_codes);
        }
    }
    Sums s;
    s.err = EPL == 16 ? e0 + e1 : e0;
    s.wd = wd;
    s.ew = ew;
    return s;
}

// Element pass, DIRECT form with the decision sums of metric COS:
//   w^ = fl(ss*y), num = sum fma(fl(c*w), w^), den = sum fma(fl(c*w^), w^), chunks of 8 and the tree;
// err is formed as well when WANT_ERR (the blk_err output).
template <int EPL, bool CODES, bool WANT_ERR, bool TIES = false, class SRC>
__device__ __forceinline__ Sums eval_direct(const float (&w)[EPL], const float (&cb)[EPL], const SRC& src, float ss, int a,
                                            bool wide_codes, uint32_t (&codes)[EPL / 4], unsigned long long* tie = nullptr)
{
    float e0 = 0.0f, e1 = 0.0f, n0 = 0.0f, n1 = 0.0f, d0 = 0.0f, d1 = 0.0f;
    if (CODES) {
#pragma unroll
        for (int j = 0; j < EPL / 4; ++j) codes[j] = 0;
    }
#pragma unroll
    for (int i0 = 0; i0 < EPL; i0 += 4) {
        Rec r[4];
        float xe[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t bo;
            src.get(i0 + j, xe[j], bo);
            r[j] = read_rec<CODES || TIES, CODES>(bo, a);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = i0 + j;
            const bool up = xe[j] > r[j].thr;
            if constexpr (TIES) *tie |= __builtin_amdgcn_ballot_w64(xe[j] == r[j].thr);
            const float yv = up ? r[j].yhi : r[j].ylo;
            const float what = ss * yv;
            const float cw = cb[i] * w[i];
            const float cwh = cb[i] * what;
            if (i < 8) { n0 = __fmaf_rn(cw, what, n0); d0 = __fmaf_rn(cwh, what, d0); }
            else       { n1 = __fmaf_rn(cw, what, n1); d1 = __fmaf_rn(cwh, what, d1); }
            if (WANT_ERR) {
                const float d = __fmaf_rn(-ss, yv, w[i]);
                const float cd = cb[i] * d;
                if (i < 8) e0 = __fmaf_rn(cd, d, e0); else e1 = __fmaf_rn(cd, d, e1);
            }
            put_code<EPL, CODES>(codes, i, (uint32_t)r[j].clo + (up ? 1u : 0u), wide_codes);
        }
    }
    Sums s;
    s.err = EPL == 16 ? e0 + e1 : e0;
    s.wd = EPL == 16 ? n0 + n1 : n0;
    s.ew = EPL == 16 ? d0 + d1 : d0;
    return s;
}

// Cosine inputs straight from the codebook values in the scaled domain, where the block scale
// cancels: cos = sign(s) <w,y>_c / sqrt(||w||_c^2 ||y||_c^2).  Used when the residual form would cancel.
// (y is read as the table holds it, halved: the ratio does not change.)
template <int EPL, int LPB, bool THR, class SRC>
__device__ __forceinline__ void direct_cosine_sums(const float (&cb)[EPL], const float (&w)[EPL], const SRC& src, bool nonzero, bool negative,
                                                   int a, float& ny_out, float& dy_out)
{
    float ny = 0.0f, dy = 0.0f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        float xe;
        uint32_t bo;
        src.get(i, xe, bo);
        const Rec r = read_rec<THR, false>(bo, a);
        const float yv = xe > r.thr ? r.yhi : r.ylo;
        ny = __fmaf_rn(cb[i] * w[i], yv, ny);
        dy = __fmaf_rn(cb[i], yv * yv, dy);
    }
    const float nsum = group_sum<LPB>(negative ? -ny : ny), dsum = group_sum<LPB>(dy);
    ny_out = nonzero ? nsum : 0.0f;                    // a zero scale reconstructs nothing
    dy_out = nonzero ? dsum : 0.0f;
}

// Candidate after the cross-lane tree
struct Cand {
    float err;    // decision score of WSE / MSE; the weighted error in COS mode when wanted
    float ny;     // cosine numerator   (cos = ny / sqrt(||w||^2 dy))
    float dy;     // cosine denominator part
    bool weak;    // residual form not trustworthy for this block
};

// The cosine is a ratio of sums that all scale with the square of the block's magnitude; formed of the raw
// sums, the product ||w||^2 ||w^||^2 would leave binary32's range for blocks of very small or very large
// weights.  The value path therefore works on sums multiplied by a power of two, sc = 2^-e with
// ||w||_c^2 = m 2^e (exact, and the same bits as before wherever nothing over- or underflowed):
// wns = sc ||w||^2 lies in [1, 2), and the residual form yields sc <w,w^> and sc ||w^||^2 directly.
struct NormScale { float wns, qwns, sc, sc2; };      // sc ||w||^2, a quarter of it, sc, 2 sc

template <int LPB, int METRIC>
__device__ __forceinline__ Cand finish_residual(const Sums& s, const NormScale& n)
{
    Cand c;
    c.err = group_sum<LPB>(s.err);
    const float wd = group_sum<LPB>(s.wd);
    const float errw = METRIC == 2 ? group_sum<LPB>(s.ew) : c.err;
    c.ny = __fmaf_rn(-wd, n.sc, n.wns);
    c.dy = __fmaf_rn(errw, n.sc, __fmaf_rn(-n.sc2, wd, n.wns));
    c.weak = !(c.dy >= n.qwns);
    return c;
}

template <int LPB>
__device__ __forceinline__ Cand finish_direct(const Sums& s)
{
    Cand c;
    c.err = group_sum<LPB>(s.err);
    c.ny = group_sum<LPB>(s.wd);
    c.dy = group_sum<LPB>(s.ew);
    c.weak = false;
    return c;
}

// first / second atom of the pair with lexicographic position pi among all pairs of SOP_K_MAXA atoms
struct PairTab { int first[SOP_K_MAXP], second[SOP_K_MAXP]; };
constexpr PairTab make_pair_tab()
{
    PairTab t{};
    int pi = 0;
    for (int i = 0; i < SOP_K_MAXA; ++i)
        for (int j = i + 1; j < SOP_K_MAXA; ++j) { t.first[pi] = i; t.second[pi] = j; ++pi; }
    return t;
}
constexpr PairTab kPairTab = make_pair_tab();
template <int PI> struct PairOf { static constexpr int i = kPairTab.first[PI], j = kPairTab.second[PI]; };

// Selector of pair PI and of all following pairs (i < j in internal order): bit `slot` of the
// block's selector word, and the chosen atom's deficit into the pair's running sum.
template <int PI, int NA, int METRIC>
__device__ __forceinline__ void all_pairs(const KParams& p, const Switches& sw, const float (&score)[SOP_K_MAXA],
                                          const float (&den)[SOP_K_MAXA], const int (&dlt)[SOP_K_MAXA],
                                          int (&accp)[SOP_K_MAXP], uint32_t& bits)
{
    constexpr int i = PairOf<PI>::i, j = PairOf<PI>::j;
    static_assert(pair_index(i, j) == PI, "pair enumeration");
    if constexpr (j < NA) {
        if (__builtin_expect((sw.pair_mask >> PI) & 1u, 1)) {
            // caller's pair (a,b): selector = "b strictly better than a" (ties keep a).  The internal
            // order may have swapped the two (b is internal i): then internal j keeps the block on a tie.
            const float si = score[i], sj = score[j], ni = den[i], nj = den[j];
            const int di = dlt[i], dj = dlt[j];
            const bool flip = (sw.flip_mask >> PI) & 1u;
            // both comparisons are formed as lane masks; the wave-uniform flag picks one of them in
            // scalar registers (no branch, no per-lane select of booleans)
            const float lhs = METRIC == 1 ? sj * ni : sj, rhs = METRIC == 1 ? si * nj : si;
            const unsigned long long lt = __builtin_amdgcn_ballot_w64(METRIC == 1 ? lhs > rhs : lhs < rhs);
            const unsigned long long le = __builtin_amdgcn_ballot_w64(METRIC == 1 ? lhs >= rhs : lhs <= rhs);
            const bool pick_j = __builtin_amdgcn_inverse_ballot_w64(flip ? le : lt);
            const int chosen = pick_j ? dj : di;
            accp[PI] += chosen;
            // bit = "internal j taken"; for swapped pairs the caller's selector is its complement, put
            // right by one xor with the mask of swapped pairs after the last pair
            const int slot = (p.pair_slot_w[PI / 4] >> (8 * (PI % 4))) & 0xFF;
            bits |= (pick_j ? 1u : 0u) << slot;
        }
    }
    if constexpr (PI + 1 < SOP_K_MAXP) all_pairs<PI + 1, NA, METRIC>(p, sw, score, den, dlt, accp, bits);
}

// The weights one lane reads per step, as they come from memory
template <bool BF16, int EPL> struct RawBlk { uint4 v[BF16 ? EPL / 8 : EPL / 4]; };

template <bool BF16, int EPL>
__device__ __forceinline__ RawBlk<BF16, EPL> load_raw(const void* W, long long ldw, long long K, long long strip, long long m, int lane)
{
    RawBlk<BF16, EPL> r;
    const long long col0 = (strip * 64 + lane) * EPL;
    const bool valid = col0 < K;
    constexpr int NV = BF16 ? EPL / 8 : EPL / 4;
    const char* src = reinterpret_cast<const char*>(W) + (m * ldw + col0) * (BF16 ? 2 : 4);
#pragma unroll
    for (int i = 0; i < NV; ++i) r.v[i] = valid ? reinterpret_cast<const uint4*>(src)[i] : make_uint4(0, 0, 0, 0);
    return r;
}
template <bool BF16, int EPL>
__device__ __forceinline__ RawBlk<BF16, EPL> load_raw(const KParams& p, long long strip, long long m, int lane)
{
    return load_raw<BF16, EPL>(p.W, p.ldw, p.K, strip, m, lane);
}

template <bool BF16, int EPL>
__device__ __forceinline__ void widen(const RawBlk<BF16, EPL>& r, float (&w)[EPL])
{
    if (BF16) {
#pragma unroll
        for (int i = 0; i < EPL / 8; ++i) {
            const uint32_t v[4] = {r.v[i].x, r.v[i].y, r.v[i].z, r.v[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                w[8 * i + 2 * j] = __uint_as_float(v[j] << 16);
                w[8 * i + 2 * j + 1] = __uint_as_float(v[j] & 0xFFFF0000u);
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < EPL / 4; ++i) {
            w[4 * i] = __uint_as_float(r.v[i].x); w[4 * i + 1] = __uint_as_float(r.v[i].y);
            w[4 * i + 2] = __uint_as_float(r.v[i].z); w[4 * i + 3] = __uint_as_float(r.v[i].w);
        }
    }
}

// NA: atoms the kernel is unrolled for (2, 6 or 8).  OCC: wavefronts per SIMD the register budget is set
// for; a workgroup is 4*OCC wavefronts and fills one compute unit on its own (one copy of the tables in
// LDS per compute unit, one ticket per compute unit in the layer reduction).
// MULTI: one launch works through a list of layers (model-wide call).  The workgroups stay, the tables are
// loaded once, and every share's steps of all the layers form one sequence with one counter: a wavefront
// passes from a layer to the next without waiting for anyone, adding what it holds to the finished layer's
// sums in LDS on the way (one set of sums per layer of the launch); tickets and the conversion to ACos happen
// once, at the end of the launch, for all its layers.
// SIGNMODE 0: the scale is positive; 1: both signs of the scale are tried and the better one kept
// (signed scale word, absmax rule); 2: argmax rule, the rule fixes the sign.
template <bool BF16, int EPL, int LPB, int SIGNMODE, int METRIC, bool EMIT, int NA, int OCC, bool MULTI>
__global__ __launch_bounds__(256 * OCC, 1) void search_kernel(const KParams p)
{
    static_assert(!MULTI || !EMIT, "the model-wide kernel searches only");
    constexpr bool SIGNED = SIGNMODE == 1, ARGMAX = SIGNMODE == 2;
    constexpr int NT = 256 * OCC, NW = 4 * OCC;                                   // threads, wavefronts of the workgroup
    extern __shared__ __align__(16) char s_mem[];
    // LDS: bin table | (scale, reciprocal) table | group parameters | reduction scratch
    char* s_bins = s_mem;                                                         // [n_bins] records of 33 words
    const size_t bins_bytes = ((size_t)p.n_bins * SOP_K_BIN_BYTES + 15) & ~(size_t)15;
    float2* s_tab = reinterpret_cast<float2*>(s_mem + bins_bytes);
    float4* s_gpar = reinterpret_cast<float4*>(s_mem + bins_bytes + (((size_t)p.n_tab_codes * sizeof(float2) + 15) & ~(size_t)15));
    // reduction scratch: flag word, the final gather's totals, the workgroup's own totals (64-bit integers)
    unsigned long long* s_red = reinterpret_cast<unsigned long long*>(s_gpar + 2 * SOP_K_MAXA);
    unsigned long long* s_acc = s_red + 1 + SOP_K_NCOL;                           // [SOP_K_NCOL] this workgroup's sums (MULTI: per layer)
    const int n_acc = MULTI ? p.n_layers * SOP_K_NCOL : SOP_K_NCOL;
    __shared__ unsigned int s_next[4];                                            // next step of each SIMD's share
    {
        // 16 bytes per lane and four loads in flight before the first LDS write: a loop of one load, wait,
        // one write would spend a round trip to L2 per word and cost more than ten microseconds per launch
        // (the table has a multiple of four bins, so its size is a multiple of 16 bytes)
        const int n16 = p.n_bins * (SOP_K_BIN_BYTES / 4) / 4;
        const uint4* src = reinterpret_cast<const uint4*>(p.bins);
        uint4* dst = reinterpret_cast<uint4*>(s_bins);
        for (int i0 = threadIdx.x; i0 < n16; i0 += 4 * NT) {
            uint4 t[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] = i0 + j * NT < n16 ? src[i0 + j * NT] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i0 + j * NT < n16) dst[i0 + j * NT] = t[j];
        }
        {
            float2 t[3];                                // at most 2048 codes: three per thread are enough for 768 threads or more
            const int nt = p.n_tab_codes;
            for (int i0 = threadIdx.x; i0 < nt; i0 += 3 * NT) {
#pragma unroll
                for (int j = 0; j < 3; ++j) t[j] = i0 + j * NT < nt ? p.stab[i0 + j * NT] : make_float2(0.f, 0.f);
#pragma unroll
                for (int j = 0; j < 3; ++j)
                    if (i0 + j * NT < nt) s_tab[i0 + j * NT] = t[j];
            }
        }
        if (threadIdx.x < 4) s_next[threadIdx.x] = 0u;
        for (int i = threadIdx.x; i < n_acc; i += NT) s_acc[i] = 0ull;
        // (static indices: a lane-dependent index into the kernel arguments would copy them to scratch memory)
#pragma unroll
        for (int a = 0; a < SOP_K_MAXA; ++a)
            if ((int)threadIdx.x == a) {
                s_gpar[2 * a] = make_float4(p.tpos[a], p.tneg[a], p.bin_sc[a], p.bin_off[a]);
                s_gpar[2 * a + 1] = make_float4(p.bin_lo[a], p.bin_hi[a], 0.0f, 0.0f);
            }
    }
    __syncthreads();
    const uint32_t lds_neg = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)s_bins + SOP_K_BIN_NEGC;

    const int lane = threadIdx.x & 63;
    // the wavefront's number is the same in all its lanes: saying so keeps the row loop's counters
    // and tests in scalar registers
    const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // The workgroup's range of steps is cut into four equal shares, one per SIMD.  The hardware deals the
    // wavefronts of a workgroup out to the four SIMDs in turn, so wavefronts w, w+4, w+8, ... share a SIMD
    // (as measured on this GPU) and work on share w mod 4; were they dealt out
    // otherwise, only the balance would suffer: every share has wavefronts of its own.  The wavefronts of
    // a share take its steps one at a time from a counter in LDS: the hardware favours the oldest
    // wavefront of a SIMD, and with fixed parts the younger ones would run on alone, at a fraction of the
    // SIMD's rate, for a fifth of the kernel.  Which wavefront takes which step does not change any
    // result: all sums are integers.
    const int simd = wv & 3;
    // the share's range of steps in a layer of total_units steps
    auto share_of = [&](long long total_units, unsigned int& first, unsigned int& count) {
        const long long g0 = total_units * blockIdx.x / gridDim.x, g1 = total_units * (blockIdx.x + 1) / gridDim.x;
        first = (unsigned int)(g0 + (g1 - g0) * simd / 4);
        count = (unsigned int)(g0 + (g1 - g0) * (simd + 1) / 4) - first;
    };
    // Request side (the row loads run one step ahead of the arithmetic): the layer the next requested step
    // lies in.  One layer: sb, cnt are the share's range.  MULTI: the shares of all layers follow one another
    // in one sequence of step numbers; rq_base is the number of the first step of layer rq_l in it.
    unsigned int sb, cnt;
    int rq_l = 0;
    unsigned int rq_base = 0u, rq_M32 = 0u, rq_magic = 0u;
    const void* rq_W = nullptr;
    long long rq_ldw = 0, rq_K = 0;
    // (everything here is the same in all lanes; saying so keeps it in scalar registers: the range's
    // divisions run on the vector unit, in 32 bits: T*b/G = (T/G)*b + (T%G)*b/G with G, b below 2^16)
    auto uni = [](unsigned int x) { return (unsigned int)__builtin_amdgcn_readfirstlane((int)x); };
    auto uni64 = [&](unsigned long long x) { return ((unsigned long long)uni((unsigned int)(x >> 32)) << 32) | uni((unsigned int)x); };
    auto rq_enter = [&](int l) {
        const LayerDesc& d = p.layers[l];
        const unsigned int T = uni(d.total_units), G = gridDim.x, b = blockIdx.x;
        const unsigned int tq = T / G, tr = T - tq * G;
        const unsigned int g0 = tq * b + tr * b / G, g1 = tq * (b + 1u) + tr * (b + 1u) / G;
        const unsigned int first = g0 + (g1 - g0) * (unsigned int)simd / 4u;
        sb = uni(first);
        cnt = uni(g0 + (g1 - g0) * (unsigned int)(simd + 1) / 4u - first);
        rq_W = reinterpret_cast<const void*>(uni64((unsigned long long)reinterpret_cast<uintptr_t>(d.W)));
        rq_ldw = (long long)uni64((unsigned long long)d.ldw);
        rq_K = (long long)uni((unsigned int)d.K);
        rq_M32 = uni(d.M32); rq_magic = uni(d.m_magic);
    };
    if constexpr (MULTI) rq_enter(0);
    else share_of(p.total_units, sb, cnt);          // (the layer's own values are read from the kernel arguments where used)
    // is step v of the sequence there?  (MULTI: moves the request side on to its layer; v never decreases)
    auto seek = [&](unsigned int v) -> bool {
        if constexpr (!MULTI) return v < cnt;
        else {
            if (rq_l >= p.n_layers) return false;
            while (v - rq_base >= cnt) {
                rq_base += cnt;
                if (++rq_l >= p.n_layers) return false;
                rq_enter(rq_l);
            }
            return true;
        }
    };
    auto grab = [&]() -> unsigned int {
        unsigned int v = 0u;
        if (lane == 0) v = atomicAdd(&s_next[simd], 1u);
        return (unsigned int)__builtin_amdgcn_readfirstlane((int)v);
    };
    // step number -> (strip, row): steps run down the rows of a strip; division by multiplication with
    // floor(2^32 / M), one correction (scalar arithmetic)
    auto locate = [&](unsigned int u, long long& st, long long& row) {
        const unsigned int magic = MULTI ? rq_magic : p.m_magic, rows = MULTI ? rq_M32 : p.M32;
        unsigned int q = __umulhi(u, magic);
        unsigned int r = u - q * rows;
        if (r >= rows) { ++q; r -= rows; }
        st = q; row = r;
    };

    // running sums of 1 - cos in units of 2^-22 (integers: exact, so their order does not matter): atoms,
    // pairs, and the lanes whose block has zero norm
    int acca[SOP_K_MAXA], accp[SOP_K_MAXP], accz = 0;
#pragma unroll
    for (int i = 0; i < SOP_K_MAXA; ++i) acca[i] = 0;
#pragma unroll
    for (int i = 0; i < SOP_K_MAXP; ++i) accp[i] = 0;
    // Lane sums of a column, exact.  A row of 16 lanes is added up with data-parallel-primitive moves on the
    // vector ALU (quads, half rows, rows: every lane of the row then holds the row's sum), and the first lane
    // of each row adds its row's sum to the workgroup's 64-bit sum in LDS: four lanes to one word per column.
    // (This translation unit is compiled
    // with the compiler's atomic optimizer off: it would turn each of these adds into a loop over the
    // active lanes.)
    auto row_sum = [](int x) -> int {
        x += __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false);      // quad_perm [1,0,3,2]
        x += __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false);      // quad_perm [2,3,0,1]
        x += __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false);     // row_half_mirror
        x += __builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, false);     // row_mirror
        return x;
    };
    int cl = MULTI ? -1 : 0;                       // the layer the arithmetic is in
    // few: the lanes hold at most 15 steps (a wavefront's share of a layer of a few thousand rows: the rule at
    // a change of layer in the model-wide kernel, and at the end of a single call on such a layer).  Then a
    // lane holds at most 15 * 2^23 and a row of 16 lanes less than 2^31: one 32-bit pass per column.  In
    // general a lane holds at most 128 steps x 2^23 < 2^31: the value is split at bit 15 and both halves are
    // added over the row (below 2^19 and 2^20), then joined in 64 bits.
    auto flush = [&](int layer, bool few) {
        const int c0 = MULTI ? layer * SOP_K_NCOL : 0;
        const bool row_lead = (lane & 15) == 0;
        constexpr int NCOLS = SOP_K_MAXA + SOP_K_MAXP + 1;
        int col_of[NCOLS], val[NCOLS], n = 0;        // the live columns of this variant (compile-time list)
#pragma unroll
        for (int i = 0; i < NA; ++i) { col_of[n] = i; val[n] = acca[i]; acca[i] = 0; ++n; }
#pragma unroll
        for (int i = 0; i < SOP_K_MAXP; ++i)
            if (kPairTab.second[i] < NA) { col_of[n] = SOP_K_MAXA + i; val[n] = accp[i]; accp[i] = 0; ++n; }
        col_of[n] = SOP_K_ZCOL; val[n] = accz; accz = 0; ++n;
        // four columns at a time: their chains of moves are independent and fill each other's wait states,
        // and few values are live at once
        constexpr int B = 4;
        if (few) {
#pragma unroll
            for (int j0 = 0; j0 < NCOLS; j0 += B) {
                int rs[B];
#pragma unroll
                for (int j = 0; j < B; ++j) if (j0 + j < n) rs[j] = row_sum(val[j0 + j]);
                if (row_lead) {
#pragma unroll
                    for (int j = 0; j < B; ++j) if (j0 + j < n) atomicAdd(&s_acc[c0 + col_of[j0 + j]], (unsigned long long)(long long)rs[j]);   // (a lane's sum can be a few units below zero: sign-extended)
                }
            }
            return;
        }
#pragma unroll
        for (int j0 = 0; j0 < NCOLS; j0 += B) {
            int rl[B], rh[B];
#pragma unroll
            for (int j = 0; j < B; ++j) if (j0 + j < n) { rl[j] = row_sum(val[j0 + j] & 0x7FFF); rh[j] = row_sum(val[j0 + j] >> 15); }
            if (row_lead) {
#pragma unroll
                for (int j = 0; j < B; ++j)
                    if (j0 + j < n) atomicAdd(&s_acc[c0 + col_of[j0 + j]], (unsigned long long)(((long long)rh[j] << 15) + (long long)rl[j]));
            }
        }
    };
    // what the arithmetic needs of its layer
    const float* lc_c = nullptr;
    void* lc_sel = nullptr;
    long long lc_K = 0, lc_Bk = 0;
    unsigned int lc_Kc = 1u;

    long long strip = 0, m = 0;
    long long cur_strip = -1;
    float cb[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) cb[i] = 0.0f;
    unsigned int i_cur = grab(), i_nxt = grab();
    RawBlk<BF16, EPL> nxt;
    bool ok_cur = seek(i_cur);
    int l_nxt = rq_l;                              // layer of the row in nxt
    if (ok_cur) { locate(sb + (i_cur - rq_base), strip, m); nxt = load_raw<BF16, EPL>(MULTI ? rq_W : p.W, MULTI ? rq_ldw : p.ldw, MULTI ? rq_K : p.K, strip, m, lane); }
    int since_flush = 0;

    while (ok_cur) {
        if constexpr (MULTI) {
            if (l_nxt != cl) {
                // the arithmetic enters another layer: its channel norms are requested first, and while they
                // travel the sums the lanes hold, which belong to the layer left, join that layer's
                const int left = cl;
                cl = l_nxt;
                const LayerDesc& d = p.layers[cl];
                lc_c = reinterpret_cast<const float*>(uni64((unsigned long long)reinterpret_cast<uintptr_t>(d.c)));
                lc_sel = reinterpret_cast<void*>(uni64((unsigned long long)reinterpret_cast<uintptr_t>(d.sel_words)));
                lc_K = (long long)uni((unsigned int)d.K); lc_Bk = (long long)uni((unsigned int)d.Bk);
                lc_Kc = uni((unsigned int)d.Kc);
                cur_strip = strip;
                const long long c0 = (strip * 64 + lane) * EPL;
#pragma unroll
                for (int i = 0; i < EPL; i += 4) {
                    float4 t = c0 < lc_K ? *reinterpret_cast<const float4*>(lc_c + (unsigned int)c0 % lc_Kc + i) : make_float4(0.f, 0.f, 0.f, 0.f);
                    cb[i] = t.x; cb[i + 1] = t.y; cb[i + 2] = t.z; cb[i + 3] = t.w;
                }
                if (left >= 0) flush(left, since_flush <= 15);
                since_flush = 0;
            }
        }
        // The uniform switches below are re-read every row.  Left loop-invariant, each test would be
        // hoisted out of the loop as a 64-bit lane mask and the hundred-odd masks would spill.
        Switches sw = {p.A, p.pair_mask, p.flip_mask, p.gid_w, p.unit_tpos, p.unit_tneg, p.wide_mask, p.mirror_mask, p.selfsym_mask};
        asm volatile("" : "+s"(sw.A), "+s"(sw.pair_mask), "+s"(sw.flip_mask), "+s"(sw.gid), "+s"(sw.unit_tpos), "+s"(sw.unit_tneg), "+s"(sw.wide));
        if constexpr (SIGNED) asm volatile("" : "+s"(sw.mirror), "+s"(sw.selfsym));
        const long long cm = m, cs = strip;
        const long long col0 = (cs * 64 + lane) * EPL;
        const bool valid = col0 < (MULTI ? lc_K : p.K);
        if (cs != cur_strip) {
            cur_strip = cs;
#pragma unroll
            for (int i = 0; i < EPL; i += 4) {
                // (rows may have been folded, see KParams::Kc: the channel of a column is its index modulo the true row length)
                float4 t = valid ? *reinterpret_cast<const float4*>((MULTI ? lc_c : p.c) + (unsigned int)col0 % (MULTI ? lc_Kc : (unsigned int)p.Kc) + i) : make_float4(0.f, 0.f, 0.f, 0.f);
                cb[i] = t.x; cb[i + 1] = t.y; cb[i + 2] = t.z; cb[i + 3] = t.w;
            }
        }
        // ---- the block: one read from HBM, requested one step ahead ----
        float w[EPL];
        widen<BF16, EPL>(nxt, w);
        const bool ok_nxt = seek(i_nxt);
        l_nxt = rq_l;
        if (ok_nxt) { locate(sb + (i_nxt - rq_base), strip, m); nxt = load_raw<BF16, EPL>(MULTI ? rq_W : p.W, MULTI ? rq_ldw : p.ldw, MULTI ? rq_K : p.K, strip, m, lane); }
        // the next step opens another layer: its channel norms are asked for now (one word per lane brings
        // every cache line of the strip's norms in), so that the loads at the top of that step find them
        // near; the value is only held until the end of this step
        float c_touch = 0.0f;
        if constexpr (MULTI) {
            if (ok_nxt && l_nxt != cl) {
                const float* cn = reinterpret_cast<const float*>(uni64((unsigned long long)reinterpret_cast<uintptr_t>(p.layers[l_nxt].c)));
                const long long tc = (strip * 64 + lane) * EPL;
                if (tc < rq_K) c_touch = cn[(unsigned int)tc % uni((unsigned int)p.layers[l_nxt].Kc)];
            }
        }
        const unsigned int i_nn = grab();              // the step after the next one; used at the end of this step

        // ---- block statistics ----
        float pmax = 0.0f, nmin = 0.0f, wn0 = 0.0f, wn1 = 0.0f;
#pragma unroll
        for (int i = 0; i < EPL; i += 2) {
            pmax = fmaxf(fmaxf(pmax, w[i]), w[i + 1]);
            nmin = fminf(fminf(nmin, w[i]), w[i + 1]);
        }
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const float cw = cb[i] * w[i];
            if (i < 8) wn0 = __fmaf_rn(cw, w[i], wn0); else wn1 = __fmaf_rn(cw, w[i], wn1);
        }
        pmax = group_max<LPB>(pmax);
        float nmax = group_max<LPB>(-nmin);
        // Lanes past the end of a row hold zero weights.  Their scale would be zero, which sends the whole
        // wavefront through the scale word's subnormal branch on every row of the last strip; a unit
        // maximum keeps them on the common path.  Nothing of theirs is written, and with zero weights they
        // still add exactly 1 to every sum and to the count column, as a zero block does.
        pmax = valid ? pmax : 1.0f;
        nmax = valid ? nmax : 1.0f;
        const float wn = group_sum<LPB>(EPL == 16 ? wn0 + wn1 : wn0);
        accz += wn > 0.0f ? 0 : (1 << 22);
        // power of two that brings ||w||^2 into [1, 2) (exponent fields 1 .. 253: norms within 2^-126 .. 2^126)
        NormScale nsc;
        {
            const uint32_t eb = min(max(__float_as_uint(wn) >> 23, 1u), 253u);
            nsc.sc = __uint_as_float((254u - eb) << 23);
            nsc.sc2 = nsc.sc + nsc.sc;
            nsc.wns = wn * nsc.sc;
            nsc.qwns = 0.25f * nsc.wns;
        }

        const long long blk_in_row = (cs * 64 + lane) / LPB;
        const long long blk = cm * (MULTI ? lc_Bk : p.Bk) + blk_in_row;
        const bool leader = valid && (lane % LPB == 0);

        // per-block results of every atom that the pair stage needs: score = err (WSE / MSE) or
        // q = num*|num| (COS, 0 for a zero reconstruction), den (COS only, 1 for a zero reconstruction), 1 - cos
        float score[SOP_K_MAXA], den[SOP_K_MAXA];
        int dlt[SOP_K_MAXA];
        // state of the current scale group: scale code, scale, scaled weights and the addresses of their bin records.
        // A signed scale word keeps the scale of both signs instead and forms scaled weights and addresses inside the
        // element pass (FlySrc): the arrays of two signs would cost 64 registers and with them a wavefront per SIMD.
        int gq = 0;
        float gss = 0.0f;                              // twice the scale (the table holds halved codebook values)
        bool gnz = false, gneg = false;
        constexpr bool FLY = SIGNED && EPL == 16;       // (a lane of 8 elements has the registers for both signs' arrays)
        float gx[FLY ? 1 : EPL], gx2[(SIGNED && !FLY) ? EPL : 1];
        uint32_t gboff[FLY ? 1 : EPL], gboff2[(SIGNED && !FLY) ? EPL : 1];
        ScalePrep spP = {0, 0.0f, 0.0f, false, false}, spM = {0, 0.0f, 0.0f, false, false};
        int cur_gid = -1;                              // scale group the state above belongs to (wave-uniform)
        // Signed scale word: the two candidates of the atom before (0: positive scale sign, 1: negative), kept for an
        // atom that is its sign-negated copy.  Codebook -a under the positive sign reconstructs what a does under the
        // negative sign, and the other way round (same scale code, same residuals bit for bit, codes k <-> N-1-k),
        // unless a scaled weight lies exactly on a code boundary: there the two resolve the tie differently.  So
        // the copy takes over the kept candidates with their roles exchanged (the wave-uniform flag f0neg: candidate
        // 0 is the negative sign), unless some lane of the wavefront saw such a tie, in which case the copy is
        // evaluated like any other atom.
        // (plain scalars: copying candidate structs would drag their padding bytes through scratch memory)
        float pv_err0 = 0.0f, pv_ny0 = 0.0f, pv_dy0 = 0.0f, pv_err1 = 0.0f, pv_ny1 = 0.0f, pv_dy1 = 0.0f;
        float pv_rn0 = 0.0f, pv_rd0 = 0.0f, pv_rn1 = 0.0f, pv_rd1 = 0.0f;   // sums of the ranking score (emit mode)
        int pv_q0 = 0, pv_q1 = 0;
        uint32_t pv_codes0[EPL / 4], pv_codes1[EPL / 4];
        bool pv_f0neg = false;                         // wave-uniform: the kept candidate 0 is the negative sign (it was kept by a copy)
        bool pv_tie = true;                            // wave-uniform: the kept candidates may not be taken over
        bool pv_raw0 = false, pv_raw1 = false;         // wave-uniform: the kept cosine sums are the direct ones (not scaled)

#pragma unroll
        for (int a = 0; a < NA; ++a) {
            score[a] = 0.0f; den[a] = 1.0f; dlt[a] = 0;
            if (__builtin_expect(a < sw.A, 1)) {
                bool derived = false;
                if constexpr (SIGNED) derived = ((sw.mirror >> a) & 1u) && !pv_tie;
                const int gid = (int)((sw.gid >> (4 * a)) & 15u);
                if (!derived && gid != cur_gid) {
                    cur_gid = gid;
                    if constexpr (FLY) {
                        spP = prepare_scale(pmax, nmax, false, a, p, sw, s_tab, s_gpar);
                        spM = prepare_scale(pmax, nmax, true, a, p, sw, s_tab, s_gpar);
                    } else if constexpr (SIGNED) {
                        bool unused;
                        prepare_sign<EPL, false>(w, pmax, nmax, false, a, p, sw, s_tab, s_gpar, lds_neg, spP.q, spP.ss, spP.nonzero, gx, gboff, unused);
                        prepare_sign<EPL, false>(w, pmax, nmax, true, a, p, sw, s_tab, s_gpar, lds_neg, spM.q, spM.ss, spM.nonzero, gx2, gboff2, unused);
                    } else {
                        prepare_sign<EPL, ARGMAX>(w, pmax, nmax, false, a, p, sw, s_tab, s_gpar, lds_neg, gq, gss, gnz, gx, gboff, gneg);
                    }
                }
                const bool wide = EMIT && ((sw.wide >> a) & 1u);
                uint32_t codes[EPL / 4];
                Cand best;
                int q = gq;
                bool neg = ARGMAX ? gneg : false;
                bool raw = false;                      // best.ny, best.dy are raw sums (else multiplied by nsc.sc); per lane for signed words
                float rk_num = 0.0f, rk_dn = 0.0f;     // sums of the ranking score of the chosen sign (signed words, emit mode)
                if constexpr (SIGNED) {
                    // ---- both signs of the scale: candidate 0 (the positive sign; the negative one when f0neg) and candidate 1 ----
                    float err0, ny0, dy0, err1, ny1, dy1, rn0 = 0.0f, rd0 = 0.0f, rn1 = 0.0f, rd1 = 0.0f;
                    int q0, q1;
                    bool raw0, raw1, f0neg;
                    uint32_t codes0[EPL / 4], codes1[EPL / 4];
                    // codes of the mirrored codebook: N-1-k in every field (no borrows: every field holds at most N-1)
                    const uint32_t cmask = (uint32_t)(p.nent[a] - 1) * (wide ? 0x01010101u : 0x11111111u);
                    if (derived) {
                        err0 = pv_err0; ny0 = pv_ny0; dy0 = pv_dy0; err1 = pv_err1; ny1 = pv_ny1; dy1 = pv_dy1;
                        rn0 = pv_rn0; rd0 = pv_rd0; rn1 = pv_rn1; rd1 = pv_rd1;
                        q0 = pv_q0; q1 = pv_q1; raw0 = pv_raw0; raw1 = pv_raw1;
                        f0neg = !pv_f0neg;                 // what was the original's negative sign is the copy's positive one
                        if (EMIT) {
#pragma unroll
                            for (int j = 0; j < EPL / 4; ++j) { codes0[j] = cmask - pv_codes0[j]; codes1[j] = cmask - pv_codes1[j]; }
                        }
                    } else {
                        unsigned long long tie = 0ull;          // lanes that saw a scaled weight exactly on a code boundary
                        f0neg = false;
                        // one sign of the scale: the atom's element pass with scaled weights formed on the spot
                        const float4 gpar = s_gpar[2 * a];             // (t+, -t-, bin scale, bin offset): same address in every lane
                        auto eval_sign = [&](const ScalePrep& sp, const bool sgn, const auto& xarr, const auto& barr,
                                             float& err, float& ny, float& dy, int& qq, bool& rawf,
                                             uint32_t (&cds)[EPL / 4], float& rn, float& rd) {
                            qq = sp.q;
                            auto run = [&](const auto& src) {
                                Cand t;
                                if constexpr (METRIC == 1) t = finish_direct<LPB>(eval_direct<EPL, EMIT, EMIT, true>(w, cb, src, sp.ss, a, wide, cds, &tie));
                                else t = finish_residual<LPB, METRIC>(eval_residual<EPL, METRIC, EMIT, true>(w, cb, src, sp.ss, a, wide, cds, &tie), nsc);
                                err = t.err; ny = t.ny; dy = t.dy;
                                rawf = METRIC == 1;
                                if constexpr (METRIC != 1) {
                                    // the residual form is accurate while the reconstruction carries a fair share of the block's
                                    // norm; otherwise the whole wavefront recomputes this candidate's cosine sums directly
                                    if (__builtin_expect(__any(t.weak) != 0, 0)) {
                                        direct_cosine_sums<EPL, LPB, true>(cb, w, src, sp.nonzero, sgn, a, ny, dy);
                                        rawf = true;
                                    }
                                }
                                if constexpr (EMIT) {
                                    if (p.blk_rank) {
                                        if constexpr (METRIC == 1) { rn = t.ny; rd = t.dy; }
                                        else {
                                            uint32_t nocodes[EPL / 4];
                                            const Cand c1 = finish_direct<LPB>(eval_direct<EPL, false, false>(w, cb, src, sp.ss, a, false, nocodes));
                                            rn = c1.ny; rd = c1.dy;
                                        }
                                    }
                                }
                            };
                            // the table covers a scale rounded down by up to the factor SOP_K_BIN_SAFE; beyond it (the scale word
                            // saturated) the whole wavefront clamps its scaled weights into the table's range
                            if constexpr (!FLY) {
                                run(ArrSrc<EPL>{xarr, barr});
                            } else if (__builtin_expect(__any(sp.beyond) != 0, 0)) {
                                const float4 g2 = s_gpar[2 * a + 1];       // (table range low, high, -, -)
                                run(FlySrc<EPL, true>{w, sp.rr, gpar.z, gpar.w, g2.x, g2.y, lds_neg});
                            } else {
                                run(FlySrc<EPL, false>{w, sp.rr, gpar.z, gpar.w, 0.0f, 0.0f, lds_neg});
                            }
                        };
                        eval_sign(spP, false, gx, gboff, err0, ny0, dy0, q0, raw0, codes0, rn0, rd0);
                        // a codebook that is its own sign-negated copy reconstructs the same under both signs (away
                        // from ties), and an equal candidate never replaces the positive sign
                        if (((sw.selfsym >> a) & 1u) && (tie & __builtin_amdgcn_ballot_w64(valid)) == 0ull) {
                            err1 = err0; ny1 = ny0; dy1 = dy0; q1 = spM.q; raw1 = raw0; rn1 = rn0; rd1 = rd0;
                            if (EMIT) {
#pragma unroll
                                for (int j = 0; j < EPL / 4; ++j) codes1[j] = cmask - codes0[j];
                            }
                        } else {
                            eval_sign(spM, true, gx2, gboff2, err1, ny1, dy1, q1, raw1, codes1, rn1, rd1);
                        }
                        pv_tie = (tie & __builtin_amdgcn_ballot_w64(valid)) != 0ull;
                    }
                    pv_err0 = err0; pv_ny0 = ny0; pv_dy0 = dy0; pv_err1 = err1; pv_ny1 = ny1; pv_dy1 = dy1;
                    pv_q0 = q0; pv_q1 = q1; pv_raw0 = raw0; pv_raw1 = raw1; pv_f0neg = f0neg;
                    if (EMIT) {
                        pv_rn0 = rn0; pv_rd0 = rd0; pv_rn1 = rn1; pv_rd1 = rd1;
#pragma unroll
                        for (int j = 0; j < EPL / 4; ++j) { pv_codes0[j] = codes0[j]; pv_codes1[j] = codes1[j]; }
                    }
                    // the negative sign only when strictly better: candidate 1 is taken when it is strictly better, or, if it
                    // is the positive sign (f0neg), when it is at least as good.  Both comparisons are formed as lane masks
                    // and the wave-uniform flag picks one of them in scalar registers.
                    bool pick1;
                    if constexpr (METRIC == 1) {
                        const float bq0 = dy0 > 0.0f ? ny0 * fabsf(ny0) : 0.0f, bd0 = dy0 > 0.0f ? dy0 : 1.0f;
                        const float bq1 = dy1 > 0.0f ? ny1 * fabsf(ny1) : 0.0f, bd1 = dy1 > 0.0f ? dy1 : 1.0f;
                        const unsigned long long gt = __builtin_amdgcn_ballot_w64(bq1 * bd0 > bq0 * bd1);
                        const unsigned long long ge = __builtin_amdgcn_ballot_w64(!(bq0 * bd1 > bq1 * bd0));
                        pick1 = __builtin_amdgcn_inverse_ballot_w64(f0neg ? ge : gt);
                        score[a] = pick1 ? bq1 : bq0;
                        den[a] = pick1 ? bd1 : bd0;
                    } else {
                        const unsigned long long lt = __builtin_amdgcn_ballot_w64(err1 < err0);
                        const unsigned long long le = __builtin_amdgcn_ballot_w64(!(err0 < err1));
                        pick1 = __builtin_amdgcn_inverse_ballot_w64(f0neg ? le : lt);
                        score[a] = pick1 ? err1 : err0;
                    }
                    neg = pick1 != f0neg;
                    best.err = pick1 ? err1 : err0;
                    best.ny = pick1 ? ny1 : ny0;
                    best.dy = pick1 ? dy1 : dy0;
                    best.weak = false;
                    raw = pick1 ? raw1 : raw0;
                    q = pick1 ? q1 : q0;
                    if (EMIT) {
                        rk_num = pick1 ? rn1 : rn0; rk_dn = pick1 ? rd1 : rd0;
#pragma unroll
                        for (int j = 0; j < EPL / 4; ++j) codes[j] = pick1 ? codes1[j] : codes0[j];
                    }
                } else if constexpr (METRIC == 1) {
                    // (emit mode without a code plane, as when only the ranking scores are wanted: the pass that forms no codes)
                    if (!EMIT || p.codes) best = finish_direct<LPB>(eval_direct<EPL, EMIT, EMIT>(w, cb, ArrSrc<EPL>{gx, gboff}, gss, a, wide, codes));
                    else best = finish_direct<LPB>(eval_direct<EPL, false, EMIT>(w, cb, ArrSrc<EPL>{gx, gboff}, gss, a, wide, codes));
                    score[a] = best.dy > 0.0f ? best.ny * fabsf(best.ny) : 0.0f;
                    den[a] = best.dy > 0.0f ? best.dy : 1.0f;
                    raw = true;
                } else {
                    // (emit mode without a code plane, as when only the ranking scores are wanted: the pass that forms no codes
                    // and reads no boundaries)
                    if (!EMIT || p.codes) best = finish_residual<LPB, METRIC>(eval_residual<EPL, METRIC, EMIT>(w, cb, ArrSrc<EPL>{gx, gboff}, gss, a, wide, codes), nsc);
                    else best = finish_residual<LPB, METRIC>(eval_residual<EPL, METRIC, false>(w, cb, ArrSrc<EPL>{gx, gboff}, gss, a, wide, codes), nsc);
                    // the residual form is accurate while the reconstruction carries a fair share of
                    // the block's norm; otherwise the whole wavefront recomputes this atom directly
                    if (__builtin_expect(__any(best.weak) != 0, 0)) {
                        float ny1, dy1;
                        direct_cosine_sums<EPL, LPB, EMIT>(cb, w, ArrSrc<EPL>{gx, gboff}, gnz, ARGMAX ? gneg : false, a, ny1, dy1);
                        best.ny = ny1;
                        best.dy = dy1;
                        raw = true;
                    }
                    score[a] = best.err;
                }
                // cosine value; a vanishing reconstruction has ny = 0 and gives cos 0; a zero-norm block
                // gives exactly 1 - 0 here and is corrected through the count column
                // 3 - cos lies in [2, 4], where binary32 values are 2^-22 apart and their bit patterns count
                // those steps: the fma's own rounding (nearest, ties to even) rounds 1 - cos to the unit of
                // the integer sums, and pattern minus pattern of 2.0 is that integer (no conversion)
                // (direct sums come with the codebook's own magnitude: paired with the raw norm, as they were formed;
                // the COS metric's decision sums are raw sums of w^ and are brought to the scaled norm's units)
                const float ny_raw = best.ny, dy_raw = best.dy;
                if constexpr (METRIC == 1) { best.ny *= nsc.sc; best.dy *= nsc.sc; }
                const float rs = __frsqrt_rn(__fmaf_rn((raw && METRIC != 1) ? wn : nsc.wns, best.dy, 1.0e-37f));
                const int ia = (int)__float_as_uint(__fmaf_rn(-best.ny, rs, 3.0f)) - 0x40000000;
                dlt[a] = ia;
                acca[a] += ia;
                if (EMIT) {
                    const long long ua = p.uidx[a];
                    if (p.scale_code && leader) p.scale_code[ua * p.Nb + blk] = (uint16_t)(q | (neg ? 0x8000 : 0));
                    if (p.blk_err && leader) p.blk_err[ua * p.Nb + blk] = best.err;
                    if (p.blk_cos && leader) p.blk_cos[ua * p.Nb + blk] = wn > 0.0f ? 1.0f - __fmaf_rn(-best.ny, rs, 1.0f) : 1.0f;
                    if (p.blk_rank) {
                        // ranking score of step 2 of the per-layer search: a decision quantity, formed in binary32 from
                        // the block's tree sums num = <w,w^>_c, den = ||w^||_c^2 (chunks of 8, balanced tree) and wn:
                        // fl(fl(num / wn) * fl(|num| / den)), 1 for a block without weighted norm, 0 for a zero reconstruction
                        float num, dn;
                        if constexpr (SIGNED) { num = rk_num; dn = rk_dn; }
                        else if constexpr (METRIC == 1) { num = ny_raw; dn = dy_raw; }
                        else {
                            uint32_t nocodes[EPL / 4];
                            const Cand c1 = finish_direct<LPB>(eval_direct<EPL, false, false>(w, cb, ArrSrc<EPL>{gx, gboff}, gss, a, false, nocodes));
                            num = c1.ny; dn = c1.dy;
                        }
                        const float rank = wn > 0.0f ? (dn > 0.0f ? (num / wn) * (fabsf(num) / dn) : 0.0f) : 1.0f;
                        if (leader) p.blk_rank[ua * p.Nb + blk] = rank;
                    }
                    if (p.codes && valid) {
                        if (!wide) {
                            uint8_t* dst = p.codes + p.code_off[a] + (cm * p.K + col0) / 2;
#pragma unroll
                            for (int j = 0; j < EPL / 8; ++j) reinterpret_cast<uint32_t*>(dst)[j] = codes[j];
                        } else {
                            uint8_t* dst = p.codes + p.code_off[a] + cm * p.K + col0;
#pragma unroll
                            for (int j = 0; j < EPL / 4; ++j) reinterpret_cast<uint32_t*>(dst)[j] = codes[j];
                        }
                    }
                }
            }
        }
        // ---- selector of every requested pair: one word per block ----
        uint32_t bits = 0;
        all_pairs<0, NA, METRIC>(p, sw, score, den, dlt, accp, bits);
        bits ^= p.flip_slots;
        void* const sel_words = MULTI ? lc_sel : p.sel_words;
        if (sel_words && leader) {
            if (p.sel_u32) reinterpret_cast<uint32_t*>(sel_words)[blk] = bits;
            else reinterpret_cast<uint16_t*>(sel_words)[blk] = (uint16_t)bits;
        }
        if constexpr (MULTI) asm volatile("" :: "v"(c_touch));
        i_cur = i_nxt;
        ok_cur = ok_nxt;
        i_nxt = i_nn;
        if (++since_flush == 128) { flush(cl, false); since_flush = 0; }   // a step adds at most 2^23: a lane's sums stay below 2^31
    }

    // ---- per-workgroup sums: what the lanes still hold joins the workgroup's integer sums in LDS ----
    if (!MULTI || cl >= 0) flush(cl, since_flush <= 15);      // (since_flush: steps since the last flush)
    __syncthreads();
    if constexpr (MULTI) {
        // every layer's sums of this workgroup join the layer's replica; eight adds of a thread are in
        // flight before their returned values are consumed (see below for why they are consumed)
        for (int base = 0; base < n_acc; base += 8 * NT) {
            unsigned long long before[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int idx = base + j * NT + (int)threadIdx.x;
                before[j] = 0ull;
                if (idx < n_acc) {
                    const unsigned long long v = s_acc[idx];
                    const int layer = idx / SOP_K_NCOL, col = idx - layer * SOP_K_NCOL;
                    if (v != 0ull) before[j] = atomicAdd(p.sums + ((size_t)layer * SOP_K_REPL + blockIdx.x % SOP_K_REPL) * SOP_K_NCOL + col, v);
                }
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) asm volatile("" :: "v"(before[j]) : "memory");
        }
    } else if ((int)threadIdx.x < SOP_K_NCOL) {
        const int i = threadIdx.x;
        const unsigned long long v = s_acc[i];
        if (v != 0ull) {
            // Atomics to one address are served one after the other (about 20 ns each), so the sums
            // are kept in SOP_K_REPL replicas chosen by workgroup number.  The returned value is
            // consumed so that the add has completed at the memory side before this workgroup
            // announces itself below (all traffic here is atomic: no cache write-back, which a fence
            // would cost on every workgroup, is needed).
            const unsigned long long before = atomicAdd(p.sums + (blockIdx.x % SOP_K_REPL) * SOP_K_NCOL + i, v);
            asm volatile("" :: "v"(before) : "memory");
        }
    }
    // ---- layer reduction: every workgroup takes a ticket; the one that takes the last finishes the
    //      layer.  (One counter: the workgroups do not end at the same instant, and a second level of
    //      counters only put one more round trip to memory on the last workgroup's path.) ----
    __syncthreads();
    unsigned int* s_flag = reinterpret_cast<unsigned int*>(s_red);
    if (threadIdx.x == 0) {
        unsigned int last = 0u;
        if (atomicAdd(p.done, 1u) == gridDim.x - 1) { atomicExch(p.done, 0u); last = 1u; }
        *s_flag = last;
    }
    __syncthreads();
    if constexpr (MULTI) {
        if (*s_flag) {
            // totals of every (layer, column) over the replicas into LDS, in place of the workgroup's own sums
            // (the exchanges leave zeros for the next call), then one ACos per (layer, atom or pair)
            __syncthreads();
            for (int idx = threadIdx.x; idx < n_acc; idx += NT) {
                const int layer = idx / SOP_K_NCOL, col = idx - layer * SOP_K_NCOL;
                unsigned long long* src = p.sums + (size_t)layer * SOP_K_REPL * SOP_K_NCOL + col;
                unsigned long long part[SOP_K_REPL];
#pragma unroll
                for (int r = 0; r < SOP_K_REPL; ++r) part[r] = atomicExch(src + r * SOP_K_NCOL, 0ull);
                unsigned long long tot = 0ull;
#pragma unroll
                for (int r = 0; r < SOP_K_REPL; ++r) tot += part[r];
                s_acc[idx] = tot;
            }
            __syncthreads();
            const int per = p.A + p.P;
            for (int o = threadIdx.x; o < p.n_layers * per; o += NT) {
                const int layer = o / per, q = o - layer * per;
                int col;
                double* dst;
                const size_t row = (size_t)p.layers[layer].out_row;
                if (q < p.A) { col = q; dst = p.acos_atom ? p.acos_atom + row * p.A + p.uidx[q] : nullptr; }
                else { col = SOP_K_MAXA + p.pair_pi[q - p.A]; dst = p.acos_pair ? p.acos_pair + row * p.P + (q - p.A) : nullptr; }
                const long long z = (long long)s_acc[layer * SOP_K_NCOL + SOP_K_ZCOL];
                const long long t = (long long)s_acc[layer * SOP_K_NCOL + col];
                if (dst) *dst = 1.0 - ((double)(t - z) * (1.0 / 4194304.0)) / ((double)p.layers[layer].Nb * (double)p.lpb);
            }
        }
    } else if (*s_flag) {
        // gather the replicas (exact integer adds in LDS; the exchanges leave zeros for the next call)
        unsigned long long* s_tot = s_red + 1;
        __syncthreads();
        if ((int)threadIdx.x < SOP_K_NCOL) s_tot[threadIdx.x] = 0ull;
        __syncthreads();
        for (int idx = threadIdx.x; idx < SOP_K_REPL * SOP_K_NCOL; idx += NT) {
            const unsigned long long v = atomicExch(p.sums + idx, 0ull);
            if (v) atomicAdd(&s_tot[idx % SOP_K_NCOL], v);
        }
        __syncthreads();
        // lanes whose block had zero weighted norm (and lanes past the end of a row) added exactly 1
        // to every column; the count column takes them out again
        const long long z = (long long)s_tot[SOP_K_ZCOL];
        const int o = threadIdx.x;                 // 0..A-1 atoms (internal order), then pairs by output index
        if (o < p.A + p.P) {
            int col;
            double* dst;
            if (o < p.A) { col = o; dst = p.acos_atom ? p.acos_atom + p.uidx[o] : nullptr; }
            else { col = SOP_K_MAXA + p.pair_pi[o - p.A]; dst = p.acos_pair ? p.acos_pair + (o - p.A) : nullptr; }
            const long long t = (long long)s_tot[col];
            if (dst) *dst = 1.0 - ((double)(t - z) * (1.0 / 4194304.0)) / ((double)p.Nb * (double)p.lpb);
        }
    }
}

}  // namespace sopk

// ---- kernel table of this part ----
namespace {
// wavefronts per SIMD each variant is built for: the largest number its register need allows (a lane
// owning 8 elements needs far fewer registers than one owning 16; trying both signs, emitting codes and
// eight atoms each need more; measured on the 4096 x 11008 layer where two choices were close)
constexpr int occ_for(int epl, int sign_mode, bool emit, int na, int metric)
{
    if (na == 2) {                                   // one or two atoms: fewer registers
        if (epl == 8) return (sign_mode == 1 && emit) ? 3 : 4;
        return emit ? 2 : 3;                           // (with the per-block planes a lane of 16 elements needs more than 168 registers)
    }
    if (epl == 8) {
        if (sign_mode == 1) return emit ? 2 : 3;
        return (emit || na == 8) ? 3 : 4;
    }
    if (sign_mode == 1) return emit ? (na == 8 ? 1 : 2) : (na == 8 ? 2 : 3);
    if (emit) return 2;
    return (na == 8 || metric == 1) ? 2 : 3;        // the cosine metric keeps two more sums per candidate alive
}

// one variant: *occ = wavefronts per SIMD its registers allow (a workgroup has 4 * occ wavefronts).  mode 0: one
// layer; 2: a list of layers, which exists for the searches of more than two atoms that write no per-block
// planes; *mode_out tells which mode was given.
template <bool BF16, int EPL, int LPB, int S, bool E, int NA>
const void* variant(int mode, int* occ, int* mode_out)
{
    constexpr int MT = SOPK_PART_METRIC;
    constexpr int O = occ_for(EPL, S, E, NA, MT);
    *occ = O;
    *mode_out = 0;
    if constexpr (!E && NA != 2) {
        if (mode == 2) {
            *mode_out = 2;
            return reinterpret_cast<const void*>(&sopk::search_kernel<BF16, EPL, LPB, S, MT, E, NA, O, true>);
        }
    }
    return reinterpret_cast<const void*>(&sopk::search_kernel<BF16, EPL, LPB, S, MT, E, NA, O, false>);
}

// na_class: 0 = at most two atoms, 1 = at most six, 2 = up to eight
template <bool BF16, int EPL, int LPB>
const void* pick_geom(int sign_mode, bool emit, int na_class, int mode, int* occ, int* mode_out)
{
#define SOPK_FN(S, E, NA) variant<BF16, EPL, LPB, S, E, NA>(mode, occ, mode_out)
#define SOPK_BY_SIGN(E, NA) (sign_mode == 1 ? SOPK_FN(1, E, NA) : sign_mode == 2 ? SOPK_FN(2, E, NA) : SOPK_FN(0, E, NA))
    if (emit) return na_class == 0 ? SOPK_BY_SIGN(true, 2) : na_class == 1 ? SOPK_BY_SIGN(true, 6) : SOPK_BY_SIGN(true, 8);
    if (na_class == 0) return SOPK_BY_SIGN(false, 2);
    if (na_class == 1) return SOPK_BY_SIGN(false, 6);
    return SOPK_BY_SIGN(false, 8);
#undef SOPK_BY_SIGN
#undef SOPK_FN
}
}  // namespace

#define SOPK_CAT2(a, b, c) a##b##_##c
#define SOPK_CAT(a, b, c) SOPK_CAT2(a, b, c)

// g: block size; na_class: 0 / 1 / 2 for alphabets of at most 2 / 6 / 8 atoms; mode: 0 one layer, 2 a list of layers
// (*mode_out: the mode of the kernel returned, 0 where the one asked for does not exist).  *occ receives the
// wavefronts per SIMD the variant is built for (its workgroup has 256 * occ threads)
extern "C" const void* SOPK_CAT(sopk_part_, SOPK_PART_BF16, SOPK_PART_METRIC)(int g, int sign_mode, int emit, int na_class, int mode, int* occ, int* mode_out)
{
    constexpr bool B = SOPK_PART_BF16 != 0;
    switch (g) {
        case 8:  return pick_geom<B, 8, 1>(sign_mode, emit, na_class, mode, occ, mode_out);
        case 16: return pick_geom<B, 16, 1>(sign_mode, emit, na_class, mode, occ, mode_out);
        case 32: return pick_geom<B, 16, 2>(sign_mode, emit, na_class, mode, occ, mode_out);
        default: return pick_geom<B, 16, 4>(sign_mode, emit, na_class, mode, occ, mode_out);
    }
}
