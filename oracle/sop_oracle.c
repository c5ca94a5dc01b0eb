/*
 * CPU oracle for the per-layer pair search of "Scaled Outer Product".
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP path is checked
 * against.  It shares no code with that path and nothing in the product may call it; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg do.
 *
 * What it computes, per layer W[M,K] cut into blocks of g consecutive weights along K
 * (Section "Block Scaling": W[m,k] ~ s_W[m, floor(k/g)] * Q_W[m,k]):
 *   - absmax block scale against the codebook endpoints t+ / t-     (Section "Block Scaling",
 *     the absmax equation; "LUT-scale coupling": s = |w|max / max(LUT));
 *   - the optional per-layer power-of-two shift of all block scales  (Section "Scale Format and
 *     Metabit Allocation", paragraph on the per-layer scale shift);
 *   - rounding of the scale into a narrow SwExMy scale word          (same section, SwExMy
 *     notation);
 *   - Q = round_q(W / s): nearest codebook entry                     (Section "Block Scaling",
 *     the round_q equation);
 *   - the c-weighted inner products and the activation-weighted cosine, averaged over blocks
 *     (Section "Activation-Weighted Cosine Similarity", both equations);
 *   - the finishing reassignment: each block is evaluated under both codebooks of a pair, and
 *     under both signs of the scale when the format is signed, and the better candidate wins
 *     (Section "Per-Layer Pair Search", step 4; the metric is block error or ACos, design
 *     axis (ii)).
 *
 * Precision.  Everything that decides an integer output (scale code, element code, scale sign,
 * selector bit) is done in IEEE binary32, one rounding per written operation, with fmaf where an
 * fma is written; the file must be compiled with -ffp-contract=off.  The paper does not fix a
 * precision; binary32 is the precision the HIP path decides in.  Everything that is only a
 * value (the cosines and their layer means) is evaluated in binary64.
 *
 * Conventions where the paper is silent (each is listed in the design notes of the repository):
 *   - scale rounding: nearest representable value, ties to the lower code, saturating at
 *     max_code; subnormals of the scale format are kept; every code is a finite value;
 *   - element rounding: nearest entry, ties to the lower index; done as a count of midpoints
 *     strictly below x, midpoints formed in binary64 and rounded once to binary32;
 *   - a block sum is taken over chunks of 8 consecutive elements (sequential fma inside a
 *     chunk), chunk partials combined by a balanced binary tree in index order;
 *   - a block with zero weighted norm has cosine 1, a zero reconstruction of a non-zero block
 *     has cosine 0;
 *   - in a pair (a,b) the selector bit is 1 only when b is strictly better; the negative scale
 *     sign is taken only when strictly better.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SOPO_MAX_ENTRIES 64
#define SOPO_MAX_ATOMS 16

typedef struct {
    int sign_bits;  /* w: 0 unsigned, 1 signed                                   */
    int exp_bits;   /* x                                                          */
    int man_bits;   /* y                                                          */
    int bias;       /* exponent bias; the paper's default is 2^(x-1)-1            */
    int max_code;   /* largest magnitude code in use (<= 2^(x+y)-1)               */
} sopo_fmt;

enum { SOPO_WSE = 0, SOPO_COS = 1, SOPO_MSE = 2 };

/* ---- scale word: magnitude code q -> value (SwExMy: x exponent bits, y mantissa bits) ---- */
double sopo_scale_value(const sopo_fmt* f, int q)
{
    int y = f->man_bits;
    int e = q >> y;
    int m = q & ((1 << y) - 1);
    if (e == 0) return ldexp((double)m, 1 - f->bias - y);            /* subnormal: 0.m * 2^(1-bias) */
    return ldexp((double)((1 << y) + m), e - f->bias - y);           /* normal: 1.m * 2^(e-bias)    */
}

/* Definition of the scale rounding: scan every code, keep the nearest, ties to the lower code. */
int sopo_scale_encode_exhaustive(const sopo_fmt* f, float sp)
{
    if (!(sp < INFINITY)) return f->max_code;                        /* +inf saturates              */
    int best = 0;
    double bestd = fabs(sopo_scale_value(f, 0) - (double)sp);
    for (int q = 1; q <= f->max_code; ++q) {
        double d = fabs(sopo_scale_value(f, q) - (double)sp);
        if (d < bestd) { bestd = d; best = q; }
    }
    return best;
}

/* Same result by bisection on the increasing sequence v(q); used inside the layer loop because
 * the scan above costs 2^(x+y) evaluations per block.  The tests check the two agree. */
int sopo_scale_encode(const sopo_fmt* f, float sp)
{
    double t = (double)sp;
    if (!(sp < INFINITY) || t >= sopo_scale_value(f, f->max_code)) return f->max_code;
    if (t <= 0.0) return 0;
    int lo = 0, hi = f->max_code;                                    /* v(lo) <= t < v(hi)          */
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (sopo_scale_value(f, mid) <= t) lo = mid; else hi = mid;
    }
    double dlo = t - sopo_scale_value(f, lo), dhi = sopo_scale_value(f, hi) - t;
    return (dhi < dlo) ? hi : lo;                                    /* tie -> lower code           */
}

/* ---- block sums: chunks of 8, sequential fma in a chunk, balanced tree over chunks ---- */
static float tree_dot(const float* a, const float* b, int g)
{
    float part[64];
    int chunk = g < 8 ? g : 8;
    int n = g / chunk;
    for (int p = 0; p < n; ++p) {
        float acc = 0.0f;
        for (int i = 0; i < chunk; ++i) acc = fmaf(a[p * chunk + i], b[p * chunk + i], acc);
        part[p] = acc;
    }
    for (; n > 1; n >>= 1)
        for (int p = 0; p < n / 2; ++p) part[p] = part[2 * p] + part[2 * p + 1];
    return part[0];
}

typedef struct {
    int   q;            /* magnitude scale code                        */
    int   neg;          /* 1 when the negative scale sign was taken    */
    float err;          /* decision score of modes WSE / MSE           */
    float num, den;     /* binary32 sums used by mode COS              */
    double cosv;        /* value of the block cosine                   */
    uint8_t code[64];
} cand;

/* Ranking score of step 2 of the per-layer pair search (Section "Per-Layer Pair Search", step 2: every
 * block is scored against L_a under its own scale and the blocks are ranked; design axis (i): the
 * ranking score is the block cosine).  The ranking decides which pool a block goes to, so the score is
 * a decision quantity and is formed in binary32, one rounding per operation, from the block's binary32
 * tree sums: with num = <w,w^>_c, den = ||w^||_c^2, wn = ||w||_c^2 it is
 *     fl( fl(num / wn) * fl(|num| / den) ),
 * the block cosine squared with the cosine's sign, which ranks blocks as the cosine does.  Both
 * quotients are of the order of one whatever the block's magnitude.  A block without weighted norm has
 * cosine 1 (score 1), a zero reconstruction of a non-zero block cosine 0 (score 0). */
static float rank_score(float num, float den, float wn)
{
    if (!(wn > 0.0f)) return 1.0f;
    if (!(den > 0.0f)) return 0.0f;
    float a = num / wn;
    float b = fabsf(num) / den;
    return a * b;
}

/* cosine-mode comparison: is candidate b strictly better than candidate a?  cos = num/sqrt(wn*den);
 * wn is common, so compare num*|num|/den by cross-multiplication; a zero reconstruction has
 * cosine 0. */
static int cos_better(const cand* b, const cand* a)
{
    float qb = b->den > 0.0f ? b->num * fabsf(b->num) : 0.0f, db = b->den > 0.0f ? b->den : 1.0f;
    float qa = a->den > 0.0f ? a->num * fabsf(a->num) : 0.0f, da = a->den > 0.0f ? a->den : 1.0f;
    return (qb * da) > (qa * db);
}

static int better(const cand* b, const cand* a, int metric)
{
    return metric == SOPO_COS ? cos_better(b, a) : (b->err < a->err);
}

/* Ideal scale magnitude under the absmax rule (Section "Block Scaling", absmax scaling): no element
 * lands beyond an endpoint.  A negative scale sign swaps the roles of the endpoints. */
static float absmax_scale(const float* L, int N, float pmax, float nmax, int sigma)
{
    float tp = L[N - 1], tn = -L[0];
    float s_pos = sigma > 0 ? pmax / tp : pmax / tn;
    float s_neg = sigma > 0 ? nmax / tn : nmax / tp;
    return s_pos > s_neg ? s_pos : s_neg;
}

/* Argmax rule (Section "Block Scaling", argmax scaling): the element of largest magnitude x* is
 * mapped onto the endpoint of larger magnitude t*: s = x* / t*, so the scale's sign is that of x*
 * when t* is the positive endpoint and the opposite otherwise.  Where the paper is silent: of two
 * elements of equal magnitude and opposite sign the positive one is x*; of two endpoints of equal
 * magnitude the positive one is t*. */
static float argmax_scale(const float* L, int N, float pmax, float nmax, int* sigma)
{
    float tp = L[N - 1], tn = -L[0];
    int x_pos = pmax >= nmax, t_pos = tp >= tn;
    float amax = x_pos ? pmax : nmax;
    *sigma = (x_pos == t_pos) ? +1 : -1;
    return amax / (t_pos ? tp : tn);
}

/* One candidate: block w[g] with weights c[g], codebook L[N] (ascending) with midpoints mid[N-1],
 * ideal scale magnitude sstar, scale sign sigma (+1/-1). */
static void eval_candidate(const float* w, const float* c, int g, const float* L, const float* mid, int N,
                           float sstar, int sigma, const sopo_fmt* f, int k, int metric,
                           const float* cw, double wn_d, cand* out)
{
    float sp = sstar * (float)ldexp(1.0, k);                         /* per-layer shift 2^k          */
    int q = sopo_scale_encode(f, sp);
    float s = (float)ldexp(sopo_scale_value(f, q), -k);              /* exact by validation          */
    float r = s > 0.0f ? 1.0f / s : 0.0f;
    float ss = sigma > 0 ? s : -s;                                   /* signed effective scale       */

    float d[64], what[64], cd[64], cwh[64];
    double num_d = 0.0, den_d = 0.0;
    for (int i = 0; i < g; ++i) {
        float x = (sigma > 0 ? w[i] : -w[i]) * r;
        int code = 0;
        for (int j = 0; j < N - 1; ++j) code += (x > mid[j]);        /* ties -> lower index          */
        out->code[i] = (uint8_t)code;
        float y = L[code];
        d[i] = fmaf(-ss, y, w[i]);                                   /* w - s*y, rounded once        */
        what[i] = ss * y;
        cd[i] = (metric == SOPO_MSE) ? d[i] : c[i] * d[i];
        cwh[i] = c[i] * what[i];
        double wh = (double)ss * (double)y;
        num_d += (double)c[i] * (double)w[i] * wh;
        den_d += (double)c[i] * wh * wh;
    }
    out->q = q;
    out->neg = sigma < 0;
    out->err = tree_dot(cd, d, g);
    out->num = tree_dot(cw, what, g);
    out->den = tree_dot(cwh, what, g);
    if (wn_d == 0.0) out->cosv = 1.0;
    else if (den_d == 0.0) out->cosv = 0.0;
    else {
        double cv = num_d / sqrt(wn_d * den_d);
        out->cosv = cv > 1.0 ? 1.0 : (cv < -1.0 ? -1.0 : cv);
    }
}

/*
 * Layer search.  All pointers are host memory.  Outputs may be NULL when not wanted.
 *   W          [M][ldw] binary32 (bf16 inputs are widened exactly by the caller)
 *   c          [K] channel norms, >= 0
 *   atoms      concatenated ascending tables, n_entries[a] values each
 *   pair_ab    [2*P] atom indices (a,b) of each pair
 *   acos_pair  [P], acos_atom [A]                       binary64
 *   sel_words  [M*K/g] u32, one word per block: bit p = selector of pair p (1: the pair's second atom)
 *   scale_code [A][M*K/g] u16, bit 15 = negative sign taken, low bits = magnitude code
 *   codes      one plane per atom, planes back to back: M*K/2 bytes when n_entries <= 16 (two
 *              codes per byte, even element in the low nibble), otherwise M*K bytes
 *   blk_err    [A][M*K/g] binary32 decision score (c-weighted error; unweighted in mode MSE)
 *   blk_cos    [A][M*K/g] binary32 rounding of the block cosine
 *   blk_rank   [A][M*K/g] binary32 ranking score of step 2 (rank_score above) of the candidate kept
 * Returns 0, or a negative number for an invalid argument.
 */
int sopo_pair_search(const float* W, int64_t M, int64_t K, int64_t ldw, const float* c, int g,
                     int n_atoms, const int* n_entries, const float* atoms,
                     int n_pairs, const int* pair_ab,
                     const sopo_fmt* fmt, int k, int metric, int scale_rule,
                     double* acos_pair, double* acos_atom, uint32_t* sel_words, uint16_t* scale_code,
                     uint8_t* codes, float* blk_err, float* blk_cos, float* blk_rank, int n_threads)
{
    if (M <= 0 || K <= 0 || g <= 0 || g > 64 || K % g != 0 || ldw < K) return -1;
    if (n_atoms < 1 || n_atoms > SOPO_MAX_ATOMS) return -2;
    if (n_pairs < 0 || n_pairs > 32) return -4;
    int chunk = g < 8 ? g : 8;
    if (g % chunk != 0 || ((g / chunk) & (g / chunk - 1)) != 0) return -1;
    if (fmt->max_code < 1 || fmt->max_code >= (1 << (fmt->exp_bits + fmt->man_bits))) return -3;
    if (scale_rule != 0 && scale_rule != 1) return -3;
    if (scale_rule == 1 && fmt->sign_bits == 0) return -3;        /* the argmax scale carries a sign */

    const float* L[SOPO_MAX_ATOMS];
    float mid[SOPO_MAX_ATOMS][SOPO_MAX_ENTRIES];
    {
        const float* p = atoms;
        for (int a = 0; a < n_atoms; ++a) {
            int N = n_entries[a];
            if (N < 2 || N > SOPO_MAX_ENTRIES) return -2;
            L[a] = p;
            for (int j = 0; j + 1 < N; ++j) {
                if (!(p[j] < p[j + 1])) return -2;
                mid[a][j] = (float)(((double)p[j] + (double)p[j + 1]) * 0.5);
            }
            if (!(p[0] < 0.0f && p[N - 1] > 0.0f)) return -2;
            p += N;
        }
    }
    for (int p = 0; p < n_pairs; ++p)
        if (pair_ab[2 * p] < 0 || pair_ab[2 * p] >= n_atoms || pair_ab[2 * p + 1] < 0 || pair_ab[2 * p + 1] >= n_atoms)
            return -4;

    const int64_t Bk = K / g, Nb = M * Bk;
    int64_t code_off[SOPO_MAX_ATOMS + 1];
    code_off[0] = 0;
    for (int a = 0; a < n_atoms; ++a) code_off[a + 1] = code_off[a] + (n_entries[a] <= 16 ? M * K / 2 : M * K);
    const int is_signed = fmt->sign_bits != 0;
    double* row_sum = (double*)calloc((size_t)M * (size_t)(n_atoms + n_pairs), sizeof(double));
    if (!row_sum) return -5;
    if (sel_words) memset(sel_words, 0, (size_t)Nb * sizeof(uint32_t));

#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double* rs = row_sum + m * (n_atoms + n_pairs);
        for (int64_t j = 0; j < Bk; ++j) {
            const float* w = W + m * ldw + j * g;
            const float* cb = c + j * g;
            float pmax = 0.0f, nmax = 0.0f, cw[64];
            double wn_d = 0.0;
            for (int i = 0; i < g; ++i) {
                if (w[i] > pmax) pmax = w[i];
                if (-w[i] > nmax) nmax = -w[i];
                cw[i] = cb[i] * w[i];
                wn_d += (double)cb[i] * (double)w[i] * (double)w[i];
            }
            cand best[SOPO_MAX_ATOMS];
            for (int a = 0; a < n_atoms; ++a) {
                if (scale_rule == 1) {                             /* argmax: the rule fixes the sign */
                    int sigma;
                    float sstar = argmax_scale(L[a], n_entries[a], pmax, nmax, &sigma);
                    eval_candidate(w, cb, g, L[a], mid[a], n_entries[a], sstar, sigma, fmt, k, metric, cw, wn_d, &best[a]);
                } else {
                    eval_candidate(w, cb, g, L[a], mid[a], n_entries[a], absmax_scale(L[a], n_entries[a], pmax, nmax, +1), +1,
                                   fmt, k, metric, cw, wn_d, &best[a]);
                    if (is_signed) {
                        cand neg;
                        eval_candidate(w, cb, g, L[a], mid[a], n_entries[a], absmax_scale(L[a], n_entries[a], pmax, nmax, -1), -1,
                                       fmt, k, metric, cw, wn_d, &neg);
                        if (better(&neg, &best[a], metric)) best[a] = neg;
                    }
                }
                int64_t blk = m * Bk + j;
                rs[a] += best[a].cosv;
                if (scale_code) scale_code[(int64_t)a * Nb + blk] = (uint16_t)(best[a].q | (best[a].neg ? 0x8000 : 0));
                if (blk_err) blk_err[(int64_t)a * Nb + blk] = best[a].err;
                if (blk_cos) blk_cos[(int64_t)a * Nb + blk] = (float)best[a].cosv;
                if (blk_rank) blk_rank[(int64_t)a * Nb + blk] = rank_score(best[a].num, best[a].den, tree_dot(cw, w, g));
                if (codes) {
                    if (n_entries[a] <= 16) {
                        uint8_t* o = codes + code_off[a] + (m * K + j * g) / 2;
                        for (int i = 0; i < g; i += 2) o[i / 2] = (uint8_t)(best[a].code[i] | (best[a].code[i + 1] << 4));
                    } else {
                        uint8_t* o = codes + code_off[a] + m * K + j * g;
                        for (int i = 0; i < g; ++i) o[i] = best[a].code[i];
                    }
                }
            }
            for (int p = 0; p < n_pairs; ++p) {
                const cand* ca = &best[pair_ab[2 * p]];
                const cand* cb2 = &best[pair_ab[2 * p + 1]];
                int sel = better(cb2, ca, metric);
                rs[n_atoms + p] += sel ? cb2->cosv : ca->cosv;
                if (sel && sel_words) sel_words[m * Bk + j] |= (uint32_t)1 << p;
            }
        }
    }
    /* layer means: rows are added in index order so the result does not depend on the thread count */
    for (int a = 0; a < n_atoms + n_pairs; ++a) {
        double acc = 0.0;
        for (int64_t m = 0; m < M; ++m) acc += row_sum[m * (n_atoms + n_pairs) + a];
        acc /= (double)Nb;
        if (a < n_atoms) { if (acos_atom) acos_atom[a] = acc; }
        else if (acos_pair) acos_pair[a - n_atoms] = acc;
    }
    free(row_sum);
    return 0;
}

int sopo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
