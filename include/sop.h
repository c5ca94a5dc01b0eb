/*
 * sop.h -- C boundary of the MI355X pair-search library (libsop_hip.so).
 *
 * The library runs the data-parallel core of the per-layer pair search of "Scaled Outer Product"
 * on one gfx950 GPU: for every block of g consecutive weights along K it derives the absmax block
 * scale, rounds it into a narrow floating-point scale word, quantises the block to the nearest
 * entry of every candidate codebook ("atom"), scores the channel-norm-weighted error, sets the
 * per-block selector bit of every candidate pair and reduces to the per-layer activation-weighted
 * cosine (ACos) of every atom and pair.
 *
 * Conventions common to all calls
 *   - Every function returns a sop_status; SOP_OK is 0.  Nothing throws or aborts.  After a
 *     non-zero status sop_last_error() returns a text describing it.
 *   - "HOST" pointers are ordinary process memory, "DEVICE" pointers are memory of the GPU the
 *     context was created on.  The library never allocates or frees memory the caller sees; it
 *     owns only a small image of the codebook tables, the layer reduction's sums and a slab of
 *     scale tables inside the context, all allocated by sop_create.
 *   - sop_pair_search() is asynchronous on the given HIP stream and does no host synchronisation.
 *     Inputs are read-only; requested outputs are completely overwritten.
 *   - Block index: block j of row m has index m*(K/g) + j.
 *   - Weights and channel norms must be finite.
 */
#ifndef SOP_H
#define SOP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SOP_MAX_ATOMS   8     /* atoms in one alphabet                       */
#define SOP_MAX_ENTRIES 64    /* entries in one atom (n <= 6 bits)           */
#define SOP_DD_MAX_CANDIDATES 2047  /* grid points sop_dd_fit_grid() selects from */

typedef enum {
    SOP_OK = 0,
    SOP_EINVAL = 1,   /* null pointer, bad enum, misaligned buffer, bad pair list            */
    SOP_ESHAPE = 2,   /* M or K <= 0, g not in {8,16,32,64}, g does not divide K, ldw < K    */
    SOP_EATOM  = 3,   /* atom not strictly ascending, < 2 or > 64 entries, not two-sided, NaN,
                         two code boundaries closer than 1/650 of the atom's range, or a
                         non-zero entry below 2^-125 in magnitude                              */
    SOP_EFMT   = 4,   /* scale format or layer shift outside the supported range             */
    SOP_ENOMEM = 5,   /* workspace too small                                                 */
    SOP_EHIP   = 6    /* a HIP runtime call failed; see sop_last_error()                     */
} sop_status;

typedef enum { SOP_F32 = 0, SOP_BF16 = 1 } sop_dtype;

/* Metric of the per-block finishing reassignment (Section "Per-Layer Pair Search", design axis
 * (ii): block error or ACos).  SOP_SEL_WSE: channel-norm-weighted squared error sum_i c_i (w_i -
 * w^_i)^2 (default).  SOP_SEL_MSE: unweighted squared error.  SOP_SEL_COS: per-block weighted
 * cosine, compared without a division: with num = sum_i c_i w_i w^_i, den = sum_i c_i w^_i^2 and
 * q = num*|num|, candidate b beats candidate a when q_b*den_a > q_a*den_b (a zero reconstruction
 * counts as q = 0, den = 1). */
typedef enum { SOP_SEL_WSE = 0, SOP_SEL_COS = 1, SOP_SEL_MSE = 2 } sop_metric;

/* Scale word SwExMy in a b-bit container (Section "Scale Format and Metabit Allocation"): w sign
 * bits (0 or 1), x exponent bits, y mantissa bits.  Magnitude code q = (e << y) | f has the value
 * f/2^y * 2^(1-bias) when e == 0 and (1 + f/2^y) * 2^(e-bias) otherwise; every code is finite.
 * bias < 0 selects the default 2^(x-1)-1; max_code < 0 selects 2^(x+y)-1.  A signed format makes
 * the search try both signs of the block scale. */
typedef struct {
    int sign_bits, exp_bits, man_bits, container_bits;
    int bias;
    int max_code;
} sop_scale_fmt;

/* One codebook: n_entries values, strictly ascending, first negative and last positive.
 * `values` is a HOST pointer; the table is copied by sop_set_alphabet(). */
typedef struct {
    int n_entries;
    const float* values;
} sop_atom;

/* Output buffers, all DEVICE memory owned by the caller; a NULL member is not produced.
 * A = number of atoms, P = number of pairs, N_b = M*K/g. */
typedef struct {
    double*   acos_pair;   /* [P]   layer ACos with the per-block selector applied              */
    double*   acos_atom;   /* [A]   layer ACos of each atom alone                               */
    void*     sel_words;   /* [N_b] one selector word per block (the paper keeps the selector as a
                              per-block metabit): bit q = 1 when the second atom of pair q (index
                              in the pair list) reconstructs the block.  uint16_t words when
                              P <= 16, uint32_t words otherwise; 4-byte aligned                  */
    uint16_t* scale_code;  /* [A][N_b]  bit 15 = negative scale sign taken, low bits = code q   */
    uint8_t*  codes;       /* one plane per atom, back to back: M*K/2 bytes when the atom has
                              <= 16 entries (two codes per byte, even element in the low nibble),
                              M*K bytes otherwise                                               */
    float*    blk_cos;     /* [A][N_b]  per-block weighted cosine (value, fp32 accuracy)        */
    float*    blk_err;     /* [A][N_b]  per-block decision score (weighted error; unweighted in
                              mode SOP_SEL_MSE)                                                 */
    float*    blk_rank;    /* [A][N_b]  ranking score of step 2 of the per-layer search (Section
                              "Per-Layer Pair Search", step 2; design axis (i): block cosine): the
                              block cosine squared, with the cosine's sign, formed in binary32 from the
                              block's binary32 sums (chunks of 8 consecutive elements, sequential fma,
                              balanced tree) num = <w,w^>_c, den = ||w^||_c^2, wn = ||w||_c^2 as
                              fl(fl(num / wn) * fl(|num| / den)); 1 when wn = 0, 0 when den = 0.  It
                              orders blocks as blk_cos does but is reproducible bit for bit, so pools
                              derived from it (sop_partition) are too                            */
} sop_outputs;

typedef struct sop_ctx sop_ctx;

/* Create a context on GPU `device_ordinal`.  Allocates the device table image (a few KB).
 * Fails with SOP_EHIP when no usable GPU or HIP runtime is present: there is no CPU fallback. */
sop_status sop_create(sop_ctx** ctx, int device_ordinal);
sop_status sop_destroy(sop_ctx* ctx);

/* Install the alphabet (Section "Per-Layer Pair Search": the search runs over an alphabet of
 * candidate codebooks, each atom and its sign negation being separate candidates).  atoms is a
 * HOST array of n_atoms <= SOP_MAX_ATOMS descriptors.  Builds value and midpoint tables (midpoint
 * = binary64 mean of neighbours rounded once to binary32) and uploads them synchronously.
 * The kernel finds an element's code through a table over at most 1024 uniform bins of the scaled
 * weight with at most one code boundary per bin: an atom with two boundaries (midpoints of
 * neighbouring entries) closer than about 1/650 of its range is refused with SOP_EATOM.
 * The table holds half of every entry (the element passes multiply by twice the block scale: the
 * same product), so a non-zero entry must be at least 2^-125 in magnitude (SOP_EATOM otherwise).
 * Weights and channel norms must be finite; per-block results are exact for weighted block norms
 * sum(c w^2) within 2^-126 .. 2^126 (the cosine's value path rescales by the norm's exponent).
 * Resets the pair list to all pairs a < b in lexicographic order. */
sop_status sop_set_alphabet(sop_ctx* ctx, const sop_atom* atoms, int n_atoms);

/* Host-only self check of the element-search table the library would build for this alphabet
 * (no GPU needed): builds the table, then compares table lookups with the direct count of
 * midpoints below x on every float near each code boundary and on dense sweeps of the range.
 * Returns SOP_OK when they agree; *n_bins receives the table's bin count, *n_checked the number of
 * values compared (either may be NULL). */
sop_status sop_check_alphabet(const sop_atom* atoms, int n_atoms, int* n_bins, int64_t* n_checked);

/* Choose the candidate pairs: HOST array of P pairs (a, b) with a < b, no duplicates.
 * P = 0 (or pair_ab NULL) restores the default of all pairs.  Output index = position here. */
sop_status sop_set_pairs(sop_ctx* ctx, const int* pair_ab, int n_pairs);

/* Rule for the block scale (Section "Block Scaling").  SOP_SCALE_ABSMAX (default): the smallest scale
 * that leaves no element beyond an endpoint, s = max(max_r x / t+, max_r (-x) / (-t-)); with a signed
 * scale word the search evaluates both signs of it and keeps the better.  SOP_SCALE_ARGMAX: the
 * element of largest magnitude x* is mapped onto the endpoint of larger magnitude t*, s = x* / t*; the
 * rule fixes the sign (bit 15 of scale_code), so the scale word must have a sign bit (else SOP_EFMT
 * from sop_pair_search).  Ties: of +a and -a the positive element is x*; of endpoints of equal
 * magnitude the positive one is t*.  The rule stays set for later sop_pair_search() calls. */
typedef enum { SOP_SCALE_ABSMAX = 0, SOP_SCALE_ARGMAX = 1 } sop_scale_rule;
sop_status sop_set_scale_rule(sop_ctx* ctx, sop_scale_rule rule);

/* Bytes of DEVICE workspace sop_pair_search() needs for this shape.  This version needs none and
 * reports 0 (the layer reduction keeps a few words inside the context); the workspace arguments of
 * sop_pair_search() are accepted for callers written against a version that did, and may be
 * NULL / 0. */
sop_status sop_workspace_bytes(sop_ctx* ctx, int64_t M, int64_t K, int g, size_t* bytes);

/* The per-layer search (Section "Block Scaling": absmax scale and round_q; Section "Scale Format
 * and Metabit Allocation": scale word and per-layer shift; Section "Activation-Weighted Cosine
 * Similarity": ACos; Section "Per-Layer Pair Search", step 4: finishing reassignment).
 *   W_dev       DEVICE, M rows of K elements, row stride ldw elements, dtype fp32 or bf16;
 *               base pointer and row stride must be multiples of 16 bytes
 *   c_dev       DEVICE, K channel norms (fp32, >= 0), 16-byte aligned
 *   g           block size along K: 8, 16, 32 or 64; must divide K
 *   fmt         scale word format; layer_shift_k multiplies every ideal block scale by 2^k before
 *               rounding and divides the decoded scale by it (|k| <= 64)
 *   metric      SOP_SEL_WSE, SOP_SEL_MSE or SOP_SEL_COS
 *   workspace   DEVICE, at least sop_workspace_bytes() bytes (0: may be NULL)
 *   out         HOST pointer to the struct of DEVICE output pointers
 *   hip_stream  a hipStream_t (NULL = the default stream)
 * Arguments are validated before anything is launched.  Calls on one context must not overlap
 * with sop_set_alphabet / sop_set_pairs, nor with each other on the GPU (the context holds the
 * running sums of the layer reduction): issue them on one stream, or use one context per stream. */
sop_status sop_pair_search(sop_ctx* ctx, const void* W_dev, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                           const float* c_dev, int g, sop_scale_fmt fmt, int layer_shift_k, sop_metric metric,
                           void* workspace_dev, size_t workspace_bytes, const sop_outputs* out, void* hip_stream);

/* The table of (scale, reciprocal) per scale code that sop_pair_search() reads for (fmt, layer_shift_k),
 * written ahead of time.  Optional: a call that finds the table missing writes it itself with one small
 * kernel on its stream before its search kernel (the tables live in memory the context allocated at its
 * creation, 160 of them, the least recently used one is replaced; nothing is allocated or copied from the host,
 * and the host never waits).  Asynchronous on hip_stream; the search calls that use the table must be ordered
 * after it (same stream, or an event). */
sop_status sop_prepare_scale(sop_ctx* ctx, sop_scale_fmt fmt, int layer_shift_k, void* hip_stream);

/* sop_pair_search() for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments (without the workspace), same kernels, same results bit
 * for bit; the call itself calls no hipMalloc / hipFree and no allocating library routine.  What
 * sop_pair_search() keeps in memory of the context allocated on demand (the running sums and ticket
 * counters of the layer reduction, the table of (scale, reciprocal) per scale code) lives here in a
 * statically allocated device array of SOP_STATIC_SCRATCH_BYTES bytes that is part of the library's device
 * image: every GPU the library runs on holds one copy until the process ends.  A small kernel at the start
 * of the call clears the sums and writes the scale table for (fmt, layer_shift_k); it is launched on
 * hip_stream before the search kernel (no memset node, so the pair may be captured into a graph).
 * Limit: the scale word may have at most SOP_STATIC_MAX_CODES magnitude codes (max_code < 2048, i.e.
 * x + y <= 11); a wider word is refused with SOP_EFMT (sop_pair_search() decodes such words arithmetically).
 * The context must have been created and given its alphabet beforehand (those calls allocate).  All static
 * calls on one GPU share the one array, whatever the context or stream: calls that overlap on a GPU race;
 * issue them on one stream or order them with events.  The first call of a kernel variant on a context
 * queries its occupancy (no allocation). */
#define SOP_STATIC_MAX_CODES     2048
#define SOP_STATIC_SCRATCH_BYTES (2560 + 8 * SOP_STATIC_MAX_CODES)
sop_status sop_pair_search_static(sop_ctx* ctx, const void* W_dev, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                  const float* c_dev, int g, sop_scale_fmt fmt, int layer_shift_k, sop_metric metric,
                                  const sop_outputs* out, void* hip_stream);

/* Text of the last error on this context (or of the last failed sop_create when ctx is NULL). */
const char* sop_last_error(sop_ctx* ctx);

/* ---- host-side atom builders (Section "Per-Layer Pair Search", alphabet list; Section "Primary
 * Formats" for the sinh grid).  `out` is a HOST array of 2^n_bits floats, ascending. ---- */

/* NormalFloat grid: Gaussian quantiles, 2^(n-1) positive and 2^(n-1)-1 negative entries plus an
 * exact zero, endpoints -1 and +1.  n_bits in 2..6. */
sop_status sop_atom_nf(int n_bits, float* out);
/* Sinh grid sinh(alpha t) + c on 2^n uniform t in [-1,1], divided by its largest magnitude
 * (the paper uses alpha = 1.5, c = -0.02). */
sop_status sop_atom_sh(int n_bits, double alpha, double c, float* out);
/* Sign-negated atom, re-sorted ascending.  in and out may not overlap. */
sop_status sop_atom_negate(const float* in, int n_entries, float* out);
/* Weighted 1-D Lloyd iteration on HOST samples (weights may be NULL = uniform): each sample goes
 * to its nearest centroid (ties to the lower), every centroid moves to the weighted mean of its
 * cell, empty cells stay; `centroids` holds the start grid on entry and the result on return. */
sop_status sop_lloyd_1d(const double* samples, const double* weights, int64_t n_samples,
                        double* centroids, int n_centroids, int iters);
/* Block-optimum-fitted grid: the n_draws HOST N(0,1) draws are cut into blocks of g, each block
 * is divided by its signed absmax element, Lloyd runs from the NormalFloat grid; afterwards the
 * endpoints are set to -1 and +1 and the entry nearest zero to 0. */
sop_status sop_atom_bof(int n_bits, const double* draws, int64_t n_draws, int g, int iters, float* out);

/* The search over the linear layers of a model in one call (Section "Per-Layer Pair Search": the pair is
 * chosen per layer; the result is a table of per-layer ACos for every atom and pair, which the format
 * allocation of the later pipeline steps reads).  layers: HOST array of n_layers descriptors of DEVICE
 * tensors that share dtype, block size, scale format and metric; each has its own shape, channel norms
 * and layer shift.  acos_pair_table_dev: DEVICE [n_layers][P] doubles (may be NULL), acos_atom_table_dev:
 * DEVICE [n_layers][A] doubles (may be NULL; not both).  sel_words_dev of a layer may be NULL (search
 * mode without selector words).  Every layer is validated before the first launch; an error names the
 * layer in sop_last_error().  Asynchronous on hip_stream.  Alphabets of more than two atoms are searched
 * by one launch per distinct layer shift (and per 1024 layers) that works through the list; the results
 * equal those of sop_pair_search on each layer bit for bit.  Smaller alphabets run one kernel per layer
 * on two streams of the library's own, which start after the work already queued on hip_stream and
 * which hip_stream waits for.  The call may wait on the host until the layer list of the launch before
 * last has been copied to the device (two pinned staging buffers are used in turn), i.e. the host runs
 * at most two such launches ahead of the device. */
typedef struct {
    const void*  W_dev;
    int64_t      M, K, ldw;
    const float* c_dev;
    int          layer_shift_k;
    void*        sel_words_dev;
} sop_layer;
sop_status sop_pair_search_layers(sop_ctx* ctx, const sop_layer* layers, int n_layers, sop_dtype dtype, int g,
                                  sop_scale_fmt fmt, sop_metric metric, double* acos_pair_table_dev,
                                  double* acos_atom_table_dev, void* hip_stream);

/* ---- data-derived codebook ("DD" atom; Section "Per-Layer Pair Search", steps 1 and 3: a
 * data-adaptive atom is fitted per layer from a histogram of the layer's weights; design axis (iii):
 * uniform or channel-norm-weighted updates).  Two steps: a statistics pass on the GPU and a
 * weighted Lloyd fit on the histogram on the host. ----
 *
 * Histogram, in exact integer arithmetic (binary32 operations, one rounding each):
 *   cmax = max_k c_k, cs = 2^20 / cmax (c_dev NULL: every c_k = 1);
 *   per block of g weights: a = max |w_i| (blocks with a = 0 are skipped), r = 1 / a;
 *   per weight: x = w_i * r, mass = rint(c_i * cs)  (units of 2^-20 cmax),
 *               bin = clamp(floor(x * H/2 + H/2), 0, H-1);    hist[bin] += mass.
 * The result does not depend on the order of addition. */

/* W_dev, dtype, M, K, ldw, c_dev (may be NULL), g as in sop_pair_search(); n_bins = H, a power of
 * two within 64..8192; row_step >= 1: only rows 0, row_step, 2*row_step, ... enter the histogram
 * (1 = the whole layer; the pass is bound by LDS atomics, not by HBM, so a sample of the rows is
 * the cheap way to a fit of the same quality); block_mask_dev: DEVICE or NULL, one byte per block
 * (index m*(K/g) + j): only blocks with a non-zero byte enter (the fitting pool of step 3 of the pair
 * search); hist_dev: DEVICE, H 64-bit integers, overwritten.
 * Asynchronous on the stream; needs no workspace.  Calls on one context must not overlap on the
 * GPU (the context holds the running histogram). */
sop_status sop_dd_histogram(sop_ctx* ctx, const void* W_dev, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                            const float* c_dev, int g, int n_bins, int64_t row_step, const uint8_t* block_mask_dev,
                            int64_t* hist_dev, void* hip_stream);

/* Weighted Lloyd iteration on a histogram (all HOST memory): bin b stands for its centre
 * -1 + (2b+1)/H and goes, whole, to that centre's cell (cell = number of midpoints of the current
 * grid strictly below the centre); every non-empty cell's entry moves to the mass-weighted mean of
 * its bins' centres (exact integer sums, one binary64 division); the grid is re-sorted; `iters`
 * rounds from the ascending start grid `init`.  `out` receives n_entries binary32 values.
 * SOP_EATOM when the result is not strictly ascending or not two-sided (it could not serve as an
 * atom). */
sop_status sop_dd_fit(const int64_t* hist, int n_bins, int n_entries, int iters, const float* init, float* out);

/* Grid-constrained data-derived codebook (Section "Per-Layer Pair Search", step 1: the entries of a
 * data-adaptive codebook are selected among the grid points of the deployed LUT value format by a
 * dynamic programme on the histogram, so that no snap-to-grid displacement follows the fit; step 3
 * uses the same construction on the fitting pool).  All HOST memory.
 *   hist, n_bins   as sop_dd_histogram() writes them (bin b stands for its centre -1 + (2b+1)/H)
 *   cand           n_cand candidate values in the histogram's domain, strictly ascending, within
 *                  [-4, 4] (grid value / normalisation target; sop_weight_grid() lists a format's values)
 *   chosen         receives n_entries ascending indices into cand: the selection with the least
 *                  sum over bins of mass * (centre - nearest chosen value)^2 (a bin goes, whole, to
 *                  the value nearest its centre, ties to the lower value); among selections whose
 *                  costs agree to rounding (about 1e-14 relative) the one found first is returned
 *   cost           HOST or NULL: receives that sum (mass units times squared domain units)
 * Exact optimum by dynamic programming over (number of values chosen, last value chosen):
 * O(n_entries * n_cand^2) operations and n_cand^2 doubles of host memory (0.1 ms for 16 of the 63
 * E2M3 values, 1.3 ms for 16 of the 255 E4M3 values, 2 s at the limits: 64 of 2047).  SOP_EATOM when the candidates are not ascending or the
 * selection is not two-sided (it could not serve as an atom). */
sop_status sop_dd_fit_grid(const int64_t* hist, int n_bins, const double* cand, int n_cand, int n_entries,
                           int* chosen, double* cost);

/* ---- per-layer scale shift (Section "Scale Format and Metabit Allocation", paragraph "Per-layer
 * scale shift": all block scales of a layer are multiplied by 2^k before they are rounded into the
 * scale word, k* maximising the fraction of block scales in the format's normal range).  Two steps:
 * a statistics pass on the GPU and the choice of k* on the host; k* is then passed to
 * sop_pair_search() as layer_shift_k. ----
 *
 * Histogram of the ideal block scales sc = max(pmax / t_pos, nmax / t_neg) (the absmax rule against
 * a codebook with last entry t_pos and first entry -t_neg; IEEE binary32 divisions): writing
 * sc = m * 2^e with 1/2 <= m < 1, hist[e + 160] counts the blocks with that e, and
 * hist[320 + e + 160] those among them whose m exceeds the m of the format's largest value.
 * Blocks with sc = 0 are not counted.  hist_dev: DEVICE, 640 64-bit integers, overwritten.
 * SOP_ESHAPE for a layer of 2^31 or more wavefront steps (a step is 64 lanes x 8 or 16 weights:
 * about 10^12 weights).  Asynchronous; needs no workspace; calls on one context must not overlap on
 * the GPU. */
sop_status sop_scale_histogram(sop_ctx* ctx, const void* W_dev, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw, int g,
                               float t_pos, float t_neg, sop_scale_fmt fmt, int64_t* hist_dev, void* hip_stream);

/* k* from such a histogram (HOST memory).  Normal range = [2^(1-bias), value(max_code)], both ends
 * included; n_blocks = M*K/g is the denominator of the fraction (zero scales are in no range);
 * candidates are the shifts within [-64, 64] that sop_pair_search() accepts for the format; among
 * equally good shifts the smallest |k| wins, then the non-negative one.  *fraction (may be NULL)
 * receives the fraction reached. */
sop_status sop_layer_shift(const int64_t* hist, int64_t n_blocks, sop_scale_fmt fmt, int* k_star, double* fraction);

/* ---- layer-scope weight formats (Section "Primary Formats", paragraph "Block-scaled FP6 versus
 * POT-scaled FP8": the baseline E4M3^0sUE8M0 is bare E4M3 weights with one power-of-two scale per
 * layer; Appendix "Format string grammar": ^0 = layer-max scope).  The block-scaled side of that
 * comparison is sop_pair_search() with the E2M3 grid as an atom; its layer error is the sum of the
 * blk_err plane (sop_sum_f32). ---- */

/* An ExMy weight grid: magnitudes value(q), q = 0..max_code (bias < 0: 2^(x-1)-1; max_code < 0:
 * 2^(x+y)-1, every code finite), both signs, one zero: 2*max_code+1 values. */
typedef struct { int exp_bits, man_bits, bias, max_code; } sop_weight_fmt;

/* The distinct values of an ExMy weight grid, ascending, both signs and one zero (Section "SOP
 * Methodology", paragraph "LUT value format": LUT entries live on a small floating-point grid such
 * as E2M3 or E4M3).  top > 0 keeps only magnitudes up to top (a normalisation target below the
 * format's largest value); top <= 0 keeps all.  values: HOST, room for 2*max_code+1 doubles;
 * n_values receives the count.  x + y <= 10. */
sop_status sop_weight_grid(sop_weight_fmt wfmt, double top, double* values, int* n_values);

/* One scale for the whole layer by the block rule with the layer as the block: s* = max(pmax, nmax)
 * / value(max_code), times 2^k, rounded into the scale word `sfmt` (nearest, ties to the lower
 * code), s = value(q) * 2^-k; every weight goes to the nearest grid value of x = w / s (ties to the
 * lower value); d = w - s*y.
 *   out_dev    DEVICE, 4 doubles: sum c_k d^2, sum d^2, sum c_k w^2, scale code q
 *   codes_dev  DEVICE or NULL: [M*K] uint16 index of every weight's value in the ascending grid
 *   c_dev      DEVICE or NULL (c = 1); K must be a multiple of 8 (bf16) or 4 (fp32)
 * The products and the sums over the 8 (bf16) or 4 (fp32) weights a lane reads at a time are
 * binary32; these enter binary64 sums in an order fixed by the GPU's size (reproducible on one GPU;
 * within about 1e-7 relative of the exact sums).  Asynchronous; no workspace; calls on
 * one context must not overlap on the GPU. */
sop_status sop_layer_scope_error(sop_ctx* ctx, const void* W_dev, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                 const float* c_dev, sop_weight_fmt wfmt, sop_scale_fmt sfmt, int layer_shift_k,
                                 double* out_dev, uint16_t* codes_dev, void* hip_stream);

/* Calibration, not part of the method: a plain read of n_bytes (a multiple of 16) of DEVICE memory at
 * x_dev (16-byte aligned) by SOP_READ_PROBE_WORDS workgroups, which is what every statistics pass above
 * must at least do; its time is the floor their rooflines are judged against (the published HBM peak is
 * not reachable by a kernel, and the reachable rate depends on the buffer's size).
 * out_dev: DEVICE, SOP_READ_PROBE_WORDS uint32 words, overwritten: word b = exclusive-or of the 32-bit
 * words workgroup b read; the exclusive-or of all of them is that of the whole buffer.  Asynchronous. */
#define SOP_READ_PROBE_WORDS 2048
sop_status sop_read_probe(sop_ctx* ctx, const void* x_dev, int64_t n_bytes, uint32_t* out_dev, void* hip_stream);

/* Calibration: the rate at which the vector ALUs take one kind of instruction (not part of the method; it
 * is what the "alu" roofline of the search kernel is read against).  Launches n_cu * waves_per_simd * 256
 * threads so that every SIMD holds waves_per_simd wavefronts (one workgroup per compute unit up to four
 * wavefronts per SIMD, two for six and eight, workgroups of four wavefronts for five and seven); every lane
 * executes iters * 64 instructions of the kind on eight independent chains, without memory traffic:
 *   kind 0 v_fmac_f32 (registers only)   1 v_max_f32   2 v_fma_f32 with a scalar-register operand
 *        3 v_cmp_lt_f32 + v_cndmask_b32  4 v_mul_f32   5 v_mad_u32_u24   6 v_fma_f32 + v_max_f32 alternating
 *        7 v_add_f32  8 v_and_b32  9 v_add_u32  10 v_lshrrev_b32  11 v_lshlrev_b32  12 v_cvt_i32_f32  13 v_med3_f32
 *        14 v_rcp_f32  (7..14 tell an instruction's class; their values are not meant to be checked)
 *   kinds 15..18: the element pass of the search kernel on its own (per iteration six passes over 16 elements: a
 *        table look-up in LDS at a bin that differs from lane to lane, the choice between the two values, residual
 *        fma, c*d, error fma, cosine-sum fma; iters * 96 elements per lane): 15 with 12-byte look-ups (boundary and
 *        two values, 6 vector instructions per element), 16 with 8-byte look-ups (two values, the boundary is their
 *        sum: 7 instructions; what the search kernel does), 17 and 18 the arithmetic of 16 and 15 on register values
 *        without look-ups.  What LDS costs beside the arithmetic (values not meant to be checked).
 * a, b: the two operand values (chains start at (thread % 8) / 8 + chain number).
 * out_dev: DEVICE, n_cu * waves_per_simd * 256 floats, overwritten: the sum ((x0+x1)+(x2+x3))+((x4+x5)+(x6+x7))
 * of the lane's chain values.  waves_per_simd 1..8, iters 1..2^20.  Asynchronous.
 * *n_out (HOST, may be NULL) receives the number of floats written (threads launched). */
#define SOP_ISSUE_PROBE_KINDS 19
sop_status sop_issue_probe(sop_ctx* ctx, int kind, int waves_per_simd, int iters, float a, float b,
                           float* out_dev, int* n_out, void* hip_stream);

/* out_dev[0] = sum of the n binary32 values at x_dev, accumulated in binary64 in a fixed order. */
sop_status sop_sum_f32(sop_ctx* ctx, const float* x_dev, int64_t n, double* out_dev, void* hip_stream);

/* ---- block ranking and pools (Section "Per-Layer Pair Search", step 2: every block is scored
 * against L_a under its own scale and ranked, the best-ranked p% stay with L_a; step 3: the rest is
 * the pool L_b is fitted on; design axes (i) ranking score = block cosine or unweighted block error,
 * (iv) pool defined by a rank). ----
 *   score_dev   DEVICE, n_blocks binary32 scores, no NaN (a blk_cos or blk_err plane of an emitting
 *               sop_pair_search() call), 16-byte aligned
 *   n_top       size asked of the first pool, 0 .. n_blocks (the caller turns p% into a count)
 *   higher_is_better  non-zero for a cosine, zero for an error
 *   pool_b_dev  DEVICE, n_blocks bytes, 4-byte aligned: 1 = the block ranks strictly worse than tau
 *               (fitting pool of L_b; feeds sop_dd_histogram as block mask), 0 = it stays with L_a
 *   tau_dev     DEVICE, 1 float: the score of the block of rank n_top (+inf / -inf when n_top = 0)
 *   n_a_dev     DEVICE, 1 int64: blocks at least as good as tau (>= n_top: blocks that tie with tau
 *               all stay; +0 and -0 tie)
 * Exact (integer counting), reproducible, asynchronous, no workspace; calls on one context must not
 * overlap on the GPU. */
sop_status sop_partition(sop_ctx* ctx, const float* score_dev, int64_t n_blocks, int64_t n_top, int higher_is_better,
                         uint8_t* pool_b_dev, float* tau_dev, int64_t* n_a_dev, void* hip_stream);

/* The same ranking for several sizes of the first pool at once (Section "Per-Layer Pair Search": the search
 * sweeps the partition parameter p; steps 2 and 3 for every p of the sweep from one ranking and one pass over
 * the weights).  n_top: HOST, n_levels (1..8) non-decreasing sizes of the first pool, so that the fitting pools
 * are nested: pool j = the blocks ranked strictly worse than tau_j, pool 0 the largest.
 *   level_dev   DEVICE, n_blocks bytes, 4-byte aligned: the number of pools the block belongs to
 *               (0 .. n_levels); block b is in pool j exactly when level[b] > j
 *   tau_dev     DEVICE, n_levels floats; n_a_dev  DEVICE, n_levels int64: as in sop_partition(), per threshold
 * Each (tau_j, n_a_j, pool j) equals what sop_partition() returns for n_top[j].  Exact, asynchronous, no
 * workspace; calls on one context must not overlap on the GPU. */
sop_status sop_partition_levels(sop_ctx* ctx, const float* score_dev, int64_t n_blocks, const int64_t* n_top, int n_levels,
                                int higher_is_better, uint8_t* level_dev, float* tau_dev, int64_t* n_a_dev, void* hip_stream);

/* sop_dd_histogram() for nested pools: level_dev as sop_partition_levels() writes it; hist_dev: DEVICE,
 * [n_levels][n_bins] 64-bit integers, overwritten: row j is the histogram of pool j (the blocks of level > j),
 * equal to sop_dd_histogram() with pool j as block mask.  One pass over the weights.  n_levels * n_bins must
 * not exceed 8192. */
sop_status sop_dd_histogram_levels(sop_ctx* ctx, const void* W_dev, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                   const float* c_dev, int g, int n_bins, int64_t row_step, const uint8_t* level_dev, int n_levels,
                                   int64_t* hist_dev, void* hip_stream);

/* ---- materialisation (Section "Scale Format and Metabit Allocation", paragraphs "The SwExMy
 * notation", "Bit placement" and "Worked examples"; Section "Per-Layer Pair Search": one metabit per
 * block names the codebook; introduction: a block of g n-bit codes is g*n/8 bytes). ----
 * Per block: the scale word in its container of fmt.container_bits <= 16 bits, one uint16 per block:
 * sign at bit b-1 when fmt.sign_bits = 1; magnitude code (exponent then mantissa) above the low-end
 * metabits; the selector in the first metabit (bit b-1 without a sign bit, bit m-1 with one, m = b -
 * w - x - y); remaining metabits zero.  And the block's codes as a little-endian string of n-bit
 * fields (code i in bits i*n .. i*n+n-1; n = bits needed for the larger codebook).
 *   scale_a_dev / codes_a_dev / entries_a   one atom's plane of an emitting search: scale_code
 *               [N_b] (bit 15 = sign) and code plane (layout as in sop_outputs.codes), 8-byte aligned
 *   scale_b_dev / codes_b_dev / entries_b   the second atom, or NULL, NULL, 0: single codebook
 *   sel_words_dev, sel_word_bytes, pair_q   the search's selector words (2 or 4 bytes each) and the
 *               pair's bit; selector 1 = the block takes atom b.  NULL with a single codebook
 *   words_dev   DEVICE, N_b uint16;   payload_dev  DEVICE, N_b * g*n/8 bytes, 8-byte aligned
 *   n_bits_out  HOST, may be NULL: receives n
 * SOP_EFMT when two codebooks meet a format without a metabit.  Asynchronous; no workspace. */
sop_status sop_pack_blocks(sop_ctx* ctx, int64_t M, int64_t K, int g, sop_scale_fmt fmt,
                           const uint16_t* scale_a_dev, const uint8_t* codes_a_dev, int entries_a,
                           const uint16_t* scale_b_dev, const uint8_t* codes_b_dev, int entries_b,
                           const void* sel_words_dev, int sel_word_bytes, int pair_q,
                           uint16_t* words_dev, uint8_t* payload_dev, int* n_bits_out, void* hip_stream);

/* ---- the per-layer pair search as one call (Section "Per-Layer Pair Search": step 1 per-atom scoring, step 2
 * block ranking and the top-p% pool, step 3 the second codebook fitted on the rest, step 4 the finishing
 * reassignment; the search sweeps the atoms and the partition parameter p and keeps the best (L_a, p, L_b)). ----
 * Candidates examined: every pair of atoms of the given alphabet; and, for every atom a and every p of the sweep,
 * the pair (a, L_b) with L_b fitted on the blocks that a serves worst (the ranking score is blk_rank, the pool
 * the blocks ranked strictly worse than the block of rank round(p * N_b / 100), halves up; the fit is
 * sop_dd_fit() on sop_dd_histogram() of that pool, or sop_dd_fit_grid() when a grid is given; an empty pool
 * leaves the start grid).  The winner has the largest layer ACos under step 4's reassignment; among equal
 * values the first in this order wins: pairs of atoms in lexicographic order, then atom by atom, p by p.
 * A fitted codebook that cannot serve as an atom (SOP_EATOM from the fit or from the table construction) drops
 * its candidate (NaN in acos_fitted).
 * An alphabet of more than SOP_MAX_ATOMS atoms (at most SOP_LAYER_MAX_ATOMS) is covered by several searches of at
 * most eight atoms each: the halves [0, 8) and [8, A) whole (every atom's own ACos and ranking plane, the pairs inside
 * a half) and the pairs across the halves four atoms against four, at most six searches; every pair is scored in exactly
 * one of them, with the arithmetic of a search that holds both atoms. */
#define SOP_LAYER_MAX_P 7
#define SOP_LAYER_MAX_ATOMS 16
#define SOP_LAYER_MAX_PAIRS 120
typedef struct {
    int           n_p;                         /* values of p in the sweep, 0..7 (0: pairs of atoms only)            */
    double        p_percent[SOP_LAYER_MAX_P];  /* non-decreasing, each within [0, 100]                               */
    int           fit_entries, fit_iters;      /* entries of L_b (2..64), Lloyd rounds of the free fit                */
    int           fit_bins;                    /* histogram bins (power of two, n_p * fit_bins <= 8192)               */
    const float*  fit_init;                    /* HOST, fit_entries ascending values: start grid (NULL: the first atom) */
    int           weighted_fit;                /* non-zero: channel-norm-weighted histogram (design axis (iii))       */
    const double* fit_grid;                    /* HOST or NULL: ascending candidate values, L_b is selected among them */
    int           n_fit_grid;
    int           pack;                        /* non-zero: the winner is searched once more and packed               */
} sop_layer_opts;
typedef struct {
    int    kind;                               /* 0: both codebooks are atoms of the alphabet; 1: L_b was fitted      */
    int    a, b;                               /* atom indices (b = -1 when fitted)                                   */
    int    j;                                  /* index of the winner's p in the sweep (fitted only)                  */
    double p_percent;                          /* the winner's p (0 for kind 0)                                       */
    double acos;                               /* its layer ACos                                                      */
    int    n_entries_b;
    float  table_b[SOP_MAX_ENTRIES];           /* the second codebook                                                 */
    double acos_fixed[SOP_LAYER_MAX_PAIRS];    /* every pair of atoms, lexicographic; NaN beyond the alphabet's pairs */
    double acos_atom[SOP_LAYER_MAX_ATOMS];     /* every atom alone                                                    */
    double acos_fitted[SOP_LAYER_MAX_ATOMS][SOP_LAYER_MAX_P];   /* (a, p_j); NaN: not examined or dropped             */
    int    n_bits;                             /* bits per code of the packed payload (pack only)                     */
} sop_layer_result;

/* Bytes of DEVICE workspace sop_search_layer() needs (the ranking scores of every atom, A * N_b floats, make up
 * most of it). */
sop_status sop_search_layer_workspace(sop_ctx* ctx, int64_t M, int64_t K, int g, int n_atoms, const sop_layer_opts* opts, size_t* bytes);

/* W_dev, dtype, M, K, ldw, c_dev, g, fmt, layer_shift_k, metric as in sop_pair_search(); atoms: HOST, n_atoms
 * (1..16) codebooks; workspace_dev: DEVICE, 256-byte aligned, at least sop_search_layer_workspace() bytes;
 * result: HOST; words_dev / payload_dev: DEVICE outputs of the packing as in sop_pack_blocks() (pack only: N_b
 * uint16 and N_b * g*n/8 bytes with n = bits of the larger of the two codebooks; the scale word needs a metabit).
 * The call queues its kernels on hip_stream and waits for the stream twice (the pool histograms are fitted on the
 * host; the ACos values decide the winner); the packing is queued and not waited for.  It replaces the context's
 * alphabet and pair list: afterwards the context has no alphabet set.  The first call on a context allocates
 * pinned host staging (a few MB).  Calls on one context must not overlap. */
sop_status sop_search_layer(sop_ctx* ctx, const void* W_dev, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw, const float* c_dev,
                            int g, sop_scale_fmt fmt, int layer_shift_k, sop_metric metric, const sop_atom* atoms, int n_atoms,
                            const sop_layer_opts* opts, void* workspace_dev, size_t workspace_bytes, sop_layer_result* result,
                            uint16_t* words_dev, uint8_t* payload_dev, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SOP_H */
