// Launch parameters shared by the host side of the library and its kernels (passed by value).
#ifndef SOP_KPARAMS_H
#define SOP_KPARAMS_H
#include <stdint.h>

#define SOP_K_MAXA 8                 /* atoms                                        */
#define SOP_K_MAXP 28                /* pairs i < j among SOP_K_MAXA atoms           */
#define SOP_K_NCOL (SOP_K_MAXA + SOP_K_MAXP + 1)   /* sum columns: atoms, pairs, zero-norm lane count */
#define SOP_K_ZCOL (SOP_K_MAXA + SOP_K_MAXP)
#define SOP_K_REPL 8                 /* replicas of the layer sums (spreads same-address atomics) */
#define SOP_K_MAXBINS 1024           /* bins of the element-search table                        */
#define SOP_K_MAXTABCODES 2048       /* scale codes whose (scale, reciprocal) pair is tabulated */
#define SOP_K_BIN_WORDS (4 * SOP_K_MAXA + 1)   /* words of one bin record (odd: conflict-free banks)  */
#define SOP_K_BIN_BYTES (4 * SOP_K_BIN_WORDS)
#define SOP_K_BIN_MAGIC 12582912.0f  /* 1.5 * 2^23: one unit in the last place is 1               */
/* bits(MAGIC + v) = 0x4B400000 + v; the 24-bit multiply sees 0x400000 + v: subtract its product */
#define SOP_K_BIN_NEGC (0u - 0x400000u * (unsigned)SOP_K_BIN_BYTES)
/* The bin table covers scaled weights from BIN_EXT * L[0] to BIN_EXT * L[N-1]: a block scale that
 * was rounded down (by at most a factor 1.5, in the subnormal range of the scale word) leaves every
 * scaled weight inside the table without a clamp.  Blocks whose scale saturated take a clamped path,
 * selected when ideal scale / rounded scale exceeds BIN_SAFE. */
#define SOP_K_BIN_EXT 1.5625f
#define SOP_K_BIN_SAFE 1.55f

#if defined(__HIPCC__) || defined(__HIP__)
#define SOP_K_HD __host__ __device__
#else
#define SOP_K_HD
struct float2 { float x, y; };       /* (host-only translation units see the launch parameters' layout without a HIP header) */
#endif

/* position of (i,j), i < j, in the lexicographic list of all pairs of SOP_K_MAXA atoms */
SOP_K_HD constexpr int pair_index(int i, int j) { return i * (2 * SOP_K_MAXA - i - 1) / 2 + (j - i - 1); }

/* One bin of the element-search table.  For every atom the bin holds at most one code boundary.
 * The two values are stored HALVED (exactly; the element passes multiply by twice the block scale): the boundary
 * between two neighbouring entries then equals the binary32 sum of the two stored values, and the passes that only
 * choose between the values form it with one addition instead of reading it. */
struct BinRec {
    float thr[SOP_K_MAXA];      // the boundary inside the bin (+inf when there is none)
    float ylo[SOP_K_MAXA];      // half of the codebook value at and below the boundary
    float yhi[SOP_K_MAXA];      // half of the codebook value above the boundary
    int   code_lo[SOP_K_MAXA];  // code at and below the boundary
    int   pad;
};

/* Atoms are handled in an internal order in which atoms with equal endpoints (one "scale group":
 * same ideal scale, same scale code, same scaled weights) are adjacent, and an atom that is the
 * sign-negated copy of another follows it directly where the grouping allows. */
struct KParams {
    // inputs
    const void*   W;
    const float*  c;
    const BinRec* bins;              // [n_bins], atoms in internal order
    const float2* stab;              // [n_tab_codes] (twice the scale value(q) * 2^-k, the scale's reciprocal), or null
    long long M, K, ldw;             // as the kernel walks the layer: rows may be folded (see Kc)
    long long Kc;                    // true row length.  When the rows lie back to back (ldw == K) and 64 lanes do not divide a
                                     // row's lanes, the host folds f rows into one of f*K columns (M/f rows): the last strip of
                                     // every row then wastes fewer lanes (none when 64 divides f*K/EPL).  Block and element
                                     // indices are unchanged by this; only the channel of a column becomes its index modulo Kc.
    long long Bk;                    // blocks per row
    long long Nb;                    // blocks in the layer
    long long strips;                // 64-lane strips per row
    long long total_units;           // strips * M
    long long n_waves;               // wavefronts launched (multiple of 4)
    unsigned int M32, m_magic;       // M, and floor(2^32 / M) (2^32 - 1 for M = 1): step number -> (strip, row)
    int A, P, lpb;
    int n_bins;
    int n_tab_codes;                 // 0: scale and reciprocal are computed arithmetically
    // scale word
    int man_bits, bias, max_code, k;
    float pow2k;                     // 2^k
    float sub_quantum;               // 2^(1-bias-man_bits-k)
    // atoms, internal order
    float tpos[SOP_K_MAXA], tneg[SOP_K_MAXA];      // t+ and -t-
    float bin_sc[SOP_K_MAXA], bin_off[SOP_K_MAXA]; // bin = bits(fma(x, sc, off)) - bits(magic)
    float bin_lo[SOP_K_MAXA], bin_hi[SOP_K_MAXA];  // range of x the table covers (clamped path)
    unsigned int gid_w;                            // 4 bits per atom: its scale group (atoms of a group are adjacent)
    unsigned int mirror_mask;                      // bit a: atom a is the sign-negated copy of atom a-1 (signed scale words take its candidates over)
    unsigned int selfsym_mask;                     // bit a: atom a is its own sign-negated copy
    alignas(8) unsigned char nent[SOP_K_MAXA];     // entries of the atom
    unsigned int unit_tpos, unit_tneg;             // bit a: the endpoint is exactly 1 (no division needed)
    unsigned int wide_mask;                        // bit a: more than 16 entries (one byte per code)
    alignas(8) unsigned char uidx[SOP_K_MAXA];     // caller's index of the atom
    long long code_off[SOP_K_MAXA];                // byte offset of the atom's code plane
    unsigned int pair_mask;                           // bit pair_index(i,j): the pair is requested
    unsigned int flip_mask;                           // bit pair_index(i,j): the caller's first atom is internal j
    unsigned int flip_slots;                          // bit q: output pair q is such a swapped pair
    // (byte arrays sit on 8-byte boundaries so that the kernels fetch them with scalar loads)
    unsigned int pair_slot_w[SOP_K_MAXP / 4];          // byte pi%4 of word pi/4: output index of pair pi = pair_index(i,j)
    alignas(8) unsigned char pair_pi[SOP_K_MAXP + 4];  // pair_index(i,j) of output o
    // outputs
    // layer sums of 1-cos in fixed point (2^-22 units): every workgroup adds its share with integer
    // atomics (order-independent, so the result is reproducible); the workgroup that finishes last
    // turns them into the ACos outputs and leaves sums and counter at zero for the next call
    unsigned long long* sums;        // [SOP_K_REPL][SOP_K_NCOL]
    unsigned int* done;              // workgroups finished (zero between calls; room for 1 + SOP_K_REPL words)
    double*   acos_pair;
    double*   acos_atom;
    void*     sel_words;             // [Nb] selector word of every block
    int       sel_u32;               // 1: 32-bit selector words, 0: 16-bit
    uint16_t* scale_code;
    uint8_t*  codes;
    float*    blk_cos;
    float*    blk_err;
    float*    blk_rank;              // [A][Nb] ranking score of step 2 (signed squared block cosine, binary32 decision quantity)
    // model-wide kernel: the layers of one launch (W, c, M, K, ldw, Nb, sel_words above are then unused); sums is
    // [n_layers][SOP_K_REPL][SOP_K_NCOL], acos_pair / acos_atom are tables with rows of P / A values (a layer names its row)
    const struct LayerDesc* layers;
    int n_layers;
};

/* One layer of a model-wide launch (72 bytes, read with scalar loads) */
struct LayerDesc {
    const void*  W;
    const float* c;
    void*        sel_words;          // or NULL
    long long    ldw;
    long long    Nb;
    int          Bk;
    int          out_row;            // row of the ACos tables this layer's results go to
    unsigned int M32, m_magic;       // rows, floor(2^32 / rows)
    int          K;
    unsigned int total_units;        // strips * rows
    int          Kc;                 // true row length (rows may be folded as in KParams)
    int          pad;
};

/* Statistics pass of the data-derived codebook */
#define SOP_K_DD_THREADS 1024
#define SOP_K_DD_MAXBINS 8192
struct DdParams {
    const void*  W;
    const float* c;                  // null: uniform weights
    const unsigned char* block_mask; // null: every block; else [M*K/g], non-zero = the block enters
    int n_levels;                    // 0: plain mask.  L >= 1: the mask byte is a level 0..L; a block of level l >= 1 enters
                                     // histogram l-1 of L (n_bins bins each), and the result holds, for every j, the sum of
                                     // the histograms j .. L-1 (the pool of every block of level > j)
    int n_planes;                    // levels only: P >= 1 level planes, plane_stride bytes apart (one per codebook whose pools are
    long long plane_stride;          // wanted): one pass over the weights fills P * L histograms, laid out [plane][level][bin]
    long long M, K, ldw, Bk;
    long long row_step, Ms;          // every row_step-th row is used: Ms = ceil(M / row_step) rows
    long long strips, total_units, n_waves;  // total_units = strips * Ms
    int n_bins;
    unsigned long long* acc;         // [n_bins] running histogram of the layer (zero between calls)
    unsigned int* done;              // workgroups finished
    long long* hist;                 // [n_bins] output
};

/* Statistics pass of the per-layer scale shift */
#define SOP_K_FL_THREADS 1024
#define SOP_K_FL_BINS 320            /* binary exponents -160 .. 159 of sc = m * 2^e, 1/2 <= m < 1 */
struct FlParams {
    const void* W;
    long long M, K, ldw;
    long long strips, total_units, n_waves;
    int units_per_wg, units_rem;     // total_units = workgroups * units_per_wg + units_rem
    float t_pos, t_neg;              // endpoints t+ and -t- of the codebook
    float m_top;                     // m of the scale format's largest value
    unsigned long long* acc;         // [2 * SOP_K_FL_BINS] running counts (zero between calls)
    unsigned int* done;
    long long* hist;                 // [2][SOP_K_FL_BINS] output
};

/* Read-rate calibration kernel: workgroups (of 256 threads) of one launch */
#define SOP_K_PROBE_WG 2048

/* Layer-scope weight formats and the binary64 sum */
#define SOP_K_LS_MAXWG 2048
#define SOP_K_LS_MAXREP 64           /* copies of the running layer maxima */
struct LsParams {
    const void*  W;                  // weights (or the binary32 array of the sum kernel)
    const float* c;                  // null: c = 1
    long long M, K, ldw;
    long long strips, total_units, n_waves;   // sum kernel: total_units = number of elements
    int w_man, w_bias, w_max_code;   // weight grid ExMy
    int s_man, s_bias, s_max_code;   // scale word
    int k;
    float pow2k;
    unsigned int* maxbits;           // [SOP_K_LS_MAXREP][32], two words used: bit patterns of the largest positive / negative weight (zero between calls)
    unsigned long long* part;        // [SOP_K_LS_MAXWG][3] workgroup partials (bit patterns of doubles)
    unsigned int* done;              // [17] tickets: over the groups, then per group of workgroups
    double* out;                     // [4] weighted error, plain error, ||W||_c^2, scale code   (sum kernel: [1])
    uint16_t* codes;                 // optional [M*K] index into the ascending signed grid
};

/* Ranking of the blocks by a per-block score (exact selection of the score of a given rank) */
#define SOP_K_SEL_THREADS 256         /* pool-mask kernel */
#define SOP_K_CNT_THREADS 1024        /* counting kernels */
#define SOP_K_SEL_BINS 2048          /* 11 + 11 + 10 bits of the 32-bit key over three passes */
struct SelParams {
    const float* score;              // [n]
    long long n, n_top;              // 1 <= n_top <= n (n_top == 0: all_b)
    int higher;                      // 1: a larger score ranks better
    int all_b;                       // 1: every block goes to the second pool
    unsigned int* hist;              // [3][SOP_K_SEL_BINS] digit counts of the passes (zero when the call starts)
    unsigned int* hist_other;        // [3][SOP_K_SEL_BINS] the set the next call counts into: cleared by this call
    unsigned char* pool_b;           // [n] 1 = ranked strictly worse than the threshold
    float* tau;                      // [1] the threshold score
    long long* n_a;                  // [1] blocks that stay in the first pool
};

/* Ranking with several thresholds at once (the sweep over the partition parameter p): nested pools */
#define SOP_K_SEL_MAXLEV 8
#define SOP_K_SELM_WORDS ((1 + 2 * SOP_K_SEL_MAXLEV) * SOP_K_SEL_BINS)   /* one set of digit counts */
/* what the passes of such a ranking hand on, per score plane (written by a one-workgroup kernel after each counting pass) */
struct SelMState {
    unsigned int prefix[SOP_K_SEL_MAXLEV];       // digits of every threshold's key fixed so far
    unsigned int rank_in[SOP_K_SEL_MAXLEV];      // rank wanted among the keys with those digits
    unsigned int above[SOP_K_SEL_MAXLEV];        // keys above those digits
    int alias[SOP_K_SEL_MAXLEV];                 // first threshold with the same digits so far (its histogram is the one used)
    unsigned long long tkey[SOP_K_SEL_MAXLEV];   // after the last pass: the threshold's key (2^32: every block ranks worse)
};
struct SelMParams {
    const float* score;              // [n]
    long long n;
    int higher;                      // 1: a larger score ranks better
    int n_levels;                    // thresholds, 1 .. SOP_K_SEL_MAXLEV
    long long n_top[SOP_K_SEL_MAXLEV];   // non-decreasing sizes of the first pool (0: every block goes to the second pool)
    unsigned int* hist;              // pass 0: [SOP_K_SEL_BINS]; pass 1: [MAXLEV][BINS]; pass 2: [MAXLEV][BINS] (zero when the call starts)
    unsigned int* hist_other;        // the set the next call counts into: cleared by this call
    unsigned char* level;            // [n] number of thresholds the block ranks strictly worse than
    float* tau;                      // [n_levels] threshold scores
    long long* n_a;                  // [n_levels] blocks at least as good as the threshold
    SelMState* state;                // [n_planes]
    // several score planes in one launch (blockIdx.y names the plane): plane q reads score + q * n, counts into
    // hist + q * SOP_K_SELM_WORDS and writes level + q * n, tau / n_a + q * SOP_K_SEL_MAXLEV
    int n_planes;
    int n_clear;                     // planes of hist_other that hold counts (the calls that counted into that set may have
                                     // had more planes than this one): all of them are cleared
};

/* Packing of scale words and code payloads */
struct PackParams {
    long long Nb, Bk;                // blocks, blocks per row
    long long M, K;
    int g, n_bits;
    int wide_a, wide_b;              // 1: the atom's plane holds one byte per code (else two codes per byte)
    const uint16_t* scale_a; const uint16_t* scale_b;   // [Nb] bit 15 = sign, low bits = magnitude code
    const unsigned char* codes_a; const unsigned char* codes_b;
    const void* sel_words;           // null: single codebook
    int sel_u32, pair_q;
    int sign_pos, mag_shift, sel_pos;   // bit positions inside the container (-1: absent)
    uint16_t* words;                 // [Nb]
    unsigned char* payload;          // [Nb][g*n_bits/8]
};
#endif
