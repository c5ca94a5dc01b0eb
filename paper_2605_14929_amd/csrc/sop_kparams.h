// Launch parameters shared by the host side of the library and its kernels (passed by value).
#ifndef SOP_KPARAMS_H
#define SOP_KPARAMS_H
#include <stdint.h>

#define SOP_K_MAXA 8                 /* atoms                                        */
#define SOP_K_MAXP 28                /* pairs i < j among SOP_K_MAXA atoms           */
#define SOP_K_NCOL (SOP_K_MAXA + SOP_K_MAXP)
#define SOP_K_MAXBINS 512            /* bins of the element-search table                        */
#define SOP_K_MAXTABCODES 2048       /* scale codes whose (scale, reciprocal) pair is tabulated */
#define SOP_K_BIN_WORDS (4 * SOP_K_MAXA + 1)   /* words of one bin record (odd: conflict-free banks)  */
#define SOP_K_BIN_BYTES (4 * SOP_K_BIN_WORDS)
#define SOP_K_BIN_MAGIC 12582912.0f  /* 1.5 * 2^23: one unit in the last place is 1               */
/* bits(MAGIC + v) = 0x4B400000 + v; the 24-bit multiply sees 0x400000 + v: subtract its product */
#define SOP_K_BIN_NEGC (0u - 0x400000u * (unsigned)SOP_K_BIN_BYTES)

#if defined(__HIPCC__)
#define SOP_K_HD __host__ __device__
#else
#define SOP_K_HD
#endif

/* position of (i,j), i < j, in the lexicographic list of all pairs of SOP_K_MAXA atoms */
SOP_K_HD constexpr int pair_index(int i, int j) { return i * (2 * SOP_K_MAXA - i - 1) / 2 + (j - i - 1); }

/* One bin of the element-search table.  For every atom the bin holds at most one code boundary. */
struct BinRec {
    float thr[SOP_K_MAXA];      // the boundary inside the bin (+inf when there is none)
    float ylo[SOP_K_MAXA];      // codebook value at and below the boundary
    float yhi[SOP_K_MAXA];      // codebook value above the boundary
    int   code_lo[SOP_K_MAXA];  // code at and below the boundary
    int   pad;
};

/* Atoms are handled in an internal order in which atoms with equal endpoints (one "scale group":
 * same ideal scale, same scale code, same scaled weights) are adjacent. */
struct KParams {
    // inputs
    const void*   W;
    const float*  c;
    const BinRec* bins;              // [n_bins], atoms in internal order
    const float2* stab;              // [n_tab_codes] (scale * 2^-k, its reciprocal), or null
    long long M, K, ldw;
    long long Bk;                    // blocks per row
    long long Nb;                    // blocks in the layer
    long long Wr;                    // selector words per row
    long long strips;                // 64-lane strips per row
    long long total_units;           // strips * M
    long long n_waves;               // wavefronts launched (multiple of 4)
    int A, P, lpb;
    int n_bins;
    int n_tab_codes;                 // 0: scale and reciprocal are computed arithmetically
    // scale word
    int man_bits, bias, max_code, k;
    float pow2k;                     // 2^k
    float sub_quantum;               // 2^(1-bias-man_bits-k)
    // atoms, internal order
    float tpos[SOP_K_MAXA], tneg[SOP_K_MAXA];      // t+ and -t-
    float bin_sc[SOP_K_MAXA], bin_off[SOP_K_MAXA]; // bin = bits(fma(clamp(x), sc, off)) - bits(magic)
    unsigned int grp_first_mask;                   // bit a: first atom of its scale group
    unsigned int unit_tpos, unit_tneg;             // bit a: the endpoint is exactly 1 (no division needed)
    unsigned int wide_mask;                        // bit a: more than 16 entries (one byte per code)
    unsigned char uidx[SOP_K_MAXA];                // caller's index of the atom
    long long code_off[SOP_K_MAXA];                // byte offset of the atom's code plane
    unsigned int pair_mask;                           // bit pair_index(i,j): the pair is requested
    unsigned int flip_mask;                           // bit pair_index(i,j): the caller's first atom is internal j
    signed char pair_slot[SOP_K_MAXP];                // output index of pair pair_index(i,j), or -1
    unsigned char pair_col[SOP_K_MAXP];               // rank of output o's pair among the requested pairs, by pair_index
    // outputs
    float*    partial;               // [NCOL][n_waves/4] per-workgroup sums of 1-cos
    double*   acos_pair;
    double*   acos_atom;
    uint32_t* sel_bits;
    uint16_t* scale_code;
    uint8_t*  codes;
    float*    blk_cos;
    float*    blk_err;
};
#endif
