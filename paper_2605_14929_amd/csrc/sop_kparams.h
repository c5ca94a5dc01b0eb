// Launch parameters shared by the host side of the library and its kernels (passed by value).
#ifndef SOP_KPARAMS_H
#define SOP_KPARAMS_H
#include <stdint.h>

#define SOP_K_MAXA 8                 /* atoms                                        */
#define SOP_K_MAXP 28                /* pairs i < j among SOP_K_MAXA atoms           */
#define SOP_K_NCOL (SOP_K_MAXA + SOP_K_MAXP)
#define SOP_K_MAXBINS 1024           /* bins of the element-search table per atom    */
#define SOP_K_MAXTABCODES 2048       /* scale codes whose (scale, reciprocal) pair is tabulated */
#define SOP_K_BIN_MAGIC 786432.0f    /* 1.5 * 2^19: one unit in the last place is 1/16 */

#if defined(__HIPCC__)
#define SOP_K_HD __host__ __device__
#else
#define SOP_K_HD
#endif

/* position of (i,j), i < j, in the lexicographic list of all pairs of SOP_K_MAXA atoms */
SOP_K_HD constexpr int pair_index(int i, int j) { return i * (2 * SOP_K_MAXA - i - 1) / 2 + (j - i - 1); }

/* One record of the element-search table: the bin holds at most one code boundary. */
struct alignas(16) BinRec {
    float thr;       // the boundary inside the bin (+inf when there is none)
    float ylo, yhi;  // codebook value at and below / above the boundary
    int   code_lo;   // code at and below the boundary
};

/* Atoms are handled in an internal order in which atoms with equal endpoints (one "scale group":
 * same ideal scale, same scale code, same scaled weights) are adjacent. */
struct KParams {
    // inputs
    const void*   W;
    const float*  c;
    const BinRec* bins;              // [A][n_bins], internal atom order
    const float2* stab;              // [n_tab_codes] (scale * 2^-k, its reciprocal), or null
    long long M, K, ldw;
    long long Bk;                    // blocks per row
    long long Nb;                    // blocks in the layer
    long long Wr;                    // selector words per row
    long long strips;                // 64-lane strips per row
    long long total_units;           // strips * M
    long long n_waves;               // wavefronts launched (multiple of 4)
    int A, P, lpb;
    int n_bins;                      // power of two
    int n_tab_codes;                 // 0: scale and reciprocal are computed arithmetically
    // scale word
    int man_bits, bias, max_code, k;
    float pow2k;                     // 2^k
    float sub_quantum;               // 2^(1-bias-man_bits-k)
    // atoms, internal order
    float tpos[SOP_K_MAXA], tneg[SOP_K_MAXA];      // t+ and -t-
    float bin_sc[SOP_K_MAXA], bin_off[SOP_K_MAXA]; // bin = floor(fma(clamp(x), sc, off)) - magic
    int nent[SOP_K_MAXA];
    unsigned char grp_first[SOP_K_MAXA];           // 1: first atom of its scale group
    unsigned char uidx[SOP_K_MAXA];                // caller's index of the atom
    long long code_off[SOP_K_MAXA];                // byte offset of the atom's code plane
    signed char pair_slot[SOP_K_MAXA * SOP_K_MAXA];   // [i*MAXA+j], i<j internal: output index or -1
    unsigned char pair_flip[SOP_K_MAXA * SOP_K_MAXA]; // 1: the caller's first atom is internal j
    unsigned char pair_col[SOP_K_MAXP];               // pair_index(i,j) of output o
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
