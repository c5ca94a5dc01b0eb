// Launch parameters shared by the host side of the library and its kernels (passed by value).
#ifndef SOP_KPARAMS_H
#define SOP_KPARAMS_H
#include <stdint.h>

#define SOP_K_MAXA 8                 /* atoms                                        */
#define SOP_K_MAXP 28                /* pairs a < b among SOP_K_MAXA atoms           */
#define SOP_K_TAB 64                 /* padded table length per atom                 */

#if defined(__HIPCC__) || defined(__CUDACC__)
#define SOP_K_HD __host__ __device__
#else
#define SOP_K_HD
#endif

/* position of (a,b), a < b, in the lexicographic list of all pairs of SOP_K_MAXA atoms */
SOP_K_HD constexpr int pair_index(int a, int b) { return a * (2 * SOP_K_MAXA - a - 1) / 2 + (b - a - 1); }

struct KParams {
    // inputs
    const void*  W;
    const float* c;
    const float* tab_mid;            // [MAXA][TAB] midpoints, padded with +inf
    const float* tab_val;            // [MAXA][TAB] values
    long long M, K, ldw;
    long long Bk;                    // blocks per row
    long long Nb;                    // blocks in the layer
    long long Wr;                    // selector words per row
    long long strips;                // 64-lane strips per row
    long long total_units;           // strips * M
    long long n_waves;               // wavefronts launched (multiple of 4)
    int A, P, lpb;
    // scale word
    int man_bits, bias, max_code, k;
    float pow2k;                     // 2^k
    float sub_quantum;               // 2^(1-bias-man_bits-k)
    // atoms
    float tpos[SOP_K_MAXA], tneg[SOP_K_MAXA];   // t+ and -t-
    int half0[SOP_K_MAXA];           // first step of the binary search (padded length / 2)
    int nent[SOP_K_MAXA];
    long long code_off[SOP_K_MAXA];
    signed char pair_slot[SOP_K_MAXA * SOP_K_MAXA];   // output index of pair (a,b) or -1
    unsigned char pair_col[SOP_K_MAXP];               // pair_index(a,b) of output o
    // outputs
    float*    partial;               // [n_waves][MAXA+MAXP]
    double*   acos_pair;
    double*   acos_atom;
    uint32_t* sel_bits;
    uint16_t* scale_code;
    uint8_t*  codes;
    float*    blk_cos;
    float*    blk_err;
};
#endif
