// Driver of the CPU sanitizer build: the library's host-only translation unit (sop_host.cpp) and the C oracle
// (oracle/sop_oracle.c), compiled with -fsanitize=address,undefined, are run through their entry points on
// small inputs, error paths included.  tests/test_host_sanitize.py builds and runs it; any report of a
// sanitizer, any unexpected status or a disagreement between the two sides' atom builders fails the test.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/sop.h"
#include "../paper_2605_14929_amd/csrc/sop_host.h"

extern "C" {
typedef struct { int sign_bits, exp_bits, man_bits, bias, max_code; } sopo_fmt;
double sopo_scale_value(const sopo_fmt* f, int q);
int sopo_scale_encode(const sopo_fmt* f, float sp);
int sopo_scale_encode_exhaustive(const sopo_fmt* f, float sp);
int sopo_pair_search(const float* W, int64_t M, int64_t K, int64_t ldw, const float* c, int g, int n_atoms, const int* n_entries,
                     const float* atoms, int n_pairs, const int* pair_ab, const sopo_fmt* fmt, int k, int metric, int scale_rule,
                     double* acos_pair, double* acos_atom, uint32_t* sel_words, uint16_t* scale_code, uint8_t* codes, float* blk_err,
                     float* blk_cos, float* blk_rank, int n_threads);
}

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("CHECK failed line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uni() { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return ((rng_state >> 11) + 0.5) / 9007199254740992.0; }
static double gauss() { return std::sqrt(-2.0 * std::log(uni())) * std::cos(6.283185307179586 * uni()); }

int main()
{
    // ---- atom builders and their error paths ----
    std::vector<std::vector<float>> nf(7), sh(7);
    for (int n = 2; n <= 6; ++n) { nf[n].resize(1u << n); CHECK(sop_atom_nf(n, nf[n].data()) == SOP_OK); CHECK(nf[n].front() == -1.0f && nf[n].back() == 1.0f); }
    for (int n = 1; n <= 6; ++n) { sh[n].resize(1u << n); CHECK(sop_atom_sh(n, 1.5, -0.02, sh[n].data()) == SOP_OK); }
    CHECK(sop_atom_nf(1, nf[2].data()) == SOP_EINVAL && sop_atom_nf(7, nf[2].data()) == SOP_EINVAL && sop_atom_nf(4, nullptr) == SOP_EINVAL);
    CHECK(sop_atom_sh(4, -1.0, 0.0, sh[4].data()) == SOP_EINVAL);
    std::vector<float> nnf(16), nsh(16), bof(16), nbof(16);
    CHECK(sop_atom_negate(nf[4].data(), 16, nnf.data()) == SOP_OK && sop_atom_negate(sh[4].data(), 16, nsh.data()) == SOP_OK);
    std::vector<double> draws(1 << 14);
    for (double& d : draws) d = gauss();
    CHECK(sop_atom_bof(4, draws.data(), (int64_t)draws.size(), 16, 30, bof.data()) == SOP_OK);
    CHECK(bof.front() == -1.0f && bof.back() == 1.0f);
    CHECK(sop_atom_bof(4, draws.data(), 8, 16, 30, bof.data()) == SOP_EINVAL);
    CHECK(sop_atom_negate(bof.data(), 16, nbof.data()) == SOP_OK);
    {
        std::vector<double> x(1000), cent = {0.1, 0.4, 0.9};
        for (size_t i = 0; i < x.size(); ++i) x[i] = (i + 0.5) / x.size();
        CHECK(sop_lloyd_1d(x.data(), nullptr, (int64_t)x.size(), cent.data(), 3, 200) == SOP_OK);
        CHECK(std::fabs(cent[0] - 1.0 / 6) < 2e-3 && std::fabs(cent[1] - 0.5) < 2e-3 && std::fabs(cent[2] - 5.0 / 6) < 2e-3);
        CHECK(sop_lloyd_1d(x.data(), nullptr, 0, cent.data(), 3, 1) == SOP_EINVAL);
    }
    // ---- element-search table: construction and self check ----
    auto atom = [](const std::vector<float>& v) { sop_atom a; a.n_entries = (int)v.size(); a.values = v.data(); return a; };
    {
        sop_atom six[6] = {atom(nf[4]), atom(sh[4]), atom(bof), atom(nnf), atom(nsh), atom(nbof)};
        int nb = 0; int64_t nc = 0;
        CHECK(sop_check_alphabet(six, 6, &nb, &nc) == SOP_OK && nb >= 16 && nc > 100000);
        sop_atom five[4] = {atom(nf[5]), atom(sh[5]), atom(nf[6]), atom(sh[3])};
        CHECK(sop_check_alphabet(five, 4, &nb, nullptr) == SOP_OK);
        std::vector<double> grid(2 * 64 + 1); int ng = 0;
        sop_weight_fmt e2m3 = {2, 3, -1, -1};
        CHECK(sop_weight_grid(e2m3, 0.0, grid.data(), &ng) == SOP_OK && ng == 63);
        std::vector<float> g63(63);
        for (int i = 0; i < 63; ++i) g63[i] = (float)(grid[i] / 7.5);
        sop_atom one[1] = {atom(g63)};
        CHECK(sop_check_alphabet(one, 1, &nb, nullptr) == SOP_OK);
        std::vector<float> bad = {0.5f, -0.5f}, onesided = {0.1f, 0.5f}, close = {-1.0f, 0.0f, 1e-6f, 2e-6f, 1.0f};
        sop_atom b1[1] = {atom(bad)}, b2[1] = {atom(onesided)}, b3[1] = {atom(close)};
        CHECK(sop_check_alphabet(b1, 1, nullptr, nullptr) == SOP_EATOM && sop_check_alphabet(b2, 1, nullptr, nullptr) == SOP_EATOM);
        CHECK(sop_check_alphabet(b3, 1, nullptr, nullptr) == SOP_EATOM);
        CHECK(sop_check_alphabet(six, 9, nullptr, nullptr) == SOP_EATOM && sop_check_alphabet(nullptr, 1, nullptr, nullptr) == SOP_EINVAL);
        CHECK(soph::host_last_error()[0] != 0);                     // (what sop_last_error(NULL) returns)
    }
    // ---- fits on histograms ----
    {
        const int H = 1024;
        std::vector<int64_t> hist(H, 0);
        for (int i = 0; i < 200000; ++i) {
            double x = gauss() * 0.35; x = x < -1 ? -1 : (x > 1 ? 1 : x);
            int b = (int)std::floor(x * H / 2 + H / 2); b = b < 0 ? 0 : (b > H - 1 ? H - 1 : b);
            hist[b] += 1 + (int64_t)(uni() * 1000);
        }
        std::vector<float> out(16);
        CHECK(sop_dd_fit(hist.data(), H, 16, 20, nf[4].data(), out.data()) == SOP_OK);
        for (int j = 0; j + 1 < 16; ++j) CHECK(out[j] < out[j + 1]);
        CHECK(sop_dd_fit(hist.data(), 1000, 16, 20, nf[4].data(), out.data()) == SOP_EINVAL);
        std::vector<int64_t> empty(H, 0);
        (void)sop_dd_fit(empty.data(), H, 16, 5, nf[4].data(), out.data());             // an empty histogram keeps the start grid
        std::vector<double> grid(2 * 256 + 1); int ng = 0;
        sop_weight_fmt e4m3 = {4, 3, -1, -1};
        CHECK(sop_weight_grid(e4m3, 0.0, grid.data(), &ng) == SOP_OK && ng == 255);
        for (int i = 0; i < ng; ++i) grid[i] /= 480.0;
        std::vector<int> chosen(16); double cost = -1;
        CHECK(sop_dd_fit_grid(hist.data(), H, grid.data(), ng, 16, chosen.data(), &cost) == SOP_OK && cost >= 0);
        for (int j = 0; j + 1 < 16; ++j) CHECK(chosen[j] < chosen[j + 1] && chosen[j] >= 0 && chosen[j + 1] < ng);
        CHECK(sop_dd_fit_grid(hist.data(), H, grid.data(), 8, 16, chosen.data(), nullptr) == SOP_EINVAL);
        std::swap(grid[3], grid[4]);
        CHECK(sop_dd_fit_grid(hist.data(), H, grid.data(), ng, 16, chosen.data(), nullptr) == SOP_EATOM);
        sop_weight_fmt badw = {9, 3, -1, -1};
        CHECK(sop_weight_grid(badw, 0.0, grid.data(), &ng) == SOP_EFMT);
    }
    // ---- layer shift ----
    {
        std::vector<int64_t> h(640, 0);
        for (int e = -20; e <= -8; ++e) { h[e + 160] = 1000 + e; h[320 + e + 160] = 10; }
        const sop_scale_fmt fmts[3] = {{0, 4, 4, 8, -1, -1}, {1, 4, 3, 8, -1, -1}, {1, 8, 7, 16, 119, 244 * 128 + 127}};
        for (const sop_scale_fmt& f : fmts) {
            int k = 999; double frac = -1;
            CHECK(sop_layer_shift(h.data(), 20000, f, &k, &frac) == SOP_OK && k >= -64 && k <= 64 && frac >= 0 && frac <= 1);
        }
        sop_scale_fmt bad = {0, 9, 4, 16, -1, -1}; int k;
        CHECK(sop_layer_shift(h.data(), 20000, bad, &k, nullptr) == SOP_EFMT && sop_layer_shift(h.data(), 0, fmts[0], &k, nullptr) == SOP_EINVAL);
    }
    // ---- the oracle: every block size, metric, sign mode and scale rule, every output, two threads ----
    {
        const int64_t M = 6, K = 256;
        std::vector<float> W(M * K), c(K);
        for (float& v : W) v = (float)(gauss() / std::sqrt(uni() + 0.05));
        for (int i = 0; i < 16; ++i) W[K + i] = 0.0f;                                    // a zero block
        W[2 * K + 5] = 1e-30f; W[3 * K + 7] = 3e6f;
        for (float& v : c) v = (float)std::exp(gauss());
        c[9] = 0.0f;
        std::vector<float> flat;
        const std::vector<float>* tabs[4] = {&nf[4], &sh[4], &nnf, &nf[5]};
        int nent[4], pairs[12], np = 0;
        for (int a = 0; a < 4; ++a) { nent[a] = (int)tabs[a]->size(); flat.insert(flat.end(), tabs[a]->begin(), tabs[a]->end()); }
        for (int a = 0; a < 4; ++a) for (int b = a + 1; b < 4; ++b) { pairs[2 * np] = a; pairs[2 * np + 1] = b; ++np; }
        const sopo_fmt fmts[3] = {{0, 4, 4, 7, 255}, {1, 4, 3, 7, 127}, {1, 8, 7, 119, 244 * 128 + 127}};
        for (int g : {8, 16, 32, 64})
            for (const sopo_fmt& f : fmts)
                for (int metric = 0; metric < 3; ++metric)
                    for (int rule = 0; rule < 2; ++rule) {
                        if (rule == 1 && f.sign_bits == 0) continue;
                        const int64_t Nb = M * K / g;
                        std::vector<double> ap(np), aa(4);
                        std::vector<uint32_t> sel(Nb);
                        std::vector<uint16_t> sc(4 * Nb);
                        std::vector<uint8_t> codes(3 * M * K / 2 + M * K);
                        std::vector<float> be(4 * Nb), bc(4 * Nb), br(4 * Nb);
                        const int rc = sopo_pair_search(W.data(), M, K, K, c.data(), g, 4, nent, flat.data(), np, pairs, &f, g == 16 ? 2 : 0, metric, rule,
                                                        ap.data(), aa.data(), sel.data(), sc.data(), codes.data(), be.data(), bc.data(), br.data(), 2);
                        CHECK(rc == 0);
                        for (double v : aa) CHECK(v > 0.5 && v <= 1.0 + 1e-12);
                    }
        CHECK(sopo_pair_search(W.data(), M, 250, 250, c.data(), 16, 4, nent, flat.data(), np, pairs, &fmts[0], 0, 0, 0,
                               nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 1) < 0);
        for (const sopo_fmt& f : fmts)
            for (int i = 0; i < 2000; ++i) {
                const float s = (float)std::exp((uni() - 0.5) * 40.0);
                CHECK(sopo_scale_encode(&f, s) == sopo_scale_encode_exhaustive(&f, s));
            }
    }
    if (failures) { std::printf("%d checks failed\n", failures); return 1; }
    std::printf("sanitize ok\n");
    return 0;
}
