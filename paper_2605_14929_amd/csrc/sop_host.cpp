// Host-only part of libsop_hip.so: see sop_host.h.  Nothing here touches the GPU or includes a HIP header.
#include "sop_host.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>

using soph::AlphabetPlan;
using soph::dd_bins_ok;
using soph::FmtRange;
using soph::resolve_fmt;

namespace {
thread_local std::string g_host_err;
uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
float u2f(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }
// order-preserving map between finite floats and integers
int64_t ford(float f) { const uint32_t u = f2u(f); return (u & 0x80000000u) ? -(int64_t)(u & 0x7FFFFFFFu) : (int64_t)u; }
float funord(int64_t k) { return k < 0 ? u2f(0x80000000u | (uint32_t)(-k)) : u2f((uint32_t)k); }


sop_status planfail(std::string* err, sop_status s, const char* msg) { if (err) *err = msg; return s; }
}  // namespace

sop_status soph::host_fail(sop_status s, const std::string& msg) { g_host_err = msg; return s; }
const char* soph::host_last_error() { return g_host_err.c_str(); }

// Bin of a scaled weight, exactly as the kernel computes it: clamp to the range the table covers
// (the kernel skips the clamp when it knows the value is inside), one fma whose constant term
// carries 1.5*2^23 (so the sum is rounded to an integer), bin = low bits.
static int bin_of(float x, float xl, float xh, float sc, float off)
{
    const float xc = std::fmin(std::fmax(x, xl), xh);
    const float t = std::fmaf(xc, sc, off);
    return (int)(f2u(t) - f2u(SOP_K_BIN_MAGIC));
}

// Fill atom slot `ia` of the bin records for the table range [xl, xh] (wider than the atom: values
// beyond the atom's endpoints take its first / last entry); false when some bin would hold two code
// boundaries or the binning leaves [0, n_bins).
static bool build_bins(const std::vector<float>& L, float xl, float xh, float sc, float off, int n_bins, int ia, BinRec* rec)
{
    const int N = (int)L.size();
    const float inf = std::numeric_limits<float>::infinity();
    std::vector<float> mid(N - 1);
    for (int j = 0; j + 1 < N; ++j) mid[j] = (float)(((double)L[j] + (double)L[j + 1]) * 0.5);
    auto code_of = [&](float x) { int c = 0; for (int j = 0; j + 1 < N; ++j) c += x > mid[j]; return c; };
    const int b_lo = bin_of(xl, xl, xh, sc, off), b_hi = bin_of(xh, xl, xh, sc, off);
    if (b_lo < 0 || b_hi >= n_bins || b_lo > b_hi) return false;
    // Quick rejection (the caller tries bin counts in ascending order, and most fail): two neighbouring code
    // boundaries with a float above the second one still in the first one's bin put two boundaries into
    // that bin.  (Where this does not decide, the full construction below does.)
    for (int j = 0; j + 2 < N; ++j) {
        const int bj = bin_of(mid[j], xl, xh, sc, off);
        if (mid[j] >= xl && mid[j + 1] < xh && bj > b_lo && bj < b_hi && bin_of(mid[j + 1], xl, xh, sc, off) == bj &&
            bin_of(std::nextafter(mid[j + 1], inf), xl, xh, sc, off) == bj)
            return false;
    }
    // first[j] = smallest float in [xl, xh] whose bin is >= j (the binning is monotone in x)
    std::vector<float> first(n_bins + 1, inf);
    for (int j = 0; j <= b_lo; ++j) first[j] = xl;
    for (int j = b_lo + 1; j <= b_hi; ++j) {
        int64_t lo = ford(first[j - 1]), hi = ford(xh);              // bin(lo) < j <= bin(hi)
        if (bin_of(funord(lo), xl, xh, sc, off) >= j) { first[j] = funord(lo); continue; }
        // the bin changes where x*sc + off passes j - 1/2 above the constant: a bracket of a few floats around
        // that x, used if it holds the change (the bisection then takes 7 steps instead of 30)
        {
            const float est = (float)(((double)j - 0.5 + ((double)SOP_K_BIN_MAGIC - (double)off)) / (double)sc);
            if (std::isfinite(est)) {
                const int64_t elo = std::max(lo, ford(est) - 64), ehi = std::min(hi, ford(est) + 64);
                if (elo < ehi && bin_of(funord(elo), xl, xh, sc, off) < j && bin_of(funord(ehi), xl, xh, sc, off) >= j) { lo = elo; hi = ehi; }
            }
        }
        while (hi - lo > 1) {
            const int64_t m = lo + (hi - lo) / 2;
            if (bin_of(funord(m), xl, xh, sc, off) >= j) hi = m; else lo = m;
        }
        first[j] = funord(hi);
    }
    for (int j = 0; j < n_bins; ++j) {
        // floats of bin j: [first[j], pred(first[j+1])]; everything below xl falls into bin(xl),
        // everything above xh into bin(xh)
        int c0 = 0, c1 = 0;
        if (j < b_lo || j > b_hi || !(first[j] < first[j + 1])) {     // never addressed
            c0 = c1 = 0;
        } else {
            c0 = j == b_lo ? 0 : code_of(first[j]);
            c1 = j == b_hi ? N - 1 : code_of(std::nextafter(first[j + 1], -inf));
        }
        if (c1 - c0 > 1) return false;
        rec[j].thr[ia] = c1 > c0 ? mid[c0] : inf;
        rec[j].ylo[ia] = 0.5f * L[c0];               // halves (exact: plan_alphabet refuses entries whose half is not)
        rec[j].yhi[ia] = 0.5f * L[c1];
        rec[j].code_lo[ia] = c0;
    }
    return true;
}


// Validate the atoms, form the scale groups and build the bin table (host only).
sop_status soph::plan_alphabet(std::string* err, const sop_atom* atoms, int n_atoms, AlphabetPlan& pl)
{
    if (!atoms) return planfail(err, SOP_EINVAL, "atoms is NULL");
    if (n_atoms < 1 || n_atoms > SOP_K_MAXA) return planfail(err, SOP_EATOM, "1..8 atoms supported");
    pl.tabs.assign(n_atoms, {});
    pl.n_atoms = n_atoms;
    for (int a = 0; a < n_atoms; ++a) {
        const int N = atoms[a].n_entries;
        const float* L = atoms[a].values;
        if (!L) return planfail(err, SOP_EINVAL, "atom values pointer is NULL");
        if (N < 2 || N > SOP_MAX_ENTRIES) return planfail(err, SOP_EATOM, "an atom needs 2..64 entries");
        for (int j = 0; j < N; ++j) {
            if (!std::isfinite(L[j])) return planfail(err, SOP_EATOM, "atom entry is not finite");
            if (j && !(L[j - 1] < L[j])) return planfail(err, SOP_EATOM, "atom entries must be strictly ascending");
        }
        if (!(L[0] < 0.0f && L[N - 1] > 0.0f)) return planfail(err, SOP_EATOM, "an atom must have a negative first and a positive last entry");
        // the table holds half of every entry, exactly
        for (int j = 0; j < N; ++j) {
            const volatile float h = 0.5f * L[j];
            if (h + h != L[j]) return planfail(err, SOP_EATOM, "atom entry too small: a non-zero entry must be at least 2^-125 in magnitude");
        }
        // The search kernels that write no codes form a code boundary as the binary32 sum of its neighbours' halves
        // instead of reading it.  That sum is the boundary (the binary64 mean rounded once to binary32): both round the
        // same real number once, the binary64 mean being exact whenever its low bits can matter.  Checked, not assumed:
        for (int j = 0; j + 1 < N; ++j) {
            const volatile float hs = 0.5f * L[j] + 0.5f * L[j + 1];
            if (hs != (float)(((double)L[j] + (double)L[j + 1]) * 0.5))
                return planfail(err, SOP_EATOM, "atom entries whose code boundary is not the sum of their halves (not expected for finite entries)");
        }
        pl.tabs[a].assign(L, L + N);
    }
    // Scale groups: equal endpoints; internal order = groups by first appearance.  An atom that is the
    // sign-negated copy of another (L'[k] = -L[N-1-k]) is placed directly after it where it can be: inside a
    // group with symmetric endpoints, and at the seam between a group and the group of mirrored endpoints,
    // which then follows it.  Under a signed scale word such a copy needs no evaluation of its own.
    auto same_ends = [&](int a, int b) { return pl.tabs[a].front() == pl.tabs[b].front() && pl.tabs[a].back() == pl.tabs[b].back(); };
    auto is_copy = [&](int a, int b) {                       // b is the sign-negated copy of a
        const std::vector<float>&A = pl.tabs[a], &B = pl.tabs[b];
        if (A.size() != B.size()) return false;
        for (size_t k = 0; k < A.size(); ++k) if (B[k] != -A[A.size() - 1 - k]) return false;
        // (a boundary at zero is no obstacle: the kernel finds a scaled weight on a code boundary by a floating-point
        // comparison, under which -0 and +0 are equal)
        return true;
    };
    int n = 0, n_groups = 0;
    bool used[SOP_K_MAXA] = {false};
    auto place = [&](int a, int g, int mir) { used[a] = true; pl.order[n] = a; pl.gid[n] = g; pl.mirror[n] = mir; pl.selfsym[n] = is_copy(a, a); ++n; };
    auto copy_of = [&](int a, bool same_group) {             // an unused sign-negated copy of a, inside or outside a's group
        for (int b = 0; b < n_atoms; ++b)
            if (!used[b] && b != a && same_ends(a, b) == same_group && is_copy(a, b)) return b;
        return -1;
    };
    for (int a = 0; a < n_atoms; ++a) {
        if (used[a]) continue;
        const int g = n_groups++;
        std::vector<int> members;
        for (int b = a; b < n_atoms; ++b) if (!used[b] && same_ends(a, b)) members.push_back(b);
        // the member placed last is one whose copy lives in the group of mirrored endpoints (if there is one)
        int seam = -1, seam_copy = -1;
        for (int b : members) { const int cb = copy_of(b, false); if (cb >= 0) { seam = b; seam_copy = cb; break; } }
        for (int b : members) {
            if (used[b] || b == seam) continue;
            place(b, g, 0);
            if (!pl.selfsym[n - 1]) { const int cb = copy_of(b, true); if (cb >= 0) place(cb, g, 1); }
        }
        if (seam >= 0) {
            place(seam, g, 0);
            const int g2 = n_groups++;
            place(seam_copy, g2, 1);
            for (int b = 0; b < n_atoms; ++b) {               // the rest of the mirrored group
                if (used[b] || !same_ends(seam_copy, b)) continue;
                place(b, g2, 0);
                if (!pl.selfsym[n - 1]) { const int cb = copy_of(b, true); if (cb >= 0) place(cb, g2, 1); }
            }
        }
    }
    // smallest bin count for which every bin of every atom holds at most one code boundary.  The
    // table spans SOP_K_BIN_EXT times the atom's range, so that a block whose scale was rounded down
    // needs no clamp.
    static const int kBinCounts[] = {16, 24, 32, 40, 48, 56, 64, 80, 96, 112, 128, 160, 192, 256, 384, 512, 768, 1024};
    for (int nb : kBinCounts) {
        pl.img.assign((size_t)nb, BinRec{});
        bool ok = true;
        for (int i = 0; i < n_atoms && ok; ++i) {
            const std::vector<float>& L = pl.tabs[pl.order[i]];
            const float xl = L.front() * SOP_K_BIN_EXT, xh = L.back() * SOP_K_BIN_EXT;
            // the additive constant is an integer-valued float, so the rounded sum lies within
            // [-0.5, nb-1] of 1.5*2^23: bins 0 .. nb-1
            pl.sc[i] = (float)(((double)nb - 1.5) / ((double)xh - (double)xl));
            pl.off[i] = (float)((double)SOP_K_BIN_MAGIC - (double)xl * (double)pl.sc[i]);
            pl.lo[i] = xl; pl.hi[i] = xh;
            ok = build_bins(L, xl, xh, pl.sc[i], pl.off[i], nb, i, pl.img.data());
        }
        if (ok) { pl.n_bins = nb; break; }
    }
    if (!pl.n_bins) return planfail(err, SOP_EATOM, "atom entries are too closely spaced (two code boundaries within 1/650 of the atom's range)");
    return SOP_OK;
}


static sop_status check_plan(const sop_atom* atoms, int n_atoms, AlphabetPlan& pl)
{
    std::string err;
    const sop_status s = soph::plan_alphabet(&err, atoms, n_atoms, pl);
    return s == SOP_OK ? s : soph::host_fail(s, err);
}

extern "C" sop_status sop_check_alphabet(const sop_atom* atoms, int n_atoms, int* n_bins, int64_t* n_checked)
{
    AlphabetPlan pl;
    if (sop_status s = check_plan(atoms, n_atoms, pl)) return s;
    int64_t checked = 0;
    const float inf = std::numeric_limits<float>::infinity();
    for (int i = 0; i < n_atoms; ++i) {
        const std::vector<float>& L = pl.tabs[pl.order[i]];
        const int N = (int)L.size();
        const float xl = L.front(), xh = L.back();
        std::vector<float> mid(N - 1);
        for (int j = 0; j + 1 < N; ++j) mid[j] = (float)(((double)L[j] + (double)L[j + 1]) * 0.5);
        auto check = [&](float x) {
            int code = 0;
            for (int j = 0; j + 1 < N; ++j) code += x > mid[j];
            const int b = bin_of(x, pl.lo[i], pl.hi[i], pl.sc[i], pl.off[i]);
            if (b < 0 || b >= pl.n_bins) return false;
            const BinRec& r = pl.img[b];
            const bool up = x > r.thr[i];
            ++checked;
            // (the table holds halves; the boundary formed as their sum must choose the same value wherever it is used)
            const volatile float thr2 = r.ylo[i] + r.yhi[i];
            const float v_up = x > thr2 ? r.yhi[i] : r.ylo[i];
            if (v_up + v_up != L[code]) return false;
            const float v = up ? r.yhi[i] : r.ylo[i];
            return r.code_lo[i] + (up ? 1 : 0) == code && v + v == L[code];
        };
        bool ok = true;
        // every float within 64 steps of a code boundary or of an endpoint, a uniform sweep, and
        // values far outside the range
        for (int j = 0; j < N + 1 && ok; ++j) {
            const float centre = j == 0 ? xl : (j == N ? xh : mid[j - 1]);
            float lo = centre, hi = centre;
            for (int t = 0; t < 64 && ok; ++t) { ok = check(lo) && check(hi); lo = std::nextafter(lo, -inf); hi = std::nextafter(hi, inf); }
        }
        for (int t = 0; t <= 200000 && ok; ++t) ok = check(xl * 2.0f + (xh - xl) * 2.0f * (float)t / 200000.0f);
        for (int64_t k = ford(pl.lo[i]); k <= ford(pl.hi[i]) && ok; k += 4099) ok = check(funord(k));
        ok = ok && check(pl.lo[i]) && check(pl.hi[i]) && check(std::nextafter(pl.lo[i], -inf)) && check(std::nextafter(pl.hi[i], inf));
        ok = ok && check(-inf) && check(inf) && check(-3.0e38f) && check(3.0e38f) && check(0.0f) && check(-0.0f);
        if (!ok) return soph::host_fail(SOP_EATOM, "sop_check_alphabet: the bin table disagrees with the direct search");
    }
    if (n_bins) *n_bins = pl.n_bins;
    if (n_checked) *n_checked = checked;
    return SOP_OK;
}


// ------------------------------------------------------------------ host atom builders
// Inverse standard normal CDF: bisection start refined by Newton steps on erfc (binary64).
static double norm_ppf(double prob)
{
    double lo = -12.0, hi = 12.0;
    for (int i = 0; i < 80; ++i) {
        const double mid = 0.5 * (lo + hi);
        if (0.5 * std::erfc(-mid / std::sqrt(2.0)) < prob) lo = mid; else hi = mid;
    }
    double z = 0.5 * (lo + hi);
    for (int i = 0; i < 3; ++i) {
        const double cdf = 0.5 * std::erfc(-z / std::sqrt(2.0));
        const double pdf = std::exp(-0.5 * z * z) / std::sqrt(2.0 * M_PI);
        if (pdf > 0) z -= (cdf - prob) / pdf;
    }
    return z;
}

static void nf_grid(int n_bits, std::vector<double>& v)
{
    const int npos = 1 << (n_bits - 1), nneg = npos - 1;
    const double delta = 0.5 * ((1.0 - 1.0 / 32.0) + (1.0 - 1.0 / 30.0));
    v.clear();
    for (int i = 0; i < nneg; ++i) v.push_back(-norm_ppf(delta + (0.5 - delta) * i / nneg));
    v.push_back(0.0);
    for (int i = 0; i < npos; ++i) v.push_back(norm_ppf(delta + (0.5 - delta) * i / npos));
    double mx = 0;
    for (double t : v) mx = std::max(mx, std::fabs(t));
    for (double& t : v) t /= mx;
    std::sort(v.begin(), v.end());
}

extern "C" sop_status sop_atom_nf(int n_bits, float* out)
{
    if (!out || n_bits < 2 || n_bits > 6) return SOP_EINVAL;
    std::vector<double> v;
    nf_grid(n_bits, v);
    for (size_t i = 0; i < v.size(); ++i) out[i] = (float)v[i];
    return SOP_OK;
}

extern "C" sop_status sop_atom_sh(int n_bits, double alpha, double cc, float* out)
{
    if (!out || n_bits < 1 || n_bits > 6 || !(alpha > 0)) return SOP_EINVAL;
    const int N = 1 << n_bits;
    std::vector<double> v(N);
    double mx = 0;
    for (int i = 0; i < N; ++i) {
        const double t = -1.0 + 2.0 * i / (N - 1);
        v[i] = std::sinh(alpha * t) + cc;
        mx = std::max(mx, std::fabs(v[i]));
    }
    for (int i = 0; i < N; ++i) out[i] = (float)(v[i] / mx);
    return SOP_OK;
}

extern "C" sop_status sop_atom_negate(const float* in, int n, float* out)
{
    if (!in || !out || n < 1) return SOP_EINVAL;
    for (int i = 0; i < n; ++i) out[i] = -in[n - 1 - i];
    return SOP_OK;
}

extern "C" sop_status sop_lloyd_1d(const double* x, const double* wt, int64_t n, double* cent, int nc, int iters)
{
    if (!x || !cent || n < 1 || nc < 2 || nc > 4096 || iters < 0) return SOP_EINVAL;
    std::sort(cent, cent + nc);
    std::vector<double> mids(nc - 1), sw(nc), swx(nc);
    for (int it = 0; it < iters; ++it) {
        for (int j = 0; j + 1 < nc; ++j) mids[j] = 0.5 * (cent[j] + cent[j + 1]);
        std::fill(sw.begin(), sw.end(), 0.0);
        std::fill(swx.begin(), swx.end(), 0.0);
        for (int64_t i = 0; i < n; ++i) {
            // cell = number of midpoints strictly below the sample (ties to the lower centroid)
            const int cell = (int)(std::lower_bound(mids.begin(), mids.end(), x[i]) - mids.begin());
            const double wi = wt ? wt[i] : 1.0;
            sw[cell] += wi;
            swx[cell] += wi * x[i];
        }
        for (int j = 0; j < nc; ++j) if (sw[j] > 0) cent[j] = swx[j] / sw[j];
        std::sort(cent, cent + nc);
    }
    return SOP_OK;
}

extern "C" sop_status sop_atom_bof(int n_bits, const double* draws, int64_t n_draws, int g, int iters, float* out)
{
    if (!draws || !out || n_bits < 2 || n_bits > 6 || g < 1 || n_draws < g || iters < 0) return SOP_EINVAL;
    const int64_t nb = n_draws / g;
    std::vector<double> x((size_t)(nb * g));
    for (int64_t b = 0; b < nb; ++b) {
        const double* blk = draws + b * g;
        double piv = blk[0];
        for (int i = 1; i < g; ++i) if (std::fabs(blk[i]) > std::fabs(piv)) piv = blk[i];
        for (int i = 0; i < g; ++i) x[(size_t)(b * g + i)] = blk[i] / piv;
    }
    std::vector<double> cent;
    nf_grid(n_bits, cent);
    const int N = (int)cent.size();
    sop_status s = sop_lloyd_1d(x.data(), nullptr, (int64_t)x.size(), cent.data(), N, iters);
    if (s != SOP_OK) return s;
    cent[0] = -1.0; cent[N - 1] = 1.0;
    int z = 0;
    for (int j = 1; j < N; ++j) if (std::fabs(cent[j]) < std::fabs(cent[z])) z = j;
    cent[z] = 0.0;
    std::sort(cent.begin(), cent.end());
    for (int j = 0; j < N; ++j) out[j] = (float)cent[j];
    return SOP_OK;
}


extern "C" sop_status sop_dd_fit(const int64_t* hist, int n_bins, int n_entries, int iters, const float* init, float* out)
{
    if (!hist || !init || !out) return soph::host_fail(SOP_EINVAL, "sop_dd_fit: NULL argument");
    if (!dd_bins_ok(n_bins) || n_entries < 2 || n_entries > SOP_MAX_ENTRIES || iters < 0) return soph::host_fail(SOP_EINVAL, "sop_dd_fit: bad n_bins, n_entries or iters");
    for (int b = 0; b < n_bins; ++b) if (hist[b] < 0) return soph::host_fail(SOP_EINVAL, "sop_dd_fit: negative histogram entry");
    std::vector<double> cent(init, init + n_entries), mids(n_entries - 1);
    for (int j = 0; j + 1 < n_entries; ++j)
        if (!(cent[j] < cent[j + 1])) return soph::host_fail(SOP_EATOM, "sop_dd_fit: the start grid must be strictly ascending");
    // A bin stands for its centre -1 + (2b+1)/H and goes, whole, to that centre's cell (cell = number of
    // midpoints strictly below the centre).  The centres ascend with b, so a cell is a run of bins and its
    // mass and first moment are differences of prefix sums (exact integers); the run's end for a midpoint is
    // found by bisection on the same binary64 expression of the centre that defines the cell.
    std::vector<unsigned __int128> pm(n_bins + 1), pf(n_bins + 1);
    pm[0] = 0; pf[0] = 0;
    for (int b = 0; b < n_bins; ++b) {
        pm[b + 1] = pm[b] + (unsigned __int128)hist[b];
        pf[b + 1] = pf[b] + (unsigned __int128)hist[b] * (unsigned)(2 * b + 1);
    }
    auto centre = [n_bins](int b) { return -1.0 + (2.0 * (double)b + 1.0) / (double)n_bins; };
    for (int it = 0; it < iters; ++it) {
        for (int j = 0; j + 1 < n_entries; ++j) mids[j] = 0.5 * (cent[j] + cent[j + 1]);
        int lo_bin = 0;                               // first bin of the current cell
        for (int j = 0; j < n_entries; ++j) {
            int end = n_bins;                         // one past the last bin of cell j
            if (j + 1 < n_entries) {
                // smallest b >= lo_bin with mids[j] < centre(b): those bins belong to later cells
                int lo = lo_bin, hi = n_bins;
                while (lo < hi) {
                    const int mid = (lo + hi) / 2;
                    if (mids[j] < centre(mid)) hi = mid; else lo = mid + 1;
                }
                end = lo;
            }
            const unsigned __int128 mass = pm[end] - pm[lo_bin], first = pf[end] - pf[lo_bin];
            if (mass > 0) cent[j] = ((double)first / (double)mass) / (double)n_bins - 1.0;
            lo_bin = end;
        }
        std::sort(cent.begin(), cent.end());
    }
    for (int j = 0; j < n_entries; ++j) out[j] = (float)cent[j];
    for (int j = 0; j + 1 < n_entries; ++j)
        if (!(out[j] < out[j + 1])) return soph::host_fail(SOP_EATOM, "sop_dd_fit: the fitted grid is not strictly ascending in binary32 (too little data)");
    if (!(out[0] < 0.0f && out[n_entries - 1] > 0.0f)) return soph::host_fail(SOP_EATOM, "sop_dd_fit: the fitted grid is one-sided");
    return SOP_OK;
}

extern "C" sop_status sop_weight_grid(sop_weight_fmt wfmt, double top, double* values, int* n_values)
{
    if (!values || !n_values) return soph::host_fail(SOP_EINVAL, "sop_weight_grid: NULL argument");
    const int x = wfmt.exp_bits, y = wfmt.man_bits;
    if (x < 1 || x > 8 || y < 0 || y > 10 || x + y > 10) return soph::host_fail(SOP_EFMT, "sop_weight_grid: need 1<=x<=8, 0<=y<=10, x+y<=10");
    const int bias = wfmt.bias < 0 ? (1 << (x - 1)) - 1 : wfmt.bias;
    const int max_code = wfmt.max_code < 0 ? (1 << (x + y)) - 1 : wfmt.max_code;
    if (max_code < 1 || max_code >= (1 << (x + y)) || bias > 127) return soph::host_fail(SOP_EFMT, "sop_weight_grid: bad bias or max_code");
    if (top != top) return soph::host_fail(SOP_EINVAL, "sop_weight_grid: top is NaN");
    // magnitudes ascend with the code; a format without mantissa bits has no subnormal step above zero
    std::vector<double> mag;
    for (int q = 0; q <= max_code; ++q) {
        const int e = q >> y, f = q & ((1 << y) - 1);
        const double v = e == 0 ? std::ldexp((double)f, 1 - bias - y) : std::ldexp((double)((1 << y) + f), e - bias - y);
        if (top > 0.0 && v > top) break;
        if (mag.empty() || v > mag.back()) mag.push_back(v);
    }
    if (mag.size() < 2) return soph::host_fail(SOP_EINVAL, "sop_weight_grid: top leaves no value besides zero");
    int n = 0;
    for (size_t i = mag.size(); i-- > 1;) values[n++] = -mag[i];
    for (size_t i = 0; i < mag.size(); ++i) values[n++] = mag[i];
    *n_values = n;
    return SOP_OK;
}

extern "C" sop_status sop_dd_fit_grid(const int64_t* hist, int n_bins, const double* cand, int n_cand, int n_entries,
                                      int* chosen, double* cost)
{
    if (!hist || !cand || !chosen) return soph::host_fail(SOP_EINVAL, "sop_dd_fit_grid: NULL argument");
    if (!dd_bins_ok(n_bins)) return soph::host_fail(SOP_EINVAL, "sop_dd_fit_grid: n_bins must be a power of two within 64..8192");
    if (n_entries < 2 || n_entries > SOP_MAX_ENTRIES || n_cand < n_entries || n_cand > SOP_DD_MAX_CANDIDATES)
        return soph::host_fail(SOP_EINVAL, "sop_dd_fit_grid: need 2 <= n_entries <= 64 and n_entries <= n_cand <= 2047");
    for (int b = 0; b < n_bins; ++b) if (hist[b] < 0) return soph::host_fail(SOP_EINVAL, "sop_dd_fit_grid: negative histogram entry");
    for (int c = 0; c < n_cand; ++c) {
        if (!std::isfinite(cand[c]) || std::fabs(cand[c]) > 4.0) return soph::host_fail(SOP_EATOM, "sop_dd_fit_grid: candidates must be finite and within [-4, 4]");
        if (c > 0 && !(cand[c - 1] < cand[c])) return soph::host_fail(SOP_EATOM, "sop_dd_fit_grid: candidates must be strictly ascending");
    }
    const int H = n_bins, G = n_cand, N = n_entries;
    // Bin b stands for its centre, numerator u_b = 2b+1-H in units of 1/H.  Prefix sums of the mass and of
    // its first and second moments in these integer units are exact in 128 bits (mass < 2^63, |u| < 2^13);
    // they are rounded once to the x87 extended format (64-bit significand), so the cost of sending a run of
    // bins to one value, (S2 - 2a*S1 + a*a*S0) / H^2 with a = value * H (exact: H is a power of two), keeps
    // some 15 digits after the cancellation between its terms.
    std::vector<long double> p0(H + 1), p1(H + 1), p2(H + 1);
    {
        __int128 s0 = 0, s1 = 0, s2 = 0;
        p0[0] = p1[0] = p2[0] = 0.0L;
        for (int b = 0; b < H; ++b) {
            const __int128 m = hist[b], u = 2 * b + 1 - H;
            s0 += m; s1 += m * u; s2 += m * u * u;
            p0[b + 1] = (long double)s0; p1[b + 1] = (long double)s1; p2[b + 1] = (long double)s2;
        }
    }
    std::vector<long double> a(G);
    for (int c = 0; c < G; ++c) a[c] = (long double)cand[c] * (long double)H;
    auto run = [&](int c, int lo, int hi) -> double {              // bins [lo, hi) sent to candidate c, times H^2
        if (hi <= lo) return 0.0;
        const long double v = (p2[hi] - p2[lo]) - 2.0L * a[c] * (p1[hi] - p1[lo]) + a[c] * a[c] * (p0[hi] - p0[lo]);
        return v > 0.0L ? (double)v : 0.0;
    };
    std::vector<double> centre(H);
    for (int b = 0; b < H; ++b) centre[b] = -1.0 + (2.0 * (double)b + 1.0) / (double)H;
    std::vector<int> upto(G);                                      // number of bins with centre <= candidate
    {
        int j = 0;
        for (int c = 0; c < G; ++c) { while (j < H && centre[j] <= cand[c]) ++j; upto[c] = j; }
    }
    // Cost of two neighbouring chosen values c' < c: the bins above c' up to c go to the nearer of the two
    // (centre <= midpoint: the lower):
    //   pair(c', c) = run(c'; first bin above c', split) + run(c; split, first bin above c),
    // split = number of bins whose centre is at most the midpoint; for a fixed c' it rises with c, so one
    // sweep over the bins serves a whole row.  Stored with c as the row: the search below reads a row in order.
    std::vector<double> pair_cost((size_t)G * G);
    for (int cp = 0; cp < G; ++cp) {
        int j = upto[cp];
        for (int c = cp + 1; c < G; ++c) {
            const double mid = 0.5 * (cand[cp] + cand[c]);
            while (j < H && centre[j] <= mid) ++j;
            pair_cost[(size_t)c * G + cp] = run(cp, upto[cp], j) + run(c, j, upto[c]);
        }
    }
    // best[k][c]: least cost of the bins at or below candidate c when c is the k-th chosen value;
    //   best[1][c] = all those bins sent to c,  best[k][c] = min over c' < c of best[k-1][c'] + pair(c', c);
    // the bins above the last chosen value are added at the end.
    std::vector<double> best((size_t)(N + 1) * G, HUGE_VAL);
    std::vector<int> from((size_t)(N + 1) * G, -1);
    for (int c = 0; c < G; ++c) best[(size_t)1 * G + c] = run(c, 0, upto[c]);
    for (int k = 2; k <= N; ++k) {
        const double* prev = &best[(size_t)(k - 1) * G];
        for (int c = k - 1; c < G; ++c) {
            const double* pc = &pair_cost[(size_t)c * G];
            double bv = HUGE_VAL; int bp = -1;
            for (int cp = k - 2; cp < c; ++cp) {
                const double v = prev[cp] + pc[cp];
                if (v < bv) { bv = v; bp = cp; }                  // equal sums: the lower candidate stays
            }
            best[(size_t)k * G + c] = bv; from[(size_t)k * G + c] = bp;
        }
    }
    double total = HUGE_VAL; int last = -1;
    for (int c = N - 1; c < G; ++c) {
        const double v = best[(size_t)N * G + c] + run(c, upto[c], H);
        if (v < total) { total = v; last = c; }
    }
    if (last < 0) return soph::host_fail(SOP_EINVAL, "sop_dd_fit_grid: no selection found");
    for (int k = N, c = last; k >= 1; --k) { chosen[k - 1] = c; c = from[(size_t)k * G + c]; }
    if (cost) *cost = total / ((double)H * (double)H);
    if (!(cand[chosen[0]] < 0.0 && cand[chosen[N - 1]] > 0.0)) return soph::host_fail(SOP_EATOM, "sop_dd_fit_grid: the selected grid is one-sided");
    return SOP_OK;
}


bool soph::resolve_fmt(const sop_scale_fmt& fmt, FmtRange& r)
{
    const int x = fmt.exp_bits, y = fmt.man_bits, w = fmt.sign_bits;
    if ((w != 0 && w != 1) || x < 1 || x > 8 || y < 0 || y > 10 || x + y > 15) return false;
    r.x = x; r.y = y;
    r.bias = fmt.bias < 0 ? (1 << (x - 1)) - 1 : fmt.bias;
    r.max_code = fmt.max_code < 0 ? (1 << (x + y)) - 1 : fmt.max_code;
    if (r.max_code < 1 || r.max_code >= (1 << (x + y)) || r.bias < 0 || r.bias > 127) return false;
    const int e = r.max_code >> y, f = r.max_code & ((1 << y) - 1);
    r.lo = std::ldexp(1.0, 1 - r.bias);
    r.hi = e == 0 ? std::ldexp((double)f, 1 - r.bias - y) : std::ldexp((double)((1 << y) + f), e - r.bias - y);
    return true;
}

extern "C" sop_status sop_layer_shift(const int64_t* hist, int64_t n_blocks, sop_scale_fmt fmt, int* k_star, double* fraction)
{
    if (!hist || !k_star) return soph::host_fail(SOP_EINVAL, "sop_layer_shift: NULL argument");
    if (n_blocks < 1) return soph::host_fail(SOP_EINVAL, "sop_layer_shift: n_blocks must be positive");
    FmtRange r;
    if (!resolve_fmt(fmt, r)) return soph::host_fail(SOP_EFMT, "scale format: need w in {0,1}, 1<=x<=8, 0<=y<=10, x+y<=15, valid bias and max_code");
    // block scale m * 2^e (1/2 <= m < 1) times 2^k lies in [lo, hi = m_top * 2^e_top] exactly when
    //   e + k >= e_lo  and  ( e + k < e_top  or  ( e + k == e_top and m <= m_top ) )
    int e_lo, e_top;
    (void)std::frexp(r.lo, &e_lo);
    (void)std::frexp((float)r.hi, &e_top);
    const int emax = std::max(r.max_code >> r.y, 1);
    long long best_count = -1;
    int best_k = 0;
    for (int mag = 0; mag <= 64; ++mag) {
        for (int sgn = 0; sgn < 2; ++sgn) {             // candidates by |k|, the non-negative one first
            if (mag == 0 && sgn == 1) continue;
            const int k = sgn ? -mag : mag;
            // the shifts sop_pair_search() accepts for this format
            if (1 - r.bias - r.y - k < -126 || 1 - r.bias - k > 126 || emax - r.bias - k > 125) continue;
            long long count = 0;
            for (int b = 0; b < SOP_K_FL_BINS; ++b) {
                const int e = b - 160 + k;
                if (e < e_lo || e > e_top) continue;
                count += hist[b];
                if (e == e_top) count -= hist[SOP_K_FL_BINS + b];
            }
            if (count > best_count) { best_count = count; best_k = k; }
        }
    }
    *k_star = best_k;
    if (fraction) *fraction = (double)best_count / (double)n_blocks;
    return SOP_OK;
}

