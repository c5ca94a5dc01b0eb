// Host side of libsop_hip.so: context, argument validation, table image, launch parameters, and
// the host atom builders.  See include/sop.h for the contract of every entry point.
#include "../../include/sop.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <string>
#include <vector>

#include "sop_kparams.h"

extern "C" hipError_t sopk_launch(const KParams* p, int is_bf16, int g, int is_signed, int metric, int emit, void* stream);

struct sop_ctx {
    int device = 0;
    int n_atoms = 0, n_pairs = 0;
    int nent[SOP_K_MAXA] = {0};
    float tpos[SOP_K_MAXA] = {0}, tneg[SOP_K_MAXA] = {0};
    int half0[SOP_K_MAXA] = {0};
    int pairs[2 * SOP_K_MAXP] = {0};
    float* d_tab = nullptr;          // [2][MAXA][TAB]: midpoints then values
    long long target_waves = 0;
    std::string err;
};

static thread_local std::string g_create_err;

static sop_status fail(sop_ctx* c, sop_status s, const std::string& msg)
{
    if (c) c->err = msg; else g_create_err = msg;
    return s;
}
static sop_status hipfail(sop_ctx* c, hipError_t e, const char* what)
{
    return fail(c, SOP_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

extern "C" const char* sop_last_error(sop_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

extern "C" sop_status sop_create(sop_ctx** out, int device)
{
    if (!out) return fail(nullptr, SOP_EINVAL, "sop_create: ctx is NULL");
    *out = nullptr;
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n <= 0) return fail(nullptr, SOP_EHIP, "sop_create: no HIP device available (there is no CPU fallback)");
    if (device < 0 || device >= n) return fail(nullptr, SOP_EINVAL, "sop_create: device ordinal out of range");
    int prev = 0;
    (void)hipGetDevice(&prev);
    if ((e = hipSetDevice(device)) != hipSuccess) return hipfail(nullptr, e, "hipSetDevice");
    sop_ctx* c = new sop_ctx();
    c->device = device;
    hipDeviceProp_t prop;
    if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) { delete c; return hipfail(nullptr, e, "hipGetDeviceProperties"); }
    // one range of (strip,row) steps per resident wavefront: 4 SIMDs per CU, a few waves per SIMD
    long long wps = 4;
    if (const char* s = getenv("SOP_WAVES_PER_SIMD")) { long long v = atoll(s); if (v >= 1 && v <= 16) wps = v; }
    c->target_waves = (long long)prop.multiProcessorCount * 4 * wps;
    if ((e = hipMalloc((void**)&c->d_tab, sizeof(float) * 2 * SOP_K_MAXA * SOP_K_TAB)) != hipSuccess) { delete c; return hipfail(nullptr, e, "hipMalloc(table image)"); }
    (void)hipSetDevice(prev);
    *out = c;
    return SOP_OK;
}

extern "C" sop_status sop_destroy(sop_ctx* c)
{
    if (!c) return SOP_OK;
    if (c->d_tab) (void)hipFree(c->d_tab);
    delete c;
    return SOP_OK;
}

static void default_pairs(sop_ctx* c)
{
    int p = 0;
    for (int a = 0; a < c->n_atoms; ++a)
        for (int b = a + 1; b < c->n_atoms; ++b) { c->pairs[2 * p] = a; c->pairs[2 * p + 1] = b; ++p; }
    c->n_pairs = p;
}

extern "C" sop_status sop_set_alphabet(sop_ctx* c, const sop_atom* atoms, int n_atoms)
{
    if (!c) return SOP_EINVAL;
    if (!atoms) return fail(c, SOP_EINVAL, "sop_set_alphabet: atoms is NULL");
    if (n_atoms < 1 || n_atoms > SOP_K_MAXA) return fail(c, SOP_EATOM, "sop_set_alphabet: 1..8 atoms supported");
    std::vector<float> img(2 * SOP_K_MAXA * SOP_K_TAB, 0.0f);
    float* mid = img.data();
    float* val = img.data() + SOP_K_MAXA * SOP_K_TAB;
    for (int i = 0; i < SOP_K_MAXA * SOP_K_TAB; ++i) mid[i] = std::numeric_limits<float>::infinity();
    for (int a = 0; a < n_atoms; ++a) {
        const int N = atoms[a].n_entries;
        const float* L = atoms[a].values;
        if (!L) return fail(c, SOP_EINVAL, "sop_set_alphabet: atom values pointer is NULL");
        if (N < 2 || N > SOP_MAX_ENTRIES) return fail(c, SOP_EATOM, "sop_set_alphabet: an atom needs 2..64 entries");
        for (int j = 0; j < N; ++j) {
            if (!std::isfinite(L[j])) return fail(c, SOP_EATOM, "sop_set_alphabet: atom entry is not finite");
            if (j && !(L[j - 1] < L[j])) return fail(c, SOP_EATOM, "sop_set_alphabet: atom entries must be strictly ascending");
        }
        if (!(L[0] < 0.0f && L[N - 1] > 0.0f)) return fail(c, SOP_EATOM, "sop_set_alphabet: an atom must have a negative first and a positive last entry");
        int npad = 2;
        while (npad < N) npad <<= 1;
        for (int j = 0; j < N; ++j) val[a * SOP_K_TAB + j] = L[j];
        for (int j = N; j < SOP_K_TAB; ++j) val[a * SOP_K_TAB + j] = L[N - 1];
        for (int j = 0; j + 1 < N; ++j) mid[a * SOP_K_TAB + j] = (float)(((double)L[j] + (double)L[j + 1]) * 0.5);
        c->nent[a] = N;
        c->half0[a] = npad / 2;
        c->tpos[a] = L[N - 1];
        c->tneg[a] = -L[0];
    }
    int prev = 0;
    (void)hipGetDevice(&prev);
    hipError_t e = hipSetDevice(c->device);
    if (e == hipSuccess) e = hipMemcpy(c->d_tab, img.data(), img.size() * sizeof(float), hipMemcpyHostToDevice);
    (void)hipSetDevice(prev);
    if (e != hipSuccess) return hipfail(c, e, "upload of the table image");
    c->n_atoms = n_atoms;
    default_pairs(c);
    return SOP_OK;
}

extern "C" sop_status sop_set_pairs(sop_ctx* c, const int* pair_ab, int n_pairs)
{
    if (!c) return SOP_EINVAL;
    if (c->n_atoms < 1) return fail(c, SOP_EINVAL, "sop_set_pairs: set the alphabet first");
    if (!pair_ab || n_pairs == 0) { default_pairs(c); return SOP_OK; }
    if (n_pairs < 0 || n_pairs > SOP_K_MAXP) return fail(c, SOP_EINVAL, "sop_set_pairs: too many pairs");
    bool seen[SOP_K_MAXA * SOP_K_MAXA] = {false};
    for (int p = 0; p < n_pairs; ++p) {
        const int a = pair_ab[2 * p], b = pair_ab[2 * p + 1];
        if (a < 0 || b >= c->n_atoms || a >= b) return fail(c, SOP_EINVAL, "sop_set_pairs: need 0 <= a < b < n_atoms");
        if (seen[a * SOP_K_MAXA + b]) return fail(c, SOP_EINVAL, "sop_set_pairs: duplicate pair");
        seen[a * SOP_K_MAXA + b] = true;
    }
    std::memcpy(c->pairs, pair_ab, sizeof(int) * 2 * n_pairs);
    c->n_pairs = n_pairs;
    return SOP_OK;
}

static sop_status shape_check(sop_ctx* c, int64_t M, int64_t K, int g)
{
    if (M <= 0 || K <= 0) return fail(c, SOP_ESHAPE, "M and K must be positive");
    if (g != 8 && g != 16 && g != 32 && g != 64) return fail(c, SOP_ESHAPE, "block size g must be 8, 16, 32 or 64");
    if (K % g != 0) return fail(c, SOP_ESHAPE, "g must divide K");
    return SOP_OK;
}

static long long plan_waves(const sop_ctx* c, int64_t M, int64_t K, int g)
{
    const int epl = g < 16 ? g : 16;
    const long long lanes = K / epl, strips = (lanes + 63) / 64, units = strips * M;
    long long w = std::min<long long>(c->target_waves, units);
    w = (w + 3) / 4 * 4;
    return std::max<long long>(w, 4);
}

extern "C" sop_status sop_workspace_bytes(sop_ctx* c, int64_t M, int64_t K, int g, size_t* bytes)
{
    if (!c) return SOP_EINVAL;
    if (!bytes) return fail(c, SOP_EINVAL, "sop_workspace_bytes: bytes is NULL");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    *bytes = (size_t)plan_waves(c, M, K, g) * (SOP_K_MAXA + SOP_K_MAXP) * sizeof(float);
    return SOP_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" sop_status sop_pair_search(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                      const float* cn, int g, sop_scale_fmt fmt, int k, sop_metric metric,
                                      void* ws, size_t ws_bytes, const sop_outputs* out, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!W || !cn || !out) return fail(c, SOP_EINVAL, "sop_pair_search: W, c and out must not be NULL");
    if (c->n_atoms < 1) return fail(c, SOP_EINVAL, "sop_pair_search: no alphabet set");
    if (dtype != SOP_F32 && dtype != SOP_BF16) return fail(c, SOP_EINVAL, "sop_pair_search: dtype must be SOP_F32 or SOP_BF16");
    if (metric == SOP_SEL_COS) return fail(c, SOP_EINVAL, "sop_pair_search: SOP_SEL_COS is not available in this build");
    if (metric != SOP_SEL_WSE && metric != SOP_SEL_MSE) return fail(c, SOP_EINVAL, "sop_pair_search: unknown metric");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    if (ldw < K) return fail(c, SOP_ESHAPE, "ldw must be at least K");
    const int esz = dtype == SOP_BF16 ? 2 : 4;
    if (!aligned16(W) || (ldw * esz) % 16 != 0) return fail(c, SOP_EINVAL, "W and its row stride must be multiples of 16 bytes");
    if (!aligned16(cn)) return fail(c, SOP_EINVAL, "c must be 16-byte aligned");
    if ((out->sel_bits && (reinterpret_cast<uintptr_t>(out->sel_bits) & 3u)) || (out->codes && (reinterpret_cast<uintptr_t>(out->codes) & 3u)) ||
        (out->scale_code && (reinterpret_cast<uintptr_t>(out->scale_code) & 1u)))
        return fail(c, SOP_EINVAL, "output buffers must be naturally aligned");

    // ---- scale format ----
    const int x = fmt.exp_bits, y = fmt.man_bits, w = fmt.sign_bits;
    if ((w != 0 && w != 1) || x < 1 || x > 8 || y < 0 || y > 10 || x + y > 15) return fail(c, SOP_EFMT, "scale format: need w in {0,1}, 1<=x<=8, 0<=y<=10, x+y<=15");
    if (fmt.container_bits != 0 && (fmt.container_bits < w + x + y || fmt.container_bits > 16)) return fail(c, SOP_EFMT, "scale format: container must hold w+x+y bits and be at most 16");
    const int bias = fmt.bias < 0 ? (1 << (x - 1)) - 1 : fmt.bias;
    const int max_code = fmt.max_code < 0 ? (1 << (x + y)) - 1 : fmt.max_code;
    if (max_code < 1 || max_code >= (1 << (x + y))) return fail(c, SOP_EFMT, "scale format: max_code out of range");
    if (k < -64 || k > 64) return fail(c, SOP_EFMT, "layer shift k must be within [-64, 64]");
    if (bias < 0 || bias > 126) return fail(c, SOP_EFMT, "scale format: bias must be within [0, 126]");
    const int emax = max_code >> y;
    // every scale value, the subnormal quantum and every reciprocal must be normal binary32 numbers
    if (1 - bias - y - k < -126 || 1 - bias - k > 126 || std::max(emax, 1) - bias - k > 125)
        return fail(c, SOP_EFMT, "scale format with this layer shift leaves binary32's normal range (choose bias / max_code / k accordingly)");

    const int epl = g < 16 ? g : 16, lpb = g / epl;
    KParams p;
    std::memset(&p, 0, sizeof(p));
    p.W = W; p.c = cn;
    p.tab_mid = c->d_tab; p.tab_val = c->d_tab + SOP_K_MAXA * SOP_K_TAB;
    p.M = M; p.K = K; p.ldw = ldw;
    p.Bk = K / g; p.Nb = M * p.Bk; p.Wr = (p.Bk + 31) / 32;
    p.strips = (K / epl + 63) / 64;
    p.total_units = p.strips * M;
    p.n_waves = plan_waves(c, M, K, g);
    p.A = c->n_atoms; p.P = c->n_pairs; p.lpb = lpb;
    p.man_bits = y; p.bias = bias; p.max_code = max_code; p.k = k;
    p.pow2k = std::ldexp(1.0f, k);
    p.sub_quantum = std::ldexp(1.0f, 1 - bias - y - k);
    long long off = 0;
    for (int a = 0; a < c->n_atoms; ++a) {
        p.tpos[a] = c->tpos[a]; p.tneg[a] = c->tneg[a]; p.half0[a] = c->half0[a]; p.nent[a] = c->nent[a];
        p.code_off[a] = off;
        off += c->nent[a] <= 16 ? M * K / 2 : M * K;
    }
    std::memset(p.pair_slot, -1, sizeof(p.pair_slot));
    for (int q = 0; q < c->n_pairs; ++q) {
        const int a = c->pairs[2 * q], b = c->pairs[2 * q + 1];
        p.pair_slot[a * SOP_K_MAXA + b] = (signed char)q;
        p.pair_col[q] = (unsigned char)pair_index(a, b);
    }
    const size_t need = (size_t)p.n_waves * (SOP_K_MAXA + SOP_K_MAXP) * sizeof(float);
    if (!ws || ws_bytes < need) return fail(c, SOP_ENOMEM, "workspace is NULL or smaller than sop_workspace_bytes()");
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(c, SOP_EINVAL, "workspace must be 256-byte aligned");
    p.partial = static_cast<float*>(ws);
    p.acos_pair = c->n_pairs ? out->acos_pair : nullptr;
    p.acos_atom = out->acos_atom;
    p.sel_bits = c->n_pairs ? out->sel_bits : nullptr;
    p.scale_code = out->scale_code; p.codes = out->codes; p.blk_cos = out->blk_cos; p.blk_err = out->blk_err;
    const int emit = (p.scale_code || p.codes || p.blk_cos || p.blk_err) ? 1 : 0;

    int prev = 0;
    (void)hipGetDevice(&prev);
    hipError_t e = hipSuccess;
    if (prev != c->device) e = hipSetDevice(c->device);
    if (e == hipSuccess) e = sopk_launch(&p, dtype == SOP_BF16, g, w, (int)metric, emit, stream);
    if (prev != c->device) (void)hipSetDevice(prev);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
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
