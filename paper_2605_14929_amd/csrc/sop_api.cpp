// Host side of libsop_hip.so: context, argument validation, table images, launch parameters, and
// the host atom builders.  See include/sop.h for the contract of every entry point.
#include "../../include/sop.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <map>
#include <string>
#include <tuple>
#include <vector>

#include "sop_kparams.h"
#include "sop_host.h"

using soph::AlphabetPlan;
using soph::dd_bins_ok;
using soph::FmtRange;
using soph::resolve_fmt;

extern "C" const void* sopk_search_kernel(int is_bf16, int g, int sign_mode, int metric, int emit, int na_class, int mode, int* occ, int* mode_out);
extern "C" int sopk_variant_index(int is_bf16, int g, int sign_mode, int metric, int emit, int na_class, int mode);
extern "C" hipError_t sopk_launch(const void* fn, const KParams* p, int n_wg, int occ, size_t dyn_lds, void* stream);
extern "C" hipError_t sopk_dd_launch(const DdParams* p, int is_bf16, int g, void* stream);
extern "C" hipError_t sopk_fl_launch(const FlParams* p, int is_bf16, int g, void* stream);
extern "C" int sopk_fl_weights_per_lane(int is_bf16, int g);
extern "C" hipError_t sopk_ls_launch(const LsParams* p, int is_bf16, void* stream);
extern "C" hipError_t sopk_sum_launch(const LsParams* p, void* stream);
extern "C" hipError_t sopk_issue_probe_launch(int kind, int n_wg, int n_threads, int iters, float a, float b, float* out, void* stream);
extern "C" hipError_t sopk_probe_launch(const void* x, long long n16, unsigned int* out, void* stream);
extern "C" hipError_t sopk_sel_launch(const SelParams* p, int n_wg_count, int n_wg, void* stream);
extern "C" hipError_t sopk_selm_launch(const SelMParams* p, int n_wg_count, int n_wg, void* stream);
extern "C" hipError_t sopk_pack_launch(const PackParams* p, void* stream);

namespace {

struct ScaleTab { float2* dev = nullptr; int n = 0; };
struct ScaleSlot { std::tuple<int, int, int, int, int> key; bool used = false; unsigned long long age = 0; };

}  // namespace

static constexpr int kLanes = 2;          // streams of its own that sop_pair_search_layers deals the layers out to
static constexpr int kMaxLayers = 1024;  // layers of one launch of the model-wide kernel (more are dealt with in several launches)
static constexpr int kStabSlots = 160;   // (scale, reciprocal) tables kept on the device: more than the layer shifts one call can name (129)
static constexpr size_t kSumsWords = SOP_K_REPL * SOP_K_NCOL + SOP_K_REPL + 1;   // one set of layer sums and tickets, in 64-bit words

// ---- scratch of the entry point that allocates nothing (sop_pair_search_static) ----
// One set of layer sums with its ticket counters, then the (scale, reciprocal) table of the call's scale
// word.  The array lives in the library's device image: every GPU the library runs on holds its own copy
// at its own address until the process ends.  Host code never uses the array's name as an address: the
// address on a device comes from hipGetSymbolAddress (static_scratch_of) and is what kernels are given.
static constexpr size_t kStaticSumsBytes = (kSumsWords * sizeof(unsigned long long) + 255) & ~(size_t)255;
static constexpr size_t kStaticBytes = kStaticSumsBytes + (size_t)SOP_STATIC_MAX_CODES * sizeof(float2);
static_assert(kStaticBytes == SOP_STATIC_SCRATCH_BYTES, "the header states the size of the static scratch");
static __device__ __align__(256) unsigned char sop_static_scratch[kStaticBytes];
static constexpr int kMaxDevices = 64;
static unsigned char* g_static_ptr[kMaxDevices] = {nullptr};   // per device, filled once by static_scratch_of()

// Address of this device's copy of the scratch array (the device must be current).
static hipError_t static_scratch_of(int device, unsigned char** out)
{
    *out = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_static_ptr[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(sop_static_scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_static_ptr[device] = static_cast<unsigned char*>(ptr);
    }
    *out = g_static_ptr[device];
    return hipSuccess;
}

// Start of a static call: the sums and tickets are cleared (an earlier call that did not finish may have left
// anything there) and the scale table of this call's scale word and layer shift is written:
// value(q) * 2^-k (exact) and its IEEE reciprocal, the same values the host builds for sop_pair_search.
__global__ void static_prologue_kernel(unsigned long long* sums, int n_words, float2* tab, int n_codes, int y, int bias, int k)
{
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i < n_words) sums[i] = 0ull;
    if (i < n_codes) {
        const int e = i >> y, f = i & ((1 << y) - 1);
        const float s = e == 0 ? ldexpf((float)f, 1 - bias - y - k) : ldexpf((float)((1 << y) + f), e - bias - y - k);
        tab[i] = make_float2(s + s, s > 0.0f ? 1.0f / s : 0.0f);      // (twice the scale, its reciprocal)
    }
}

struct sop_ctx {
    int device = 0;
    int n_cu = 0;
    size_t lds_max = 0;                   // LDS one workgroup may use
    LayerDesc* d_ldesc = nullptr;         // [kMaxLayers] layer list of the model-wide kernel
    unsigned long long* d_msums = nullptr; // its sums [kMaxLayers][SOP_K_REPL][SOP_K_NCOL] and tickets (zero between calls)
    LayerDesc* h_ldesc[2] = {nullptr, nullptr};   // pinned staging for the layer list, used in turn
    hipEvent_t ldesc_copied[2] = {nullptr, nullptr};  // the copy out of each staging buffer has run
    bool ldesc_pending[2] = {false, false};
    int ldesc_turn = 0;
    int n_atoms = 0, n_pairs = 0;
    // caller's order
    std::vector<std::vector<float>> tables;
    int pairs[2 * SOP_K_MAXP] = {0};
    // internal order: atoms of one scale group (equal endpoints) adjacent
    int order[SOP_K_MAXA] = {0};          // internal index -> caller's index
    int gid[SOP_K_MAXA] = {0};            // scale group of the internal atom
    int mirror[SOP_K_MAXA] = {0};         // 1: the internal atom is the sign-negated copy of the one before it
    int selfsym[SOP_K_MAXA] = {0};        // 1: the atom is its own sign-negated copy
    float tpos[SOP_K_MAXA] = {0}, tneg[SOP_K_MAXA] = {0}, bin_sc[SOP_K_MAXA] = {0}, bin_off[SOP_K_MAXA] = {0};
    float bin_lo[SOP_K_MAXA] = {0}, bin_hi[SOP_K_MAXA] = {0};
    int nent[SOP_K_MAXA] = {0};
    int n_bins = 0;
    BinRec* d_bins = nullptr;             // [MAXBINS] capacity: the context's own image of the element-search table
    BinRec* d_bins_cur = nullptr;         // the image the searches read (d_bins, or an image inside a caller's workspace during sop_search_layer)
    BinRec* h_bins = nullptr;             // pinned staging for table images of sop_search_layer (allocated at its first call)
    char* h_res = nullptr;                // pinned staging for its results
    hipEvent_t stage_done = nullptr;      // the last copy out of h_bins has run
    bool stage_pending = false;
    unsigned long long* d_ls = nullptr;   // [3*SOP_K_LS_MAXWG] workgroup partials, one spare word, 17 ticket counters (u32) from word 3*MAXWG+1, then SOP_K_LS_MAXREP copies of the layer maxima (2 x u32 each, 128 bytes apart) from word 3*MAXWG+16; zero between calls
    unsigned long long* d_ddacc = nullptr; // [SOP_K_DD_MAXBINS] running DD histogram + (one word further) its finished-workgroup counter; zero between calls
    unsigned int* d_sel = nullptr;        // [2][3][SOP_K_SEL_BINS] two sets of digit counts of the block ranking: a call counts into set sel_set and clears the other
    int sel_set = 0;
    unsigned int* d_selm = nullptr;       // [2][SOP_K_MAXA][SOP_K_SELM_WORDS] two sets of digit counts of the ranking with several thresholds (one per score plane of a launch)
    int selm_set = 0;
    int selm_dirty[2] = {0, 0};           // planes of each set of the batched ranking's digit counts that hold counts
    SelMState* d_selstate = nullptr;      // [SOP_K_MAXA] what the passes of that ranking hand on, per score plane
    unsigned long long* d_sums = nullptr; // two sets of [SOP_K_REPL][SOP_K_NCOL] layer sums followed by their ticket counters; zero between calls
    hipStream_t lane_stream[kLanes] = {};   // sop_pair_search_layers deals the layers out to streams of its own
    hipEvent_t lane_event[kLanes + 1] = {};  // one per stream (join) and one for the fork
    float2* d_stab = nullptr;             // [kStabSlots][SOP_K_MAXTABCODES] (scale * 2^-k, reciprocal) tables, written by a kernel on first use
    ScaleSlot stab_slot[kStabSlots];      // what each slot holds: (x, y, bias, max_code, k); the least recently used one is replaced
    unsigned long long stab_clock = 0;
    int scale_rule = 0;                   // 0: absmax, 1: argmax
    unsigned char* static_scratch = nullptr;   // this device's copy of sop_static_scratch (looked up by sop_create)
    int occ_blocks[864];                  // resident workgroups per CU of each kernel variant (0 = unknown)
    size_t occ_lds[864];
    std::string err;
};


static sop_status fail(sop_ctx* c, sop_status s, const std::string& msg)
{
    if (c) c->err = msg; else (void)soph::host_fail(s, msg);
    return s;
}
static sop_status hipfail(sop_ctx* c, hipError_t e, const char* what)
{
    return fail(c, SOP_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

namespace {
struct DeviceGuard {
    int prev = 0;
    bool switched = false;
    hipError_t err = hipSuccess;
    explicit DeviceGuard(int dev) { (void)hipGetDevice(&prev); if (prev != dev) { err = hipSetDevice(dev); switched = err == hipSuccess; } }
    ~DeviceGuard() { if (switched) (void)hipSetDevice(prev); }
};
}  // namespace

extern "C" const char* sop_last_error(sop_ctx* ctx) { return ctx ? ctx->err.c_str() : soph::host_last_error(); }

extern "C" sop_status sop_create(sop_ctx** out, int device)
{
    if (!out) return fail(nullptr, SOP_EINVAL, "sop_create: ctx is NULL");
    *out = nullptr;
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n <= 0) return fail(nullptr, SOP_EHIP, "sop_create: no HIP device available (there is no CPU fallback)");
    if (device < 0 || device >= n) return fail(nullptr, SOP_EINVAL, "sop_create: device ordinal out of range");
    DeviceGuard guard(device);
    if (guard.err != hipSuccess) return hipfail(nullptr, guard.err, "hipSetDevice");
    sop_ctx* c = new sop_ctx();
    c->device = device;
    std::memset(c->occ_blocks, 0, sizeof(c->occ_blocks));
    std::memset(c->occ_lds, 0, sizeof(c->occ_lds));
    hipDeviceProp_t prop;
    if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) { delete c; return hipfail(nullptr, e, "hipGetDeviceProperties"); }
    c->n_cu = prop.multiProcessorCount;
    c->lds_max = prop.sharedMemPerBlock;
    if ((e = hipMalloc((void**)&c->d_bins, sizeof(BinRec) * SOP_K_MAXBINS)) != hipSuccess) { delete c; return hipfail(nullptr, e, "hipMalloc(table image)"); }
    if ((e = hipMalloc((void**)&c->d_sums, sizeof(unsigned long long) * kLanes * kSumsWords)) != hipSuccess ||
        (e = hipMemset(c->d_sums, 0, sizeof(unsigned long long) * kLanes * kSumsWords)) != hipSuccess) {
        (void)hipFree(c->d_bins); if (c->d_sums) (void)hipFree(c->d_sums);
        delete c;
        return hipfail(nullptr, e, "hipMalloc(layer sums)");
    }
    if ((e = hipMalloc((void**)&c->d_ddacc, sizeof(unsigned long long) * (SOP_K_DD_MAXBINS + 1))) != hipSuccess ||
        (e = hipMemset(c->d_ddacc, 0, sizeof(unsigned long long) * (SOP_K_DD_MAXBINS + 1))) != hipSuccess) {
        (void)hipFree(c->d_bins); (void)hipFree(c->d_sums); if (c->d_ddacc) (void)hipFree(c->d_ddacc);
        delete c;
        return hipfail(nullptr, e, "hipMalloc(histogram)");
    }
    if ((e = hipMalloc((void**)&c->d_ls, sizeof(unsigned long long) * (3 * SOP_K_LS_MAXWG + 2 + 9 + 5 + 16 * SOP_K_LS_MAXREP))) != hipSuccess ||
        (e = hipMemset(c->d_ls, 0, sizeof(unsigned long long) * (3 * SOP_K_LS_MAXWG + 2 + 9 + 5 + 16 * SOP_K_LS_MAXREP))) != hipSuccess) {
        (void)hipFree(c->d_bins); (void)hipFree(c->d_sums); (void)hipFree(c->d_ddacc); if (c->d_ls) (void)hipFree(c->d_ls);
        delete c;
        return hipfail(nullptr, e, "hipMalloc(partials)");
    }
    if ((e = hipMalloc((void**)&c->d_sel, sizeof(unsigned int) * (6 * SOP_K_SEL_BINS))) != hipSuccess ||
        (e = hipMemset(c->d_sel, 0, sizeof(unsigned int) * (6 * SOP_K_SEL_BINS))) != hipSuccess) {
        (void)hipFree(c->d_bins); (void)hipFree(c->d_sums); (void)hipFree(c->d_ddacc); (void)hipFree(c->d_ls); if (c->d_sel) (void)hipFree(c->d_sel);
        delete c;
        return hipfail(nullptr, e, "hipMalloc(rank counts)");
    }
    if ((e = hipMalloc((void**)&c->d_stab, sizeof(float2) * (size_t)kStabSlots * SOP_K_MAXTABCODES)) != hipSuccess) {
        (void)hipFree(c->d_bins); (void)hipFree(c->d_sums); (void)hipFree(c->d_ddacc); (void)hipFree(c->d_ls); (void)hipFree(c->d_sel);
        delete c;
        return hipfail(nullptr, e, "hipMalloc(scale tables)");
    }
    if ((e = hipMalloc((void**)&c->d_selm, sizeof(unsigned int) * 2 * SOP_K_MAXA * SOP_K_SELM_WORDS)) != hipSuccess ||
        (e = hipMemset(c->d_selm, 0, sizeof(unsigned int) * 2 * SOP_K_MAXA * SOP_K_SELM_WORDS)) != hipSuccess ||
        (e = hipMalloc((void**)&c->d_selstate, sizeof(SelMState) * SOP_K_MAXA)) != hipSuccess) {
        (void)hipFree(c->d_bins); (void)hipFree(c->d_sums); (void)hipFree(c->d_ddacc); (void)hipFree(c->d_ls); (void)hipFree(c->d_sel); (void)hipFree(c->d_stab); if (c->d_selm) (void)hipFree(c->d_selm);
        delete c;
        return hipfail(nullptr, e, "hipMalloc(rank counts of the sweep)");
    }
    const size_t msums_bytes = sizeof(unsigned long long) * ((size_t)kMaxLayers * SOP_K_REPL * SOP_K_NCOL + SOP_K_REPL + 1);
    if ((e = hipMalloc((void**)&c->d_ldesc, sizeof(LayerDesc) * kMaxLayers)) != hipSuccess ||
        (e = hipMalloc((void**)&c->d_msums, msums_bytes)) != hipSuccess || (e = hipMemset(c->d_msums, 0, msums_bytes)) != hipSuccess ||
        (e = hipHostMalloc((void**)&c->h_ldesc[0], sizeof(LayerDesc) * kMaxLayers, hipHostMallocDefault)) != hipSuccess ||
        (e = hipHostMalloc((void**)&c->h_ldesc[1], sizeof(LayerDesc) * kMaxLayers, hipHostMallocDefault)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&c->ldesc_copied[0], hipEventDisableTiming)) != hipSuccess ||
        (e = hipEventCreateWithFlags(&c->ldesc_copied[1], hipEventDisableTiming)) != hipSuccess) {
        (void)hipFree(c->d_bins); (void)hipFree(c->d_sums); (void)hipFree(c->d_ddacc); (void)hipFree(c->d_ls); (void)hipFree(c->d_sel); (void)hipFree(c->d_selm); (void)hipFree(c->d_stab);
        if (c->d_ldesc) (void)hipFree(c->d_ldesc);
        if (c->d_msums) (void)hipFree(c->d_msums);
        for (int i = 0; i < 2; ++i) { if (c->h_ldesc[i]) (void)hipHostFree(c->h_ldesc[i]); if (c->ldesc_copied[i]) (void)hipEventDestroy(c->ldesc_copied[i]); }
        delete c;
        return hipfail(nullptr, e, "hipMalloc(layer list)");
    }
    if ((e = static_scratch_of(device, &c->static_scratch)) != hipSuccess) {
        hipError_t keep = e;
        sop_destroy(c);
        return hipfail(nullptr, keep, "hipGetSymbolAddress(static scratch)");
    }
    *out = c;
    return SOP_OK;
}

extern "C" sop_status sop_destroy(sop_ctx* c)
{
    if (!c) return SOP_OK;
    {
        DeviceGuard guard(c->device);
        if (c->d_bins) (void)hipFree(c->d_bins);
        if (c->d_sums) (void)hipFree(c->d_sums);
        if (c->d_ddacc) (void)hipFree(c->d_ddacc);
        if (c->d_ls) (void)hipFree(c->d_ls);
        if (c->d_sel) (void)hipFree(c->d_sel);
        if (c->d_selm) (void)hipFree(c->d_selm);
        if (c->d_selstate) (void)hipFree(c->d_selstate);
        if (c->d_ldesc) (void)hipFree(c->d_ldesc);
        if (c->d_msums) (void)hipFree(c->d_msums);
        for (int i = 0; i < 2; ++i) { if (c->h_ldesc[i]) (void)hipHostFree(c->h_ldesc[i]); if (c->ldesc_copied[i]) (void)hipEventDestroy(c->ldesc_copied[i]); }
        if (c->h_bins) (void)hipHostFree(c->h_bins);
        if (c->h_res) (void)hipHostFree(c->h_res);
        if (c->stage_done) (void)hipEventDestroy(c->stage_done);
        for (hipStream_t s : c->lane_stream) if (s) (void)hipStreamDestroy(s);
        for (hipEvent_t ev : c->lane_event) if (ev) (void)hipEventDestroy(ev);
        if (c->d_stab) (void)hipFree(c->d_stab);
    }
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

static sop_status plan_alphabet(sop_ctx* c, const sop_atom* atoms, int n_atoms, AlphabetPlan& pl)
{
    std::string err;
    const sop_status s = soph::plan_alphabet(&err, atoms, n_atoms, pl);
    return s == SOP_OK ? s : fail(c, s, err);
}

// Plan the alphabet and make it the context's current one.  d_img == nullptr: the context's own image, copied
// synchronously.  Otherwise the image goes through the pinned buffer h_stage to d_img with a copy on `st`
// (the host does not wait), and the searches launched from now on read d_img.
static sop_status install_alphabet(sop_ctx* c, const sop_atom* atoms, int n_atoms, BinRec* d_img, BinRec* h_stage, hipStream_t st)
{
    AlphabetPlan pl;
    if (sop_status s = plan_alphabet(c, atoms, n_atoms, pl)) return s;
    {
        DeviceGuard guard(c->device);
        hipError_t e = guard.err;
        if (e == hipSuccess) {
            if (d_img) {
                std::memcpy(h_stage, pl.img.data(), pl.img.size() * sizeof(BinRec));
                e = hipMemcpyAsync(d_img, h_stage, pl.img.size() * sizeof(BinRec), hipMemcpyHostToDevice, st);
            } else e = hipMemcpy(c->d_bins, pl.img.data(), pl.img.size() * sizeof(BinRec), hipMemcpyHostToDevice);
        }
        if (e != hipSuccess) return hipfail(c, e, "upload of the table image");
    }
    c->d_bins_cur = d_img ? d_img : c->d_bins;
    c->tables.swap(pl.tabs);
    c->n_atoms = n_atoms;
    c->n_bins = pl.n_bins;
    for (int i = 0; i < n_atoms; ++i) {
        const std::vector<float>& L = c->tables[pl.order[i]];
        c->order[i] = pl.order[i]; c->gid[i] = pl.gid[i]; c->mirror[i] = pl.mirror[i]; c->selfsym[i] = pl.selfsym[i];
        c->tpos[i] = L.back(); c->tneg[i] = -L.front(); c->nent[i] = (int)L.size();
        c->bin_sc[i] = pl.sc[i]; c->bin_off[i] = pl.off[i]; c->bin_lo[i] = pl.lo[i]; c->bin_hi[i] = pl.hi[i];
    }
    default_pairs(c);                      // (the occupancy cache is keyed by variant and LDS size: it stays valid)
    return SOP_OK;
}

extern "C" sop_status sop_set_alphabet(sop_ctx* c, const sop_atom* atoms, int n_atoms)
{
    if (!c) return SOP_EINVAL;
    return install_alphabet(c, atoms, n_atoms, nullptr, nullptr, nullptr);
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

extern "C" sop_status sop_set_scale_rule(sop_ctx* c, sop_scale_rule rule)
{
    if (!c) return SOP_EINVAL;
    if (rule != SOP_SCALE_ABSMAX && rule != SOP_SCALE_ARGMAX) return fail(c, SOP_EINVAL, "sop_set_scale_rule: unknown rule");
    c->scale_rule = rule == SOP_SCALE_ARGMAX ? 1 : 0;
    return SOP_OK;
}

static sop_status shape_check(sop_ctx* c, int64_t M, int64_t K, int g)
{
    if (M <= 0 || K <= 0) return fail(c, SOP_ESHAPE, "M and K must be positive");
    if (g != 8 && g != 16 && g != 32 && g != 64) return fail(c, SOP_ESHAPE, "block size g must be 8, 16, 32 or 64");
    if (K % g != 0) return fail(c, SOP_ESHAPE, "g must divide K");
    return SOP_OK;
}

// upper bound of the workgroups one launch uses: 8 resident wavefronts per SIMD

extern "C" sop_status sop_workspace_bytes(sop_ctx* c, int64_t M, int64_t K, int g, size_t* bytes)
{
    if (!c) return SOP_EINVAL;
    if (!bytes) return fail(c, SOP_EINVAL, "sop_workspace_bytes: bytes is NULL");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    *bytes = 0;                      // the layer reduction keeps its few words inside the context
    return SOP_OK;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Rows folded into one for the search kernel (see KParams::Kc): the power of two f <= 64 dividing M that leaves
// the fewest idle lanes in the last 64-lane strip of a row of f*K columns; 1 when the rows do not lie back to back.
static int row_fold(int64_t M, int64_t K, int64_t ldw, int epl)
{
    if (ldw != K) return 1;
    int best = 1;
    double best_waste = 1e9;
    for (int f = 1; f <= 64 && M % f == 0 && K * f < (1ll << 24); f *= 2) {
        const int64_t lanes = K * f / epl, strips = (lanes + 63) / 64;
        const double waste = (double)(strips * 64 - lanes) / (double)lanes;
        if (waste < best_waste - 1e-12) { best_waste = waste; best = f; }
    }
    return best;
}

// (twice the scale, reciprocal) of every code of a scale word: 2 * value(q) * 2^-k (exact; the table of codebook values holds halves) and the IEEE reciprocal of value(q) * 2^-k.
// The tables live in a slab the context allocated at its creation; a table that is not there yet is written
// by a small kernel on the caller's stream ahead of the kernel that reads it (no allocation, no copy from the
// host, no synchronisation), into the slot that was used longest ago.
__global__ void scale_table_kernel(float2* tab, int n_codes, int y, int bias, int k)
{
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i < n_codes) {
        const int e = i >> y, f = i & ((1 << y) - 1);
        const float s = e == 0 ? ldexpf((float)f, 1 - bias - y - k) : ldexpf((float)((1 << y) + f), e - bias - y - k);
        tab[i] = make_float2(s + s, s > 0.0f ? 1.0f / s : 0.0f);      // (twice the scale, its reciprocal)
    }
}

static sop_status scale_table(sop_ctx* c, int x, int y, int bias, int max_code, int k, void* stream, ScaleTab* out)
{
    const auto key = std::make_tuple(x, y, bias, max_code, k);
    int slot = -1, oldest = -1;
    for (int i = 0; i < kStabSlots && slot < 0; ++i)
        if (c->stab_slot[i].used && c->stab_slot[i].key == key) slot = i;
    for (int i = 0; i < kStabSlots && slot < 0; ++i) {            // a free slot, else the one used longest ago
        if (!c->stab_slot[i].used) { oldest = i; break; }
        if (oldest < 0 || c->stab_slot[i].age < c->stab_slot[oldest].age) oldest = i;
    }
    const int n = max_code + 1;
    if (slot < 0) {
        slot = oldest;
        float2* dst = c->d_stab + (size_t)slot * SOP_K_MAXTABCODES;
        scale_table_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(dst, n, y, bias, k);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hipfail(c, e, "kernel launch (scale table)");
        c->stab_slot[slot].key = key;
        c->stab_slot[slot].used = true;
    }
    c->stab_slot[slot].age = ++c->stab_clock;
    out->dev = c->d_stab + (size_t)slot * SOP_K_MAXTABCODES;
    out->n = n;
    return SOP_OK;
}

// launch == false: validate everything and prepare the tables the call needs, but launch nothing
static sop_status pair_search_impl(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                   const float* cn, int g, sop_scale_fmt fmt, int k, sop_metric metric,
                                   void* ws, size_t ws_bytes, const sop_outputs* out, void* stream, bool launch, int sums_set = 0,
                                   KParams* p_out = nullptr, size_t* lds_out = nullptr, bool use_static = false)
{
    if (!c) return SOP_EINVAL;
    if (!W || !cn || !out) return fail(c, SOP_EINVAL, "sop_pair_search: W, c and out must not be NULL");
    if (c->n_atoms < 1) return fail(c, SOP_EINVAL, "sop_pair_search: no alphabet set");
    if (dtype != SOP_F32 && dtype != SOP_BF16) return fail(c, SOP_EINVAL, "sop_pair_search: dtype must be SOP_F32 or SOP_BF16");
    if (metric != SOP_SEL_WSE && metric != SOP_SEL_MSE && metric != SOP_SEL_COS) return fail(c, SOP_EINVAL, "sop_pair_search: unknown metric");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    if (ldw < K) return fail(c, SOP_ESHAPE, "ldw must be at least K");
    const int esz = dtype == SOP_BF16 ? 2 : 4;
    if (!aligned16(W) || (ldw * esz) % 16 != 0) return fail(c, SOP_EINVAL, "W and its row stride must be multiples of 16 bytes");
    if (!aligned16(cn)) return fail(c, SOP_EINVAL, "c must be 16-byte aligned");
    if ((out->sel_words && (reinterpret_cast<uintptr_t>(out->sel_words) & 3u)) || (out->codes && (reinterpret_cast<uintptr_t>(out->codes) & 3u)) ||
        (out->scale_code && (reinterpret_cast<uintptr_t>(out->scale_code) & 1u)) ||
        ((reinterpret_cast<uintptr_t>(out->blk_cos) | reinterpret_cast<uintptr_t>(out->blk_err) | reinterpret_cast<uintptr_t>(out->blk_rank)) & 3u))
        return fail(c, SOP_EINVAL, "output buffers must be naturally aligned");

    // ---- scale format ----
    const int x = fmt.exp_bits, y = fmt.man_bits, w = fmt.sign_bits;
    if ((w != 0 && w != 1) || x < 1 || x > 8 || y < 0 || y > 10 || x + y > 15) return fail(c, SOP_EFMT, "scale format: need w in {0,1}, 1<=x<=8, 0<=y<=10, x+y<=15");
    if (fmt.container_bits != 0 && (fmt.container_bits < w + x + y || fmt.container_bits > 16)) return fail(c, SOP_EFMT, "scale format: container must hold w+x+y bits and be at most 16");
    if (c->scale_rule == 1 && w == 0) return fail(c, SOP_EFMT, "the argmax scale rule needs a scale word with a sign bit");
    const int bias = fmt.bias < 0 ? (1 << (x - 1)) - 1 : fmt.bias;
    const int max_code = fmt.max_code < 0 ? (1 << (x + y)) - 1 : fmt.max_code;
    if (max_code < 1 || max_code >= (1 << (x + y))) return fail(c, SOP_EFMT, "scale format: max_code out of range");
    if (k < -64 || k > 64) return fail(c, SOP_EFMT, "layer shift k must be within [-64, 64]");
    if (bias < 0 || bias > 127) return fail(c, SOP_EFMT, "scale format: bias must be within [0, 127]");
    const int emax = max_code >> y;
    // every scale value, the subnormal quantum and every reciprocal must be normal binary32 numbers
    if (1 - bias - y - k < -126 || 1 - bias - k > 126 || std::max(emax, 1) - bias - k > 125)
        return fail(c, SOP_EFMT, "scale format with this layer shift leaves binary32's normal range (choose bias / max_code / k accordingly)");

    (void)ws; (void)ws_bytes;         // no workspace is needed (sop_workspace_bytes reports 0)
    if (use_static) {
        if (max_code >= SOP_STATIC_MAX_CODES)
            return fail(c, SOP_EFMT, "sop_pair_search_static: the scale word has more magnitude codes than the static scale table holds (2048); use sop_pair_search");
        if (!c->static_scratch) return fail(c, SOP_EHIP, "sop_pair_search_static: the static scratch of this device was not found");
    }

    const int epl = g < 16 ? g : 16, lpb = g / epl;
    const int A = c->n_atoms;
    KParams p;
    std::memset(&p, 0, sizeof(p));
    p.W = W; p.c = cn;
    p.bins = c->d_bins_cur;
    const int64_t Mu = M, Ku = K;                       // the caller's shape (output planes are laid out by it)
    const int fold = row_fold(M, K, ldw, epl);
    p.Kc = K;
    M /= fold; K *= fold; ldw = fold > 1 ? K : ldw;     // from here on: the shape the kernel walks
    p.M = M; p.K = K; p.ldw = ldw;
    p.Bk = K / g; p.Nb = M * p.Bk;
    p.strips = (K / epl + 63) / 64;
    p.total_units = p.strips * M;
    if (p.total_units >= (1ll << 31) || M >= (1ll << 31)) return fail(c, SOP_ESHAPE, "the layer has more than 2^31 strip rows");
    p.M32 = (unsigned int)M;
    p.m_magic = M == 1 ? 0xFFFFFFFFu : (unsigned int)((1ull << 32) / (unsigned long long)M);
    p.A = A; p.P = c->n_pairs; p.lpb = lpb;
    p.n_bins = c->n_bins;
    p.man_bits = y; p.bias = bias; p.max_code = max_code; p.k = k;
    p.pow2k = std::ldexp(1.0f, k);
    p.sub_quantum = std::ldexp(1.0f, 1 - bias - y - k);
    // code planes are laid out in the caller's atom order
    long long plane_off[SOP_K_MAXA], off = 0;
    for (int a = 0; a < A; ++a) { plane_off[a] = off; off += c->tables[a].size() <= 16 ? Mu * Ku / 2 : Mu * Ku; }
    int internal_of[SOP_K_MAXA];
    for (int i = 0; i < A; ++i) {
        p.tpos[i] = c->tpos[i]; p.tneg[i] = c->tneg[i]; p.bin_sc[i] = c->bin_sc[i]; p.bin_off[i] = c->bin_off[i];
        p.bin_lo[i] = c->bin_lo[i]; p.bin_hi[i] = c->bin_hi[i];
        p.gid_w |= (unsigned)c->gid[i] << (4 * i);
        if (c->mirror[i]) p.mirror_mask |= 1u << i;
        if (c->selfsym[i]) p.selfsym_mask |= 1u << i;
        p.nent[i] = (unsigned char)c->nent[i];
        if (c->tpos[i] == 1.0f) p.unit_tpos |= 1u << i;
        if (c->tneg[i] == 1.0f) p.unit_tneg |= 1u << i;
        if (c->nent[i] > 16) p.wide_mask |= 1u << i;
        p.uidx[i] = (unsigned char)c->order[i];
        p.code_off[i] = plane_off[c->order[i]];
        internal_of[c->order[i]] = i;
    }
    for (int q = 0; q < c->n_pairs; ++q) {
        const int ia = internal_of[c->pairs[2 * q]], ib = internal_of[c->pairs[2 * q + 1]];
        const int i = std::min(ia, ib), j = std::max(ia, ib), pi = pair_index(i, j);
        p.pair_mask |= 1u << pi;
        if (ia > ib) { p.flip_mask |= 1u << pi; p.flip_slots |= 1u << q; }
        p.pair_slot_w[pi / 4] |= (unsigned)q << (8 * (pi % 4));
        p.pair_pi[q] = (unsigned char)pi;
    }
    p.sums = use_static ? reinterpret_cast<unsigned long long*>(c->static_scratch) : c->d_sums + (size_t)sums_set * kSumsWords;
    p.done = reinterpret_cast<unsigned int*>(p.sums + SOP_K_REPL * SOP_K_NCOL);
    p.acos_pair = c->n_pairs ? out->acos_pair : nullptr;
    p.acos_atom = out->acos_atom;
    p.sel_words = c->n_pairs ? out->sel_words : nullptr;
    p.sel_u32 = c->n_pairs > 16 ? 1 : 0;
    p.scale_code = out->scale_code; p.codes = out->codes; p.blk_cos = out->blk_cos; p.blk_err = out->blk_err; p.blk_rank = out->blk_rank;
    const int emit = (p.scale_code || p.codes || p.blk_cos || p.blk_err || p.blk_rank) ? 1 : 0;

    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    if (use_static) {
        p.stab = reinterpret_cast<const float2*>(c->static_scratch + kStaticSumsBytes);
        p.n_tab_codes = max_code + 1;
    } else if (max_code < SOP_K_MAXTABCODES) {
        ScaleTab t;
        if (sop_status s = scale_table(c, x, y, bias, max_code, k, stream, &t)) return s;
        p.stab = t.dev;
        p.n_tab_codes = t.n;
    }
    const int na_class = A > 6 ? 2 : (A > 2 ? 1 : 0);
    const int sign_mode = c->scale_rule == 1 ? 2 : w;
    int occ = 1, mode = 0;
    const void* fn = sopk_search_kernel(dtype == SOP_BF16, g, sign_mode, (int)metric, emit, na_class, 0, &occ, &mode);
    const int vi = sopk_variant_index(dtype == SOP_BF16, g, sign_mode, (int)metric, emit, na_class, 0);
    const size_t dyn_lds = (((size_t)p.n_bins * SOP_K_BIN_BYTES + 15) & ~(size_t)15) + (((size_t)p.n_tab_codes * sizeof(float2) + 15) & ~(size_t)15) +
                           2 * SOP_K_MAXA * sizeof(float4) + (1 + 2 * SOP_K_NCOL) * sizeof(unsigned long long);
    if (p_out) *p_out = p;
    if (lds_out) *lds_out = dyn_lds;
    hipError_t e = hipSuccess;
    if (c->occ_blocks[vi] == 0 || c->occ_lds[vi] != dyn_lds) {
        if (dyn_lds > 48 * 1024) {
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds);
            if (e != hipSuccess) return hipfail(c, e, "hipFuncSetAttribute(dynamic LDS)");
        }
        int nb = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, 256 * occ, dyn_lds);
        if (e != hipSuccess) return hipfail(c, e, "hipOccupancyMaxActiveBlocksPerMultiprocessor");
        if (nb < 1) return fail(c, SOP_EHIP, "the kernel does not fit on a compute unit with this alphabet and scale format");
        c->occ_blocks[vi] = nb;
        c->occ_lds[vi] = dyn_lds;
    }
    // one workgroup of 4*occ wavefronts per compute unit; each takes a contiguous range of (strip,row) steps
    const long long waves_per_wg = 4 * occ;
    long long wg = std::min<long long>(c->n_cu, (p.total_units + waves_per_wg - 1) / waves_per_wg);
    wg = std::max<long long>(wg, 1);
    p.n_waves = wg * waves_per_wg;
    if (!launch) return SOP_OK;
    if (use_static) {
        const int n_words = (int)kSumsWords, n_thr = std::max(n_words, p.n_tab_codes);
        static_prologue_kernel<<<dim3((unsigned)((n_thr + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
            p.sums, n_words, reinterpret_cast<float2*>(c->static_scratch + kStaticSumsBytes), p.n_tab_codes, y, bias, k);
        if ((e = hipGetLastError()) != hipSuccess) return hipfail(c, e, "kernel launch (static prologue)");
    }
    e = sopk_launch(fn, &p, (int)wg, occ, dyn_lds, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

extern "C" sop_status sop_pair_search(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                      const float* cn, int g, sop_scale_fmt fmt, int k, sop_metric metric,
                                      void* ws, size_t ws_bytes, const sop_outputs* out, void* stream)
{
    return pair_search_impl(c, W, dtype, M, K, ldw, cn, g, fmt, k, metric, ws, ws_bytes, out, stream, true);
}

extern "C" sop_status sop_prepare_scale(sop_ctx* c, sop_scale_fmt fmt, int k, void* stream)
{
    if (!c) return SOP_EINVAL;
    const int x = fmt.exp_bits, y = fmt.man_bits, w = fmt.sign_bits;
    if ((w != 0 && w != 1) || x < 1 || x > 8 || y < 0 || y > 10 || x + y > 15) return fail(c, SOP_EFMT, "scale format: need w in {0,1}, 1<=x<=8, 0<=y<=10, x+y<=15");
    const int bias = fmt.bias < 0 ? (1 << (x - 1)) - 1 : fmt.bias;
    const int max_code = fmt.max_code < 0 ? (1 << (x + y)) - 1 : fmt.max_code;
    if (max_code < 1 || max_code >= (1 << (x + y))) return fail(c, SOP_EFMT, "scale format: max_code out of range");
    if (k < -64 || k > 64 || bias < 0 || bias > 127) return fail(c, SOP_EFMT, "layer shift k must be within [-64, 64], bias within [0, 127]");
    if (1 - bias - y - k < -126 || 1 - bias - k > 126 || std::max(max_code >> y, 1) - bias - k > 125)
        return fail(c, SOP_EFMT, "scale format with this layer shift leaves binary32's normal range (choose bias / max_code / k accordingly)");
    if (max_code >= SOP_K_MAXTABCODES) return SOP_OK;            // such words are decoded arithmetically: nothing to prepare
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    ScaleTab t;
    return scale_table(c, x, y, bias, max_code, k, stream, &t);
}

extern "C" sop_status sop_pair_search_static(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                             const float* cn, int g, sop_scale_fmt fmt, int k, sop_metric metric,
                                             const sop_outputs* out, void* stream)
{
    return pair_search_impl(c, W, dtype, M, K, ldw, cn, g, fmt, k, metric, nullptr, 0, out, stream, true, 0, nullptr, nullptr, true);
}

extern "C" sop_status sop_pair_search_layers(sop_ctx* c, const sop_layer* layers, int n_layers, sop_dtype dtype, int g,
                                             sop_scale_fmt fmt, sop_metric metric, double* acos_pair_table, double* acos_atom_table,
                                             void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!layers || n_layers < 1) return fail(c, SOP_EINVAL, "sop_pair_search_layers: no layers");
    if (!acos_pair_table && !acos_atom_table) return fail(c, SOP_EINVAL, "sop_pair_search_layers: no output table");
    if ((reinterpret_cast<uintptr_t>(acos_pair_table) | reinterpret_cast<uintptr_t>(acos_atom_table)) & 7u)
        return fail(c, SOP_EINVAL, "sop_pair_search_layers: tables must be 8-byte aligned");
    // The layers go through the model-wide kernel: one launch works through a list of layers, its wavefronts
    // passing from layer to layer without a pause (tables loaded once, tickets once), on the caller's stream.
    // Layers are grouped by their layer shift (the scale table in LDS belongs to one shift): a launch per
    // shift, and per kMaxLayers layers.  Where that kernel does not exist (alphabets of one or two atoms) or
    // the tables leave no room in LDS for the layers' sums, there is one kernel per layer, dealt out to two
    // streams of the library's own (each with its own set of layer sums) so that a layer's table load and
    // first rows overlap its predecessor's tail; both streams start after the work already queued on the
    // caller's stream, and the caller's stream continues after both.
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = hipSuccess;
    // ---- every layer is validated before anything is launched (this also prepares the tables of the call);
    //      the format part of the kernel parameters is kept per distinct shift ----
    std::map<int, std::pair<KParams, size_t>> by_shift;
    for (int l = 0; l < n_layers; ++l) {
        const sop_layer& L = layers[l];
        sop_outputs o;
        std::memset(&o, 0, sizeof(o));
        o.acos_atom = acos_atom_table;            // (any non-NULL output: nothing is written in this pass)
        o.acos_pair = acos_pair_table;
        o.sel_words = L.sel_words_dev;
        KParams pk;
        size_t ldsk = 0;
        const sop_status s = pair_search_impl(c, L.W_dev, dtype, L.M, L.K, L.ldw, L.c_dev, g, fmt, L.layer_shift_k, metric,
                                              nullptr, 0, &o, stream, false, 0, &pk, &ldsk);
        if (s != SOP_OK) { c->err = "layer " + std::to_string(l) + ": " + c->err; return s; }
        by_shift.emplace(L.layer_shift_k, std::make_pair(pk, ldsk));
    }
    if (n_layers > 1) {
        const int na_class = c->n_atoms > 6 ? 2 : (c->n_atoms > 2 ? 1 : 0);
        const int sign_mode = c->scale_rule == 1 ? 2 : fmt.sign_bits;
        int occ = 1, mode = 0;
        const void* fn = sopk_search_kernel(dtype == SOP_BF16, g, sign_mode, (int)metric, 0, na_class, 2, &occ, &mode);
        const size_t lds0 = by_shift.begin()->second.second;          // (the same for every shift: table sizes do not depend on it)
        const size_t per_layer = SOP_K_NCOL * sizeof(unsigned long long), slack = 256;     // (the kernel's few static words)
        const long long room = c->lds_max > lds0 + slack ? (long long)((c->lds_max - lds0 - slack) / per_layer) : 0;
        const int chunk = (int)std::min<long long>(kMaxLayers, room);
        if (mode == 2 && chunk >= 2) {
            const int vi = sopk_variant_index(dtype == SOP_BF16, g, sign_mode, (int)metric, 0, na_class, 2);
            const int epl = g < 16 ? g : 16;
            for (const auto& kv : by_shift) {
                std::vector<int> idx;                                 // the layers of this shift, in the caller's order
                for (int l = 0; l < n_layers; ++l) if (layers[l].layer_shift_k == kv.first) idx.push_back(l);
                for (size_t i0 = 0; i0 < idx.size(); i0 += (size_t)chunk) {
                    const int n = (int)std::min<size_t>((size_t)chunk, idx.size() - i0);
                    const int turn = c->ldesc_turn;
                    c->ldesc_turn ^= 1;
                    if (c->ldesc_pending[turn]) {                              // the copy that last used this staging buffer has run?
                        if ((e = hipEventSynchronize(c->ldesc_copied[turn])) != hipSuccess) return hipfail(c, e, "hipEventSynchronize(layer list)");
                        c->ldesc_pending[turn] = false;
                    }
                    LayerDesc* h = c->h_ldesc[turn];
                    for (int i = 0; i < n; ++i) {
                        const int l = idx[i0 + i];
                        const sop_layer& L = layers[l];
                        LayerDesc& d = h[i];
                        const int fold = row_fold(L.M, L.K, L.ldw, epl);
                        const int64_t Mf = L.M / fold, Kf = L.K * fold;
                        d.W = L.W_dev; d.c = L.c_dev; d.sel_words = c->n_pairs ? L.sel_words_dev : nullptr; d.ldw = fold > 1 ? Kf : L.ldw;
                        d.Bk = (int)(Kf / g); d.Nb = L.M * (L.K / g);
                        d.out_row = l;
                        d.M32 = (unsigned int)Mf;
                        d.m_magic = Mf == 1 ? 0xFFFFFFFFu : (unsigned int)((1ull << 32) / (unsigned long long)Mf);
                        d.K = (int)Kf; d.Kc = (int)L.K; d.pad = 0;
                        d.total_units = (unsigned int)(((Kf / epl + 63) / 64) * Mf);
                    }
                    if ((e = hipMemcpyAsync(c->d_ldesc, h, sizeof(LayerDesc) * n, hipMemcpyHostToDevice, (hipStream_t)stream)) != hipSuccess ||
                        (e = hipEventRecord(c->ldesc_copied[turn], (hipStream_t)stream)) != hipSuccess)
                        return hipfail(c, e, "copy of the layer list");
                    c->ldesc_pending[turn] = true;
                    KParams p = kv.second.first;
                    p.W = nullptr; p.c = nullptr; p.sel_words = nullptr;
                    p.layers = c->d_ldesc;
                    p.n_layers = n;
                    p.sums = c->d_msums;
                    p.done = reinterpret_cast<unsigned int*>(c->d_msums + (size_t)kMaxLayers * SOP_K_REPL * SOP_K_NCOL);
                    p.acos_pair = c->n_pairs > 0 ? acos_pair_table : nullptr;
                    p.acos_atom = acos_atom_table;
                    const size_t dyn_lds = lds0 + (size_t)n * per_layer;
                    if (c->occ_blocks[vi] == 0 || c->occ_lds[vi] != dyn_lds) {
                        if (dyn_lds > 48 * 1024 && (e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds)) != hipSuccess)
                            return hipfail(c, e, "hipFuncSetAttribute(dynamic LDS)");
                        int nb = 0;
                        if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, 256 * occ, dyn_lds)) != hipSuccess)
                            return hipfail(c, e, "hipOccupancyMaxActiveBlocksPerMultiprocessor");
                        if (nb < 1) return fail(c, SOP_EHIP, "the model-wide kernel does not fit on a compute unit with this alphabet and scale format");
                        c->occ_blocks[vi] = nb;
                        c->occ_lds[vi] = dyn_lds;
                    }
                    if ((e = sopk_launch(fn, &p, c->n_cu, occ, dyn_lds, stream)) != hipSuccess) return hipfail(c, e, "kernel launch");
                }
            }
            return SOP_OK;
        }
    }
    // ---- otherwise: one kernel per layer, dealt out to streams of the library's own ----
    const int n_lanes = std::min(n_layers, kLanes);     // (three or four streams measured no faster than two)
    const bool lanes = n_lanes > 1;
    for (int i = 0; i < n_lanes && e == hipSuccess; ++i)
        if (!c->lane_stream[i]) e = hipStreamCreateWithFlags(&c->lane_stream[i], hipStreamNonBlocking);
    for (int i = 0; i <= kLanes && e == hipSuccess; ++i)
        if (!c->lane_event[i]) e = hipEventCreateWithFlags(&c->lane_event[i], hipEventDisableTiming);
    if (e != hipSuccess) return hipfail(c, e, "stream / event creation");
    if (lanes) {
        e = hipEventRecord(c->lane_event[kLanes], (hipStream_t)stream);
        for (int i = 0; i < n_lanes && e == hipSuccess; ++i) e = hipStreamWaitEvent(c->lane_stream[i], c->lane_event[kLanes], 0);
        if (e != hipSuccess) return hipfail(c, e, "stream fork");
    }
    for (int l = 0; l < n_layers; ++l) {
        const sop_layer& L = layers[l];
        sop_outputs o;
        std::memset(&o, 0, sizeof(o));
        o.acos_pair = acos_pair_table && c->n_pairs > 0 ? acos_pair_table + (size_t)l * c->n_pairs : nullptr;
        o.acos_atom = acos_atom_table ? acos_atom_table + (size_t)l * c->n_atoms : nullptr;
        o.sel_words = L.sel_words_dev;
        const int lane = lanes ? l % n_lanes : 0;
        void* st = lanes ? (void*)c->lane_stream[lane] : stream;
        const sop_status s = pair_search_impl(c, L.W_dev, dtype, L.M, L.K, L.ldw, L.c_dev, g, fmt, L.layer_shift_k, metric,
                                              nullptr, 0, &o, st, true, lane);
        if (s != SOP_OK) {
            c->err = "layer " + std::to_string(l) + ": " + c->err;
            if (lanes) {                                                  // rejoin what was launched
                for (int i = 0; i < n_lanes; ++i)
                    if (hipEventRecord(c->lane_event[i], c->lane_stream[i]) == hipSuccess) (void)hipStreamWaitEvent((hipStream_t)stream, c->lane_event[i], 0);
            }
            return s;
        }
    }
    if (lanes) {
        for (int i = 0; i < n_lanes; ++i) {
            if ((e = hipEventRecord(c->lane_event[i], c->lane_stream[i])) != hipSuccess ||
                (e = hipStreamWaitEvent((hipStream_t)stream, c->lane_event[i], 0)) != hipSuccess)
                return hipfail(c, e, "stream join");
        }
    }
    return SOP_OK;
}

// ------------------------------------------------------------------ data-derived codebook (DD atom)
static sop_status dd_histogram_impl(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                    const float* cn, int g, int n_bins, int64_t row_step, const uint8_t* block_mask, int n_levels,
                                    int64_t* hist, void* stream, int n_planes = 1, int64_t plane_stride = 0)
{
    if (!c) return SOP_EINVAL;
    if (!W || !hist) return fail(c, SOP_EINVAL, "sop_dd_histogram: W and hist must not be NULL");
    if (dtype != SOP_F32 && dtype != SOP_BF16) return fail(c, SOP_EINVAL, "sop_dd_histogram: dtype must be SOP_F32 or SOP_BF16");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    if (ldw < K) return fail(c, SOP_ESHAPE, "ldw must be at least K");
    const int esz = dtype == SOP_BF16 ? 2 : 4;
    if (!aligned16(W) || (ldw * esz) % 16 != 0) return fail(c, SOP_EINVAL, "W and its row stride must be multiples of 16 bytes");
    if (cn && !aligned16(cn)) return fail(c, SOP_EINVAL, "c must be 16-byte aligned");
    if (!dd_bins_ok(n_bins)) return fail(c, SOP_EINVAL, "n_bins must be a power of two within 64..8192");
    if (n_planes < 1 || (n_planes > 1 && n_levels < 1)) return fail(c, SOP_EINVAL, "several level planes need levels");
    if (n_levels < 0 || n_levels > 255 || (long long)std::max(n_levels, 1) * n_planes * n_bins > SOP_K_DD_MAXBINS)
        return fail(c, SOP_EINVAL, "sop_dd_histogram_levels: n_levels * n_bins must not exceed 8192");
    if (n_levels > 0 && !block_mask) return fail(c, SOP_EINVAL, "sop_dd_histogram_levels: level_dev must not be NULL");
    if (reinterpret_cast<uintptr_t>(hist) & 7u) return fail(c, SOP_EINVAL, "hist must be 8-byte aligned");
    if (row_step < 1) return fail(c, SOP_EINVAL, "row_step must be at least 1");
    const int epl = g < 16 ? g : 16;
    DdParams p;
    std::memset(&p, 0, sizeof(p));
    p.n_planes = n_planes; p.plane_stride = plane_stride;
    p.W = W; p.c = cn; p.block_mask = block_mask; p.n_levels = n_levels; p.M = M; p.K = K; p.ldw = ldw; p.Bk = K / g;
    p.row_step = row_step; p.Ms = (M + row_step - 1) / row_step;
    p.strips = (K / epl + 63) / 64;
    p.total_units = p.strips * p.Ms;
    const long long waves_per_wg = SOP_K_DD_THREADS / 64;
    long long wg = std::min<long long>(c->n_cu, (p.total_units + waves_per_wg - 1) / waves_per_wg);
    p.n_waves = std::max<long long>(wg, 1) * waves_per_wg;
    p.n_bins = n_bins;
    p.acc = c->d_ddacc;
    p.done = reinterpret_cast<unsigned int*>(c->d_ddacc + SOP_K_DD_MAXBINS);
    p.hist = reinterpret_cast<long long*>(hist);
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_dd_launch(&p, dtype == SOP_BF16, g, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

extern "C" sop_status sop_dd_histogram(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                       const float* cn, int g, int n_bins, int64_t row_step, const uint8_t* block_mask, int64_t* hist, void* stream)
{
    return dd_histogram_impl(c, W, dtype, M, K, ldw, cn, g, n_bins, row_step, block_mask, 0, hist, stream);
}

extern "C" sop_status sop_dd_histogram_levels(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw,
                                              const float* cn, int g, int n_bins, int64_t row_step, const uint8_t* level, int n_levels,
                                              int64_t* hist, void* stream)
{
    if (c && n_levels < 1) return fail(c, SOP_EINVAL, "sop_dd_histogram_levels: n_levels must be at least 1");
    return dd_histogram_impl(c, W, dtype, M, K, ldw, cn, g, n_bins, row_step, level, n_levels, hist, stream);
}

// ------------------------------------------------------------------ per-layer scale shift
extern "C" sop_status sop_scale_histogram(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw, int g,
                                          float t_pos, float t_neg, sop_scale_fmt fmt, int64_t* hist, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!W || !hist) return fail(c, SOP_EINVAL, "sop_scale_histogram: W and hist must not be NULL");
    if (dtype != SOP_F32 && dtype != SOP_BF16) return fail(c, SOP_EINVAL, "sop_scale_histogram: dtype must be SOP_F32 or SOP_BF16");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    if (ldw < K) return fail(c, SOP_ESHAPE, "ldw must be at least K");
    const int esz = dtype == SOP_BF16 ? 2 : 4;
    if (!aligned16(W) || (ldw * esz) % 16 != 0) return fail(c, SOP_EINVAL, "W and its row stride must be multiples of 16 bytes");
    if (!(t_pos > 0.0f) || !(t_neg > 0.0f) || !std::isfinite(t_pos) || !std::isfinite(t_neg)) return fail(c, SOP_EATOM, "endpoints must be positive and finite (t_neg is the magnitude of the first entry)");
    FmtRange r;
    if (!resolve_fmt(fmt, r)) return fail(c, SOP_EFMT, "scale format: need w in {0,1}, 1<=x<=8, 0<=y<=10, x+y<=15, valid bias and max_code");
    if (reinterpret_cast<uintptr_t>(hist) & 7u) return fail(c, SOP_EINVAL, "hist must be 8-byte aligned");
    const int epl = sopk_fl_weights_per_lane(dtype == SOP_BF16, g);   // 16 or 32 bytes per lane and step
    FlParams p;
    std::memset(&p, 0, sizeof(p));
    p.W = W; p.M = M; p.K = K; p.ldw = ldw;
    p.strips = (K / epl + 63) / 64;
    p.total_units = p.strips * M;
    const long long waves_per_wg = SOP_K_FL_THREADS / 64;
    // one large workgroup per compute unit: every workgroup adds its counts to the same few words of the
    // running histogram, and atomics to one address are served one after the other
    long long wg = std::min<long long>((long long)c->n_cu, (p.total_units + waves_per_wg - 1) / waves_per_wg);
    p.n_waves = std::max<long long>(wg, 1) * waves_per_wg;
    // the kernel keeps unit numbers in 32 bits
    if (p.total_units >= (1ll << 31) - 4096) return fail(c, SOP_ESHAPE, "the layer has more than 2^31 wavefront steps");
    p.units_per_wg = (int)(p.total_units / std::max<long long>(wg, 1));
    p.units_rem = (int)(p.total_units % std::max<long long>(wg, 1));
    p.t_pos = t_pos; p.t_neg = t_neg;
    int e_top;
    p.m_top = std::frexp((float)r.hi, &e_top);
    p.acc = c->d_ddacc;              // the context's running-histogram words serve both statistics passes
    p.done = reinterpret_cast<unsigned int*>(c->d_ddacc + SOP_K_DD_MAXBINS);
    p.hist = reinterpret_cast<long long*>(hist);
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_fl_launch(&p, dtype == SOP_BF16, g, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

// ------------------------------------------------------------------ layer-scope weight formats
extern "C" sop_status sop_layer_scope_error(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw, const float* cn,
                                            sop_weight_fmt wfmt, sop_scale_fmt sfmt, int k, double* out, uint16_t* codes, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!W || !out) return fail(c, SOP_EINVAL, "sop_layer_scope_error: W and out must not be NULL");
    if (dtype != SOP_F32 && dtype != SOP_BF16) return fail(c, SOP_EINVAL, "sop_layer_scope_error: dtype must be SOP_F32 or SOP_BF16");
    if (M <= 0 || K <= 0) return fail(c, SOP_ESHAPE, "M and K must be positive");
    const int epl = dtype == SOP_BF16 ? 8 : 4, esz = dtype == SOP_BF16 ? 2 : 4;
    if (K % epl != 0) return fail(c, SOP_ESHAPE, "K must be a multiple of 16 bytes of weights");
    if (ldw < K) return fail(c, SOP_ESHAPE, "ldw must be at least K");
    if (!aligned16(W) || (ldw * esz) % 16 != 0) return fail(c, SOP_EINVAL, "W and its row stride must be multiples of 16 bytes");
    if (cn && !aligned16(cn)) return fail(c, SOP_EINVAL, "c must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(out) & 7u) || (codes && (reinterpret_cast<uintptr_t>(codes) & 3u))) return fail(c, SOP_EINVAL, "out must be 8-byte aligned, codes 4-byte aligned");
    FmtRange rs, rw;
    if (!resolve_fmt(sfmt, rs)) return fail(c, SOP_EFMT, "scale format: need w in {0,1}, 1<=x<=8, 0<=y<=10, x+y<=15, valid bias and max_code");
    sop_scale_fmt wf = {0, wfmt.exp_bits, wfmt.man_bits, 0, wfmt.bias, wfmt.max_code};
    if (!resolve_fmt(wf, rw)) return fail(c, SOP_EFMT, "weight format: need 1<=x<=8, 0<=y<=10, x+y<=15, valid bias and max_code");
    if (k < -64 || k > 64) return fail(c, SOP_EFMT, "layer shift k must be within [-64, 64]");
    const int semax = std::max(rs.max_code >> rs.y, 1), wemax = std::max(rw.max_code >> rw.y, 1);
    if (1 - rs.bias - rs.y - k < -126 || 1 - rs.bias - k > 126 || semax - rs.bias - k > 125)
        return fail(c, SOP_EFMT, "scale format with this layer shift leaves binary32's normal range");
    if (1 - rw.bias - rw.y < -126 || wemax - rw.bias > 125) return fail(c, SOP_EFMT, "weight format leaves binary32's normal range");
    LsParams p;
    std::memset(&p, 0, sizeof(p));
    p.W = W; p.c = cn; p.M = M; p.K = K; p.ldw = ldw;
    p.strips = (K / epl + 63) / 64;
    p.total_units = p.strips * M;
    long long wg = std::min<long long>(std::min<long long>((long long)c->n_cu * 4, SOP_K_LS_MAXWG), (p.total_units + 3) / 4);
    p.n_waves = std::max<long long>(wg, 1) * 4;
    p.w_man = rw.y; p.w_bias = rw.bias; p.w_max_code = rw.max_code;
    p.s_man = rs.y; p.s_bias = rs.bias; p.s_max_code = rs.max_code;
    p.k = k; p.pow2k = std::ldexp(1.0f, k);
    p.part = c->d_ls;
    p.maxbits = reinterpret_cast<unsigned int*>(c->d_ls + 3 * SOP_K_LS_MAXWG + 16);   // 128-byte aligned: one cache line per copy
    p.done = reinterpret_cast<unsigned int*>(c->d_ls + 3 * SOP_K_LS_MAXWG + 1);
    p.out = out; p.codes = codes;
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_ls_launch(&p, dtype == SOP_BF16, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

extern "C" sop_status sop_read_probe(sop_ctx* c, const void* x, int64_t n_bytes, uint32_t* out, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!x || !out || n_bytes < 16 || n_bytes % 16 != 0) return fail(c, SOP_EINVAL, "sop_read_probe: x and out must not be NULL, n_bytes a positive multiple of 16");
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(out) & 3u)) return fail(c, SOP_EINVAL, "sop_read_probe: misaligned pointer");
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_probe_launch(x, (long long)(n_bytes / 16), out, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

extern "C" sop_status sop_issue_probe(sop_ctx* c, int kind, int waves_per_simd, int iters, float a, float b, float* out, int* n_out, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (kind < 0 || kind >= SOP_ISSUE_PROBE_KINDS || waves_per_simd < 1 || waves_per_simd > 8 || iters < 1 || iters > (1 << 20) || !out)
        return fail(c, SOP_EINVAL, "sop_issue_probe: kind 0..18, waves_per_simd 1..8, iters 1..2^20, out not NULL");
    if (reinterpret_cast<uintptr_t>(out) & 3u) return fail(c, SOP_EINVAL, "sop_issue_probe: misaligned pointer");
    // every SIMD is to hold exactly waves_per_simd wavefronts: one workgroup per compute unit with that many wavefronts
    // per SIMD (up to four), two such workgroups for six and eight, else workgroups of four wavefronts
    int n_wg = c->n_cu * waves_per_simd, n_threads = 256;
    if (waves_per_simd <= 4) { n_wg = c->n_cu; n_threads = 256 * waves_per_simd; }
    else if (waves_per_simd % 2 == 0) { n_wg = 2 * c->n_cu; n_threads = 128 * waves_per_simd; }
    if (n_out) *n_out = n_wg * n_threads;
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_issue_probe_launch(kind, n_wg, n_threads, iters, a, b, out, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

extern "C" sop_status sop_sum_f32(sop_ctx* c, const float* x, int64_t n, double* out, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!x || !out || n < 1) return fail(c, SOP_EINVAL, "sop_sum_f32: x and out must not be NULL, n positive");
    if ((reinterpret_cast<uintptr_t>(x) & 3u) || (reinterpret_cast<uintptr_t>(out) & 7u)) return fail(c, SOP_EINVAL, "sop_sum_f32: misaligned pointer");
    LsParams p;
    std::memset(&p, 0, sizeof(p));
    p.W = x; p.total_units = n;
    long long wg = std::min<long long>(std::min<long long>((long long)c->n_cu * 4, SOP_K_LS_MAXWG), (n + 255) / 256);
    p.n_waves = std::max<long long>(wg, 1) * 4;
    p.part = c->d_ls;
    p.done = reinterpret_cast<unsigned int*>(c->d_ls + 3 * SOP_K_LS_MAXWG + 1);
    p.out = out;
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_sum_launch(&p, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

// ------------------------------------------------------------------ block ranking and pools (step 2)
extern "C" sop_status sop_partition(sop_ctx* c, const float* score, int64_t n_blocks, int64_t n_top, int higher_is_better,
                                    uint8_t* pool_b, float* tau, int64_t* n_a, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!score || !pool_b || !tau || !n_a) return fail(c, SOP_EINVAL, "sop_partition: score, pool_b, tau and n_a must not be NULL");
    if (n_blocks < 1 || n_blocks > 0x7FFFFFFFll) return fail(c, SOP_ESHAPE, "sop_partition: n_blocks must lie in 1 .. 2^31-1");
    if (n_top < 0 || n_top > n_blocks) return fail(c, SOP_EINVAL, "sop_partition: n_top must lie in 0 .. n_blocks");
    if (!aligned16(score)) return fail(c, SOP_EINVAL, "sop_partition: score must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(pool_b) & 3u) || (reinterpret_cast<uintptr_t>(tau) & 3u) || (reinterpret_cast<uintptr_t>(n_a) & 7u))
        return fail(c, SOP_EINVAL, "sop_partition: pool_b and tau must be 4-byte aligned, n_a 8-byte aligned");
    SelParams p;
    std::memset(&p, 0, sizeof(p));
    p.score = score; p.n = n_blocks; p.n_top = n_top; p.higher = higher_is_better ? 1 : 0; p.all_b = n_top == 0;
    p.hist = c->d_sel + (c->sel_set ? 3 * SOP_K_SEL_BINS : 0); p.hist_other = c->d_sel + (c->sel_set ? 0 : 3 * SOP_K_SEL_BINS);
    p.pool_b = pool_b; p.tau = tau; p.n_a = reinterpret_cast<long long*>(n_a);
    const long long quads = std::max<long long>((n_blocks / 4 + SOP_K_SEL_THREADS - 1) / SOP_K_SEL_THREADS, 1);
    const int n_wg = (int)std::min<long long>((long long)c->n_cu * 4, quads);
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    const long long cquads = std::max<long long>((n_blocks / 4 + SOP_K_CNT_THREADS - 1) / SOP_K_CNT_THREADS, 1);
    const int n_wg_count = (int)std::min<long long>(std::max(c->n_cu / 2, 1), cquads);
    hipError_t e = sopk_sel_launch(&p, n_wg_count, n_wg, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    if (!p.all_b) c->sel_set ^= 1;
    return SOP_OK;
}

// n_planes score planes of n_blocks scores each, back to back, ranked in the same launches (the per-layer
// procedure ranks the blocks under every atom at once): level, tau and n_a hold one row per plane
// (tau / n_a rows of SOP_K_SEL_MAXLEV entries)
static sop_status partition_levels_impl(sop_ctx* c, const float* score, int64_t n_blocks, const int64_t* n_top, int n_levels,
                                        int higher_is_better, uint8_t* level, float* tau, int64_t* n_a, int n_planes, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!score || !n_top || !level || !tau || !n_a) return fail(c, SOP_EINVAL, "sop_partition_levels: score, n_top, level_dev, tau and n_a must not be NULL");
    if (n_blocks < 1 || n_blocks > 0x7FFFFFFFll) return fail(c, SOP_ESHAPE, "sop_partition_levels: n_blocks must lie in 1 .. 2^31-1");
    if (n_levels < 1 || n_levels > SOP_K_SEL_MAXLEV) return fail(c, SOP_EINVAL, "sop_partition_levels: 1 .. 8 thresholds");
    for (int j = 0; j < n_levels; ++j) {
        if (n_top[j] < 0 || n_top[j] > n_blocks) return fail(c, SOP_EINVAL, "sop_partition_levels: n_top must lie in 0 .. n_blocks");
        if (j && n_top[j] < n_top[j - 1]) return fail(c, SOP_EINVAL, "sop_partition_levels: n_top must not decrease (the pools are nested)");
    }
    if (!aligned16(score)) return fail(c, SOP_EINVAL, "sop_partition_levels: score must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(level) & 3u) || (reinterpret_cast<uintptr_t>(tau) & 3u) || (reinterpret_cast<uintptr_t>(n_a) & 7u))
        return fail(c, SOP_EINVAL, "sop_partition_levels: level_dev and tau must be 4-byte aligned, n_a 8-byte aligned");
    SelMParams p;
    std::memset(&p, 0, sizeof(p));
    p.score = score; p.n = n_blocks; p.higher = higher_is_better ? 1 : 0; p.n_levels = n_levels;
    bool any = false;
    for (int j = 0; j < n_levels; ++j) { p.n_top[j] = n_top[j]; any = any || n_top[j] != 0; }
    p.hist = c->d_selm + (c->selm_set ? (size_t)SOP_K_MAXA * SOP_K_SELM_WORDS : 0); p.hist_other = c->d_selm + (c->selm_set ? 0 : (size_t)SOP_K_MAXA * SOP_K_SELM_WORDS);
    p.level = level; p.tau = tau; p.n_a = reinterpret_cast<long long*>(n_a);
    p.n_planes = n_planes;
    p.n_clear = c->selm_dirty[c->selm_set ^ 1];
    p.state = c->d_selstate;
    if (n_planes > 1 && (n_blocks & 3)) return fail(c, SOP_EINVAL, "ranking of several planes: the number of blocks must be a multiple of four");
    const long long quads = std::max<long long>((n_blocks / 4 + SOP_K_SEL_THREADS - 1) / SOP_K_SEL_THREADS, 1);
    const int n_wg = (int)std::min<long long>((long long)c->n_cu * 4, quads);
    const long long cquads = std::max<long long>((n_blocks / 4 + SOP_K_CNT_THREADS - 1) / SOP_K_CNT_THREADS, 1);
    const int n_wg_count = (int)std::min<long long>(std::max(c->n_cu / 2, 1), cquads);
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_selm_launch(&p, n_wg_count, n_wg, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    c->selm_dirty[c->selm_set ^ 1] = 0;
    if (any) { c->selm_dirty[c->selm_set] = std::max(c->selm_dirty[c->selm_set], n_planes); c->selm_set ^= 1; }
    return SOP_OK;
}

extern "C" sop_status sop_partition_levels(sop_ctx* c, const float* score, int64_t n_blocks, const int64_t* n_top, int n_levels,
                                           int higher_is_better, uint8_t* level, float* tau, int64_t* n_a, void* stream)
{
    return partition_levels_impl(c, score, n_blocks, n_top, n_levels, higher_is_better, level, tau, n_a, 1, stream);
}

// ------------------------------------------------------------------ scale words and code payloads
static int code_bits_of(int n_entries) { int n = 1; while ((1 << n) < n_entries) ++n; return n; }

extern "C" sop_status sop_pack_blocks(sop_ctx* c, int64_t M, int64_t K, int g, sop_scale_fmt fmt,
                                      const uint16_t* scale_a, const uint8_t* codes_a, int entries_a,
                                      const uint16_t* scale_b, const uint8_t* codes_b, int entries_b,
                                      const void* sel_words, int sel_word_bytes, int pair_q,
                                      uint16_t* words, uint8_t* payload, int* n_bits_out, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (sop_status s = shape_check(c, M, K, g)) return s;
    if (!scale_a || !codes_a || !words || !payload) return fail(c, SOP_EINVAL, "sop_pack_blocks: scale_a, codes_a, words and payload must not be NULL");
    if (entries_a < 2 || entries_a > SOP_MAX_ENTRIES) return fail(c, SOP_EATOM, "sop_pack_blocks: entries_a out of range");
    const bool two = scale_b || codes_b || sel_words;
    if (two) {
        if (!scale_b || !codes_b || !sel_words) return fail(c, SOP_EINVAL, "sop_pack_blocks: a second codebook needs scale_b, codes_b and sel_words");
        if (entries_b < 2 || entries_b > SOP_MAX_ENTRIES) return fail(c, SOP_EATOM, "sop_pack_blocks: entries_b out of range");
        if (sel_word_bytes != 2 && sel_word_bytes != 4) return fail(c, SOP_EINVAL, "sop_pack_blocks: selector words are 2 or 4 bytes wide");
        if (pair_q < 0 || pair_q >= 8 * sel_word_bytes || pair_q >= SOP_K_MAXP) return fail(c, SOP_EINVAL, "sop_pack_blocks: pair index outside the selector word");
        if (reinterpret_cast<uintptr_t>(sel_words) & (uintptr_t)(sel_word_bytes - 1)) return fail(c, SOP_EINVAL, "sop_pack_blocks: sel_words misaligned");
    }
    const int w = fmt.sign_bits, x = fmt.exp_bits, y = fmt.man_bits, b = fmt.container_bits;
    if ((w != 0 && w != 1) || x < 1 || y < 0 || b < 1 || b > 16 || x + y > 15 || b - w - x - y < 0)
        return fail(c, SOP_EFMT, "sop_pack_blocks: not a SwExMy word in a container of at most 16 bits");
    const int m = b - w - x - y;
    if (two && m == 0) return fail(c, SOP_EFMT, "sop_pack_blocks: the scale format has no metabit for the selector");
    auto mis = [](const void* q, uintptr_t a) { return (reinterpret_cast<uintptr_t>(q) & (a - 1)) != 0; };
    if (mis(codes_a, 8) || (two && mis(codes_b, 8)) || mis(payload, 8) || mis(scale_a, 2) || (two && mis(scale_b, 2)) || mis(words, 2))
        return fail(c, SOP_EINVAL, "sop_pack_blocks: code planes and payload must be 8-byte aligned, 16-bit arrays 2-byte aligned");
    PackParams p;
    std::memset(&p, 0, sizeof(p));
    p.M = M; p.K = K; p.g = g; p.Bk = K / g; p.Nb = M * (K / g);
    p.n_bits = code_bits_of(two ? std::max(entries_a, entries_b) : entries_a);
    p.wide_a = entries_a > 16; p.wide_b = two && entries_b > 16;
    p.scale_a = scale_a; p.scale_b = two ? scale_b : nullptr;
    p.codes_a = codes_a; p.codes_b = two ? codes_b : nullptr;
    p.sel_words = two ? sel_words : nullptr; p.sel_u32 = sel_word_bytes == 4; p.pair_q = two ? pair_q : 0;
    p.sign_pos = w ? b - 1 : -1;
    p.mag_shift = w ? m : (m > 0 ? m - 1 : 0);
    p.sel_pos = !two ? -1 : (w ? m - 1 : b - 1);
    p.words = words; p.payload = payload;
    if (n_bits_out) *n_bits_out = p.n_bits;
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = sopk_pack_launch(&p, stream);
    if (e != hipSuccess) return hipfail(c, e, "kernel launch");
    return SOP_OK;
}

// ------------------------------------------------------------------ the per-layer procedure (steps 1 to 4 and the sweep over p)
namespace {
constexpr size_t kImgBytes = sizeof(BinRec) * SOP_K_MAXBINS;
size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }
struct LayerWs {
    size_t rank, level, hist, tau, na, acos, bins, sc, codes, sel, total;
    int n_img;
};
// An alphabet of more than eight atoms is covered by several searches of at most eight atoms each (the kernel unrolls over
// eight): the two halves [0, 8) and [8, A) whole, which also gives every atom's own ACos and ranking plane, and the pairs
// across the halves by quarters (four atoms of one half with four of the other): at most six searches.
constexpr int kFixedMax = 6;
constexpr int kAcosPer = SOP_K_MAXP + SOP_K_MAXA;          // doubles per such search: its pairs, then its atoms
// acos region, in doubles: kFixedMax searches of the fixed alphabet, then per atom a: 8 pairs (a, L_b(p_j))
constexpr int kAcosFit = kFixedMax * kAcosPer;
constexpr int kAcosAll = kAcosFit + SOP_LAYER_MAX_ATOMS * 8;
LayerWs layer_ws(int64_t M, int64_t K, int g, int A, int n_p, int bins, int pack)
{
    const size_t Nb = (size_t)(M * (K / g));
    LayerWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += up256(bytes); return o; };
    w.rank = take((size_t)A * Nb * sizeof(float));
    w.level = take((size_t)A * up256(Nb));
    w.hist = take((size_t)A * std::max(n_p, 1) * bins * sizeof(long long));
    w.tau = take((size_t)SOP_LAYER_MAX_ATOMS * SOP_K_SEL_MAXLEV * sizeof(float));
    w.na = take((size_t)SOP_LAYER_MAX_ATOMS * SOP_K_SEL_MAXLEV * sizeof(long long));
    w.acos = take((size_t)kAcosAll * sizeof(double));
    w.n_img = kFixedMax + A + 2;                       // the searches of the fixed alphabet, one per atom's sweep, one spare, the winner
    w.bins = take((size_t)w.n_img * kImgBytes);
    w.sc = take(pack ? 2 * Nb * sizeof(uint16_t) : 0);
    w.codes = take(pack ? 2 * (size_t)(M * K) : 0);
    w.sel = take(pack ? Nb * sizeof(uint16_t) : 0);
    w.total = off;
    return w;
}
sop_status layer_opts_check(sop_ctx* c, int n_atoms, const sop_layer_opts* o)
{
    if (!o) return fail(c, SOP_EINVAL, "sop_search_layer: opts is NULL");
    if (n_atoms < 1 || n_atoms > SOP_LAYER_MAX_ATOMS) return fail(c, SOP_EATOM, "sop_search_layer: 1..16 atoms");
    if (o->n_p < 0 || o->n_p > SOP_LAYER_MAX_P) return fail(c, SOP_EINVAL, "sop_search_layer: at most 7 values of p (the atom and its fitted codebooks form one alphabet of 8)");
    for (int j = 0; j < o->n_p; ++j) {
        if (!(o->p_percent[j] >= 0.0 && o->p_percent[j] <= 100.0)) return fail(c, SOP_EINVAL, "sop_search_layer: p must lie in [0, 100]");
        if (j && o->p_percent[j] < o->p_percent[j - 1]) return fail(c, SOP_EINVAL, "sop_search_layer: the values of p must not decrease");
    }
    if (o->n_p > 0) {
        if (o->fit_entries < 2 || o->fit_entries > SOP_MAX_ENTRIES || o->fit_iters < 0) return fail(c, SOP_EINVAL, "sop_search_layer: fit_entries within 2..64, fit_iters >= 0");
        if (!dd_bins_ok(o->fit_bins) || (long long)o->fit_bins * o->n_p > SOP_K_DD_MAXBINS) return fail(c, SOP_EINVAL, "sop_search_layer: fit_bins a power of two within 64..8192 with n_p * fit_bins <= 8192");
        if (o->fit_grid && (o->n_fit_grid < o->fit_entries || o->n_fit_grid > SOP_DD_MAX_CANDIDATES)) return fail(c, SOP_EINVAL, "sop_search_layer: the grid needs fit_entries .. 2047 candidates");
    }
    return SOP_OK;
}
}  // namespace

extern "C" sop_status sop_search_layer_workspace(sop_ctx* c, int64_t M, int64_t K, int g, int n_atoms, const sop_layer_opts* o, size_t* bytes)
{
    if (!c) return SOP_EINVAL;
    if (!bytes) return fail(c, SOP_EINVAL, "sop_search_layer_workspace: bytes is NULL");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    if (sop_status s = layer_opts_check(c, n_atoms, o)) return s;
    *bytes = layer_ws(M, K, g, n_atoms, o->n_p, o->n_p ? o->fit_bins : 64, o->pack).total;
    return SOP_OK;
}

extern "C" sop_status sop_search_layer(sop_ctx* c, const void* W, sop_dtype dtype, int64_t M, int64_t K, int64_t ldw, const float* cn, int g,
                                       sop_scale_fmt fmt, int k, sop_metric metric, const sop_atom* atoms, int n_atoms,
                                       const sop_layer_opts* o, void* ws, size_t ws_bytes, sop_layer_result* res,
                                       uint16_t* words, uint8_t* payload, void* stream)
{
    if (!c) return SOP_EINVAL;
    if (!res || !atoms) return fail(c, SOP_EINVAL, "sop_search_layer: atoms and result must not be NULL");
    if (sop_status s = shape_check(c, M, K, g)) return s;
    if (sop_status s = layer_opts_check(c, n_atoms, o)) return s;
    const int A = n_atoms, n_p = o->n_p, bins = n_p ? o->fit_bins : 64;
    if (A < 2 && n_p == 0) return fail(c, SOP_EINVAL, "sop_search_layer: one atom and no sweep leave no pair to examine");
    if (o->pack && (!words || !payload)) return fail(c, SOP_EINVAL, "sop_search_layer: packing needs words_dev and payload_dev");
    const LayerWs L = layer_ws(M, K, g, A, n_p, bins, o->pack);
    if (!ws || ws_bytes < L.total) return fail(c, SOP_ENOMEM, "sop_search_layer: workspace too small (see sop_search_layer_workspace)");
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(c, SOP_EINVAL, "sop_search_layer: workspace must be 256-byte aligned");
    for (int a = 0; a < A; ++a)
        if (!atoms[a].values || atoms[a].n_entries < 2 || atoms[a].n_entries > SOP_MAX_ENTRIES) return fail(c, SOP_EATOM, "sop_search_layer: an atom needs 2..64 entries");
    std::vector<float> init;
    if (n_p) {
        if (o->fit_init) init.assign(o->fit_init, o->fit_init + o->fit_entries);
        else {
            if (atoms[0].n_entries != o->fit_entries) return fail(c, SOP_EINVAL, "sop_search_layer: without fit_init the first atom is the start grid and must have fit_entries values");
            init.assign(atoms[0].values, atoms[0].values + o->fit_entries);
        }
    }
    const int64_t Nb = M * (K / g);
    char* base = static_cast<char*>(ws);
    hipStream_t st = (hipStream_t)stream;
    DeviceGuard guard(c->device);
    if (guard.err != hipSuccess) return hipfail(c, guard.err, "hipSetDevice");
    hipError_t e = hipSuccess;
    // pinned staging, allocated once per context
    const size_t res_bytes = (size_t)SOP_LAYER_MAX_ATOMS * SOP_K_DD_MAXBINS * sizeof(long long) + (size_t)kAcosAll * sizeof(double);
    if (!c->h_bins) {
        if ((e = hipHostMalloc((void**)&c->h_bins, (size_t)(kFixedMax + SOP_LAYER_MAX_ATOMS + 2) * kImgBytes, hipHostMallocDefault)) != hipSuccess ||
            (e = hipHostMalloc((void**)&c->h_res, res_bytes, hipHostMallocDefault)) != hipSuccess ||
            (e = hipEventCreateWithFlags(&c->stage_done, hipEventDisableTiming)) != hipSuccess)
            return hipfail(c, e, "pinned staging of sop_search_layer");
    }
    if (c->stage_pending) {                            // an earlier call's copies out of the staging buffers have run?
        if ((e = hipEventSynchronize(c->stage_done)) != hipSuccess) return hipfail(c, e, "hipEventSynchronize(staging)");
        c->stage_pending = false;
    }
    // whatever happens below, the context ends up reading its own image again, with no alphabet set
    struct Restore { sop_ctx* c; ~Restore() { c->d_bins_cur = c->d_bins; c->n_atoms = 0; c->n_pairs = 0; } } restore{c};
    auto img = [&](int i) { return reinterpret_cast<BinRec*>(base + L.bins + (size_t)i * kImgBytes); };
    auto himg = [&](int i) { return reinterpret_cast<BinRec*>(reinterpret_cast<char*>(c->h_bins) + (size_t)i * kImgBytes); };
    double* d_acos = reinterpret_cast<double*>(base + L.acos);
    float* d_rank = reinterpret_cast<float*>(base + L.rank);

    // ---- step 1 for every atom, and every pair of fixed atoms: searches of at most eight atoms each, those of the two
    //      halves with the ranking scores out ----
    struct Fixed { int n, atom[SOP_K_MAXA], n_pairs, pr[2 * SOP_K_MAXP]; bool whole; };
    std::vector<Fixed> fx;
    {
        auto add = [&](int lo0, int hi0, int lo1, int hi1) {       // atoms [lo0, hi0) and [lo1, hi1); the second range empty: all pairs of the first
            Fixed f;
            std::memset(&f, 0, sizeof(f));
            for (int a = lo0; a < hi0; ++a) f.atom[f.n++] = a;
            const int n0 = f.n;
            for (int a = lo1; a < hi1; ++a) f.atom[f.n++] = a;
            f.whole = lo1 >= hi1;
            if (f.whole) { for (int i = 0; i < n0; ++i) for (int j = i + 1; j < n0; ++j) { f.pr[2 * f.n_pairs] = i; f.pr[2 * f.n_pairs + 1] = j; ++f.n_pairs; } }
            else for (int i = 0; i < n0; ++i) for (int j = n0; j < f.n; ++j) { f.pr[2 * f.n_pairs] = i; f.pr[2 * f.n_pairs + 1] = j; ++f.n_pairs; }
            fx.push_back(f);
        };
        if (A <= SOP_K_MAXA) add(0, A, 0, 0);
        else {
            add(0, SOP_K_MAXA, 0, 0);
            add(SOP_K_MAXA, A, 0, 0);
            for (int q0 = 0; q0 < SOP_K_MAXA; q0 += 4)
                for (int q1 = SOP_K_MAXA; q1 < A; q1 += 4) add(q0, q0 + 4, q1, std::min(q1 + 4, A));
        }
    }
    for (size_t i = 0; i < fx.size(); ++i) {
        const Fixed& f = fx[i];
        sop_atom sub[SOP_K_MAXA];
        for (int t = 0; t < f.n; ++t) sub[t] = atoms[f.atom[t]];
        if (sop_status s = install_alphabet(c, sub, f.n, img((int)i), himg((int)i), st)) return s;
        if (f.n_pairs) { if (sop_status s = sop_set_pairs(c, f.pr, f.n_pairs)) return s; }
        sop_outputs out;
        std::memset(&out, 0, sizeof(out));
        out.acos_pair = d_acos + i * kAcosPer;
        out.acos_atom = d_acos + i * kAcosPer + SOP_K_MAXP;
        out.blk_rank = (n_p && f.whole) ? d_rank + (size_t)f.atom[0] * Nb : nullptr;      // (a half's atoms are consecutive: so are their planes)
        if (sop_status s = pair_search_impl(c, W, dtype, M, K, ldw, cn, g, fmt, k, metric, nullptr, 0, &out, stream, true)) return s;
    }
    // ---- steps 2 and 3 for every atom and every p: one ranking with n_p thresholds, one pass over the weights ----
    int64_t tops[SOP_K_SEL_MAXLEV] = {0};
    for (int j = 0; j < n_p; ++j) {
        const double v = std::floor(o->p_percent[j] * (double)Nb / 100.0 + 0.5);      // nearest count, halves up
        tops[j] = v < 0.0 ? 0 : (v > (double)Nb ? Nb : (int64_t)v);
    }
    long long* d_hist = reinterpret_cast<long long*>(base + L.hist);
    if (n_p) {
        // all atoms' planes are ranked by the same four launches when they lie back to back with whole float4s (N_b
        // a multiple of four); the level planes are N_b bytes apart then
        const bool batch = (Nb & 3) == 0;
        const size_t lstride = batch ? (size_t)Nb : up256((size_t)Nb);
        uint8_t* d_level = reinterpret_cast<uint8_t*>(base + L.level);
        for (int a0 = 0; batch && a0 < A; a0 += SOP_K_MAXA)           // (the batched ranking takes eight planes a call)
            if (sop_status s = partition_levels_impl(c, d_rank + (size_t)a0 * Nb, Nb, tops, n_p, 1, d_level + (size_t)a0 * lstride,
                                                     reinterpret_cast<float*>(base + L.tau) + a0 * SOP_K_SEL_MAXLEV,
                                                     reinterpret_cast<int64_t*>(base + L.na) + a0 * SOP_K_SEL_MAXLEV, std::min(SOP_K_MAXA, A - a0), stream)) return s;
        // one pass over the weights fills the pool histograms of as many atoms as the histogram pass has room for
        const int per_pass = std::max(1, SOP_K_DD_MAXBINS / (n_p * bins));
        for (int a = 0; a < A; a += per_pass) {
            const int na = std::min(per_pass, A - a);
            if (!batch)
                for (int b = a; b < a + na; ++b)
                    if (sop_status s = partition_levels_impl(c, d_rank + (size_t)b * Nb, Nb, tops, n_p, 1, d_level + b * lstride, reinterpret_cast<float*>(base + L.tau),
                                                             reinterpret_cast<int64_t*>(base + L.na), 1, stream)) return s;
            if (sop_status s = dd_histogram_impl(c, W, dtype, M, K, ldw, o->weighted_fit ? cn : nullptr, g, bins, 1, d_level + a * lstride, n_p,
                                                 reinterpret_cast<int64_t*>(d_hist + (size_t)a * n_p * bins), stream, na, (int64_t)lstride)) return s;
        }
    }
    long long* h_hist = reinterpret_cast<long long*>(c->h_res);
    double* h_acos = reinterpret_cast<double*>(c->h_res + (size_t)SOP_LAYER_MAX_ATOMS * SOP_K_DD_MAXBINS * sizeof(long long));
    if (n_p) {
        if ((e = hipMemcpyAsync(h_hist, d_hist, (size_t)A * n_p * bins * sizeof(long long), hipMemcpyDeviceToHost, st)) != hipSuccess ||
            (e = hipStreamSynchronize(st)) != hipSuccess) return hipfail(c, e, "copy of the pool histograms");
    }
    // ---- the fits (host), and step 4 for one atom's whole sweep per search: alphabet (a, L_b(p_0), L_b(p_1), ...) ----
    std::vector<std::vector<float>> fitted((size_t)A * std::max(n_p, 1));
    std::vector<int> slot_of((size_t)A * std::max(n_p, 1), -1);       // position of (a, j) in the acos region, -1: candidate dropped
    int spare_uses = 0;
    auto score = [&](int a, const std::vector<int>& js, int image, int out_base) -> sop_status {
        std::vector<sop_atom> al(1 + js.size());
        al[0] = atoms[a];
        for (size_t i = 0; i < js.size(); ++i) { al[1 + i].n_entries = o->fit_entries; al[1 + i].values = fitted[(size_t)a * n_p + js[i]].data(); }
        if (sop_status s = install_alphabet(c, al.data(), (int)al.size(), img(image), himg(image), st)) return s;
        int pr[2 * SOP_K_MAXA];
        for (size_t i = 0; i < js.size(); ++i) { pr[2 * i] = 0; pr[2 * i + 1] = 1 + (int)i; }
        if (sop_status s = sop_set_pairs(c, pr, (int)js.size())) return s;
        sop_outputs out;
        std::memset(&out, 0, sizeof(out));
        out.acos_pair = d_acos + out_base;
        if (sop_status s = pair_search_impl(c, W, dtype, M, K, ldw, cn, g, fmt, k, metric, nullptr, 0, &out, stream, true)) return s;
        for (size_t i = 0; i < js.size(); ++i) slot_of[(size_t)a * n_p + js[i]] = out_base + (int)i;
        return SOP_OK;
    };
    for (int a = 0; a < A && n_p; ++a) {
        std::vector<int> js;
        for (int j = 0; j < n_p; ++j) {
            const long long* h = h_hist + ((size_t)a * n_p + j) * bins;
            bool any = false;
            for (int b = 0; b < bins && !any; ++b) any = h[b] != 0;
            std::vector<float>& Lb = fitted[(size_t)a * n_p + j];
            Lb.assign(o->fit_entries, 0.0f);
            sop_status fs = SOP_OK;
            if (!any) Lb = init;                                   // an empty pool: the start grid stands in
            else if (o->fit_grid) {
                std::vector<int> chosen(o->fit_entries);
                fs = sop_dd_fit_grid(reinterpret_cast<const int64_t*>(h), bins, o->fit_grid, o->n_fit_grid, o->fit_entries, chosen.data(), nullptr);
                if (fs == SOP_OK) for (int t = 0; t < o->fit_entries; ++t) Lb[t] = (float)o->fit_grid[chosen[t]];
            } else fs = sop_dd_fit(reinterpret_cast<const int64_t*>(h), bins, o->fit_entries, o->fit_iters, init.data(), Lb.data());
            if (fs == SOP_OK) js.push_back(j);
            else if (fs != SOP_EATOM) return fail(c, fs, std::string("sop_search_layer: fit: ") + soph::host_last_error());
        }
        if (js.empty()) continue;
        sop_status s = score(a, js, kFixedMax + a, kAcosFit + 8 * a);
        if (s == SOP_EATOM && js.size() > 1) {
            // some fitted codebook cannot be searched next to the others (entries too closely spaced for the
            // element-search table): the candidates are scored one by one, through one spare image, and
            // those that fail alone are dropped
            for (size_t i = 0; i < js.size(); ++i) {
                if (spare_uses++ && (e = hipStreamSynchronize(st)) != hipSuccess) return hipfail(c, e, "hipStreamSynchronize");
                s = score(a, std::vector<int>(1, js[i]), kFixedMax + A, kAcosFit + 8 * a + (int)i);
                if (s != SOP_OK && s != SOP_EATOM) return s;
            }
        } else if (s != SOP_OK && s != SOP_EATOM) return s;
    }
    if ((e = hipMemcpyAsync(h_acos, d_acos, (size_t)(kAcosFit + 8 * A) * sizeof(double), hipMemcpyDeviceToHost, st)) != hipSuccess ||
        (e = hipStreamSynchronize(st)) != hipSuccess) return hipfail(c, e, "copy of the ACos values");
    // ---- the best (L_a, p, L_b): the largest layer ACos, the first one among equals (fixed pairs in their
    //      order, then atom by atom, p by p) ----
    std::memset(res, 0, sizeof(*res));
    res->a = -1; res->b = -1;
    const double nan = std::numeric_limits<double>::quiet_NaN();
    for (int q = 0; q < SOP_LAYER_MAX_PAIRS; ++q) res->acos_fixed[q] = nan;
    for (int a = 0; a < SOP_LAYER_MAX_ATOMS; ++a) res->acos_atom[a] = nan;
    for (size_t i = 0; i < fx.size(); ++i) {
        const Fixed& f = fx[i];
        for (int t = 0; t < f.n_pairs; ++t) {
            const int a = f.atom[f.pr[2 * t]], b = f.atom[f.pr[2 * t + 1]];
            res->acos_fixed[a * (2 * A - a - 1) / 2 + (b - a - 1)] = h_acos[i * kAcosPer + t];
        }
        if (f.whole) for (int t = 0; t < f.n; ++t) res->acos_atom[f.atom[t]] = h_acos[i * kAcosPer + SOP_K_MAXP + t];
    }
    for (int a = 0; a < SOP_LAYER_MAX_ATOMS; ++a) {
        for (int j = 0; j < SOP_LAYER_MAX_P; ++j) {
            const int sl = (a < A && j < n_p) ? slot_of[(size_t)a * n_p + j] : -1;
            res->acos_fitted[a][j] = sl >= 0 ? h_acos[sl] : nan;
        }
    }
    bool have = false;
    {
        int q = 0;
        for (int a = 0; a < A; ++a)
            for (int b = a + 1; b < A; ++b, ++q)
                if (!have || res->acos_fixed[q] > res->acos) { have = true; res->kind = 0; res->a = a; res->b = b; res->p_percent = 0.0; res->acos = res->acos_fixed[q]; }
    }
    for (int a = 0; a < A; ++a)
        for (int j = 0; j < n_p; ++j) {
            const double v = res->acos_fitted[a][j];
            if (v == v && (!have || v > res->acos)) { have = true; res->kind = 1; res->a = a; res->b = -1; res->j = j; res->p_percent = o->p_percent[j]; res->acos = v; }
        }
    if (!have) return fail(c, SOP_EATOM, "sop_search_layer: no candidate could be scored");
    const float* tb = res->kind == 0 ? atoms[res->b].values : fitted[(size_t)res->a * n_p + res->j].data();
    res->n_entries_b = res->kind == 0 ? atoms[res->b].n_entries : o->fit_entries;
    std::memcpy(res->table_b, tb, sizeof(float) * res->n_entries_b);
    // ---- materialisation of the winner ----
    if (o->pack) {
        sop_atom two[2] = {atoms[res->a], {res->n_entries_b, res->table_b}};
        if (sop_status s = install_alphabet(c, two, 2, img(kFixedMax + A + 1), himg(kFixedMax + A + 1), st)) return s;
        uint16_t* sc = reinterpret_cast<uint16_t*>(base + L.sc);
        uint8_t* codes = reinterpret_cast<uint8_t*>(base + L.codes);
        const size_t plane_a = two[0].n_entries <= 16 ? (size_t)(M * K / 2) : (size_t)(M * K);
        sop_outputs out;
        std::memset(&out, 0, sizeof(out));
        out.acos_pair = d_acos; out.scale_code = sc; out.codes = codes; out.sel_words = base + L.sel;
        if (sop_status s = pair_search_impl(c, W, dtype, M, K, ldw, cn, g, fmt, k, metric, nullptr, 0, &out, stream, true)) return s;
        if (sop_status s = sop_pack_blocks(c, M, K, g, fmt, sc, codes, two[0].n_entries, sc + Nb, codes + plane_a, two[1].n_entries,
                                           base + L.sel, 2, 0, words, payload, &res->n_bits, stream)) return s;
    }
    if ((e = hipEventRecord(c->stage_done, st)) != hipSuccess) return hipfail(c, e, "hipEventRecord");
    c->stage_pending = true;
    return SOP_OK;
}
