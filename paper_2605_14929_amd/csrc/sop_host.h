// Host-only part of the library (no GPU code, no HIP headers): codebook builders, the element-search table,
// the fits on histograms and the choice of the layer shift.  Kept in a translation unit of its own so that it
// can be built for the CPU alone, e.g. with the sanitizers.
#ifndef SOP_HOST_H
#define SOP_HOST_H
#include <string>
#include <vector>

#include "../../include/sop.h"
#include "sop_kparams.h"

namespace soph {

// status and text of a failed host-only call (what sop_last_error(NULL) returns), per thread
sop_status host_fail(sop_status s, const std::string& msg);
const char* host_last_error();

struct AlphabetPlan {
    std::vector<std::vector<float>> tabs;      // caller's order
    int n_atoms = 0;
    int order[SOP_K_MAXA] = {0}, gid[SOP_K_MAXA] = {0}, mirror[SOP_K_MAXA] = {0}, selfsym[SOP_K_MAXA] = {0};
    float sc[SOP_K_MAXA] = {0}, off[SOP_K_MAXA] = {0}, lo[SOP_K_MAXA] = {0}, hi[SOP_K_MAXA] = {0};
    int n_bins = 0;
    std::vector<BinRec> img;
};
// Validate the atoms, form the scale groups and build the bin table; on failure *err receives the text.
sop_status plan_alphabet(std::string* err, const sop_atom* atoms, int n_atoms, AlphabetPlan& pl);

inline bool dd_bins_ok(int n_bins) { return n_bins >= 64 && n_bins <= SOP_K_DD_MAXBINS && (n_bins & (n_bins - 1)) == 0; }

struct FmtRange { int x, y, bias, max_code; double lo, hi; };
// resolves the defaults and checks the format as sop_pair_search() does
bool resolve_fmt(const sop_scale_fmt& fmt, FmtRange& r);

}  // namespace soph
#endif
