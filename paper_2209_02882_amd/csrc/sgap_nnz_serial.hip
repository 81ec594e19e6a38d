// Nnz-balanced schedule, serial strategy: the plan (tile size, merge mode) and
// the dispatch of the launch to the translation units that hold the kernel
// instances.
#include "sgap_common.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

// Tile size and merge mode of the serial kernel for a given layout; the
// zeroing pass must be launched with the same merge_log2.
NnzPlan plan_nnz_serial(int group, int lc, int vec)
{
    NnzPlan p;
    // keep every entry lane busy: tile >= lanes * group; 1024 or 2048 positions
    p.tile = (kBlock / lc) * group > 1024 ? 2048 : 1024;
    const int nslots = p.tile / group + 1;
    p.merge = nslots * (lc * vec * 4 + 8) <= kMergeLdsBudget;
    int lg = 0;
    while ((1 << lg) < (p.merge ? p.tile : group)) ++lg;
    p.merge_log2 = lg;
    return p;
}

// per-layout launchers, defined in sgap_nnz_serial_lc*.hip
hipError_t launch_nnz_serial_lc1_2(const SpmmArgs&, int, int, int, int64_t, int, bool, hipStream_t);
hipError_t launch_nnz_serial_lc4_8(const SpmmArgs&, int, int, int, int64_t, int, bool, hipStream_t);
hipError_t launch_nnz_serial_lc16_32(const SpmmArgs&, int, int, int, int64_t, int, bool, hipStream_t);
hipError_t launch_nnz_serial_lc64(const SpmmArgs&, int, int, int, int64_t, int, bool, hipStream_t);

hipError_t launch_nnz_serial(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, hipStream_t s)
{
    const NnzPlan plan = plan_nnz_serial(a.group, lc, vec);
    switch (lc) {
        case 1: case 2: return launch_nnz_serial_lc1_2(a, lc, vec, compute_units, nnz_hint, plan.tile, plan.merge, s);
        case 4: case 8: return launch_nnz_serial_lc4_8(a, lc, vec, compute_units, nnz_hint, plan.tile, plan.merge, s);
        case 16: case 32:
            return launch_nnz_serial_lc16_32(a, lc, vec, compute_units, nnz_hint, plan.tile, plan.merge, s);
        case 64: return launch_nnz_serial_lc64(a, lc, vec, compute_units, nnz_hint, plan.tile, plan.merge, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgap
