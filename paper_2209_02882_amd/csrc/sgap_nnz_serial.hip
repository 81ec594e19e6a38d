// Nnz-balanced schedule, serial strategy: the plan (tile size, merge mode) and
// the dispatch of the launch to the translation units that hold the kernel
// instances.
#include "sgap_common.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

// Tile size and merge mode of the serial kernel for a given layout; the
// zeroing pass must be launched with the same merge_log2.  forced_tile > 0
// overrides the choice of the tile size.
NnzPlan plan_nnz_serial(int group, int lc, int vec, int64_t nnz_hint, int compute_units, int forced_tile)
{
    NnzPlan p;
    // keep every entry lane busy: tile >= lanes * group; 1024 or 2048 positions
    p.tile = (kBlock / lc) * group > 1024 ? 2048 : 1024;
    // A small matrix gives the chip only a few tiles per workgroup, or fewer
    // tiles than the chip holds workgroups (about 4 per compute unit).  Rate a
    // tile size by the share of the chip that is busy over the rounds of
    // tiles, the last of which is only partly filled, and take the largest
    // tile that keeps 85 % busy, else the best one.
    // No tile below half a step of the workgroup (a step gives every entry lane
    // `group` positions; below half a step most lanes idle, which costs more
    // than it gains: powerlaw at N=16, G=32: 0.069 against 0.032 ms), nor below 256.
    const int step = (kBlock / lc) * group;
    const int min_tile = step / 2 >= p.tile ? p.tile : (step / 2 > 256 ? step / 2 : 256);
    if (forced_tile >= 1024 || (forced_tile > 0 && vec == 4)) {
        p.tile = forced_tile;
    } else if (nnz_hint > 0 && vec == 4 && lc >= 8) {
        // (narrower passes do too little per entry to pay for more, smaller tiles:
        // powerlaw at N=16 runs 0.032 ms with the full tile, 0.044 ms with the balanced one)
        const double resident = 4.0 * compute_units;
        int best_tile = p.tile;
        double best_busy = 0.0;
        for (int tile = p.tile; tile >= min_tile; tile /= 2) {
            const double rounds = (double)((nnz_hint + tile - 1) / tile) / resident;
            const double whole = (double)(int64_t)(rounds + 0.999999);
            const double busy_share = rounds / whole;
            if (busy_share > best_busy + 1e-9) {
                best_busy = busy_share;
                best_tile = tile;
            }
            if (busy_share >= 0.85) break;
        }
        p.tile = best_tile;
    }
    auto fits = [&](int tile) { return (tile / group + 1) * (lc * vec * 4 + 8) <= kMergeLdsBudget; };
    // merging a tile's partial sums on chip is worth a smaller tile: the
    // alternative is a global atomic add per partial sum
    if (forced_tile == 0 && vec == 4)
        while (!fits(p.tile) && p.tile / 2 >= min_tile) p.tile /= 2;
    p.merge = fits(p.tile);
    p.lc = lc;
    if (!p.merge && forced_tile == 0) {
        // most of the LDS, the smallest tile this vector width has, and if need be narrower passes
        // (against a global atomic add per flush: stencil27 G = 1 and 2 33 and 15.9 ms -> 22.9 and 6.6, rmat
        // G = 1 44 -> 7.7, skewed G = 4 23.4 -> 13.7; skewed G = 1, whose long rows meet on one slot either
        // way, is the one loss: 82 -> 95)
        const int small = vec == 4 ? 256 : 1024;
        auto fits_most = [&](int lanes) { return (small / group + 1) * (lanes * vec * 4 + 8) <= kMergeLdsLimit; };
        int lanes = lc;
        while (!fits_most(lanes) && lanes > 1) lanes /= 2;
        if (fits_most(lanes)) {
            p.tile = small;
            p.lc = lanes;
            p.merge = true;
        }
    }
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

hipError_t launch_nnz_serial(const SpmmArgs& a, int lc, int vec, const NnzPlan& plan, int compute_units,
                             int64_t nnz_hint, hipStream_t s)
{
    lc = plan.lc;  // the plan may have narrowed the layout
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
