// Instances of the nnz-balanced serial kernel for 1 or 2 chunk lanes per stored entry.
#include "sgap_nnz_serial_impl.hpp"

namespace sgap {

hipError_t launch_nnz_serial_lc1_2(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, int tile,
                                   bool merge, hipStream_t s)
{
    const nnz_serial_detail::Launch f{a, compute_units, nnz_hint, offsets_fit_32(a), tile, merge, s};
    switch (lc) {
        case 1: return f.run<1>(vec);
        case 2: return f.run<2>(vec);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgap
