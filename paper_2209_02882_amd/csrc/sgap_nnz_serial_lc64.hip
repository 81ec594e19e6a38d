// Instances of the nnz-balanced serial kernel for 64 chunk lanes per stored entry.
#include "sgap_nnz_serial_impl.hpp"

namespace sgap {

hipError_t launch_nnz_serial_lc64(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, int tile,
                                  bool merge, hipStream_t s)
{
    const nnz_serial_detail::Launch f{a, compute_units, nnz_hint, offsets_fit_32(a), tile, merge, s};
    switch (lc) {
        case 64: return f.run<64>(vec);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgap
