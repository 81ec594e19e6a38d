// Instances of the nnz-balanced serial kernel for 16 or 32 chunk lanes per stored entry.
#include "sgap_nnz_serial_impl.hpp"

namespace sgap {

hipError_t launch_nnz_serial_lc16_32(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, int tile,
                                     bool merge, hipStream_t s)
{
    const nnz_serial_detail::Launch f{a, compute_units, nnz_hint, offsets_fit_32(a), tile, merge, s};
    switch (lc) {
        case 16: return f.run<16>(vec);
        case 32: return f.run<32>(vec);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgap
