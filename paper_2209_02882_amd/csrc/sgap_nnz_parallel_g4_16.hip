// Instances of the nnz-balanced parallel kernel for group sizes 4, 16.
#include "sgap_nnz_parallel_impl.hpp"

namespace sgap {

hipError_t launch_nnz_parallel_g4_16(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, bool merge,
                                     hipStream_t s)
{
    using nnz_parallel_detail::launch_group;
    switch (a.group) {
        case 4: return launch_group<4>(a, lc, vec, compute_units, nnz_hint, merge, s);
        case 16: return launch_group<16>(a, lc, vec, compute_units, nnz_hint, merge, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgap
