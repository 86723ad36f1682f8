// mu <= 6: the kernel with 32 lanes per row and key-independent LDS banks.
#include "biq_launch.h"

#include "biq_query_wide.h"

namespace biq {
namespace {

template <bool FUSED>
hipError_t launch_wide_mu(int mu, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    switch (mu) {
        case 1: return launch_large_lds<query_wide_kernel<1, FUSED>, true>(qp, grid, threads, lds, s);
        case 2: return launch_large_lds<query_wide_kernel<2, FUSED>, true>(qp, grid, threads, lds, s);
        case 3: return launch_large_lds<query_wide_kernel<3, FUSED>, true>(qp, grid, threads, lds, s);
        case 4: return launch_large_lds<query_wide_kernel<4, FUSED>, true>(qp, grid, threads, lds, s);
        case 5: return launch_large_lds<query_wide_kernel<5, FUSED>, true>(qp, grid, threads, lds, s);
        case 6: return launch_large_lds<query_wide_kernel<6, FUSED>, true>(qp, grid, threads, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_wide(bool fused, int mu, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    return fused ? launch_wide_mu<true>(mu, qp, grid, threads, lds, s)
                 : launch_wide_mu<false>(mu, qp, grid, threads, lds, s);
}

}  // namespace biq
