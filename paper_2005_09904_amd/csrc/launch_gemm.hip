// mu = 8, two input vectors per pass: the batched table kernel and its half-table variant.
#include "biq_launch.h"

#include "biq_gemm8x2.h"
#include "biq_gemm8x2h.h"

namespace biq {
namespace {

template <bool FUSED>
hipError_t launch_gemm8x2_q(int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    switch (q) {
        case 1: return launch_large_lds<gemm8x2_kernel<1, FUSED>, true>(qp, grid, threads, lds, s);
        case 2: return launch_large_lds<gemm8x2_kernel<2, FUSED>, true>(qp, grid, threads, lds, s);
        case 3: return launch_large_lds<gemm8x2_kernel<3, FUSED>, true>(qp, grid, threads, lds, s);
        case 4: return launch_large_lds<gemm8x2_kernel<4, FUSED>, true>(qp, grid, threads, lds, s);
    }
    return hipErrorInvalidValue;
}

template <bool FUSED>
hipError_t launch_gemm8x2h_q(int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    switch (q) {
        case 1: return launch_large_lds<gemm8x2h_kernel<1, FUSED>, true>(qp, grid, threads, lds, s);
        case 2: return launch_large_lds<gemm8x2h_kernel<2, FUSED>, true>(qp, grid, threads, lds, s);
        case 3: return launch_large_lds<gemm8x2h_kernel<3, FUSED>, true>(qp, grid, threads, lds, s);
        case 4: return launch_large_lds<gemm8x2h_kernel<4, FUSED>, true>(qp, grid, threads, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemm8x2(bool fused, int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    return fused ? launch_gemm8x2_q<true>(q, qp, grid, threads, lds, s)
                 : launch_gemm8x2_q<false>(q, qp, grid, threads, lds, s);
}

hipError_t launch_lstm8x2h(int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    switch (q) {
        case 1: return launch_large_lds<lstm8x2h_kernel<1>, true>(qp, grid, threads, lds, s);
        case 2: return launch_large_lds<lstm8x2h_kernel<2>, true>(qp, grid, threads, lds, s);
        case 3: return launch_large_lds<lstm8x2h_kernel<3>, true>(qp, grid, threads, lds, s);
        case 4: return launch_large_lds<lstm8x2h_kernel<4>, true>(qp, grid, threads, lds, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm8x2h(bool fused, int q, const QueryParams& qp, int grid, int threads, int lds,
                           hipStream_t s) {
    return fused ? launch_gemm8x2h_q<true>(q, qp, grid, threads, lds, s)
                 : launch_gemm8x2h_q<false>(q, qp, grid, threads, lds, s);
}

}  // namespace biq
