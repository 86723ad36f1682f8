// mu = 8, one input vector: the streaming GEMV kernel and its half-table variant.
#include "biq_launch.h"

#include "biq_gemv8.h"
#include "biq_gemv8h.h"

namespace biq {
namespace {

template <int Q, bool FUSED, int MAXT>
hipError_t launch_gemv8_inst(const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    if (threads > MAXT) return hipErrorInvalidValue;
    return launch_large_lds<gemv8_kernel<Q, FUSED, MAXT>, true>(qp, grid, threads, lds, s);
}

template <bool FUSED>
hipError_t launch_gemv8_q(int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    switch (q) {
        case 1: return launch_gemv8_inst<1, FUSED, 1024>(qp, grid, threads, lds, s);
        case 2: return launch_gemv8_inst<2, FUSED, 1024>(qp, grid, threads, lds, s);
        case 3: return launch_gemv8_inst<3, FUSED, 1024>(qp, grid, threads, lds, s);
        case 4:
            // 4 planes: up to 512 threads run an instantiation with a deeper key ring (more registers)
            return threads <= 512 ? launch_gemv8_inst<4, FUSED, 512>(qp, grid, threads, lds, s)
                                  : launch_gemv8_inst<4, FUSED, 1024>(qp, grid, threads, lds, s);
    }
    return hipErrorInvalidValue;
}

template <bool FUSED>
hipError_t launch_gemv8h_q(int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    switch (q) {
        case 1: return launch_large_lds<gemv8h_kernel<1, FUSED>, true>(qp, grid, threads, lds, s);
        case 2: return launch_large_lds<gemv8h_kernel<2, FUSED>, true>(qp, grid, threads, lds, s);
        case 3: return launch_large_lds<gemv8h_kernel<3, FUSED>, true>(qp, grid, threads, lds, s);
        case 4: return launch_large_lds<gemv8h_kernel<4, FUSED>, true>(qp, grid, threads, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_gemv8(bool fused, int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    return fused ? launch_gemv8_q<true>(q, qp, grid, threads, lds, s)
                 : launch_gemv8_q<false>(q, qp, grid, threads, lds, s);
}

hipError_t launch_lstm8h(int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    switch (q) {
        case 1: return launch_large_lds<lstm8h_kernel<1>, true>(qp, grid, threads, lds, s);
        case 2: return launch_large_lds<lstm8h_kernel<2>, true>(qp, grid, threads, lds, s);
        case 3: return launch_large_lds<lstm8h_kernel<3>, true>(qp, grid, threads, lds, s);
        case 4: return launch_large_lds<lstm8h_kernel<4>, true>(qp, grid, threads, lds, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemv8h(bool fused, int q, const QueryParams& qp, int grid, int threads, int lds, hipStream_t s) {
    return fused ? launch_gemv8h_q<true>(q, qp, grid, threads, lds, s)
                 : launch_gemv8h_q<false>(q, qp, grid, threads, lds, s);
}

}  // namespace biq
