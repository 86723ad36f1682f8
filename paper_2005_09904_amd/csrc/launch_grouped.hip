// Grouped launch: several small problems of one kernel family in one dispatch.
#include "biq_launch.h"

#include "biq_grouped.h"

namespace biq {
namespace {

template <int KIND>
hipError_t launch_grouped_q(int q, const GroupParams& g, int grid, int lds, hipStream_t s) {
    switch (q) {
        case 1: return launch_large_lds<grouped_kernel<KIND, 1>, true>(g, grid, 1024, lds, s);
        case 2: return launch_large_lds<grouped_kernel<KIND, 2>, true>(g, grid, 1024, lds, s);
        case 3: return launch_large_lds<grouped_kernel<KIND, 3>, true>(g, grid, 1024, lds, s);
        case 4: return launch_large_lds<grouped_kernel<KIND, 4>, true>(g, grid, 1024, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_grouped(int kind, int q, const GroupParams& g, int grid, int lds, hipStream_t s) {
    switch (kind) {
        case GROUP_GEMV8: return launch_grouped_q<GROUP_GEMV8>(q, g, grid, lds, s);
        case GROUP_GEMV8H: return launch_grouped_q<GROUP_GEMV8H>(q, g, grid, lds, s);
        case GROUP_GEMM8X2H: return launch_grouped_q<GROUP_GEMM8X2H>(q, g, grid, lds, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace biq
