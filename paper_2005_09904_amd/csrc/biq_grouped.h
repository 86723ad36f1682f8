// Several small multiplies in one dispatch (grouped launch).
//
// A small layer's run time is one dependent dispatch (about 2.5 us) plus the latency of one table
// build and one round of key loads, whatever its size (Table IV's batch-1 column shows the same
// plateau on the paper's GPU).  Layers that do not depend on each other - the sub-layers of a
// Transformer block, the gates and directions of LSTM layers (Sec. II-C) - can share that cost:
// the grid of this kernel is the concatenation of the grids of up to kGroupMax problems, each
// workgroup finds its problem from a prefix table in the kernel arguments and then runs the
// ordinary kernel body on it.  All problems of a launch use the same kernel family and plane
// count (the host groups them accordingly); shapes, batch sizes and buffers are free.
#pragma once

#include "biq_gemm8x2h.h"
#include "biq_gemv8.h"
#include "biq_gemv8h.h"

namespace biq {

constexpr int kGroupMax = 16;

struct GroupParams {
    QueryParams p[kGroupMax];
    int first_wg[kGroupMax + 1];  // first workgroup of each problem; [count] = grid size
    int count;
};

enum GroupKind { GROUP_GEMV8 = 0, GROUP_GEMV8H = 1, GROUP_GEMM8X2H = 2 };

template <int KIND, int Q>
__global__ __launch_bounds__(1024) void grouped_kernel(const GroupParams g) {
    const int wg_all = blockIdx.x;
    int i = 0;
    while (i + 1 < g.count && wg_all >= g.first_wg[i + 1]) ++i;  // the same for the whole workgroup
    const QueryParams& p = g.p[i];
    const int wg = wg_all - g.first_wg[i];
    if constexpr (KIND == GROUP_GEMV8) gemv8_body<Q, true, 1024>(p, wg);
    else if constexpr (KIND == GROUP_GEMV8H) gemv8h_body<Q, true, false>(p, wg);
    else gemm8x2h_body<Q, true, false>(p, wg);
}

}  // namespace biq
