// Large-batch path: input vectors scaled and split into fp16 terms, and the unpack + MFMA contraction.
#include "biq_launch.h"

namespace biq {
namespace {

template <int Q, int RPW, int CT, int WS>
hipError_t launch_unpack_inst(const UnpackParams& up, int grid, int lds, hipStream_t s) {
    if constexpr (WS == 4 && Q * RPW * CT == 8) {
        return hipErrorInvalidValue;  // not built (register file, LDS): the planner rejects it
    } else {
        if (lds != UnpackGeom<CT, WS>::LDS_BYTES) return hipErrorInvalidValue;
        return launch_large_lds<unpack_mfma_kernel<Q, RPW, CT, WS>, false>(up, grid, kUnpackThreads, lds, s);
    }
}

template <int CT, int WS>
hipError_t launch_unpack_qr(int q, int rpw, const UnpackParams& up, int grid, int lds, hipStream_t s) {
    switch (q * 8 + rpw) {
        case 1 * 8 + 1: return launch_unpack_inst<1, 1, CT, WS>(up, grid, lds, s);
        case 1 * 8 + 2: return launch_unpack_inst<1, 2, CT, WS>(up, grid, lds, s);
        case 1 * 8 + 4: return launch_unpack_inst<1, 4, CT, WS>(up, grid, lds, s);
        case 2 * 8 + 1: return launch_unpack_inst<2, 1, CT, WS>(up, grid, lds, s);
        case 2 * 8 + 2: return launch_unpack_inst<2, 2, CT, WS>(up, grid, lds, s);
        case 3 * 8 + 1: return launch_unpack_inst<3, 1, CT, WS>(up, grid, lds, s);
        case 4 * 8 + 1: return launch_unpack_inst<4, 1, CT, WS>(up, grid, lds, s);
    }
    return hipErrorInvalidValue;  // the planner admits no other combination
}

}  // namespace

hipError_t launch_unpack(int q, int rpw, int ct, int ws, const UnpackParams& up, int grid, int lds,
                         hipStream_t s) {
    switch (ct * 8 + ws) {
        case 1 * 8 + 1: return launch_unpack_qr<1, 1>(q, rpw, up, grid, lds, s);
        case 1 * 8 + 2: return launch_unpack_qr<1, 2>(q, rpw, up, grid, lds, s);
        case 1 * 8 + 4: return launch_unpack_qr<1, 4>(q, rpw, up, grid, lds, s);
        case 2 * 8 + 1: return launch_unpack_qr<2, 1>(q, rpw, up, grid, lds, s);
        case 2 * 8 + 2: return launch_unpack_qr<2, 2>(q, rpw, up, grid, lds, s);
        case 2 * 8 + 4: return launch_unpack_qr<2, 4>(q, rpw, up, grid, lds, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_xsplit(int ct, const float* X, mfma_u32x4* Xf, int* colexp, int n, int batch, int steps,
                         int padded_batch, hipStream_t s) {
    // one workgroup per (padded) input vector, in blocks of 64 workgroups = 8 line groups x 8 vectors
    const unsigned grid = (unsigned)((padded_batch + 63) / 64 * 64);
    if (ct == 2)
        hipLaunchKernelGGL(xsplit_kernel<2>, dim3(grid), dim3(kXsplitThreads), 0, s, X, Xf, colexp, n, batch,
                           padded_batch, steps);
    else if (ct == 1)
        hipLaunchKernelGGL(xsplit_kernel<1>, dim3(grid), dim3(kXsplitThreads), 0, s, X, Xf, colexp, n, batch,
                           padded_batch, steps);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace biq
