// Large-batch path, two scaled fp16 terms per input element (plan.input_terms = 2).
#include "biq_launch_unpack.inc"

namespace biq {

hipError_t launch_unpack_2term(int q, int rpw, int ct, int ws, const UnpackParams& up, int grid, int lds,
                               hipStream_t s) {
    return launch_unpack_terms<2>(q, rpw, ct, ws, up, grid, lds, s);
}

hipError_t launch_xsplit_2term(int ct, const float* X, mfma_u32x4* Xf, int* colexp, int n, int batch, int steps,
                               int padded_batch, hipStream_t s) {
    return launch_xsplit_terms<2>(ct, X, Xf, colexp, n, batch, steps, padded_batch, s);
}

}  // namespace biq
