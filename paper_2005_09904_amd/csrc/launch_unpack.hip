// Large-batch path, exact input split (three bf16 terms): the input split and the unpack + MFMA
// contraction; the entry points that pick the number of terms.
#include "biq_launch_unpack.inc"

namespace biq {

hipError_t launch_unpack_2term(int q, int rpw, int ct, int ws, const UnpackParams& up, int grid, int lds,
                               hipStream_t s);
hipError_t launch_xsplit_2term(int ct, const float* X, mfma_u32x4* Xf, int* colexp, int n, int batch, int steps,
                               int padded_batch, hipStream_t s);

hipError_t launch_unpack(int terms, int q, int rpw, int ct, int ws, const UnpackParams& up, int grid, int lds,
                         hipStream_t s) {
    if (terms == 3) return launch_unpack_terms<3>(q, rpw, ct, ws, up, grid, lds, s);
    if (terms == 2) return launch_unpack_2term(q, rpw, ct, ws, up, grid, lds, s);
    return hipErrorInvalidValue;
}

hipError_t launch_xsplit(int terms, int ct, const float* X, mfma_u32x4* Xf, int* colexp, int n, int batch,
                         int steps, int padded_batch, hipStream_t s) {
    if (terms == 3) return launch_xsplit_terms<3>(ct, X, Xf, colexp, n, batch, steps, padded_batch, s);
    if (terms == 2) return launch_xsplit_2term(ct, X, Xf, colexp, n, batch, steps, padded_batch, s);
    return hipErrorInvalidValue;
}

}  // namespace biq
