// The small kernels: key packing, index extraction, tables to device memory, sum of partial
// results, quantiser.
#include "biq_launch.h"

#include "biq_quantize.h"

namespace biq {

hipError_t launch_reduce_splits(const float* partial, float* Y, long long count, int splits, hipStream_t s) {
    const bool vec4 = (count % 4 == 0) && ((reinterpret_cast<uintptr_t>(partial) & 15) == 0) &&
                      ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
    if (vec4)
        hipLaunchKernelGGL(reduce_splits_kernel<4>, dim3((unsigned)((count / 4 + 255) / 256)), dim3(256), 0, s,
                           partial, Y, count, splits);
    else
        hipLaunchKernelGGL(reduce_splits_kernel<1>, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s,
                           partial, Y, count, splits);
    return hipGetLastError();
}

hipError_t launch_pack(const int8_t* B, uint32_t* K, long long key_rows, int n, int stride_dw, hipStream_t s) {
    const long long total = key_rows * stride_dw;
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (n % 16 == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0)
        hipLaunchKernelGGL(pack_kernel<true>, dim3(grid), dim3(256), 0, s, B, K, key_rows, n, stride_dw);
    else
        hipLaunchKernelGGL(pack_kernel<false>, dim3(grid), dim3(256), 0, s, B, K, key_rows, n, stride_dw);
    return hipGetLastError();
}

namespace {

template <typename KEY>
hipError_t launch_unpack_keys_t(int mu, const uint32_t* K, KEY* keys, long long key_rows, int C, int stride_dw,
                                hipStream_t s) {
#define BIQ_UNPACK_CASE(MU)                                                                          \
    case MU: {                                                                                       \
        const long long total = key_rows * ((C + KeyUnit<MU>::UK - 1) / KeyUnit<MU>::UK);            \
        hipLaunchKernelGGL((unpack_keys_kernel<MU, KEY>), dim3((unsigned)((total + 255) / 256)),     \
                           dim3(256), 0, s, K, keys, key_rows, C, stride_dw);                        \
        break;                                                                                       \
    }
    switch (mu) {
        BIQ_UNPACK_CASE(1) BIQ_UNPACK_CASE(2) BIQ_UNPACK_CASE(3) BIQ_UNPACK_CASE(4) BIQ_UNPACK_CASE(5)
        BIQ_UNPACK_CASE(6) BIQ_UNPACK_CASE(7) BIQ_UNPACK_CASE(8) BIQ_UNPACK_CASE(9) BIQ_UNPACK_CASE(10)
        default: return hipErrorInvalidValue;
    }
#undef BIQ_UNPACK_CASE
    return hipGetLastError();
}

}  // namespace

hipError_t launch_unpack_keys(int mu, bool wide_keys, const uint32_t* K, void* keys, long long key_rows, int C,
                              int stride_dw, hipStream_t s) {
    return wide_keys ? launch_unpack_keys_t<uint16_t>(mu, K, static_cast<uint16_t*>(keys), key_rows, C, stride_dw, s)
                     : launch_unpack_keys_t<uint8_t>(mu, K, static_cast<uint8_t*>(keys), key_rows, C, stride_dw, s);
}

hipError_t launch_build_lut(int mu, const float* X, float* LUT, int n, int batch, int C, hipStream_t s) {
    const int HG = mu > 4 ? (1 << (mu - 4)) : 1;
    const bool vec4 = (batch % 4 == 0) && ((reinterpret_cast<uintptr_t>(LUT) & 15) == 0);
    const int bv = vec4 ? batch / 4 : batch;
    // box of a workgroup: up to 64 vector groups, then key groups, then chunks, 256 threads in all
    int lta = 0, lth = 0;
    while (lta < 6 && (1 << lta) < bv) ++lta;
    while (lta + lth < 8 && (1 << lth) < HG) ++lth;
    const int ltc = 8 - lta - lth;
    const long long a_tiles = ((long long)bv + (1 << lta) - 1) >> lta;
    const long long h_tiles = ((long long)HG + (1 << lth) - 1) >> lth;
    const long long c_tiles = ((long long)C + (1 << ltc) - 1) >> ltc;
    const long long boxes = a_tiles * h_tiles * c_tiles;
    if (boxes > 0x7fffffffll) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)boxes;
#define BIQ_LUT_CASE(MU)                                                                           \
    case MU:                                                                                       \
        if (vec4)                                                                                  \
            hipLaunchKernelGGL((build_lut_kernel<MU, 4>), dim3(grid), dim3(256), 0, s, X, LUT, n,  \
                               batch, C, lta, lth, ltc, (int)a_tiles, (int)h_tiles);               \
        else                                                                                       \
            hipLaunchKernelGGL((build_lut_kernel<MU, 1>), dim3(grid), dim3(256), 0, s, X, LUT, n,  \
                               batch, C, lta, lth, ltc, (int)a_tiles, (int)h_tiles);               \
        break;
    switch (mu) {
        BIQ_LUT_CASE(1) BIQ_LUT_CASE(2) BIQ_LUT_CASE(3) BIQ_LUT_CASE(4) BIQ_LUT_CASE(5)
        BIQ_LUT_CASE(6) BIQ_LUT_CASE(7) BIQ_LUT_CASE(8) BIQ_LUT_CASE(9) BIQ_LUT_CASE(10)
        default: return hipErrorInvalidValue;
    }
#undef BIQ_LUT_CASE
    return hipGetLastError();
}

hipError_t launch_quantize(const float* W, uint32_t* K, float* alpha, int m, int n, int q, int stride_dw,
                           hipStream_t s) {
    if (n > kQuantMaxN) return hipErrorInvalidValue;
#define BIQ_QUANT_CASE(EPT, WPR)                                                                   \
    hipLaunchKernelGGL((quantize_wave_kernel<EPT, WPR>), dim3((m + (4 / WPR) - 1) / (4 / WPR)),   \
                       dim3(kQuantThreads), 0, s, W, K, alpha, m, n, q, stride_dw)
    if (n <= 64 * 8) BIQ_QUANT_CASE(8, 1);
    else if (n <= 64 * 16) BIQ_QUANT_CASE(16, 1);
    else if (n <= 64 * 32) BIQ_QUANT_CASE(32, 1);
    else if (n <= 64 * 64) BIQ_QUANT_CASE(64, 1);
    else if (n <= 64 * 128) BIQ_QUANT_CASE(128, 1);
    else if (n <= 64 * 64 * 4) BIQ_QUANT_CASE(64, 4);    // four waves per row
    else BIQ_QUANT_CASE(128, 4);
#undef BIQ_QUANT_CASE
    return hipGetLastError();
}

}  // namespace biq
