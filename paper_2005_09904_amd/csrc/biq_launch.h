// Internal interface between the C ABI (biq_api.hip: argument checks, planner) and the
// translation units that instantiate and launch the kernels (launch_*.hip).  One kernel family
// per translation unit, so that the library builds in parallel.  Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "biq_kernels.h"
#include "biq_unpack_mfma.h"

namespace biq {

constexpr int kLdsPerCu = 160 * 1024;  // gfx950: LDS of one CU, the most a workgroup can ask for

// Opt-in to dynamic LDS above 48 KiB and, for the kernels that address LDS absolutely
// (lds_read_abs), the proof that dynamic LDS starts at address 0: a kernel's dynamic LDS follows
// its static LDS, so a kernel whose code object reports 0 bytes of static LDS has its
// `extern __shared__` array at LDS address 0.  Both belong to (function, device): `granted` is the
// instantiation's bitmap of devices already done (devices >= 64 are done every time).
// Concurrent first calls from several threads at worst do the work twice.
inline hipError_t grant_large_lds(const void* kern, unsigned long long& granted, bool needs_lds_base_0) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && ((__atomic_load_n(&granted, __ATOMIC_RELAXED) >> dev) & 1ull)) return hipSuccess;
    if (needs_lds_base_0) {
        hipFuncAttributes attr;
        e = hipFuncGetAttributes(&attr, kern);
        if (e != hipSuccess) return e;
        if (attr.sharedSizeBytes != 0) return hipErrorInvalidDeviceFunction;  // never launch it
    }
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsPerCu);
    if (e == hipSuccess && dev >= 0 && dev < 64) __atomic_fetch_or(&granted, 1ull << dev, __ATOMIC_RELAXED);
    return e;
}

// Launch of a kernel that needs more than 48 KiB of dynamic LDS; one opt-in bitmap per kernel.
// ABS_LDS: the kernel reads its tables through absolute LDS addresses.
template <auto Kern, bool ABS_LDS, typename Params>
hipError_t launch_large_lds(const Params& params, int grid, int threads, int lds, hipStream_t s) {
    static unsigned long long granted = 0;
    if (hipError_t e = grant_large_lds(reinterpret_cast<const void*>(Kern), granted, ABS_LDS); e != hipSuccess)
        return e;
    hipLaunchKernelGGL(Kern, dim3(grid), dim3(threads), lds, s, params);
    return hipGetLastError();
}

// ---- lookup-table query kernels (fused: tables built from X in LDS; else copied from p.LUT) ----
hipError_t launch_query_generic(bool fused, int mu, int bt, const QueryParams& p, int grid, int threads,
                                int lds, hipStream_t s);
hipError_t launch_wide(bool fused, int mu, const QueryParams& p, int grid, int threads, int lds, hipStream_t s);
hipError_t launch_gemv8(bool fused, int q, const QueryParams& p, int grid, int threads, int lds, hipStream_t s);
hipError_t launch_gemv8h(bool fused, int q, const QueryParams& p, int grid, int threads, int lds, hipStream_t s);
hipError_t launch_gemm8x2(bool fused, int q, const QueryParams& p, int grid, int threads, int lds, hipStream_t s);
hipError_t launch_gemm8x2h(bool fused, int q, const QueryParams& p, int grid, int threads, int lds, hipStream_t s);

// ---- fused LSTM cell step (half-table kernels with the cell update as epilogue) ----
hipError_t launch_lstm8h(int q, const QueryParams& p, int grid, int threads, int lds, hipStream_t s);
hipError_t launch_lstm8x2h(int q, const QueryParams& p, int grid, int threads, int lds, hipStream_t s);

// ---- several small problems in one dispatch (kind: GroupKind) ----
struct GroupParams;
hipError_t launch_grouped(int kind, int q, const GroupParams& g, int grid, int lds, hipStream_t s);

// ---- unpack + MFMA path ----
// (terms: 3 = exact split into bf16 terms, 2 = two scaled fp16 terms)
hipError_t launch_xsplit(int terms, int ct, const float* X, mfma_u32x4* Xf, int* colexp, int n, int batch,
                         int steps, int padded_batch, hipStream_t s);
hipError_t launch_unpack(int terms, int q, int rpw, int ct, int ws, const UnpackParams& up, int grid, int lds,
                         hipStream_t s);

// ---- the small kernels ----
// Y[i] = sum over the `splits` partial results [splits][count], in a fixed order.
hipError_t launch_reduce_splits(const float* partial, float* Y, long long count, int splits, hipStream_t s);
hipError_t launch_pack(const int8_t* B, uint32_t* K, long long key_rows, int n, int stride_dw, hipStream_t s);
hipError_t launch_unpack_keys(int mu, bool wide_keys, const uint32_t* K, void* keys, long long key_rows, int C,
                              int stride_dw, hipStream_t s);
hipError_t launch_build_lut(int mu, const float* X, float* LUT, int n, int batch, int C, hipStream_t s);
hipError_t launch_quantize(const float* W, uint32_t* K, float* alpha, int m, int n, int q, int stride_dw,
                           hipStream_t s);

}  // namespace biq
