// Binary-coding quantisation of a weight matrix, row by row (Sec. II-B, Eq. 1):
// w ~ sum_i alpha_i b_i, b_i in {-1,+1}^n.  The paper only names the heuristic ("greedy
// approximation"); this is the greedy procedure Eq. 1 suggests, one plane at a time on the
// residual r (r = w at the start):
//     b_i = sign(r) (sign(0) = +1),  alpha_i = mean |r|,  r <- r - alpha_i b_i
// Each step is the exact minimiser of Eq. 1 for q = 1 applied to the residual.  The signs are
// written straight in the packed key format (bit j of the row <-> element j, +1 <-> 1), the
// scales as alpha[q][m]: the outputs feed biq_gemm without a pass over int8 signs.
//
// Two kernels.  Rows up to 8192 elements: one wave per row, the residual in registers (element
// j = 64*t + lane, so one ballot per t is two key dwords), no barriers.  Longer rows (up to
// 32768): one workgroup per row, the residual in LDS.  Sums are taken in a fixed order (per lane
// over its strided elements, then a butterfly inside the wave, then over the waves), so the
// result does not depend on timing.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace biq {

constexpr int kQuantThreads = 256;
constexpr int kQuantMaxN = 32768;

__global__ __launch_bounds__(kQuantThreads) void quantize_kernel(const float* __restrict__ W,
                                                                 uint32_t* __restrict__ K,
                                                                 float* __restrict__ alpha, int m, int n,
                                                                 int q, int stride_dw) {
    extern __shared__ __align__(16) float qlds[];   // [n] residual, then [4] wave sums
    float* const wave_sums = qlds + ((n + 3) & ~3);
    const int row = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const float* wrow = W + (size_t)row * n;

    if ((n & 3) == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0) {
        for (int j = tid * 4; j < n; j += kQuantThreads * 4)
            *reinterpret_cast<float4*>(qlds + j) = *reinterpret_cast<const float4*>(wrow + j);
    } else {
        for (int j = tid; j < n; j += kQuantThreads) qlds[j] = wrow[j];
    }
    __syncthreads();

    const int stride_bits = stride_dw * 32;
    for (int i = 0; i < q; ++i) {
        float s = 0.0f;
        for (int j = tid; j < n; j += kQuantThreads) s += fabsf(qlds[j]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) wave_sums[wave] = s;
        __syncthreads();
        const float a = (((wave_sums[0] + wave_sums[1]) + wave_sums[2]) + wave_sums[3]) / (float)n;
        if (tid == 0) alpha[(size_t)i * m + row] = a;
        uint32_t* krow = K + ((size_t)i * m + row) * stride_dw;
        // 64 consecutive elements per wave and step: one ballot = two key dwords
        for (int j0 = wave * 64; j0 < stride_bits; j0 += kQuantThreads) {
            const int j = j0 + lane;
            bool plus = false;
            if (j < n) {
                const float v = qlds[j];
                plus = !(v < 0.0f);
                qlds[j] = v - (plus ? a : -a);
            }
            const unsigned long long mask = __ballot(plus);
            if (lane == 0) {
                krow[j0 >> 5] = (uint32_t)mask;
                krow[(j0 >> 5) + 1] = (uint32_t)(mask >> 32);
            }
        }
        __syncthreads();
    }
}

// One wave per row, EPT elements per lane (n <= 64 * EPT).
template <int EPT>
__global__ __launch_bounds__(kQuantThreads) void quantize_wave_kernel(const float* __restrict__ W,
                                                                      uint32_t* __restrict__ K,
                                                                      float* __restrict__ alpha, int m,
                                                                      int n, int q, int stride_dw) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * (kQuantThreads / 64) + (threadIdx.x >> 6);
    if (row >= m) return;
    const float* wrow = W + (size_t)row * n;
    // All loads are issued unconditionally (addresses clamped into the row) so that they are in
    // flight together; elements past n are then zeroed and stay zero.
    float r[EPT];
#pragma unroll
    for (int t = 0; t < EPT; ++t) r[t] = wrow[min(64 * t + lane, n - 1)];
#pragma unroll
    for (int t = 0; t < EPT; ++t) r[t] = (64 * t + lane < n) ? r[t] : 0.0f;
    const int steps = stride_dw / 2;  // 64-bit groups of the packed row (stride is a multiple of 16 bytes)
    int nvalid = (n - lane + 63) >> 6;  // this lane holds elements of steps 0 .. nvalid - 1
    for (int i = 0; i < q; ++i) {
        // (keeps the EPT "step is valid" predicates from being hoisted out of this loop into
        // 2 * EPT scalar registers)
        asm volatile("" : "+v"(nvalid));
        float s = 0.0f;
#pragma unroll
        for (int t = 0; t < EPT; ++t) s += fabsf(r[t]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
        const float a = s / (float)n;
        if (lane == 0) alpha[(size_t)i * m + row] = a;
        uint32_t* krow = K + ((size_t)i * m + row) * stride_dw;
        // lane t (and t - 64) keeps the 64 sign bits of step t: the row's keys leave in one or two
        // coalesced stores instead of one small store per step
        int keep_lo[(EPT + 63) / 64], keep_hi[(EPT + 63) / 64];
#pragma unroll
        for (int u = 0; u < (EPT + 63) / 64; ++u) { keep_lo[u] = 0; keep_hi[u] = 0; }
#pragma unroll
        for (int t = 0; t < EPT; ++t) {
            const bool valid = t < nvalid;
            const unsigned long long mask = __ballot(valid && !(r[t] < 0.0f));
            // r -= copysign(a, r), with sign(0) = +1: -0.0 never occurs (x - x = +0.0)
            const float rn = r[t] - __uint_as_float((__float_as_uint(r[t]) & 0x80000000u) | __float_as_uint(a));
            r[t] = valid ? rn : 0.0f;
            // v_writelane_b32: the (wave-uniform) mask halves go into lane t of the keep registers.
            // The mask comes from a VALU compare; the assembler text is not seen by the compiler's
            // hazard recogniser, hence the explicit wait states before the first read.
            asm("s_nop 4\n\tv_writelane_b32 %0, %1, %2" : "+v"(keep_lo[t >> 6]) : "s"((uint32_t)mask), "n"(t & 63));
            asm("v_writelane_b32 %0, %1, %2" : "+v"(keep_hi[t >> 6]) : "s"((uint32_t)(mask >> 32)), "n"(t & 63));
        }
#pragma unroll
        for (int u = 0; u < (EPT + 63) / 64; ++u) {
            const int t = 64 * u + lane;
            if (t < EPT && t < steps)
                *reinterpret_cast<uint2*>(krow + 2 * t) = make_uint2((uint32_t)keep_lo[u], (uint32_t)keep_hi[u]);
        }
    }
}

}  // namespace biq
