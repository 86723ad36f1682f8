// Binary-coding quantisation of a weight matrix, row by row (Sec. II-B, Eq. 1):
// w ~ sum_i alpha_i b_i, b_i in {-1,+1}^n.  The paper only names the heuristic ("greedy
// approximation"); this is the greedy procedure Eq. 1 suggests, one plane at a time on the
// residual r (r = w at the start):
//     b_i = sign(r) (sign(0) = +1),  alpha_i = mean |r|,  r <- r - alpha_i b_i
// Each step is the exact minimiser of Eq. 1 for q = 1 applied to the residual.  The signs are
// written straight in the packed key format (bit j of the row <-> element j, +1 <-> 1), the
// scales as alpha[q][m]: the outputs feed biq_gemm without a pass over int8 signs.
//
// The residual lives in registers.  Rows up to 8192 elements: one wave per row (element
// j = 64*t + lane, so one ballot per t is two key dwords), no barriers.  Longer rows (up to
// 32768): the four waves of a workgroup share a row, one barrier per plane for the sum.  Sums
// are taken in a fixed order (per lane over its strided elements, then a butterfly inside the
// wave, then over the waves), so the result does not depend on timing.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace biq {

constexpr int kQuantThreads = 256;
constexpr int kQuantMaxN = 32768;

// WPR waves per row (1: four rows per workgroup; 4: one row per workgroup), EPT elements per
// lane: n <= 64 * EPT * WPR.  Lane l of wave w (of the row's WPR waves) holds elements
// j = (t * WPR + w) * 64 + l, t = 0 .. EPT-1: the ballot of step t is the 64-bit word t * WPR + w
// of the packed row.
template <int EPT, int WPR>
__global__ __launch_bounds__(kQuantThreads) void quantize_wave_kernel(const float* __restrict__ W,
                                                                      uint32_t* __restrict__ K,
                                                                      float* __restrict__ alpha, int m,
                                                                      int n, int q, int stride_dw) {
    __shared__ float wave_sums[2][4];   // WPR = 4: the waves' partial sums, double buffered over the planes
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wsub = wave % WPR;
    const int row = blockIdx.x * (kQuantThreads / 64 / WPR) + wave / WPR;
    if (row >= m) return;   // WPR = 4: whole workgroup
    const float* wrow = W + (size_t)row * n;
    // All loads are issued unconditionally (addresses clamped into the row) so that they are in
    // flight together; elements past n are then zeroed and stay zero.
    float r[EPT];
#pragma unroll
    for (int t = 0; t < EPT; ++t) r[t] = wrow[min((t * WPR + wsub) * 64 + lane, n - 1)];
#pragma unroll
    for (int t = 0; t < EPT; ++t) r[t] = ((t * WPR + wsub) * 64 + lane < n) ? r[t] : 0.0f;
    const int words = stride_dw / 2;  // 64-bit words of the packed row (stride is a multiple of 16 bytes)
    // this lane holds elements of steps 0 .. nvalid - 1
    int nvalid = max(0, (n - lane - 64 * wsub + 64 * WPR - 1) / (64 * WPR));
    for (int i = 0; i < q; ++i) {
        // (keeps the EPT "step is valid" predicates from being hoisted out of this loop into
        // 2 * EPT scalar registers)
        asm volatile("" : "+v"(nvalid));
        float s = 0.0f;
#pragma unroll
        for (int t = 0; t < EPT; ++t) s += fabsf(r[t]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
        if constexpr (WPR > 1) {
            if (lane == 0) wave_sums[i & 1][wave] = s;
            __syncthreads();
            s = ((wave_sums[i & 1][0] + wave_sums[i & 1][1]) + wave_sums[i & 1][2]) + wave_sums[i & 1][3];
        }
        const float a = s / (float)n;
        if (lane == 0 && wsub == 0) alpha[(size_t)i * m + row] = a;
        uint32_t* krow = K + ((size_t)i * m + row) * stride_dw;
        // lane t (and t - 64) keeps the 64 sign bits of step t: the row's keys leave in a few
        // wide stores instead of one small store per step
        int keep_lo[(EPT + 63) / 64], keep_hi[(EPT + 63) / 64];
#pragma unroll
        for (int u = 0; u < (EPT + 63) / 64; ++u) { keep_lo[u] = 0; keep_hi[u] = 0; }
#pragma unroll
        for (int t = 0; t < EPT; ++t) {
            const bool valid = t < nvalid;
            // one predicate decides the code and the residual update: b = -1 iff r < 0, so that
            // r = +0.0 and r = -0.0 (a weight may be -0.0) both take b = +1 and r - alpha (Eq. 1
            // with sign(0) = +1)
            const bool neg = r[t] < 0.0f;
            const unsigned long long mask = __ballot(valid && !neg);
            const float rn = neg ? r[t] + a : r[t] - a;
            r[t] = valid ? rn : 0.0f;
            // the (wave-uniform) mask halves go into lane t of the keep registers: a compare and two
            // selects, all visible to the compiler's hazard handling (this toolchain has no builtin
            // for v_writelane_b32)
            const bool mine = lane == (t & 63);
            keep_lo[t >> 6] = mine ? (int)(uint32_t)mask : keep_lo[t >> 6];
            keep_hi[t >> 6] = mine ? (int)(uint32_t)(mask >> 32) : keep_hi[t >> 6];
        }
#pragma unroll
        for (int u = 0; u < (EPT + 63) / 64; ++u) {
            const int t = 64 * u + lane;
            const int word = t * WPR + wsub;
            if (t < EPT && word < words)
                *reinterpret_cast<uint2*>(krow + 2 * word) = make_uint2((uint32_t)keep_lo[u], (uint32_t)keep_hi[u]);
        }
    }
}

}  // namespace biq
