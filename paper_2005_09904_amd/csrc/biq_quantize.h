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
    __shared__ uint2 mask_strip[kQuantThreads / 64][EPT];  // per wave: the sign bits of each step of a plane
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
    for (int t = 0; t < EPT; ++t) r[t] = ((t * WPR + wsub) * 64 + lane < n) ? r[t] + 0.0f : 0.0f;
    // (+ 0.0f turns a weight of -0.0 into +0.0 and changes nothing else; a residual is never -0.0
    // afterwards (x - x = +0.0 under round-to-nearest), so the sign bit of r is exactly "r < 0" and
    // sign(0) = +1 as in Eq. 1's reading: the code and the residual update below agree)
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
        // The 64 sign bits of step t are wave-uniform (a ballot); they go through a per-wave LDS
        // strip, word t, so that afterwards lane t (and t - 64) holds step t's bits and the row's
        // keys leave in a few wide stores instead of one small store per step.  A wave only reads
        // what it wrote itself: LDS operations of one wave complete in order, no barrier needed.
        uint2* const strip = mask_strip[wave];
#pragma unroll
        for (int t = 0; t < EPT; ++t) {
            const bool valid = t < nvalid;
            const unsigned long long mask = __ballot(valid && !(r[t] < 0.0f));
            // r -= copysign(a, r)
            const float rn = r[t] - __uint_as_float((__float_as_uint(r[t]) & 0x80000000u) | __float_as_uint(a));
            r[t] = valid ? rn : 0.0f;
            if (lane == 0) strip[t] = make_uint2((uint32_t)mask, (uint32_t)(mask >> 32));
        }
#pragma unroll
        for (int u = 0; u < (EPT + 63) / 64; ++u) {
            const int t = 64 * u + lane;
            const int word = t * WPR + wsub;
            if (t < EPT && word < words) *reinterpret_cast<uint2*>(krow + 2 * word) = strip[t];
        }
    }
}

}  // namespace biq
