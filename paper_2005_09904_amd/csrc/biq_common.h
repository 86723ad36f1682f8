// Shared device-side definitions of libbiq (gfx950 only).
//
// Key stream: a packed row is a little-endian bit string; the key of chunk c for
// LUT-unit MU is bits [MU*c, MU*c + MU) (paper Sec. III-B; element j <-> bit j as in
// Algorithms 1 and 3).  A lane always handles a "unit": UD consecutive dwords holding
// UK whole keys, so that no key straddles two lanes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace biq {

constexpr int kWave = 64;

template <int MU> struct KeyUnit;
// 16-byte units where MU divides 32 ...
template <> struct KeyUnit<8> { static constexpr int UD = 4, UK = 16; };
template <> struct KeyUnit<4> { static constexpr int UD = 4, UK = 32; };
template <> struct KeyUnit<2> { static constexpr int UD = 4, UK = 64; };
template <> struct KeyUnit<1> { static constexpr int UD = 4, UK = 128; };
// ... and the shortest run of whole dwords that holds whole keys otherwise
template <> struct KeyUnit<6> { static constexpr int UD = 3, UK = 16; };
template <> struct KeyUnit<3> { static constexpr int UD = 3, UK = 32; };
template <> struct KeyUnit<5> { static constexpr int UD = 5, UK = 32; };
template <> struct KeyUnit<7> { static constexpr int UD = 7, UK = 32; };
// keys wider than a byte (the sizes Eq. 6 favours for large m): 32 keys in 9 dwords, 16 in 5
template <> struct KeyUnit<9> { static constexpr int UD = 9, UK = 32; };
template <> struct KeyUnit<10> { static constexpr int UD = 5, UK = 16; };
constexpr int kMaxMu = 10;

// Key t (compile-time position) of a unit held in w[0..UD).
template <int MU, int T, int UD>
__device__ __forceinline__ uint32_t unit_key(const uint32_t (&w)[UD]) {
    constexpr int bit = T * MU;
    constexpr int d = bit >> 5;
    constexpr int s = bit & 31;
    constexpr uint32_t mask = (1u << MU) - 1u;
    if constexpr (s + MU <= 32) {
        return __builtin_amdgcn_ubfe(w[d], s, MU);
    } else {
        // key straddles dwords d and d+1
        return __builtin_amdgcn_alignbit(w[d + 1], w[d], s) & mask;
    }
}

// Loads the UD dwords of a unit starting at dword index dw0 of a packed row;
// dwords at or past the row stride read as 0 (their chunks do not exist).
template <int UD>
__device__ __forceinline__ void load_unit(const uint32_t* __restrict__ row, int dw0, int stride_dw,
                                          uint32_t (&w)[UD]) {
    if constexpr (UD == 4) {
        // stride is a multiple of 4 dwords and dw0 a multiple of 4: all or nothing
        if (dw0 < stride_dw) {
            const uint4 v = *reinterpret_cast<const uint4*>(row + dw0);
            w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
        } else {
            w[0] = w[1] = w[2] = w[3] = 0u;
        }
    } else {
#pragma unroll
        for (int i = 0; i < UD; ++i) w[i] = (dw0 + i < stride_dw) ? row[dw0 + i] : 0u;
    }
}

// ---------------------------------------------------------------------------------
// Table entries.  For one chunk x[0..8) (elements past MU or past column n are 0) the
// entry of key k = 16*h + l is  (s0 x0 + s1 x1) + ((s2 x2 + s3 x3) + hi(h))  with
//   hi(h) = (s4 x4 + s5 x5) + (s6 x6 + s7 x7),
// s_j = +1 if bit j of k is set else -1 (paper: q = M_mu . x).  Every partial is formed
// from a pair and its exact negation, so entry(~k) = -entry(k) holds bit for bit, the
// property Algorithm 1 obtains by copying negated entries.
// ---------------------------------------------------------------------------------
struct PairSums {
    float a[4];  // a[s] = (s&1 ? x0 : -x0) + (s&2 ? x1 : -x1)
};

__device__ __forceinline__ PairSums pair_sums(float x0, float x1) {
    PairSums p;
    const float s = x0 + x1, d = x0 - x1;
    p.a[0] = -s; p.a[1] = d; p.a[2] = -d; p.a[3] = s;
    return p;
}

__device__ __forceinline__ float pair_pick(const PairSums& p, uint32_t s) {
    // branch-free select of p.a[s], s in 0..3
    const float lo = (s & 1u) ? p.a[1] : p.a[0];
    const float hi = (s & 1u) ? p.a[3] : p.a[2];
    return (s & 2u) ? hi : lo;
}

// hi(h) for h in 0..15
__device__ __forceinline__ float table_hi(const float (&x)[8], uint32_t h) {
    const PairSums c = pair_sums(x[4], x[5]);
    const PairSums d = pair_sums(x[6], x[7]);
    return pair_pick(c, h & 3u) + pair_pick(d, h >> 2);
}

// The 16 entries of keys 16*h + l, l = 0..15:  A[l & 3] + (B[l >> 2] + hi(h)).  Every kernel
// that fills tables uses this one association, so fused and unfused paths agree bit for bit.
__device__ __forceinline__ void table16(const float (&x)[8], uint32_t h, float (&out)[16]) {
    const PairSums a = pair_sums(x[0], x[1]);
    const PairSums b = pair_sums(x[2], x[3]);
    const float hi = table_hi(x, h);
    float bh[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bh[j] = b.a[j] + hi;
#pragma unroll
    for (int l = 0; l < 16; ++l) out[l] = a.a[l & 3] + bh[l >> 2];
}

// The 32 entries of keys 32*hq + 16*hh + l (hh = 0, 1; l = 0..15) of one chunk, for the fused
// mu = 8 kernels: the same association as table16 (so the results are the same bits), with the
// chunk's pair sums shared by both groups of 16.
__device__ __forceinline__ void table32(const float (&x)[8], uint32_t hq, float (&out)[32]) {
    const PairSums a = pair_sums(x[0], x[1]);
    const PairSums b = pair_sums(x[2], x[3]);
    const PairSums c = pair_sums(x[4], x[5]);
    const PairSums d = pair_sums(x[6], x[7]);
    // h = 2*hq + hh: hi(h) = C[h & 3] + D[h >> 2], and h >> 2 = hq >> 1 for both hh
    const float dd = pair_pick(d, hq >> 1);
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const float hi = pair_pick(c, 2u * (hq & 1u) + (uint32_t)hh) + dd;
        float bh[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) bh[j] = b.a[j] + hi;
#pragma unroll
        for (int l = 0; l < 16; ++l) out[hh * 16 + l] = a.a[l & 3] + bh[l >> 2];
    }
}

// x[0..8) = X[col][8*c ..] with two 128-bit loads when the row allows it (vec_ok: n % 4 == 0 and X
// 16-byte aligned), else element by element with zeros past the row or the batch.
__device__ __forceinline__ void load_chunk8(const float* __restrict__ X, int n, int batch, int col, int c,
                                            bool vec_ok, float (&x)[8]) {
    if (vec_ok && col < batch && 8 * c + 8 <= n) {
        const float4* xv = reinterpret_cast<const float4*>(X + (size_t)col * n);
        const float4 a0 = xv[2 * c], a1 = xv[2 * c + 1];
        x[0] = a0.x; x[1] = a0.y; x[2] = a0.z; x[3] = a0.w;
        x[4] = a1.x; x[5] = a1.y; x[6] = a1.z; x[7] = a1.w;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int e = 8 * c + j;
            x[j] = (col < batch && e < n) ? X[(size_t)col * n + e] : 0.0f;
        }
    }
}

// The same for input vector 0 in two halves, for rows that allow 128-bit loads (n % 4 == 0, X
// 16-byte aligned), without branches: load_chunk8_raw issues both loads unconditionally from
// addresses clamped into the row (so the loads of a prefetch stay in flight together and the
// compiler can count them: s_waitcnt vmcnt(N) instead of a full drain), chunk8_zero_tail later
// zeroes the elements that lie past the row.  n >= 4.
__device__ __forceinline__ void load_chunk8_raw(const float* __restrict__ X, int n, int c, float (&x)[8]) {
    const float4* xv = reinterpret_cast<const float4*>(X);
    const int q4 = n >> 2;  // float4 pieces of the row, >= 1
    const float4 a0 = xv[min(2 * c, q4 - 1)], a1 = xv[min(2 * c + 1, q4 - 1)];
    x[0] = a0.x; x[1] = a0.y; x[2] = a0.z; x[3] = a0.w;
    x[4] = a1.x; x[5] = a1.y; x[6] = a1.z; x[7] = a1.w;
}

__device__ __forceinline__ void chunk8_zero_tail(int n, int c, float (&x)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = (8 * c + j < n) ? x[j] : 0.0f;
}

// x[j] = X[col][MU*c + j] for j < MU and inside the row, else 0
template <int MU>
__device__ __forceinline__ void load_chunk_x(const float* __restrict__ X, int n, int batch, int col,
                                             int c, float (&x)[8]) {
    static_assert(MU <= 8, "chunks of more than 8 elements use load_chunk_x10");
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int e = MU * c + j;
        x[j] = (j < MU && col < batch && e < n) ? X[(size_t)col * n + e] : 0.0f;
    }
}

// The same for chunks of 9 or 10 elements.
template <int MU>
__device__ __forceinline__ void load_chunk_x10(const float* __restrict__ X, int n, int batch, int col,
                                               int c, float (&x)[10]) {
#pragma unroll
    for (int j = 0; j < 10; ++j) {
        const long long e = (long long)MU * c + j;
        x[j] = (j < MU && col < batch && e < n) ? X[(size_t)col * n + e] : 0.0f;
    }
}

// mu = 9, 10: the 16 entries of keys 16*h + l, h = 0 .. 2^(mu-4) - 1.  One more pair sum on top of
// table16's association: A[l&3] + (B[l>>2] + (C[h&3] + (D[(h>>2)&3] + E[h>>4]))), so entry(~k) =
// -entry(k) still holds bit for bit.
__device__ __forceinline__ void table16_wide(const float (&x)[10], uint32_t h, float (&out)[16]) {
    const PairSums a = pair_sums(x[0], x[1]);
    const PairSums b = pair_sums(x[2], x[3]);
    const PairSums c = pair_sums(x[4], x[5]);
    const PairSums d = pair_sums(x[6], x[7]);
    const PairSums e = pair_sums(x[8], x[9]);
    const float hi = pair_pick(c, h & 3u) + (pair_pick(d, (h >> 2) & 3u) + pair_pick(e, h >> 4));
    float bh[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bh[j] = b.a[j] + hi;
#pragma unroll
    for (int l = 0; l < 16; ++l) out[l] = a.a[l & 3] + bh[l >> 2];
}

// Entries of one chunk for any MU (element 9 of a mu = 9 chunk is 0, so that the unused key bit
// pairs with a zero; keys with that bit set are never looked up).
template <int MU>
__device__ __forceinline__ void chunk_table16(const float* __restrict__ X, int n, int batch, int col, int c,
                                              uint32_t h, float (&out)[16]) {
    if constexpr (MU <= 8) {
        float x[8];
        load_chunk_x<MU>(X, n, batch, col, c, x);
        table16(x, h, out);
    } else {
        float x[10];
        load_chunk_x10<MU>(X, n, batch, col, c, x);
        table16_wide(x, h, out);
    }
}

}  // namespace biq
