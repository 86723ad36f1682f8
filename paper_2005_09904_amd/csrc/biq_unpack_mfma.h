// Large-batch path: "GEMM with unpacking" (Sec. IV-B, Algorithm 3) as a dense MFMA contraction.
//
// For many input vectors the product is compute bound and the lookup tables stop paying off
// (the crossover discussed with Fig. 10); the alternative the paper measures is to unpack the
// sign bits and run an ordinary GEMM.  Here the unpacking happens in registers, straight into
// the A operand of a 32x32x16 MFMA, and nothing unpacked ever reaches memory:
//   - a weight bit becomes the 16-bit float +1.0 / -1.0 (bit set <-> +1, as in Algorithm 3; the
//     kernel forms the negated value, whose sign bit is the key bit, and negates alpha);
//   - the fp32 inputs are split once into T terms of 16-bit floats, which are T B operands
//     multiplied with the same A operand; +-1 * term products are exact and the matrix cores
//     accumulate in fp32.
// T = 3, the default: x = x0 + x1 + x2 with three bf16 terms (8 significand bits each, taken by
//     truncation, so the sum is exact).  The result differs from a plain fp32 evaluation of
//     Eq. 2 only by the order of the additions.  Terms that are zero for all of a workgroup's
//     input vectors over all of a wave's part of the row are skipped (their MFMAs and loads):
//     inputs that carry fewer than 17 (9) significand bits - values that came from fp16 (bf16)
//     arithmetic - cost two thirds (one third) of the matrix instructions, with the same bits out.
// T = 2, on request (plan.input_terms = 2): every input vector is scaled by a power of two 2^e
//     (e per vector, from its largest magnitude, which lands in [2^14, 2^15)) and every scaled
//     element is split into two fp16 terms, x * 2^e = x0 + x1 + r with x0 = fp16(x * 2^e),
//     x1 = fp16(x * 2^e - x0), both rounded to nearest: |r| <= 2^-22 |x * 2^e| (or 2^-25
//     absolutely, i.e. 2^-39 of the vector's largest magnitude, where x1 is subnormal); the
//     epilogue multiplies by 2^-e.  A third fewer MFMAs for an input rounding of a quarter of
//     fp32's unit in the last place per element.  A second term that is zero for all of a
//     workgroup's input vectors (inputs holding fp16 values) is skipped here too.
// The kernel does not depend on mu: it reads the packed bitmap, which is the same for all mu.
//
// MFMA operand layout (32x32x16, wave of 64 lanes, lane = 32*h + r):
//   A: lane holds row r of the tile, 8 consecutive k of half h     -> one key byte per lane
//   B: lane holds column r, the same 8 k of half h                 -> 8 terms of one input vector
//   C: lane holds column r, rows 8*(v/4) + 4*h + v%4 for v = 0..15
// A lane loads 16 key bytes of its row at once: half 0 takes bytes [32g, 32g+16) of the row,
// half 1 bytes [32g+16, 32g+32) ("key group" g).  Each of the lane's four key dwords feeds four
// MFMA steps (see unpack_step for which bits go to which step): the k order of the contraction
// is a permutation of the columns, which the B side follows.
//
// B operands are prepared by xsplit3_kernel / xsplit2_kernel in exactly the order the main kernel consumes them:
//   Xf[col_group][step][col_tile][term 0..T-1][lane] : 16 bytes (8 terms)
// (step = MFMA step along the row, 16 per key group), so a wave's load of a fragment is one
// contiguous KiB; the waves load their fragments straight into registers, a few steps ahead.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace biq {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t mfma_u32x4 __attribute__((ext_vector_type(4)));

constexpr int kUnpackThreads = 256;     // 4 waves
constexpr int kUnpackGroupBytes = 32;   // key bytes of a row per key group (both halves)

// What depends on the number of terms T: the MFMA operand type, two of its 1.0 in a dword, and
// the instruction.
template <int T> struct UnpackOperand;
template <> struct UnpackOperand<3> {
    typedef bf16x8 vec;
    static constexpr uint32_t kOne2 = 0x3f803f80u;
    static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct UnpackOperand<2> {
    typedef f16x8 vec;
    static constexpr uint32_t kOne2 = 0x3c003c00u;
    static __device__ __forceinline__ f32x16 mfma(vec a, vec b, f32x16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};

// Time stamps of a trace build (-DBIQ_TRACE, never the product's): lane 0 of wave 0 of every
// workgroup writes the 100 MHz wall clock into slot i of its entry.
#ifdef BIQ_TRACE
__device__ unsigned long long biq_unpack_trace[8192 * 8];
#define BIQ_USTAMP(i)                                                                        \
    do {                                                                                     \
        if (threadIdx.x == 0 && blockIdx.x < 8192) {                                         \
            biq_unpack_trace[blockIdx.x * 8 + (i)] = wall_clock64();                         \
            if ((i) == 1 || (i) == 2) biq_unpack_trace[blockIdx.x * 8 + 3 + (i)] = clock64(); \
        }                                                                                    \
    } while (0)
#else
#define BIQ_USTAMP(i) do { } while (0)
#endif

struct UnpackParams {
    const uint8_t* K;        // [q][m][stride]
    const float* alpha;      // [q][m]
    const mfma_u32x4* Xf;    // prepared B operands (see above)
    const int* colexp;       // two terms: per (padded) input vector e (its B operands hold x * 2^e) and the
                             // second-term flag, packed as (e + kExpBias) | kExpSecondTerm
    const int* nterms;       // three terms: per (column group, step, column tile), how many leading terms are
                             // not all zero (1..3)
    float* out;              // Y [batch][m], or partials [splits][batch][m]
    int m, batch;
    uint32_t stride_bytes;
    int groups;              // key groups per row = ceil(stride / 32)
    int gps;                 // key groups per split
    int splits;
    int row_blocks, col_groups;
    int ntasks, tasks_per_xcd;
};

// Splits fp32 into three bf16 terms by truncation; returns them as the high halves' bit patterns.
__device__ __forceinline__ void split3(float x, uint32_t& t0, uint32_t& t1, uint32_t& t2) {
    const uint32_t b0 = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(b0);       // exact: the low 16 significand bits
    const uint32_t b1 = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(b1);      // exact: at most 8 significand bits left
    t0 = b0 >> 16;
    t1 = b1 >> 16;
    t2 = __float_as_uint(r2) >> 16;                 // exact in bf16
}

// Splits a scaled fp32 value into two fp16 terms, each rounded to nearest; the difference taken
// in between is exact in fp32.  Returns the bit patterns.
__device__ __forceinline__ void split2(float xs, uint32_t& t0, uint32_t& t1) {
    const _Float16 hi = (_Float16)xs;
    const _Float16 lo = (_Float16)(xs - (float)hi);
    t0 = __builtin_bit_cast(unsigned short, hi);
    t1 = __builtin_bit_cast(unsigned short, lo);
}

// Exact split: one thread per (col_group, step, col_tile, lane) writes the three 16-byte B
// fragments of that lane (coalesced: a wave writes whole KiB).  Columns past the batch and
// elements past n are zero.
template <int CT>
__global__ __launch_bounds__(256) void xsplit3_kernel(const float* __restrict__ X,
                                                      mfma_u32x4* __restrict__ Xf, int* __restrict__ nterms,
                                                      int n, int batch, int steps, long long total) {
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;              // (total is a multiple of 1024: whole workgroups only)
    const int lane = (int)(idx & 63);
    long long rest = idx >> 6;
    const int ct = (int)(rest % CT); rest /= CT;
    const int step = (int)(rest % steps);   // MFMA step along the row: 16 per key group
    const int cg = (int)(rest / steps);
    const int col = (cg * CT + ct) * 32 + (lane & 31);
    const int h = lane >> 5;
    const int ks = step & 3;
    // dword of the row this step works on, and its 2 x 4 consecutive elements (see unpack_step)
    const long long dw = 8ll * (step >> 4) + 4 * h + ((step >> 2) & 3);
    const long long j0 = 32 * dw + 8 * (ks >> 1) + 4 * (ks & 1);   // elements j0..j0+3 and j0+16..j0+19
    float lo[4], hi[4];
    if (col < batch && j0 + 20 <= n && (n & 3) == 0 && ((reinterpret_cast<uintptr_t>(X) & 15) == 0)) {
        const float* src = X + (size_t)col * n + j0;
        const float4 a = *reinterpret_cast<const float4*>(src);
        const float4 b = *reinterpret_cast<const float4*>(src + 16);
        lo[0] = a.x; lo[1] = a.y; lo[2] = a.z; lo[3] = a.w;
        hi[0] = b.x; hi[1] = b.y; hi[2] = b.z; hi[3] = b.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            lo[i] = (col < batch && j0 + i < n) ? X[(size_t)col * n + j0 + i] : 0.0f;
            hi[i] = (col < batch && j0 + 16 + i < n) ? X[(size_t)col * n + j0 + 16 + i] : 0.0f;
        }
    }
    uint32_t t[3][8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        split3(lo[i], t[0][2 * i], t[1][2 * i], t[2][2 * i]);
        split3(hi[i], t[0][2 * i + 1], t[1][2 * i + 1], t[2][2 * i + 1]);
    }
    mfma_u32x4 v[3];
    uint32_t any[3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        v[s].x = t[s][0] | (t[s][1] << 16);
        v[s].y = t[s][2] | (t[s][3] << 16);
        v[s].z = t[s][4] | (t[s][5] << 16);
        v[s].w = t[s][6] | (t[s][7] << 16);
        any[s] = (v[s].x | v[s].y | v[s].z | v[s].w) & 0x7fff7fffu;   // zero of either sign does not count
    }
    mfma_u32x4* dst = Xf + (idx >> 6) * (3 * 64) + lane;
#pragma unroll
    for (int s = 0; s < 3; ++s) dst[s * 64] = v[s];
    // how many leading terms this wave's (step, column tile) pair needs
    const bool need3 = __builtin_amdgcn_ballot_w64(any[2] != 0u) != 0ull;
    const bool need2 = __builtin_amdgcn_ballot_w64(any[1] != 0u) != 0ull;
    if (lane == 0) nterms[idx >> 6] = need3 ? 3 : need2 ? 2 : 1;
}

// Two scaled terms: input vectors -> B fragments (two 16-byte pieces per MFMA step and
// half-wave, see the layout above), one workgroup per (padded) input vector: largest magnitude
// -> e, then the fragments.  Vectors past the batch and elements past n are zero.  A vector
// that holds Inf or NaN is left unscaled (e = 0) and gives non-finite results, as it would in
// any evaluation of Eq. 2.  A thread reads the 8 elements of its fragments once and keeps them
// in registers across the reduction (kXsplitCached fragments per thread: n <= 32768; what is
// beyond is read twice).
// (Measured and dropped: several workgroups per vector, each reading the whole vector for the
// maximum and writing a share of the fragments - slower from n = 4096 to 16384.)
constexpr int kXsplitThreads = 1024;
constexpr int kXsplitCached = 4;
// an input vector's word in `colexp`: e + kExpBias (e = -113 .. 140), and whether its second term is non-zero anywhere
constexpr int kExpBias = 1024, kExpMask = 0xfff, kExpSecondTerm = 1 << 16;

template <int CT>
__global__ __launch_bounds__(kXsplitThreads) void xsplit2_kernel(const float* __restrict__ X,
                                                                mfma_u32x4* __restrict__ Xf,
                                                                int* __restrict__ colexp, int n, int batch,
                                                                int padded_batch, int steps) {
    __shared__ uint32_t wave_max[kXsplitThreads / 64];
    // The 8 vectors whose pieces share a 128-byte line of Xf (lanes 8k .. 8k+7 of a fragment) go
    // to workgroups on the same XCD (workgroup b runs on XCD b % 8), so that one L2 collects the
    // whole line: line group lg = col / 8 lives on XCD lg % 8.
    const int lg = ((int)blockIdx.x >> 6) * 8 + ((int)blockIdx.x & 7);
    const int col = lg * 8 + (((int)blockIdx.x >> 3) & 7);
    if (col >= padded_batch) return;
    const int tid = threadIdx.x;
    const bool real = col < batch;
    const float* xc = X + (size_t)(real ? col : 0) * n;
    const bool vec = (n & 3) == 0 && ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    const int nfrag = steps * 2;
    const int cg = col / (CT * 32), ct = (col >> 5) % CT, lr = col & 31;

    // fragment f of the vector (4 consecutive f cover one 128-byte line of X): its 8 elements in
    // operand order, and where its pieces go
    auto load_fragment = [&](int f, float (&x)[8]) {
        const int ks = f & 3, d = (f >> 2) & 3, h = (f >> 4) & 1, g = f >> 5;
        // dword of the row this step works on, and its 2 x 4 consecutive elements (see unpack_step)
        const long long dw = 8ll * g + 4 * h + d;
        const long long j0 = 32 * dw + 8 * (ks >> 1) + 4 * (ks & 1);   // elements j0..j0+3 and j0+16..j0+19
        if (real && vec && j0 + 20 <= n) {
            const float4 a = *reinterpret_cast<const float4*>(xc + j0);
            const float4 b = *reinterpret_cast<const float4*>(xc + j0 + 16);
            x[0] = a.x; x[2] = a.y; x[4] = a.z; x[6] = a.w;
            x[1] = b.x; x[3] = b.y; x[5] = b.z; x[7] = b.w;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[2 * i] = (real && j0 + i < n) ? xc[j0 + i] : 0.0f;
                x[2 * i + 1] = (real && j0 + 16 + i < n) ? xc[j0 + 16 + i] : 0.0f;
            }
        }
    };
    // the two terms of a fragment's 8 scaled elements as 16-byte pieces; returns the bits of the second
    auto split_fragment = [&](const float (&x)[8], int e, mfma_u32x4 (&v)[2]) -> uint32_t {
        uint32_t t[2][8];
#pragma unroll
        for (int i = 0; i < 8; ++i) split2(ldexpf(x[i], e), t[0][i], t[1][i]);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v[s].x = t[s][0] | (t[s][1] << 16);
            v[s].y = t[s][2] | (t[s][3] << 16);
            v[s].z = t[s][4] | (t[s][5] << 16);
            v[s].w = t[s][6] | (t[s][7] << 16);
        }
        return (v[1].x | v[1].y | v[1].z | v[1].w) & 0x7fff7fffu;    // zero of either sign does not count
    };
    auto store_fragment = [&](int f, const mfma_u32x4 (&v)[2]) {
        const int ks = f & 3, d = (f >> 2) & 3, h = (f >> 4) & 1, g = f >> 5;
        const int step = g * 16 + d * 4 + ks;  // MFMA step along the row: 16 per key group
        mfma_u32x4* dst = Xf + (((size_t)cg * steps + step) * CT + ct) * (2 * 64) + 32 * h + lr;
        dst[0] = v[0];
        dst[64] = v[1];
    };
    auto fold_max = [](uint32_t mb, const float (&x)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) mb = max(mb, __float_as_uint(x[i]) & 0x7fffffffu);
        return mb;
    };
    uint32_t mb = 0;                       // largest |x| as a bit pattern (ordered like the values)
    float held[kXsplitCached][8];
#pragma unroll
    for (int i = 0; i < kXsplitCached; ++i) {
        const int f = tid + kXsplitThreads * i;
        if (f < nfrag) {
            load_fragment(f, held[i]);
            mb = fold_max(mb, held[i]);
        }
    }
    for (int f = tid + kXsplitThreads * kXsplitCached; f < nfrag; f += kXsplitThreads) {
        float x[8];
        load_fragment(f, x);
        mb = fold_max(mb, x);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mb = max(mb, (uint32_t)__shfl_xor((int)mb, o));
    if ((tid & 63) == 0) wave_max[tid >> 6] = mb;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kXsplitThreads / 64; ++w) mb = max(mb, wave_max[w]);
    // exponent field ex: the maximum lies in [2^(ex-127), 2^(ex-126)) -> times 2^(141-ex) in
    // [2^14, 2^15); zero and subnormal vectors scale as if the maximum were 2^-126
    const int ex = (int)(mb >> 23);
    const int e = ex == 255 ? 0 : 141 - max(ex, 1);

    // The terms of the held fragments, and whether any second term is non-zero (inputs that hold
    // fp16 values have none: the main kernel then skips that term) - found before any store is
    // issued, since the barrier would wait for stores in flight.  What is not held counts as non-zero.
    mfma_u32x4 pieces[kXsplitCached][2];
    uint32_t second = nfrag > kXsplitThreads * kXsplitCached ? 1u : 0u;
#pragma unroll
    for (int i = 0; i < kXsplitCached; ++i)
        if (tid + kXsplitThreads * i < nfrag) second |= split_fragment(held[i], e, pieces[i]);
    const int need2 = __syncthreads_or(second != 0u);
    if (tid == 0) colexp[col] = (e + kExpBias) | (need2 ? kExpSecondTerm : 0);
#pragma unroll
    for (int i = 0; i < kXsplitCached; ++i) {
        const int f = tid + kXsplitThreads * i;
        if (f < nfrag) store_fragment(f, pieces[i]);
    }
    for (int f = tid + kXsplitThreads * kXsplitCached; f < nfrag; f += kXsplitThreads) {
        float x[8];
        mfma_u32x4 v[2];
        load_fragment(f, x);
        split_fragment(x, e, v);
        store_fragment(f, v);
    }
}

// MFMA step S (0..3) of key dword w -> the lane's 8 A elements (bf16 or fp16), with the OPPOSITE sign:
// -1.0 where the bit is set, +1.0 otherwise (the sign bit is the key bit; the epilogue multiplies
// by -alpha).  Element e = 2*i + hh is bit 8*(S/2) + 4*(S%2) + i + 16*hh of the dword: bits p
// and p + 16 land in the sign positions 15 and 31 of one dword with a single shift.  `one2`
// holds two 1.0 of the operand type in a VGPR so that mask-and-merge is one v_and_or_b32.
template <int S, typename V>
__device__ __forceinline__ V unpack_step(uint32_t w, uint32_t one2) {
    mfma_u32x4 d;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int p = 8 * (S >> 1) + 4 * (S & 1) + i;
        const uint32_t a = p <= 15 ? (w << (15 - p)) : (w >> (p - 15));
        d[i] = (a & 0x80008000u) | one2;
    }
    return __builtin_bit_cast(V, d);
}

// A workgroup's four waves form WS groups along the contraction ("wave splits"): group kg works
// on its own contiguous part of the workgroup's key groups, with 4 / WS waves side by side along
// the rows, and the WS partial accumulators are added through LDS in a fixed order at the end.
// LDS holds only those partial sums and the epilogue's transpose patches.
template <int CT, int WS, int T>
struct UnpackGeom {
    static constexpr int SPIECES = CT * T * 64;                  // 16-byte pieces of B per MFMA step
    static constexpr int LDS_BYTES = (WS == 1 ? 24 : 96) * 1024;
};

template <int Q, int RPW, int CT, int WS, int T>
__global__ __launch_bounds__(kUnpackThreads) void unpack_mfma_kernel(const UnpackParams p) {
    using G = UnpackGeom<CT, WS, T>;
    using Op = UnpackOperand<T>;
    using opvec = typename Op::vec;
    constexpr int RT = Q * RPW;                       // row tiles (32 key rows each) per wave
    constexpr int WROWS = 4 / WS;                     // waves side by side along the rows
    constexpr int SPIECES = G::SPIECES;
    static_assert((WS - 1) * WROWS * RT * CT * 4096 <= G::LDS_BYTES, "partial sums must fit");
    extern __shared__ __align__(16) mfma_u32x4 stage_buf[];  // partial sums, transpose patches

    const int wg = blockIdx.x;
    const int task = (wg & 7) * p.tasks_per_xcd + (wg >> 3);
    if (task >= p.ntasks) return;
    const int cg = task % p.col_groups;
    const int rest = task / p.col_groups;
    const int sp = rest % p.splits;
    const int rb = rest / p.splits;
    const int g0 = sp * p.gps;
    const int g1 = min(p.groups, g0 + p.gps);
    const int steps_total = p.groups * 16;
    const int per = (g1 - g0 + WS - 1) / WS;          // key groups per wave group (the last may get fewer)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int kg = wave / WROWS;                      // this wave's group along the contraction
    const int wrow = wave % WROWS;
    const int h = lane >> 5;
    const int lr = lane & 31;
    const int ga = g0 + kg * per;                     // this wave's key groups [ga, gb)
    const int gb = min(g1, ga + per);

    const int rbase = rb * (WROWS * 32 * RPW) + wrow * (32 * RPW);
    const uint8_t* kptr[RT];
#pragma unroll
    for (int i = 0; i < Q; ++i)
#pragma unroll
        for (int rp = 0; rp < RPW; ++rp) {
            const int row = min(rbase + rp * 32 + lr, p.m - 1);  // clamped: masked at the store
            kptr[i * RPW + rp] = p.K + ((size_t)i * p.m + row) * p.stride_bytes + 16 * h;
        }
    // All loads of the main loop are unconditional, from addresses clamped into the buffers: a
    // load behind a condition makes the compiler wait for every outstanding load at the next use
    // of any, and the keys of the next key group (from HBM, requested a whole group ahead) would
    // be waited for at every stage copy.  Keys past the wave's range or past the row are never
    // multiplied with anything but the zero fragments of the padding.
    auto load_keys = [&](int g, mfma_u32x4 (&k)[RT]) {
        const bool ok = g < gb && (uint32_t)(32 * g + 16 * h) < p.stride_bytes;
        const uint32_t off = ok ? (uint32_t)(32 * g) : 0u;
#pragma unroll
        for (int t = 0; t < RT; ++t) k[t] = *reinterpret_cast<const mfma_u32x4*>(kptr[t] + off - (ok ? 0 : 16 * h));
    };

    f32x16 acc[RT][CT];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][c][v] = 0.0f;

    uint32_t one2 = Op::kOne2;          // two 1.0 of the operand type, kept in a VGPR (see unpack_step)
    asm volatile("" : "+v"(one2));
    BIQ_USTAMP(0);

    // ---- main loop: no LDS, no barrier.  The B fragments lie in Xf in the order of use, 16 bytes
    // per lane: a wave loads them straight into registers (1 KiB per request, the four waves of a
    // workgroup hit the same lines in the vector cache), three MFMA steps ahead in a ring of four.
    // While the RT * CT * T MFMAs of a step issue, the next step's A operands are expanded from
    // the key bits and the fragments of the step three ahead are requested; the
    // sched_group_barrier sequence spells that interleaving out (left alone, the compiler puts a
    // step's expansion right in front of its MFMAs and the matrix pipe idles through it).
    const int ngroups = gb - ga;                       // key groups of this wave (<= 0: none)
    const int nsteps = ngroups * 16;
    if (ngroups > 0) {
        const mfma_u32x4* xw = p.Xf + ((size_t)cg * steps_total + (size_t)ga * 16) * SPIECES + lane;
        // the first `cnt` terms of step s (cnt is a constant wherever this is called)
        auto load_b = [&](int s, auto& b, int cnt) {   // b: opvec [CT][T] or [CT][fewer]
            constexpr int TD = sizeof(b[0]) / sizeof(b[0][0]);
            const int sc = min(s, nsteps - 1);         // past the end: the last step again, unused
            const mfma_u32x4* src = xw + (size_t)sc * SPIECES;
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int tm = 0; tm < TD; ++tm)
                    if (tm < cnt) b[c][tm] = __builtin_bit_cast(opvec, src[(c * T + tm) * 64]);
        };
        auto expand_a = [&](const mfma_u32x4 (&k)[RT], int step, opvec (&a)[RT]) {
            const int d = step >> 2, ks = step & 3;    // step 0..15 within the key group
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                const uint32_t w = k[t][d];
                a[t] = ks == 0 ? unpack_step<0, opvec>(w, one2) : ks == 1 ? unpack_step<1, opvec>(w, one2)
                     : ks == 2 ? unpack_step<2, opvec>(w, one2) : unpack_step<3, opvec>(w, one2);
            }
        };
        // Three terms: how many leading terms are not all zero anywhere in this wave's key groups
        // for this workgroup's input vectors = the largest of the counts xsplit3_kernel left for
        // them (16 * CT per key group, contiguous; lane l looks at the l-th 16 bytes, then the
        // largest over the wave).  Decided once per wave: each count gets a loop of its own; the
        // first three steps' fragments are requested with all T terms before the count is known.
        // The counts are requested first and looked at last: the keys and the first fragments
        // (all T terms) are on their way meanwhile, and loads return in order.
        int nt_wave = T;
        int4 cnt = make_int4(1, 1, 1, 1);
        int colword = kExpSecondTerm;
        if constexpr (T == 2) colword = p.colexp[cg * CT * 32 + (lane & (CT * 32 - 1))];   // the workgroup's input vectors
        if constexpr (T == 3) {
            const int4* f = reinterpret_cast<const int4*>(p.nterms + ((size_t)cg * steps_total + 16 * (size_t)ga) * CT);
            const int pieces = ngroups * 4 * CT;       // 16-byte pieces holding this wave's counts
            cnt = f[min(lane, pieces - 1)];
            for (int i = lane + 64; i < pieces; i += 64) {     // more than 16 / CT key groups per wave
                const int4 v = f[i];
                cnt = make_int4(max(cnt.x, v.x), max(cnt.y, v.y), max(cnt.z, v.z), max(cnt.w, v.w));
            }
        }
        mfma_u32x4 key[RT], keyn[RT];
        opvec bfr[4][CT][T];
        opvec af[2][RT];
        load_keys(ga, key);
        load_b(0, bfr[0], T);
        load_b(1, bfr[1], T);
        load_b(2, bfr[2], T);
        if constexpr (T == 3) {
            const int r = max(max(cnt.x, cnt.y), max(cnt.z, cnt.w));
            nt_wave = __builtin_amdgcn_ballot_w64(r >= 3) != 0ull ? 3 : __builtin_amdgcn_ballot_w64(r >= 2) != 0ull ? 2 : 1;
        }
        if constexpr (T == 2) nt_wave = __builtin_amdgcn_ballot_w64((colword & kExpSecondTerm) != 0) != 0ull ? 2 : 1;
        BIQ_USTAMP(1);
        // The whole walk over the wave's key groups with NT of the T terms.
        // The walk over the wave's key groups with NT of the T terms, fragments requested R - 1
        // steps ahead in a ring `rg` of R slots whose first three are filled.
        auto walk_ring = [&](auto ntc, auto rc, auto& rg) {
            constexpr int NT = decltype(ntc)::value;
            constexpr int R = decltype(rc)::value;
            constexpr int VPM = NT == 3 ? 2 : (8 + CT * NT - 1) / (CT * NT);  // expansion instructions to place per MFMA
#pragma unroll
            for (int j = 3; j + 1 < R; ++j) load_b(j, rg[j], NT);
            for (int gi = 0; gi < ngroups; ++gi) {
                // The first step's operands are expanded here, not during the last step of the group
                // before: written there, the compiler moves the expansion up to where the keys are
                // loaded and waits for them on the spot.
                expand_a(key, 0, af[0]);
                __builtin_amdgcn_sched_barrier(0);
                load_keys(ga + gi + 1, keyn);
#pragma unroll
                for (int st = 0; st < 16; ++st) {
                    load_b(gi * 16 + st + R - 1, rg[(st + R - 1) & (R - 1)], NT);
                    if (st + 1 < 16) expand_a(key, st + 1, af[(st + 1) & 1]);
#pragma unroll
                    for (int tm = 0; tm < NT; ++tm)
#pragma unroll
                        for (int t = 0; t < RT; ++t)
#pragma unroll
                            for (int c = 0; c < CT; ++c)
                                acc[t][c] = Op::mfma(af[st & 1][t], rg[st & (R - 1)][c][tm], acc[t][c]);
#pragma unroll
                    for (int i = 0; i < RT * CT * NT; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // MFMA
                        if (i < CT * NT) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);      // global load
                        if (VPM * i < RT * 8) __builtin_amdgcn_sched_group_barrier(0x002, VPM, 0);  // VALU
                    }
                    __builtin_amdgcn_sched_barrier(0);   // a step's instructions stay in the step
                }
#pragma unroll
                for (int t = 0; t < RT; ++t) key[t] = keyn[t];
            }
        };
        // With two or three terms, three steps ahead cover the latency of the fragments (measured:
        // a ring of 8 is no faster); with one term a step is a third as long and the ring grows
        // to 8 slots of one term, which takes fewer registers still.
        auto walk = [&](auto ntc) {
            constexpr int NT = decltype(ntc)::value;
            if constexpr (NT > 1 || T == 1) {
                walk_ring(ntc, std::integral_constant<int, 4>{}, bfr);
            } else {
                opvec ring[8][CT][NT];
#pragma unroll
                for (int j = 0; j < 3; ++j)
#pragma unroll
                    for (int c = 0; c < CT; ++c)
#pragma unroll
                        for (int tm = 0; tm < NT; ++tm) ring[j][c][tm] = bfr[j][c][tm];
                walk_ring(ntc, std::integral_constant<int, 8>{}, ring);
            }
        };
        if (T == 3 && nt_wave >= 3) walk(std::integral_constant<int, T>{});
        else if (nt_wave >= 2) walk(std::integral_constant<int, 2>{});
        else walk(std::integral_constant<int, 1>{});
    }

    BIQ_USTAMP(2);
    // The epilogue's inputs are requested here, ahead of the exchange between the wave groups,
    // all at once and without conditions (rows past m read row 0 and are never stored): -alpha
    // of the lane's rows in every row tile, and (two terms) the exponents of its input vectors.
    const bool vec_ok = ((p.m & 3) == 0) && ((reinterpret_cast<uintptr_t>(p.out) & 15) == 0) &&
                        ((reinterpret_cast<uintptr_t>(p.alpha) & 15) == 0);
    float al[RPW][4][Q][4];
    int xe[CT];
    if (kg == 0) {
#pragma unroll
        for (int rp = 0; rp < RPW; ++rp)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int row = rbase + rp * 32 + 8 * vq + 4 * h;
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    if (vec_ok) {
                        const float4 a = *reinterpret_cast<const float4*>(p.alpha + (size_t)i * p.m + (row < p.m ? row : 0));
                        al[rp][vq][i][0] = -a.x; al[rp][vq][i][1] = -a.y; al[rp][vq][i][2] = -a.z; al[rp][vq][i][3] = -a.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            al[rp][vq][i][e] = -p.alpha[(size_t)i * p.m + (row + e < p.m ? row + e : 0)];
                    }
                }
            }
#pragma unroll
        for (int c = 0; c < CT; ++c) xe[c] = T == 2 ? kExpBias - (p.colexp[(cg * CT + c) * 32 + lr] & kExpMask) : 0;
    }
    // ---- sum over the wave groups: groups 1.. hand their accumulators to group 0 through LDS ----
    if constexpr (WS > 1) {
        float4* red = reinterpret_cast<float4*>(stage_buf);   // [WS - 1][WROWS][RT * CT * 4][64 lanes]
        if (kg > 0) {
            float4* dst = red + ((size_t)((kg - 1) * WROWS + wrow) * (RT * CT * 4)) * 64 + lane;
#pragma unroll
            for (int t = 0; t < RT; ++t)
#pragma unroll
                for (int c = 0; c < CT; ++c)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq)
                        dst[((t * CT + c) * 4 + vq) * 64] =
                            make_float4(acc[t][c][4 * vq], acc[t][c][4 * vq + 1], acc[t][c][4 * vq + 2],
                                        acc[t][c][4 * vq + 3]);
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int j = 1; j < WS; ++j) {
            const float4* src = red + ((size_t)((j - 1) * WROWS + wrow) * (RT * CT * 4)) * 64 + lane;
#pragma unroll
            for (int t = 0; t < RT; ++t)
#pragma unroll
                for (int c = 0; c < CT; ++c)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const float4 v = src[((t * CT + c) * 4 + vq) * 64];
                        acc[t][c][4 * vq] += v.x;
                        acc[t][c][4 * vq + 1] += v.y;
                        acc[t][c][4 * vq + 2] += v.z;
                        acc[t][c][4 * vq + 3] += v.w;
                    }
        }
    }

    // ---- epilogue: scale by -alpha (the weights were unpacked with the opposite sign), add the
    // planes (Eq. 2), undo the input vector's scaling (two terms), store.  An accumulator tile has one input vector per lane and its 32 rows
    // spread over 4 registers x 2 half-waves; stored like that, every 128-byte line of Y[b][m]
    // would be written by 8 separate instructions.  Each tile therefore goes through a 32 x 36
    // float patch of LDS (private to the wave) and leaves as 128 contiguous bytes per 8 lanes.
    constexpr int TP = 36;                                      // patch pitch in floats (16-byte aligned rows)
    constexpr int RED_FLOATS = (WS - 1) * WROWS * RT * CT * 1024;  // partial sums above, still being read
    static_assert((RED_FLOATS + WROWS * 32 * TP) * 4 <= G::LDS_BYTES, "transpose patches must fit");
    float* const patch = reinterpret_cast<float*>(stage_buf) + RED_FLOATS + wrow * (32 * TP);
#pragma unroll
    for (int rp = 0; rp < RPW; ++rp) {
        const int row0 = rbase + rp * 32;                       // first row of this tile
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            // tile -> patch[column lr][row]
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v = 0.0f;
#pragma unroll
                    for (int i = 0; i < Q; ++i) v = fmaf(al[rp][vq][i][e], acc[i * RPW + rp][c][4 * vq + e], v);
                    y[e] = T == 2 ? ldexpf(v, xe[c]) : v;   // two terms: the lane's input vector was scaled by 2^-xe
                }
                *reinterpret_cast<float4*>(patch + lr * TP + 8 * vq + 4 * h) = make_float4(y[0], y[1], y[2], y[3]);
            }
            // patch -> Y: lane = 8 * (column in group of 8) + (4 rows), 4 column groups
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int pc = 8 * i + (lane >> 3);
                const int pr = 4 * (lane & 7);
                const float4 v = *reinterpret_cast<const float4*>(patch + pc * TP + pr);
                const int col = (cg * CT + c) * 32 + pc;
                const int row = row0 + pr;
                if (col < p.batch && row < p.m) {
                    float* dst = p.out + ((size_t)sp * p.batch + col) * p.m + row;
                    if (vec_ok) {
                        *reinterpret_cast<float4*>(dst) = v;
                    } else {
                        dst[0] = v.x;
                        if (row + 1 < p.m) dst[1] = v.y;
                        if (row + 2 < p.m) dst[2] = v.z;
                        if (row + 3 < p.m) dst[3] = v.w;
                    }
                }
            }
        }
    }
    BIQ_USTAMP(3);
}

}  // namespace biq
