// Kernels of libbiq (gfx950): key packing, table construction, LUT query.
#pragma once

#include "biq_common.h"

namespace biq {

// =====================================================================================
// biq_pack: B int8 [q*m][n] (+1/-1) -> packed sign bit stream [q*m][stride] (Sec. III-B).
// One thread per output dword (32 weights).  bit = (B > 0).
// =====================================================================================
__device__ __forceinline__ uint32_t sign_bits4(uint32_t w) {
    // w holds four int8; returns a 4-bit mask, bit i = (byte i > 0)
    const uint32_t nonzero = ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w;  // bit 7 of each byte
    const uint32_t pos = (nonzero & ~w & 0x80808080u) >> 7;          // bit 0 of each byte
    return (pos * 0x01020408u) >> 24;                                // gather to bits 0..3
}

template <bool ALIGNED16>
__global__ __launch_bounds__(256) void pack_kernel(const int8_t* __restrict__ B,
                                                   uint32_t* __restrict__ K, long long key_rows,
                                                   int n, int stride_dw) {
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long total = key_rows * stride_dw;
    if (gid >= total) return;
    const long long kr = gid / stride_dw;
    const int dw = (int)(gid - kr * stride_dw);
    const int col0 = dw * 32;
    const int8_t* row = B + kr * (long long)n;
    uint32_t bits = 0;
    if (ALIGNED16 && col0 + 32 <= n) {
        // n % 16 == 0 and B 16-byte aligned: two 128-bit loads
        const uint4 v0 = *reinterpret_cast<const uint4*>(row + col0);
        const uint4 v1 = *reinterpret_cast<const uint4*>(row + col0 + 16);
        bits = sign_bits4(v0.x) | (sign_bits4(v0.y) << 4) | (sign_bits4(v0.z) << 8) |
               (sign_bits4(v0.w) << 12) | (sign_bits4(v1.x) << 16) | (sign_bits4(v1.y) << 20) |
               (sign_bits4(v1.z) << 24) | (sign_bits4(v1.w) << 28);
    } else {
        for (int j = 0; j < 32; ++j) {
            const int col = col0 + j;
            if (col < n && row[col] > 0) bits |= 1u << j;
        }
    }
    K[gid] = bits;
}

// =====================================================================================
// biq_unpack_keys: the table indices as the query kernels extract them.
// One thread per (key row, unit); keys uint8 or uint16 [q*m][C].
// =====================================================================================
template <int MU, int T, typename KEY>
__device__ __forceinline__ void store_unit_keys(const uint32_t (&w)[KeyUnit<MU>::UD], KEY* dst,
                                                int c0, int C) {
    if constexpr (T < KeyUnit<MU>::UK) {
        if (c0 + T < C) dst[c0 + T] = (KEY)unit_key<MU, T>(w);
        store_unit_keys<MU, T + 1, KEY>(w, dst, c0, C);
    }
}

template <int MU, typename KEY>
__global__ __launch_bounds__(256) void unpack_keys_kernel(const uint32_t* __restrict__ K,
                                                          KEY* __restrict__ keys,
                                                          long long key_rows, int C, int stride_dw) {
    constexpr int UD = KeyUnit<MU>::UD, UK = KeyUnit<MU>::UK;
    const int units = (C + UK - 1) / UK;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= key_rows * units) return;
    const long long kr = gid / units;
    const int u = (int)(gid - kr * units);
    uint32_t w[UD];
    load_unit<UD>(K + kr * stride_dw, u * UD, stride_dw, w);
    store_unit_keys<MU, 0, KEY>(w, keys + kr * C, u * UK, C);
}

// =====================================================================================
// biq_build_lut: X [batch][n] -> LUT [C][2^MU][batch] in device memory (Sec. III-B).
// One thread per (chunk, VEC adjacent input vectors, group of 16 keys); VEC = 4 (16-byte
// stores) when the batch is a multiple of 4 and LUT is 16-byte aligned, else 1.  A workgroup
// owns a box of 2^lta vector groups x 2^lth key groups x 2^ltc chunks (256 threads, vector
// groups fastest: a wave's stores are contiguous runs of the table).  The box's inputs -
// MU floats per (chunk, vector), 32-byte pieces scattered over X - go through LDS once per
// workgroup: read by each thread on its own they cost the address unit one cache line per lane
// and load, 16 times over for the 16 key groups, and that, not the 64 MiB of stores, set the
// time (n = 4096, 128 vectors, mu = 8: 22.9 us; a plain fill of the table takes 11.3).
// =====================================================================================
constexpr int kLutStageFloats = 4096;   // largest box: 256 (chunk, vector group) pairs x 4 vectors x 4 floats

template <int MU, int VEC>
__global__ __launch_bounds__(256) void build_lut_kernel(const float* __restrict__ X,
                                                        float* __restrict__ LUT, int n, int batch,
                                                        int C, int lta, int lth, int ltc, int a_tiles,
                                                        int h_tiles) {
    constexpr int E = 1 << MU;
    constexpr int HG = (MU > 4) ? (1 << (MU - 4)) : 1;  // groups of 16 keys per table
    constexpr int LN = (MU > 4) ? 16 : E;               // keys per group
    constexpr int XW = MU <= 8 ? 8 : 10;                // elements table16 / table16_wide take
    __shared__ float xs[kLutStageFloats];
    const int bv = batch / VEC;                         // VEC divides batch
    const int tid = threadIdx.x;
    int box = blockIdx.x;
    const int A0 = (box % a_tiles) << lta; box /= a_tiles;
    const int H0 = (box % h_tiles) << lth;
    const int C0 = (box / h_tiles) << ltc;
    // stage: xs[chunk in box][vector in box][MU], zeros past n, C and the batch
    const int nvec = VEC << lta;
    const int staged = (nvec * MU) << ltc;
    for (int e = tid; e < staged; e += 256) {
        const int j = e % MU;
        const int r = e / MU;
        const int vec = A0 * VEC + r % nvec;
        const int c = C0 + r / nvec;
        const long long col = (long long)c * MU + j;
        xs[e] = (vec < batch && c < C && col < n) ? X[(size_t)vec * n + col] : 0.0f;
    }
    __syncthreads();
    const int ta = tid & ((1 << lta) - 1);
    const int th = (tid >> lta) & ((1 << lth) - 1);
    const int tc = tid >> (lta + lth);
    const int a = (A0 + ta) * VEC;
    const int h = H0 + th;
    const int c = C0 + tc;
    if (A0 + ta >= bv || h >= HG || c >= C) return;
    float ent[VEC][16];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        const float* src = xs + ((tc * nvec) + ta * VEC + v) * MU;
        float x[XW];
#pragma unroll
        for (int j = 0; j < XW; ++j) x[j] = j < MU ? src[j] : 0.0f;
        if constexpr (MU <= 8) table16(x, (uint32_t)h, ent[v]);
        else table16_wide(x, (uint32_t)h, ent[v]);
    }
    float* dst = LUT + ((size_t)c * E + (size_t)h * 16) * batch + a;
#pragma unroll
    for (int l = 0; l < LN; ++l) {
        if constexpr (VEC == 4) {
            *reinterpret_cast<float4*>(dst + (size_t)l * batch) =
                make_float4(ent[0][l], ent[1][l], ent[2][l], ent[3][l]);
        } else {
            dst[(size_t)l * batch] = ent[0][l];
        }
    }
}

// =====================================================================================
// Query / fused multiply (Algorithm 2 + Eq. 2), generic over MU and the batch tile BT.
//
// A workgroup owns rows [r0, r0 + rows_per_wg) (all q planes), input vectors
// [b0, b0 + BT) and the LUT tiles [sp*tps, (sp+1)*tps).  For each tile it fills LDS with
// the tables of CT chunks (built from X when FUSED, copied from device memory otherwise),
// then streams its key rows: a group of G = CT/UK lanes covers one row's segment, each
// lane looks its UK keys up, the plane sums are scaled by alpha and added, and the G lanes
// are reduced.  LDS table layout: [chunk in tile][key][BT].
// =====================================================================================
struct QueryParams {
    const uint32_t* K;
    const float* alpha;
    const float* X;    // FUSED: [batch][n]
    const float* LUT;  // !FUSED: [C][2^MU][batch]
    float* out;        // Y [batch][m] if splits == 1, else partial sums [splits][batch][m]
    int m, n, q, batch;
    int stride_dw, C;
    int CT, G, log2G;
    int tiles, tps, splits;
    int rows_per_wg, row_blocks, batch_tiles;
    int ntasks, tasks_per_xcd;
    int row_mode;  // mu = 8 kernels: 0 = 64-row blocks per wave, 1 = one row step per wave
    int xcd_skew;  // gemv8 throughput mode: rows moved from each odd-XCD workgroup to an even-XCD one
    int table_fill;  // gemv8, fused tables: 0 = direct fill from pair sums, 1 = Algorithm 1's order
    // LSTM-cell epilogue (the LSTM instantiations of the half-table kernels only): the m = 4 * hidden
    // rows are the gates i, f, g, o stacked; `out` receives h [batch][hidden]
    const float* bias;    // [4 * hidden]
    const float* c_prev;  // [batch][hidden]
    float* c_out;         // [batch][hidden]
    int hidden;
};

// One step of the textbook LSTM cell from the four gate pre-activations (bias included).
// sigma(z) = 1 / (1 + e^-z) and tanh(x) = 1 - 2 / (e^2x + 1) through the hardware exponential and
// reciprocal: absolute error of a few 2^-24 on values in [-1, 1] (and exact limits for large |z|),
// below what the fp32 summation of z itself contributes.
__device__ __forceinline__ float lstm_sigmoid(float z) { return __fdividef(1.0f, 1.0f + __expf(-z)); }
__device__ __forceinline__ float lstm_tanh(float x) { return 1.0f - __fdividef(2.0f, __expf(2.0f * x) + 1.0f); }

__device__ __forceinline__ void lstm_cell_update(float zi, float zf, float zg, float zo, float c_prev,
                                                 float& h, float& c) {
    c = fmaf(lstm_sigmoid(zf), c_prev, lstm_sigmoid(zi) * lstm_tanh(zg));
    h = lstm_sigmoid(zo) * lstm_tanh(c);
}

template <int MU, int BT, int T>
__device__ __forceinline__ void lookup_unit(const uint32_t (&w)[KeyUnit<MU>::UD],
                                            const float* __restrict__ tab, float (&acc)[BT]) {
    // tab points at the table of this lane's first chunk
    if constexpr (T < KeyUnit<MU>::UK) {
        constexpr int E = 1 << MU;
        const uint32_t key = unit_key<MU, T>(w);
        const float* p = tab + ((size_t)T * E + key) * BT;
        if constexpr (BT == 1) {
            acc[0] += p[0];
        } else if constexpr (BT == 2) {
            const float2 v = *reinterpret_cast<const float2*>(p);
            acc[0] += v.x; acc[1] += v.y;
        } else {
#pragma unroll
            for (int c4 = 0; c4 < BT / 4; ++c4) {
                const float4 v = *reinterpret_cast<const float4*>(p + 4 * c4);
                acc[4 * c4 + 0] += v.x; acc[4 * c4 + 1] += v.y;
                acc[4 * c4 + 2] += v.z; acc[4 * c4 + 3] += v.w;
            }
        }
        lookup_unit<MU, BT, T + 1>(w, tab, acc);
    }
}

template <int MU, int BT, bool FUSED>
__global__ __launch_bounds__(1024) void query_kernel(const QueryParams p) {
    constexpr int E = 1 << MU;
    constexpr int UD = KeyUnit<MU>::UD, UK = KeyUnit<MU>::UK;
    extern __shared__ __align__(16) float lds[];

    // XCD-aware task order: consecutive workgroup ids go to different XCDs, so give each
    // XCD a contiguous range of tasks; tasks that differ only in the batch tile read the
    // same keys and stay on one XCD's L2.
    const int wg = blockIdx.x;
    const int task = (wg & 7) * p.tasks_per_xcd + (wg >> 3);
    if (task >= p.ntasks) return;
    const int bt = task % p.batch_tiles;
    const int rest = task / p.batch_tiles;
    const int sp = rest % p.splits;
    const int rb = rest / p.splits;

    const int b0 = bt * BT;
    const int r0 = rb * p.rows_per_wg;
    const int r1 = min(p.m, r0 + p.rows_per_wg);
    const int tile0 = sp * p.tps;
    const int tile1 = min(p.tiles, tile0 + p.tps);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int G = p.G;
    const int L = tid & (G - 1);       // lane inside the row group
    const int grp = tid >> p.log2G;    // row group inside the workgroup
    const int ngrp = nthreads >> p.log2G;

    float* tables = lds;                                  // [CT][E][BT]
    float* yacc = lds + (size_t)p.CT * E * BT;            // [rows_per_wg][BT], only if tps > 1
    const bool multi = (tile1 - tile0) > 1;

    if (multi) {
        for (int i = tid; i < p.rows_per_wg * BT; i += nthreads) yacc[i] = 0.0f;
    }

    for (int tile = tile0; tile < tile1; ++tile) {
        const int c0 = tile * p.CT;
        __syncthreads();  // previous tile's readers are done (also orders the yacc init)
        if constexpr (FUSED) {
            constexpr int HG = (MU > 4) ? (1 << (MU - 4)) : 1;
            constexpr int LN = (MU > 4) ? 16 : E;
            const int jobs = p.CT * BT * HG;
            for (int job = tid; job < jobs; job += nthreads) {
                const int col = job % BT;
                const int r2 = job / BT;
                const int h = r2 % HG;
                const int ct = r2 / HG;
                float ent[16];
                chunk_table16<MU>(p.X, p.n, p.batch, b0 + col, c0 + ct, (uint32_t)h, ent);
                float* dst = tables + ((size_t)ct * E + h * 16) * BT + col;
                if constexpr (BT == 1 && LN >= 4) {
#pragma unroll
                    for (int l4 = 0; l4 < LN / 4; ++l4)
                        *reinterpret_cast<float4*>(dst + 4 * l4) =
                            make_float4(ent[4 * l4], ent[4 * l4 + 1], ent[4 * l4 + 2], ent[4 * l4 + 3]);
                } else {
#pragma unroll
                    for (int l = 0; l < LN; ++l) dst[l * BT] = ent[l];
                }
            }
        } else {
            const int entries = p.CT * E * BT;
            for (int e = tid; e < entries; e += nthreads) {
                const int col = e % BT;
                const int ck = e / BT;  // ct*E + key
                const int c = c0 + ck / E;
                float v = 0.0f;
                if (c < p.C && b0 + col < p.batch)
                    v = p.LUT[((size_t)c0 * E + ck) * p.batch + b0 + col];
                tables[e] = v;
            }
        }
        __syncthreads();

        const int dw0 = (c0 / UK) * UD + L * UD;  // this lane's unit inside a packed row
        const float* tab = tables + (size_t)L * UK * E * BT;
        // (row, plane) pairs are walked with the next pair's keys and scale already requested
        auto load_pair = [&](int r, int i, uint32_t (&w)[UD], float& al) {
#pragma unroll
            for (int d = 0; d < UD; ++d) w[d] = 0u;
            al = 0.0f;
            if (r < r1) {
                const size_t kr = (size_t)i * p.m + r;
                load_unit<UD>(p.K + kr * p.stride_dw, dw0, p.stride_dw, w);
                al = p.alpha[kr];
            }
        };
        uint32_t wcur[UD], wnext[UD];
        float alcur, alnext;
        load_pair(r0 + grp, 0, wcur, alcur);
        for (int r = r0 + grp; r < r1; r += ngrp) {
            float y[BT];
#pragma unroll
            for (int c = 0; c < BT; ++c) y[c] = 0.0f;
            for (int i = 0; i < p.q; ++i) {
                if (i + 1 < p.q) load_pair(r, i + 1, wnext, alnext);
                else load_pair(r + ngrp, 0, wnext, alnext);
                float acc[BT];
#pragma unroll
                for (int c = 0; c < BT; ++c) acc[c] = 0.0f;
                lookup_unit<MU, BT, 0>(wcur, tab, acc);
#pragma unroll
                for (int c = 0; c < BT; ++c) y[c] = fmaf(alcur, acc[c], y[c]);
#pragma unroll
                for (int d = 0; d < UD; ++d) wcur[d] = wnext[d];
                alcur = alnext;
            }
            // reduce over the G lanes of the row group (G is a power of two <= 64)
            for (int off = G >> 1; off > 0; off >>= 1) {
#pragma unroll
                for (int c = 0; c < BT; ++c) y[c] += __shfl_xor(y[c], off, kWave);
            }
            if (L == 0) {
                if (multi) {
                    float* ya = yacc + (size_t)(r - r0) * BT;
#pragma unroll
                    for (int c = 0; c < BT; ++c) ya[c] += y[c];
                } else {
#pragma unroll
                    for (int c = 0; c < BT; ++c)
                        if (b0 + c < p.batch)
                            p.out[((size_t)sp * p.batch + b0 + c) * p.m + r] = y[c];
                }
            }
        }
    }

    if (multi) {
        __syncthreads();
        const int rows = r1 - r0;
        for (int i = tid; i < rows * BT; i += nthreads) {
            const int c = i / rows, rr = i - c * rows;  // consecutive threads -> consecutive rows
            if (b0 + c < p.batch)
                p.out[((size_t)sp * p.batch + b0 + c) * p.m + r0 + rr] = yacc[(size_t)rr * BT + c];
        }
    }
}

// Sum of the chunk-split partials in a fixed order: Y[i] = sum_s partial[s][i].  VEC = 4: 16-byte
// accesses (count a multiple of 4, both buffers 16-byte aligned).
template <int VEC>
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ partial,
                                                            float* __restrict__ Y, long long count,
                                                            int splits) {
    const long long i = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
    if (i >= count) return;
    if constexpr (VEC == 4) {
        float4 acc = *reinterpret_cast<const float4*>(partial + i);
        for (int s = 1; s < splits; ++s) {
            const float4 v = *reinterpret_cast<const float4*>(partial + (size_t)s * count + i);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *reinterpret_cast<float4*>(Y + i) = acc;
    } else {
        float acc = partial[i];
        for (int s = 1; s < splits; ++s) acc += partial[(size_t)s * count + i];
        Y[i] = acc;
    }
}

}  // namespace biq
