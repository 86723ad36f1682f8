// LUT query for mu = 8, batch >= 2, small layers: half tables, two input vectors per pass.
//
// The batched counterpart of biq_gemv8h.h: LDS holds entries 0..127 of every table (the upper
// half is the negated lower half, Algorithm 1), a key k >= 128 reads entry ~k & 127 and the
// value enters the sum with factor -1.  A 128 KiB tile then covers 128 chunks x 2 input vectors
// instead of 64 x 2, so layers up to n = 1024 need no split of the row over workgroups and no
// second kernel for partial sums.  Used for small calls only (run time = dispatch + latencies).
//
// LDS layout.  8 lanes cover a row's 128-byte key segment, a wave load covers 8 rows.  Chunk
// c = 16*L + 4*td + e of the tile, vector v (0/1), entry idx (0..127):
//       td * 32768 + idx * 256 + v * 128 + (L + 8*e) * 4
// One address serves both vectors (128 bytes apart, one ds_read2_b32).  The bank is L + 8*e; an
// LDS half-wave is 4 rows x 8 L and row rho visits byte e = (te + rho) & 3 at static step te:
// 32 different banks for any keys.
#pragma once

#include "biq_gemv8h.h"

namespace biq {

constexpr int kGemmHalfTileChunks = 128;
constexpr int kGemmHalfTileBytes = kGemmHalfTileChunks * 128 * 2 * 4;  // 131072

__device__ __forceinline__ uint32_t gemm8x2h_slot_offset(int L, int td, int e, int v) {
    return (uint32_t)(td * 32768 + v * 128 + (L + 8 * e) * 4);
}

// Entries 0..127 of the tables of chunks [c0, c0 + 128) for input vectors b0, b0 + 1.
// One job = (vector, chunk, 32 keys): 2 x 128 x 4 = 1024 jobs; consecutive threads write
// consecutive banks.
__device__ __forceinline__ void gemm8x2h_build_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                    int b0, int tid, int nthreads) {
    const bool vec_ok = ((p.n & 3) == 0) && ((reinterpret_cast<uintptr_t>(p.X) & 15) == 0);
    for (int job = tid; job < 1024; job += nthreads) {
        const int L = job & 7, e = (job >> 3) & 3, td = (job >> 5) & 3, v = (job >> 7) & 1, hq = job >> 8;
        float x[8], ent[32];
        load_chunk8(p.X, p.n, p.batch, b0 + v, c0 + 16 * L + 4 * td + e, vec_ok, x);
        table32(x, (uint32_t)hq, ent);   // keys 32*hq .. 32*hq + 31, hq < 4: the stored half
        char* dst = lds_bytes + gemm8x2h_slot_offset(L, td, e, v) + (hq * 32) * 256;
#pragma unroll
        for (int l = 0; l < 32; ++l) *reinterpret_cast<float*>(dst + l * 256) = ent[l];
    }
}

// The same job by job for workgroups of 1024 threads (thread = job), with the inputs requested
// ahead of the first step's keys (see gemv8h_job_x_ahead).  An absent second input vector reads
// the last one again; its results are never stored.
__device__ __forceinline__ int gemm8x2h_job_chunk(int job) {
    return 16 * (job & 7) + 4 * ((job >> 5) & 3) + ((job >> 3) & 3);
}
__device__ __forceinline__ void gemm8x2h_job_x_ahead(const QueryParams& p, int c0, int b0, int job, float (&x)[8]) {
    const int col = min(b0 + ((job >> 7) & 1), p.batch - 1);
    load_chunk8_raw(p.X + (size_t)col * p.n, p.n, c0 + gemm8x2h_job_chunk(job), x);
}
__device__ __forceinline__ void gemm8x2h_job_build(const QueryParams& p, char* lds_bytes, int c0, int job,
                                                   float (&x)[8]) {
    const int L = job & 7, e = (job >> 3) & 3, td = (job >> 5) & 3, v = (job >> 7) & 1, hq = job >> 8;
    chunk8_zero_tail(p.n, c0 + gemm8x2h_job_chunk(job), x);
    float ent[32];
    table32(x, (uint32_t)hq, ent);
    char* dst = lds_bytes + gemm8x2h_slot_offset(L, td, e, v) + (hq * 32) * 256;
#pragma unroll
    for (int l = 0; l < 32; ++l) *reinterpret_cast<float*>(dst + l * 256) = ent[l];
}

// The same half tables copied from tables in device memory (LUT [C][256][batch]).
__device__ __forceinline__ void gemm8x2h_copy_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                   int b0, int tid, int nthreads) {
    for (int i = tid; i < kGemmHalfTileChunks * 128 * 2; i += nthreads) {
        const int v = i & 1, idx = (i >> 1) & 127, c = i >> 8;
        const int cL = c >> 4, td = (c >> 2) & 3, e = c & 3;
        float val = 0.0f;
        if (c0 + c < p.C && b0 + v < p.batch)
            val = p.LUT[((size_t)(c0 + c) * 256 + idx) * p.batch + b0 + v];
        *reinterpret_cast<float*>(lds_bytes + gemm8x2h_slot_offset(cL, td, e, v) + idx * 256) = val;
    }
}

// One 128-chunk tile and one pair of input vectors per workgroup, one step of 8 rows per wave
// at a time; the first step's keys and scales are requested before the tables are built.
//
// LSTM = true: the rows are the four gates i, f, g, o of an LSTM cell stacked (m = 4 * hidden); the
// 8 rows of a wave step are the 4 gates of TWO hidden units (rows 0..3 of the step: unit 2s, rows
// 4..7: unit 2s + 1), so the step's epilogue has all pre-activations of its units in one wave
// and applies the cell update for both input vectors: p.out receives h, p.c_out the new cell
// state.  rows_per_wg counts gate rows (4 per unit, a multiple of 8).
template <int Q, bool FUSED, bool LSTM>
__device__ __forceinline__ void gemm8x2h_body(const QueryParams& p, const int wg) {
    extern __shared__ __align__(16) float lds[];
    char* const lds_bytes = reinterpret_cast<char*>(lds);

    const int task = (wg & 7) * p.tasks_per_xcd + (wg >> 3);
    if (task >= p.ntasks) return;
    const int bt = task % p.batch_tiles;
    const int rest = task / p.batch_tiles;
    const int sp = rest % p.splits;
    const int rb = rest / p.splits;
    const int b0 = bt * 2;
    const int r0 = rb * p.rows_per_wg;
    const int r1 = min(p.m, r0 + p.rows_per_wg);
    const int tile = sp;  // one tile per split

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    // lookups address LDS absolutely (see lds_read_abs)
    if (lds_address_of(lds) != 0u) return;

    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    const int L = lane & 7;
    const int rsub = lane >> 3;  // row inside the wave step, 0..7
    const int rho = rsub & 3;    // byte rotation: the 4 rows of a 32-lane half get distinct values

    // v_perm_b32: S0 = key dword, S1 = base; byte 0 <- base byte 0, byte 1 <- key byte
    // (te + rho) & 3, byte 2 <- base byte 2 (td >> 1), byte 3 <- 0.
    uint32_t sel[4], sgn_sel[4], base[2][4];
#pragma unroll
    for (int te = 0; te < 4; ++te) {
        const int e = (te + rho) & 3;
        sel[te] = 0x0c020000u | ((uint32_t)(4 + e) << 8);
        sgn_sel[te] = half_table_sign_selector(e);
        base[0][te] = (uint32_t)((L + 8 * e) * 4);
        base[1][te] = base[0][te] | 0x10000u;
    }

    // In three phases (addresses, reads, signed additions) so that the reads of all 16 lookups are
    // in flight together: see gemv8h_body.
    auto lookup16 = [&](const u32x4& k, float& s0, float& s1) {
        const uint32_t w[4] = {k.x, k.y, k.z, k.w};
        uint32_t sg[4], addr[16];
        float v0[16], v1[16];
#pragma unroll
        for (int td = 0; td < 4; ++td) {
            uint32_t idx;
            half_table_prepare(w[td], idx, sg[td]);   // entry ~key & 127, negated, for keys >= 128
#pragma unroll
            for (int te = 0; te < 4; ++te) addr[4 * td + te] = __builtin_amdgcn_perm(idx, base[td >> 1][te], sel[te]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            v0[j] = lds_read_abs(addr[j] + ((j >> 2) & 1) * 32768);
            v1[j] = lds_read_abs(addr[j] + ((j >> 2) & 1) * 32768 + 128);
        }
        __builtin_amdgcn_sched_barrier(0);
        float a0 = 0.0f, a1 = 0.0f, c0 = 0.0f, c1 = 0.0f;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float sgn = half_table_sign(sg[j >> 2], sgn_sel[j & 3]);
            if (j & 1) { a1 = fmaf(v0[j], sgn, a1); c1 = fmaf(v1[j], sgn, c1); }
            else { a0 = fmaf(v0[j], sgn, a0); c0 = fmaf(v1[j], sgn, c0); }
        }
        s0 = a0 + a1;
        s1 = c0 + c1;
    };

    const uint32_t stride_bytes = (uint32_t)p.stride_dw * 4u;
    const int nrows = r1 - r0;
    const bool have_keys = (uint32_t)(tile * 128 + L * 16) < stride_bytes;
    // LSTM: the workgroup's hidden units [u0, u0 + nunits), two units (8 gate rows) per step
    const int u0 = LSTM ? rb * (p.rows_per_wg >> 2) : 0;
    const int nunits = LSTM ? min(p.hidden, u0 + (p.rows_per_wg >> 2)) - u0 : 0;
    const int nsteps = LSTM ? (nunits + 1) >> 1 : (nrows + 7) >> 3;
    // al[0..Q) = the scales of this lane's row; LSTM: al[Q] = its bias, al[Q + 1], al[Q + 2] = the
    // previous cell state of its unit for the two input vectors (requested with the keys, so that
    // the cell update waits for no memory access)
    // Unconditional, from clamped addresses (a step past the end: step 0; a row past the end: the
    // workgroup's first; a lane past the end of the row: its start), so that the compiler can
    // count the requests in flight; such lanes meet zero tables, such rows are not stored.
    auto load_step = [&](int s_want, u32x4 (&k)[Q], float (&al)[Q + 3]) {
        const int s = s_want < nsteps ? s_want : 0;
        // row of the key matrix inside a plane: LSTM: gate (rsub & 3) of unit u0 + 2s + (rsub >> 2)
        int unit = 2 * s + (rsub >> 2);
        if (LSTM && unit >= nunits) unit = 0;
        int row = LSTM ? (rsub & 3) * p.hidden + u0 + unit : r0 + 8 * s + rsub;
        if (!LSTM && row >= r1) row = r0;
        const uint32_t seg = have_keys ? (uint32_t)(tile * 128 + 16 * L) : 0u;
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            const size_t kr = (size_t)i * p.m + row;
            k[i] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(p.K) + kr * stride_bytes + seg);
            al[i] = p.alpha[kr];
        }
        if constexpr (LSTM) {
            al[Q] = p.bias[row];
            al[Q + 1] = p.c_prev[(size_t)b0 * p.hidden + u0 + unit];
            al[Q + 2] = p.c_prev[(size_t)min(b0 + 1, p.batch - 1) * p.hidden + u0 + unit];
        } else {
            al[Q] = 0.0f;
            al[Q + 1] = 0.0f;
            al[Q + 2] = 0.0f;
        }
    };
    u32x4 k[Q], kn[Q];
    float al[Q + 3], aln[Q + 3];
    // the tile's inputs, then the first step of keys, are requested before the tables are built;
    // the build waits for the inputs alone
    const bool x_ahead = FUSED && nthreads == 1024 && x_rows_vectorizable(p);
    float xa[8];
    if (x_ahead) gemm8x2h_job_x_ahead(p, tile * kGemmHalfTileChunks, b0, tid, xa);
    load_step(wave, k, al);
    if constexpr (FUSED) {
        if (x_ahead) gemm8x2h_job_build(p, lds_bytes, tile * kGemmHalfTileChunks, tid, xa);
        else gemm8x2h_build_tile(p, lds_bytes, tile * kGemmHalfTileChunks, b0, tid, nthreads);
    } else {
        gemm8x2h_copy_tile(p, lds_bytes, tile * kGemmHalfTileChunks, b0, tid, nthreads);
    }
    __syncthreads();
    for (int s = wave; s < nsteps; s += nwaves) {
        load_step(s + nwaves, kn, aln);
        float y0 = 0.0f, y1 = 0.0f;
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            float s0, s1;
            lookup16(k[i], s0, s1);
            y0 = fmaf(al[i], s0, y0);
            y1 = fmaf(al[i], s1, y1);
        }
        y0 = reduce8(y0);
        y1 = reduce8(y1);
        if constexpr (LSTM) {
            // each half of the wave holds z_i, z_f, z_g, z_o of one unit in its four groups of 8 lanes
            y0 += al[Q];
            y1 += al[Q];
            const int half = lane & 32;
            const float zi0 = __shfl(y0, half, 64), zf0 = __shfl(y0, half + 8, 64);
            const float zg0 = __shfl(y0, half + 16, 64), zo0 = __shfl(y0, half + 24, 64);
            const float zi1 = __shfl(y1, half, 64), zf1 = __shfl(y1, half + 8, 64);
            const float zg1 = __shfl(y1, half + 16, 64), zo1 = __shfl(y1, half + 24, 64);
            const int unit = 2 * s + (lane >> 5);
            if ((lane & 31) == 0 && unit < nunits) {
                const size_t u = (size_t)b0 * p.hidden + u0 + unit;
                float h, c;
                lstm_cell_update(zi0, zf0, zg0, zo0, al[Q + 1], h, c);
                p.out[u] = h;
                p.c_out[u] = c;
                if (b0 + 1 < p.batch) {
                    lstm_cell_update(zi1, zf1, zg1, zo1, al[Q + 2], h, c);
                    p.out[u + p.hidden] = h;
                    p.c_out[u + p.hidden] = c;
                }
            }
        } else {
            const int row = 8 * s + rsub;
            if (L == 0 && row < nrows) {
                float* out = p.out + ((size_t)sp * p.batch + b0) * p.m + r0 + row;
                out[0] = y0;
                if (b0 + 1 < p.batch) out[p.m] = y1;
            }
        }
#pragma unroll
        for (int i = 0; i < Q; ++i) k[i] = kn[i];
#pragma unroll
        for (int i = 0; i < Q + 3; ++i) al[i] = aln[i];
    }
}

template <int Q, bool FUSED>
__global__ __launch_bounds__(1024) void gemm8x2h_kernel(const QueryParams p) {
    gemm8x2h_body<Q, FUSED, false>(p, blockIdx.x);
}

// The LSTM cell step for two input vectors per workgroup (fused tables): see gemm8x2h_body.
template <int Q>
__global__ __launch_bounds__(1024) void lstm8x2h_kernel(const QueryParams p) {
    gemm8x2h_body<Q, true, true>(p, blockIdx.x);
}

}  // namespace biq
