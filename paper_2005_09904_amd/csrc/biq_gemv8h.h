// LUT query for mu = 8, batch = 1, small layers: half tables.
//
// Algorithm 1 fills the second half of a table by negating the first (q[2^mu - 1 - k] = -q[k]).
// This kernel does not store that half at all: LDS holds entries 0..127 of every chunk and a
// lookup with key k >= 128 reads entry ~k & 127 and negates it.  A 128 KiB tile then covers 256
// chunks (n = 2048) instead of 128, so that layers up to that width need no split of the row
// over workgroups and no second kernel to add partial sums - which is what the run time of a
// small GEMV consists of.  The price is 4 more VALU instructions per lookup, irrelevant here;
// the streaming kernel for large matrices (biq_gemv8.h) keeps full tables.
//
// LDS layout.  A row's 256-byte key segment is covered by 16 lanes (lane L holds bytes
// [16L, 16L+16)), a wave load covers 4 rows.  Chunk c = 16*L + 4*td + e of the tile (td = dword
// of the lane's 16 bytes, e = byte in the dword), entry idx (0..127):
//       td * 32768 + idx * 256 + (e >> 1) * 128 + (e & 1) * 64 + L * 4
// The bank is L + 16 * (e & 1).  LDS serves a wave in halves of 32 lanes = 2 rows x 16 L; at
// static step te the lane of row rho visits byte e = (te + rho) & 3, so the two rows of a half
// use different parities of e and the 32 lanes hit 32 different banks for any keys.
#pragma once

#include "biq_gemv8.h"

namespace biq {

constexpr int kGemvHalfTileChunks = 256;
constexpr int kGemvHalfTileBytes = kGemvHalfTileChunks * 128 * 4;  // 131072

__device__ __forceinline__ uint32_t gemv8h_slot_offset(int L, int td, int e) {
    return (uint32_t)(td * 32768 + (e >> 1) * 128 + (e & 1) * 64 + L * 4);
}

// Sum over each aligned group of 16 lanes; every lane of the group gets the total.
__device__ __forceinline__ float reduce16(float v) {
    v = reduce8(v);
    v = dpp_add<0x140>(v);  // row_mirror
    return v;
}

// Half-table lookups, the part done once per key dword (4 keys): a key k >= 128 reads entry
// ~k & 127 and its value counts negative.  idx = the four keys with every byte that has its top
// bit set inverted (v_perm_b32's selectors 8..11 replicate the top bit of bytes 1 and 3 of either
// source over a byte: with the dword and the dword shifted by one byte as sources that is a 0xff
// mask on exactly the bytes to invert), so that each byte is the entry index and has bit 7 clear;
// sgn = per byte 0x3f or 0xbf, the top byte of +1.0f / -1.0f.  4 instructions per 4 keys.
__device__ __forceinline__ void half_table_prepare(uint32_t w, uint32_t& idx, uint32_t& sgn) {
    const uint32_t inv = __builtin_amdgcn_perm(w, w << 8, 0x0b090a08u);
    idx = w ^ inv;
    // (w & 0x80808080) | 0x3f3f3f3f as one v_bfi_b32: both constants in registers (a VOP3
    // instruction takes no literal here, and the compiler otherwise emits v_and + v_or)
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(sgn) : "v"(0x80808080u), "v"(w), "v"(0x3f3f3f3fu));
}
// Selector that moves byte e of sgn to the top of 0x00800000: +-1.0f in one v_perm_b32.
__device__ __forceinline__ constexpr uint32_t half_table_sign_selector(int e) {
    return ((uint32_t)(4 + e) << 24) | 0x00020c0cu;
}
__device__ __forceinline__ float half_table_sign(uint32_t sgn, uint32_t selector) {
    return __uint_as_float(__builtin_amdgcn_perm(sgn, 0x00800000u, selector));
}

// Entries 0..127 of the tables of chunks [c0, c0 + 256), built from X into the layout above.
// One job = (chunk, 32 keys): 256 x 4 = 1024 jobs; consecutive threads write consecutive banks.
__device__ __forceinline__ void gemv8h_build_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                  int tid, int nthreads) {
    const bool vec_ok = ((p.n & 3) == 0) && ((reinterpret_cast<uintptr_t>(p.X) & 15) == 0);
    for (int job = tid; job < 1024; job += nthreads) {
        const int L = job & 15, e = (job >> 4) & 3, td = (job >> 6) & 3, hq = job >> 8;
        float x[8], ent[32];
        load_chunk8(p.X, p.n, 1, 0, c0 + 16 * L + 4 * td + e, vec_ok, x);
        table32(x, (uint32_t)hq, ent);   // keys 32*hq .. 32*hq + 31, hq < 4: the stored half
        char* dst = lds_bytes + gemv8h_slot_offset(L, td, e) + (hq * 32) * 256;
#pragma unroll
        for (int l = 0; l < 32; ++l) *reinterpret_cast<float*>(dst + l * 256) = ent[l];
    }
}

// The same job by job for workgroups of 1024 threads (thread = job): the inputs are requested
// first (raw, from clamped addresses), ahead of the first step's keys, and the build then waits
// for them alone - requested after the keys, they would arrive behind a round trip to HBM.
__device__ __forceinline__ int gemv8h_job_chunk(int job) {
    return 16 * (job & 15) + 4 * ((job >> 6) & 3) + ((job >> 4) & 3);
}
__device__ __forceinline__ void gemv8h_job_x_ahead(const QueryParams& p, int c0, int job, float (&x)[8]) {
    load_chunk8_raw(p.X, p.n, c0 + gemv8h_job_chunk(job), x);
}
__device__ __forceinline__ void gemv8h_job_build(const QueryParams& p, char* lds_bytes, int c0, int job,
                                                 float (&x)[8]) {
    const int L = job & 15, e = (job >> 4) & 3, td = (job >> 6) & 3, hq = job >> 8;
    chunk8_zero_tail(p.n, c0 + gemv8h_job_chunk(job), x);
    float ent[32];
    table32(x, (uint32_t)hq, ent);
    char* dst = lds_bytes + gemv8h_slot_offset(L, td, e) + (hq * 32) * 256;
#pragma unroll
    for (int l = 0; l < 32; ++l) *reinterpret_cast<float*>(dst + l * 256) = ent[l];
}

// The same half tables copied from tables in device memory (LUT [C][256][1]).
__device__ __forceinline__ void gemv8h_copy_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                 int tid, int nthreads) {
    for (int i = tid; i < kGemvHalfTileChunks * 128; i += nthreads) {
        const int idx = i & 127, c = i >> 7;
        const int cL = c >> 4, td = (c >> 2) & 3, e = c & 3;
        float v = 0.0f;
        if (c0 + c < p.C) v = p.LUT[(size_t)(c0 + c) * 256 + idx];
        *reinterpret_cast<float*>(lds_bytes + gemv8h_slot_offset(cL, td, e) + idx * 256) = v;
    }
}

// One step of 4 rows per wave at a time (row_mode 1) or one row per wave at a time (row_mode 2);
// a tile's first step of keys and scales is requested before its tables are built.  row_mode 1
// can walk several 256-chunk tiles per workgroup (rows up to three tiles wide then need no second
// dispatch for partial sums): the row sums are carried in LDS behind the tables.
//
// LSTM = true (row_mode 1 only): the rows are the four gates i, f, g, o of an LSTM cell stacked
// (m = 4 * hidden); the 4 rows of a wave step are the 4 gates of ONE hidden unit, so that the
// step's epilogue has all four pre-activations in one wave and applies the cell update itself:
// p.out receives h, p.c_out the new cell state.  rows_per_wg counts gate rows (4 per unit).
template <int Q, bool FUSED, bool LSTM>
__device__ __forceinline__ void gemv8h_body(const QueryParams& p, const int wg) {
    extern __shared__ __align__(16) float lds[];
    char* const lds_bytes = reinterpret_cast<char*>(lds);

    const int task = (wg & 7) * p.tasks_per_xcd + (wg >> 3);
    if (task >= p.ntasks) return;
    const int sp = task % p.splits;
    const int rb = task / p.splits;
    const int r0 = rb * p.rows_per_wg;
    const int r1 = min(p.m, r0 + p.rows_per_wg);
    const int tile0 = sp * p.tps;  // tiles [tile0, tile1) of this split: one, or (row_mode 1) a few
    const int tile1 = min(p.tiles, tile0 + p.tps);
    const int tile = tile0;

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    // lookups address LDS absolutely (see lds_read_abs)
    if (lds_address_of(lds) != 0u) return;

    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    const int L = lane & 15;
    const int rsub = lane >> 4;  // row inside the wave step, 0..3
    const int rho = rsub & 1;    // the two rows of a 32-lane half use different byte parities

    // v_perm_b32: S0 = key dword, S1 = base; byte 0 <- base byte 0, byte 1 <- key byte
    // (te + rho) & 3, byte 2 <- base byte 2 (td >> 1), byte 3 <- 0.
    uint32_t sel[4], sgn_sel[4], base[2][4];
#pragma unroll
    for (int te = 0; te < 4; ++te) {
        const int e = (te + rho) & 3;
        sel[te] = 0x0c020000u | ((uint32_t)(4 + e) << 8);
        sgn_sel[te] = half_table_sign_selector(e);
        base[0][te] = (uint32_t)((e >> 1) * 128 + (e & 1) * 64 + L * 4);
        base[1][te] = base[0][te] | 0x10000u;
    }

    // The 16 lookups of a lane's 16 key bytes, in three phases - all addresses, all reads, all
    // signed additions - so that the 16 LDS reads are in flight together (written lookup by
    // lookup, the compiler keeps at most three in flight and the loop runs at LDS latency).
    auto lookup16 = [&](const u32x4& k) -> float {
        const uint32_t w[4] = {k.x, k.y, k.z, k.w};
        uint32_t sg[4], addr[16];
        float v[16];
#pragma unroll
        for (int td = 0; td < 4; ++td) {
            uint32_t idx;
            half_table_prepare(w[td], idx, sg[td]);
#pragma unroll
            for (int te = 0; te < 4; ++te) addr[4 * td + te] = __builtin_amdgcn_perm(idx, base[td >> 1][te], sel[te]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = lds_read_abs(addr[j] + ((j >> 2) & 1) * 32768);
        __builtin_amdgcn_sched_barrier(0);
        float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float f = half_table_sign(sg[j >> 2], sgn_sel[j & 3]);
            if (j & 1) a1 = fmaf(v[j], f, a1);
            else a0 = fmaf(v[j], f, a0);
        }
        return a0 + a1;
    };

    const uint32_t stride_bytes = (uint32_t)p.stride_dw * 4u;
    const int nrows = r1 - r0;

    if (!LSTM && p.row_mode == 2) {
        // ---- one row per wave at a time: the 64 lanes hold the row's 64 key dwords (4 lookups
        // per lane and plane instead of 16), for workgroups with so few rows that most waves
        // would otherwise idle through the lookups.  Lane = 4*L1 + td1 holds dword td1 of the
        // 16-byte group L1; at static step te it visits byte (te + td1) & 3, which leaves a 2-way
        // bank conflict per half-wave (8 groups x 2 byte parities = 16 banks for 32 lanes).
        const int L1 = lane >> 2, td1 = lane & 3;
        uint32_t sel1[4], sgn_sel1[4], base1[4];
#pragma unroll
        for (int te = 0; te < 4; ++te) {
            const int e = (te + td1) & 3;
            sel1[te] = 0x0c020000u | ((uint32_t)(4 + e) << 8);
            sgn_sel1[te] = half_table_sign_selector(e);
            base1[te] = (uint32_t)((e >> 1) * 128 + (e & 1) * 64 + L1 * 4) | ((uint32_t)(td1 >> 1) << 16);
        }
        const uint32_t td_bit15 = (uint32_t)(td1 & 1) << 15;
        const bool have = (uint32_t)(tile * 256 + lane * 4) < stride_bytes;
        // unconditional, from clamped addresses (a row past the end: the workgroup's first; a lane
        // past the end of the row: its start), so that the compiler can count the requests in
        // flight; such lanes meet zero tables, such rows are not stored
        auto load_row = [&](int row, uint32_t (&kw)[Q], float (&a)[Q]) {
            const int row_c = row < nrows ? row : 0;
            const uint32_t seg = have ? (uint32_t)(tile * 256 + lane * 4) : 0u;
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                const size_t kr = (size_t)i * p.m + r0 + row_c;
                kw[i] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(p.K) + kr * stride_bytes + seg);
                a[i] = p.alpha[kr];
            }
        };
        uint32_t kw[Q], kwn[Q];
        float a1[Q], a1n[Q];
        const bool x_ahead = FUSED && nthreads == 1024 && x_rows_vectorizable(p);
        float xa[8];
        if (x_ahead) gemv8h_job_x_ahead(p, tile * kGemvHalfTileChunks, tid, xa);
        load_row(wave, kw, a1);
        if constexpr (FUSED) {
            if (x_ahead) gemv8h_job_build(p, lds_bytes, tile * kGemvHalfTileChunks, tid, xa);
            else gemv8h_build_tile(p, lds_bytes, tile * kGemvHalfTileChunks, tid, nthreads);
        } else {
            gemv8h_copy_tile(p, lds_bytes, tile * kGemvHalfTileChunks, tid, nthreads);
        }
        __syncthreads();
        for (int row = wave; row < nrows; row += nwaves) {
            load_row(row + nwaves, kwn, a1n);
            float y = 0.0f;
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                float acc = 0.0f;
                uint32_t idx, sgn;
                half_table_prepare(kw[i], idx, sgn);
#pragma unroll
                for (int te = 0; te < 4; ++te) {
                    const uint32_t addr = __builtin_amdgcn_perm(idx, base1[te], sel1[te]) | td_bit15;
                    const float v = lds_read_abs(addr);
                    acc = fmaf(v, half_table_sign(sgn, sgn_sel1[te]), acc);
                }
                y = fmaf(a1[i], acc, y);
            }
            y = reduce16(y);
            y += __shfl_xor(y, 16, 64);
            y += __shfl_xor(y, 32, 64);
            if (lane == 0) p.out[(size_t)sp * p.m + r0 + row] = y;
#pragma unroll
            for (int i = 0; i < Q; ++i) { kw[i] = kwn[i]; a1[i] = a1n[i]; }
        }
        return;
    }

    int tl = tile0;  // the tile being worked on
    // row sums carried from tile to tile (only with several tiles per workgroup): behind the tables
    float* const yacc = reinterpret_cast<float*>(lds_bytes + kGemvHalfTileBytes);
    // LSTM: the workgroup's hidden units [u0, u0 + nunits), one unit (4 gate rows) per step
    const int u0 = LSTM ? rb * (p.rows_per_wg >> 2) : 0;
    const int nunits = LSTM ? min(p.hidden, u0 + (p.rows_per_wg >> 2)) - u0 : 0;
    const int nsteps = LSTM ? nunits : (nrows + 3) >> 2;
    // al[0..Q) = the scales of this lane's row; LSTM: al[Q] = its bias, al[Q + 1] = the previous cell
    // state of its unit (requested with the keys, so that the cell update waits for no memory access).
    // Inside the loop every load is issued by every lane: a load behind a condition makes the
    // compiler wait for ALL outstanding loads before the first use of any, and the step requested
    // ahead would no longer be in flight during the lookups.  A step past the end is replaced by
    // the step `s_else` (the one being worked on: its lines are in the caches, and they differ
    // from wave to wave - sending every idle request to one address queues them on one memory
    // channel), a lane without a row or without keys reads the workgroup's first row.  What such a
    // lane loads is harmless: the tables of chunks past the end of the row are zero, sums of absent
    // rows are not stored.
    auto load_step = [&](int s_want, int s_else, u32x4 (&k)[Q], float (&al)[Q + 2]) {
        const int s = s_want < nsteps ? s_want : s_else;
        // row of the key matrix inside a plane: LSTM: gate rsub of unit u0 + s
        int row = LSTM ? rsub * p.hidden + u0 + s : r0 + 4 * s + rsub;
        if (!LSTM && row >= r1) row = r0;
        const bool have_keys = (uint32_t)(tl * 256 + L * 16) < stride_bytes;
        const uint32_t seg = have_keys ? (uint32_t)(tl * 256 + 16 * L) : 0u;
#pragma unroll
        for (int i = 0; i < Q; ++i) {
            const size_t kr = (size_t)i * p.m + row;
            k[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(
                reinterpret_cast<const char*>(p.K) + kr * stride_bytes + seg));
            al[i] = p.alpha[kr];
        }
        if constexpr (LSTM) {
            al[Q] = p.bias[row];
            al[Q + 1] = p.c_prev[u0 + s];
        } else {
            al[Q] = 0.0f;
            al[Q + 1] = 0.0f;
        }
    };
    auto do_step = [&](int s, const u32x4 (&k)[Q], const float (&al)[Q + 2]) {
        float y = 0.0f;
#pragma unroll
        for (int i = 0; i < Q; ++i) y = fmaf(al[i], lookup16(k[i]), y);
        y = reduce16(y);
        if constexpr (LSTM) {
            // the four groups of 16 lanes hold z_i, z_f, z_g, z_o of unit u0 + s
            y += al[Q];
            const float zi = __shfl(y, 0, 64), zf = __shfl(y, 16, 64), zg = __shfl(y, 32, 64), zo = __shfl(y, 48, 64);
            if (lane == 0) {
                const size_t u = (size_t)(u0 + s);
                float h, c;
                lstm_cell_update(zi, zf, zg, zo, al[Q + 1], h, c);
                p.out[u] = h;
                p.c_out[u] = c;
            }
        } else {
            const int row = 4 * s + rsub;
            if (L == 0 && row < nrows) {
                // the same lane handles this row in every tile: no synchronisation needed
                if (tl != tile0) y += yacc[row];
                if (tl + 1 < tile1) yacc[row] = y;
                else p.out[(size_t)sp * p.m + r0 + row] = y;
            }
        }
    };
    // Two steps per wave in flight: the one being worked on and the next.  (A deeper ring - three or
    // four steps requested ahead, as in the streaming kernel - was measured 5-10 % SLOWER here at
    // every size from 16 to 128 MiB of keys: with 4 rows x 256 bytes per request the extra requests
    // in flight cost more in the memory system than the latency they hide.)
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const bool busy = wave_u < nsteps;  // wave-uniform: a wave without a step requests nothing
    u32x4 k[Q], kn[Q];
    float al[Q + 2], aln[Q + 2];
    const bool x_ahead = FUSED && nthreads == 1024 && x_rows_vectorizable(p);
    float xa[8];
    BIQ_STAMP(p, 0);
    for (; tl < tile1; ++tl) {
        int s = wave_u;
        // the tile's inputs, then its first step of keys (a wave without a step: step 0 again),
        // are requested before its tables are built; the build waits for the inputs alone
        // (the inputs of a further tile were requested a tile ahead, right after the build before)
        if (x_ahead && tl == tile0) gemv8h_job_x_ahead(p, tl * kGemvHalfTileChunks, tid, xa);
        load_step(s, 0, k, al);
        BIQ_STAMP(p, 1);
        if (tl != tile0) __syncthreads();  // every wave is done with the previous tables
        if constexpr (FUSED) {
            if (x_ahead) {
                gemv8h_job_build(p, lds_bytes, tl * kGemvHalfTileChunks, tid, xa);
                if (tl + 1 < tile1) gemv8h_job_x_ahead(p, (tl + 1) * kGemvHalfTileChunks, tid, xa);
            } else {
                gemv8h_build_tile(p, lds_bytes, tl * kGemvHalfTileChunks, tid, nthreads);
            }
        } else {
            gemv8h_copy_tile(p, lds_bytes, tl * kGemvHalfTileChunks, tid, nthreads);
        }
        BIQ_STAMP(p, 4);
        __syncthreads();
        BIQ_STAMP(p, 2);
        // two steps per trip, so that the step requested ahead lands in registers of its own
        if (busy) {
            do {
                load_step(s + nwaves, s, kn, aln);
                do_step(s, k, al);
                BIQ_STAMP(p, 3);
                s += nwaves;
                if (s >= nsteps) break;
                load_step(s + nwaves, s, k, al);
                do_step(s, kn, aln);
                s += nwaves;
            } while (s < nsteps);
        }
    }
    BIQ_STAMP(p, 6);
}

template <int Q, bool FUSED>
__global__ __launch_bounds__(1024) void gemv8h_kernel(const QueryParams p) {
    gemv8h_body<Q, FUSED, false>(p, blockIdx.x);
}

// The LSTM cell step for one input vector (fused tables): see gemv8h_body.
template <int Q>
__global__ __launch_bounds__(1024) void lstm8h_kernel(const QueryParams p) {
    gemv8h_body<Q, true, true>(p, blockIdx.x);
}

}  // namespace biq
