// LUT query for mu = 8, batch >= 2: two input vectors per workgroup pass.
//
// Same structure as the GEMV kernel (biq_gemv8.h): a 128 KiB LDS tile of tables, 128-bit key
// loads, one v_perm_b32 per key byte to form the LDS address, gathers that are free of bank
// conflicts for any key values.  Here a tile is 64 chunks x 2 input vectors, so 4 lanes cover
// a row's 64-byte key segment and a wave load covers 16 rows; one address serves both vectors
// (the two entries are 128 bytes apart: Fig. 8's "entries of one key side by side", spread
// over two bank sweeps instead of adjacent words so that each sweep stays conflict-free).
//
// LDS layout.  Chunk c = 16*L + 4*td + e of the tile (L = lane in the row group, td = dword
// of the lane's 16 key bytes, e = byte in the dword), vector v (0/1), entry `key`:
//       (td >> 1) * 65536 + key * 256 + v * 128 + (L + 4*e + 16*(td & 1)) * 4
// An LDS half-wave is 8 rows x 4 L.  Row r of the half visits, at static step (td, te), byte
// e = (te + r) & 3 of dword td ^ (r >> 2): the dwords of rows 4..7 are swapped pairwise after
// the load.  (L, e, td & 1) then takes 32 different values over the half: 32 different banks.
#pragma once

#include "biq_gemv8.h"

namespace biq {

constexpr int kGemmTileChunks = 64;
constexpr int kGemmTileBytes = kGemmTileChunks * 256 * 2 * 4;  // 131072
constexpr int kGemmBT = 2;

__device__ __forceinline__ uint32_t gemm8x2_slot_offset(int L, int td, int e, int v) {
    return (uint32_t)((td >> 1) * 65536 + v * 128 + (L + 4 * e + 16 * (td & 1)) * 4);
}

// Sum over each aligned group of 4 lanes; every lane of the group gets the total.
__device__ __forceinline__ float reduce4(float v) {
    v = dpp_add<0xB1>(v);  // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);  // quad_perm [2,3,0,1]
    return v;
}

// Tables of chunks [c0, c0 + 64) for input vectors b0, b0 + 1, built from X into the LDS
// layout above.  One job = (vector, chunk, 32 keys): 2 x 64 x 8 = 1024 jobs; consecutive threads
// write consecutive banks.
__device__ __forceinline__ void gemm8x2_build_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                   int b0, int tid, int nthreads) {
    const bool vec_ok = ((p.n & 3) == 0) && ((reinterpret_cast<uintptr_t>(p.X) & 15) == 0);
    for (int job = tid; job < 1024; job += nthreads) {
        const int L = job & 3, e = (job >> 2) & 3, td = (job >> 4) & 3, v = (job >> 6) & 1, hq = job >> 7;
        float x[8], ent[32];
        load_chunk8(p.X, p.n, p.batch, b0 + v, c0 + 16 * L + 4 * td + e, vec_ok, x);
        table32(x, (uint32_t)hq, ent);
        char* dst = lds_bytes + gemm8x2_slot_offset(L, td, e, v) + (hq * 32) * 256;
#pragma unroll
        for (int l = 0; l < 32; ++l) *reinterpret_cast<float*>(dst + l * 256) = ent[l];
    }
}

// One build job (vector, chunk, 32 keys) in two halves: its 8 inputs requested ahead of time (rows
// that allow 128-bit loads; an input vector past the batch reads the last one), and the entries
// built from them (inputs past the row or past the batch count as zero).
__device__ __forceinline__ void gemm8x2_job_x_ahead(const QueryParams& p, int c0, int b0, int job, float (&x)[8]) {
    const int L = job & 3, e = (job >> 2) & 3, td = (job >> 4) & 3, v = (job >> 6) & 1;
    load_chunk8_raw(p.X + (size_t)min(b0 + v, p.batch - 1) * p.n, p.n, c0 + 16 * L + 4 * td + e, x);
}

__device__ __forceinline__ void gemm8x2_job_build(const QueryParams& p, char* lds_bytes, int c0, int b0, int job,
                                                  float (&x)[8]) {
    const int L = job & 3, e = (job >> 2) & 3, td = (job >> 4) & 3, v = (job >> 6) & 1, hq = job >> 7;
    chunk8_zero_tail(b0 + v < p.batch ? p.n : 0, c0 + 16 * L + 4 * td + e, x);
    float ent[32];
    table32(x, (uint32_t)hq, ent);
    char* dst = lds_bytes + gemm8x2_slot_offset(L, td, e, v) + (hq * 32) * 256;
#pragma unroll
    for (int l = 0; l < 32; ++l) *reinterpret_cast<float*>(dst + l * 256) = ent[l];
}

// The same tile copied from tables in device memory (LUT [C][256][batch]).
__device__ __forceinline__ void gemm8x2_copy_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                  int b0, int tid, int nthreads) {
    for (int i = tid; i < kGemmTileChunks * 256 * 2; i += nthreads) {
        const int v = i & 1, key = (i >> 1) & 255, c = i >> 9;
        const int cL = c >> 4, td = (c >> 2) & 3, e = c & 3;
        float val = 0.0f;
        if (c0 + c < p.C && b0 + v < p.batch)
            val = p.LUT[((size_t)(c0 + c) * 256 + key) * p.batch + b0 + v];
        *reinterpret_cast<float*>(lds_bytes + gemm8x2_slot_offset(cL, td, e, v) + key * 256) = val;
    }
}

template <int Q, bool FUSED>
__global__ __launch_bounds__(1024) void gemm8x2_kernel(const QueryParams p) {
    extern __shared__ __align__(16) float lds[];
    char* const lds_bytes = reinterpret_cast<char*>(lds);
    float* const yacc = lds + kGemmTileBytes / 4;  // [rows_per_wg][2], when a workgroup walks > 1 tile

    const int wg = blockIdx.x;
    const int task = (wg & 7) * p.tasks_per_xcd + (wg >> 3);
    if (task >= p.ntasks) return;
    const int bt = task % p.batch_tiles;
    const int rest = task / p.batch_tiles;
    const int sp = rest % p.splits;
    const int rb = rest / p.splits;
    const int b0 = bt * kGemmBT;
    const int r0 = rb * p.rows_per_wg;
    const int r1 = min(p.m, r0 + p.rows_per_wg);
    const int tile0 = sp * p.tps;
    const int tile1 = min(p.tiles, tile0 + p.tps);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    // lookups address LDS absolutely (see lds_read_abs in biq_gemv8.h)
    if (lds_address_of(lds) != 0u) return;

    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    const int L = lane & 3;
    const int rsub = lane >> 2;       // row group inside the wave, 0..15
    const int rho = rsub & 3;         // byte rotation
    const bool swap = (rsub & 4) != 0;  // rows 4..7 of a half-wave work on pairwise swapped dwords

    // v_perm_b32: S0 = key dword, S1 = base; byte 0 <- base byte 0, byte 1 <- key byte
    // (te + rho) & 3, byte 2 <- base byte 2, byte 3 <- 0.
    uint32_t sel[4], base[2][2][4];  // base[td >> 1][td & 1][te]
#pragma unroll
    for (int te = 0; te < 4; ++te) {
        const int e = (te + rho) & 3;
        sel[te] = 0x0c020000u | ((uint32_t)(4 + e) << 8);
#pragma unroll
        for (int t1 = 0; t1 < 2; ++t1) {
            const int td_low = t1 ^ (swap ? 1 : 0);  // dword parity this lane really holds at step t1
            const uint32_t b = (uint32_t)((L + 4 * e + 16 * td_low) * 4);
            base[0][t1][te] = b;
            base[1][t1][te] = b | 0x10000u;
        }
    }

    auto lookup16 = [&](const u32x4& k, float& s0, float& s1) {
        // rows 4..7 of each half-wave: swap dwords 0<->1 and 2<->3
        const uint32_t w[4] = {swap ? k.y : k.x, swap ? k.x : k.y, swap ? k.w : k.z, swap ? k.z : k.w};
        float a0, a1, c0, c1;
#pragma unroll
        for (int td = 0; td < 4; ++td) {
#pragma unroll
            for (int te = 0; te < 4; ++te) {
                const uint32_t addr = __builtin_amdgcn_perm(w[td], base[td >> 1][td & 1][te], sel[te]);
                const float v0 = lds_read_abs(addr);
                const float v1 = lds_read_abs(addr + 128);
                if (td == 0 && te < 2) {
                    if (te) { a1 = v0; c1 = v1; } else { a0 = v0; c0 = v1; }
                } else if (te & 1) { a1 += v0; c1 += v1; }
                else { a0 += v0; c0 += v1; }
            }
        }
        s0 = a0 + a1;
        s1 = c0 + c1;
    };

    const uint32_t stride_bytes = (uint32_t)p.stride_dw * 4u;
    const int nrows = r1 - r0;

    if (p.row_mode == 1) {
        // ---- latency mode: one tile per workgroup, one step of 16 rows per wave at a time; the
        // first step's keys are requested before the tables are built.
        const int tile = tile0;
        const bool have_keys = (uint32_t)(tile * 64 + L * 16) < stride_bytes;
        const int nsteps = (nrows + 15) >> 4;
        // unconditional, from clamped addresses (a step or row past the end: the workgroup's first
        // row; a lane past the end of the row: its start), so that the compiler can count the
        // requests in flight; such lanes meet zero tables, such rows are not stored
        auto load_step = [&](int s, u32x4 (&k)[Q], float (&al)[Q]) {
            int row = 16 * s + rsub;
            if (s >= nsteps || row >= nrows) row = 0;
            const uint32_t seg = have_keys ? (uint32_t)(tile * 64 + 16 * L) : 0u;
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                const size_t kr = (size_t)i * p.m + r0 + row;
                k[i] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(p.K) + kr * stride_bytes + seg);
                al[i] = p.alpha[kr];
            }
        };
        u32x4 k[Q], kn[Q];
        float al[Q], aln[Q];
        // the tile's inputs, then the first step of keys, are requested before the tables are
        // built; the build waits for the inputs alone
        const bool x_first = FUSED && nthreads == 1024 && x_rows_vectorizable(p);
        float xf[8];
        if (x_first) gemm8x2_job_x_ahead(p, tile * kGemmTileChunks, b0, tid, xf);
        load_step(wave, k, al);
        if constexpr (FUSED) {
            if (x_first) gemm8x2_job_build(p, lds_bytes, tile * kGemmTileChunks, b0, tid, xf);
            else gemm8x2_build_tile(p, lds_bytes, tile * kGemmTileChunks, b0, tid, nthreads);
        } else {
            gemm8x2_copy_tile(p, lds_bytes, tile * kGemmTileChunks, b0, tid, nthreads);
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
            y0 = reduce4(y0);
            y1 = reduce4(y1);
            const int row = 16 * s + rsub;
            if (L == 0 && row < nrows) {
                float* out = p.out + ((size_t)sp * p.batch + b0) * p.m + r0 + row;
                out[0] = y0;
                if (b0 + 1 < p.batch) out[p.m] = y1;
            }
#pragma unroll
            for (int i = 0; i < Q; ++i) { k[i] = kn[i]; al[i] = aln[i]; }
        }
        return;
    }

    // ---- throughput mode.  Rows in blocks of 64 per wave: in step t (0..3) row group g reads
    // row 4*g + t and the lane with L == t keeps the row's sums, so after 4 steps lane j holds
    // row j of the block.  Block b of a tile goes to wave b mod nwaves, every wave runs the same
    // number of block iterations per tile.  As in the GEMV kernel all loads are issued
    // unconditionally from clamped addresses (so the compiler can count the requests in flight
    // instead of draining them), the ring of PD steps per wave runs on across tile boundaries, and
    // the next tile's inputs are fetched a tile ahead.
    const int nblk = (nrows + 63) >> 6;
    const int iters = (nblk + nwaves - 1) / nwaves;  // block iterations per wave and tile, >= 1
    constexpr int PD = (Q == 1) ? 4 : (Q <= 3 ? 2 : 1);  // steps in flight per wave (VGPR budget 128)
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const char* kbase[Q];
    const char* abase[Q];
#pragma unroll
    for (int i = 0; i < Q; ++i) {
        kbase[i] = reinterpret_cast<const char*>(p.K) + ((size_t)i * p.m + r0) * stride_bytes;
        abase[i] = reinterpret_cast<const char*>(p.alpha + (size_t)i * p.m + r0);
    }
    float* const obase = p.out + ((size_t)sp * p.batch + b0) * p.m + r0;
    const uint32_t last_row = (uint32_t)(nrows - 1);
    auto load_iter = [&](int tile, int bk, int t, u32x4 (&k)[Q]) {
        const bool there = bk < nblk && tile < tile1;  // the same for the whole wave
        const uint32_t row = min((uint32_t)(64 * bk + 4 * rsub + t), last_row);
        const uint32_t seg = min((uint32_t)(tile * 64 + L * 16), stride_bytes - 16u);
        const uint32_t voff = there ? row * stride_bytes + seg : 0u;
#pragma unroll
        for (int i = 0; i < Q; ++i) k[i] = *reinterpret_cast<const u32x4*>(kbase[i] + voff);
    };
    const bool x_ahead = FUSED && nthreads == 1024 && x_rows_vectorizable(p);
    float xa[8];
    if (x_ahead) gemm8x2_job_x_ahead(p, tile0 * kGemmTileChunks, b0, tid, xa);
    auto build = [&](int tile) {
        if constexpr (FUSED) {
            if (x_ahead) gemm8x2_job_build(p, lds_bytes, tile * kGemmTileChunks, b0, tid, xa);
            else gemm8x2_build_tile(p, lds_bytes, tile * kGemmTileChunks, b0, tid, nthreads);
            if (x_ahead && tile + 1 < tile1) gemm8x2_job_x_ahead(p, (tile + 1) * kGemmTileChunks, b0, tid, xa);
        } else {
            gemm8x2_copy_tile(p, lds_bytes, tile * kGemmTileChunks, b0, tid, nthreads);
        }
    };

    // start-up: one step of keys per wave, the tables, then the rest of the ring
    u32x4 buf[PD][Q];
    load_iter(tile0, wave_u, 0, buf[0]);
    build(tile0);
    __syncthreads();
#pragma unroll
    for (int s = 1; s < PD; ++s) load_iter(tile0, wave_u, s, buf[s]);

    for (int tile = tile0; tile < tile1; ++tile) {
        int it = 0;
        do {
            const int bk = wave_u + it * nwaves;
            const bool last = it + 1 >= iters;
            const int next_bk = last ? wave_u : bk + nwaves;
            const int next_tile = last ? tile + 1 : tile;
            const int row_l = 64 * bk + lane;  // the row this lane finishes, relative to r0
            float al[Q], keep0[Q], keep1[Q];
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                al[i] = *reinterpret_cast<const float*>(abase[i] + 4u * min((uint32_t)row_l, last_row));
                keep0[i] = 0.0f;
                keep1[i] = 0.0f;
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (bk < nblk) {  // the same for the whole wave
#pragma unroll
                    for (int i = 0; i < Q; ++i) {
                        float s0, s1;
                        lookup16(buf[t % PD][i], s0, s1);
                        s0 = reduce4(s0);
                        s1 = reduce4(s1);
                        keep0[i] = (L == t) ? s0 : keep0[i];
                        keep1[i] = (L == t) ? s1 : keep1[i];
                    }
                }
                if (t + PD < 4) load_iter(tile, bk, t + PD, buf[t % PD]);
                else load_iter(next_tile, next_bk, t + PD - 4, buf[t % PD]);
            }
            if (bk < nblk) {
                float y0 = 0.0f, y1 = 0.0f;
#pragma unroll
                for (int i = 0; i < Q; ++i) {
                    y0 = fmaf(al[i], keep0[i], y0);
                    y1 = fmaf(al[i], keep1[i], y1);
                }
                if (tile != tile0) {
                    const float2 prev = *reinterpret_cast<const float2*>(yacc + 2 * row_l);
                    y0 += prev.x;
                    y1 += prev.y;
                }
                if (tile + 1 < tile1) {
                    *reinterpret_cast<float2*>(yacc + 2 * row_l) = make_float2(y0, y1);
                } else if (row_l < nrows) {
                    obase[row_l] = y0;
                    if (b0 + 1 < p.batch) obase[p.m + row_l] = y1;
                }
            }
        } while (++it < iters);
        if (tile + 1 < tile1) {
            __syncthreads();  // every wave is done with these tables
            build(tile + 1);
            __syncthreads();
        }
    }
}

}  // namespace biq
