// LUT query for mu = 8, batch = 1 (GEMV): the HBM-bound case.
//
// A workgroup keeps the tables of one tile of 128 chunks (128 KiB) in LDS and streams its
// rows' 128-byte key segments with 128-bit loads: 8 lanes per row segment, 8 rows per wave
// load.  Per key byte the inner loop is one v_perm_b32 (forms the LDS address), one
// ds_read_b32 and one v_add_f32.
//
// LDS layout.  Chunk c of the tile is written c = 16*L + 4*td + e (L = lane inside the row
// group, td = dword of the lane's 16 bytes, e = byte of that dword).  Entry `key` of its
// table lives at byte address
//       (td >> 1) * 65536  +  key * 256  +  (td & 1) * 128  +  (L + 8*e) * 4
// so that (a) the key sits in byte 1 of the address and v_perm_b32 can drop it there
// straight from the key dword, and (b) the LDS bank is L + 8*e, independent of the key.
// LDS serves a wave in two halves of 32 lanes = 4 rows x 8 L.  At step te the lane of row
// rho visits byte e = (te + rho) & 3 of its dword, so the 32 lanes of a half hit the 32
// banks exactly once whatever the keys are: gathers are conflict-free by construction
// (the arrangement idea of Fig. 8, applied to chunks instead of batch entries).
#pragma once

#include "biq_common.h"
#include "biq_kernels.h"

namespace biq {

// Time stamps of a trace build (-DBIQ_TRACE, never the product's): lane 0 of every wave writes the
// 100 MHz wall clock into slot i of its entry in the buffer passed as QueryParams::LUT.
#ifdef BIQ_TRACE
#define BIQ_STAMP(p, i)                                                                               \
    do {                                                                                              \
        if ((threadIdx.x & 63) == 0)                                                                  \
            reinterpret_cast<unsigned long long*>(const_cast<float*>((p).LUT))                        \
                [((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + (i)] = wall_clock64();          \
    } while (0)
#else
#define BIQ_STAMP(p, i) do { } while (0)
#endif

constexpr int kGemvTileChunks = 128;
constexpr int kGemvTileBytes = kGemvTileChunks * 256 * 4;  // 131072

__device__ __forceinline__ uint32_t gemv8_slot_offset(int L, int td, int e) {
    return (uint32_t)((td >> 1) * 65536 + (td & 1) * 128 + (L + 8 * e) * 4);
}

template <int DPP_CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), DPP_CTRL, 0xf, 0xf, true);
    return v + __int_as_float(moved);
}

// Sum over each aligned group of 8 lanes; every lane of the group gets the total.
__device__ __forceinline__ float reduce8(float v) {
    v = dpp_add<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);  // row_half_mirror
    return v;
}

// Reads LDS at an absolute byte address.  The kernels below own all of LDS (no static
// __shared__ variable), so their dynamic LDS starts at address 0 and a table offset is an
// LDS address; this keeps the per-key address arithmetic to the single v_perm_b32.
typedef __attribute__((address_space(3))) const float lds_cfloat;
__device__ __forceinline__ float lds_read_abs(uint32_t byte_addr) {
    return *reinterpret_cast<lds_cfloat*>(static_cast<uintptr_t>(byte_addr));
}
// LDS address of a pointer into __shared__ memory.
__device__ __forceinline__ uint32_t lds_address_of(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Table build of a 128-chunk tile for one input vector, from X straight into the LDS layout
// above.  One job = (chunk, 32 keys): 128 x 8 = 1024 jobs; consecutive jobs write consecutive
// banks.  gemv8_job_x fetches the job's 8 inputs, gemv8_job_build turns them into 32 entries.
__device__ __forceinline__ int gemv8_job_chunk(int job) {
    const int L = job & 7, e = (job >> 3) & 3, td = (job >> 5) & 3;
    return 16 * L + 4 * td + e;
}

// The job's 8 inputs, requested ahead of time (rows that allow 128-bit loads only).  Raw: elements
// past the row still hold clamped reads; gemv8_job_build zeroes them.
__device__ __forceinline__ void gemv8_job_x_ahead(const QueryParams& p, int c0, int job, float (&x)[8]) {
    load_chunk8_raw(p.X, p.n, c0 + gemv8_job_chunk(job), x);
}

__device__ __forceinline__ void gemv8_job_build(const QueryParams& p, char* lds_bytes, int c0, int job,
                                                float (&x)[8]) {
    const int L = job & 7, e = (job >> 3) & 3, td = (job >> 5) & 3, hq = job >> 7;
    chunk8_zero_tail(p.n, c0 + gemv8_job_chunk(job), x);
    float ent[32];
    table32(x, (uint32_t)hq, ent);
    char* dst = lds_bytes + gemv8_slot_offset(L, td, e) + (hq * 32) * 256;
#pragma unroll
    for (int l = 0; l < 32; ++l) *reinterpret_cast<float*>(dst + l * 256) = ent[l];
}

// The same 32 entries in the order of Algorithm 1 (dynamic programming): the job's two blocks of 16
// keys start from their first entry (all of the block's low four signs negative), every further
// entry of a block comes from an earlier one by adding 2 x_t (t = highest set bit of its offset in
// the block), and entries of the upper half of the table are the negated entries of the lower half:
// the job of keys [32 hq, 32 hq + 32), hq < 4, also writes keys [224 - 32 hq, 256 - 32 hq) = the
// complements, so only jobs with hq < 4 do anything here and each writes 64 entries.
__device__ __forceinline__ void gemv8_job_build_dp(const QueryParams& p, char* lds_bytes, int c0, int job,
                                                   float (&x)[8]) {
    const int L = job & 7, e = (job >> 3) & 3, td = (job >> 5) & 3, hq = job >> 7;
    if (hq >= 4) return;
    chunk8_zero_tail(p.n, c0 + gemv8_job_chunk(job), x);
    float x2[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) x2[j] = 2.0f * x[j];
    float r0 = x[0];  // entry of key 0: -(x_0 + ... + x_7)
#pragma unroll
    for (int j = 1; j < 8; ++j) r0 += x[j];
    r0 = -r0;
    // first entry of the job's two blocks: bits 5, 6 of the key from hq, bit 4 = block
    float base = r0;
    base = (hq & 1) ? base + x2[5] : base;
    base = (hq & 2) ? base + x2[6] : base;
    char* dst = lds_bytes + gemv8_slot_offset(L, td, e);
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        float r[16];
        r[0] = blk ? base + x2[4] : base;
#pragma unroll
        for (int k = 1; k < 16; ++k) {
            const int t = 31 - __builtin_clz((unsigned)k);
            r[k] = r[k - (1 << t)] + x2[t];
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int key = 32 * hq + 16 * blk + k;
            *reinterpret_cast<float*>(dst + key * 256) = r[k];
            *reinterpret_cast<float*>(dst + (255 - key) * 256) = -r[k];
        }
    }
}

__device__ __forceinline__ bool x_rows_vectorizable(const QueryParams& p) {
    return ((p.n & 3) == 0) && ((reinterpret_cast<uintptr_t>(p.X) & 15) == 0);
}

__device__ __forceinline__ void gemv8_build_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                 int tid, int nthreads) {
    const bool vec_ok = x_rows_vectorizable(p);
    for (int job = tid; job < 1024; job += nthreads) {
        float x[8];
        load_chunk8(p.X, p.n, 1, 0, c0 + gemv8_job_chunk(job), vec_ok, x);
        gemv8_job_build(p, lds_bytes, c0, job, x);
    }
}

// The same tile copied from tables in device memory (LUT [C][256][1]).
__device__ __forceinline__ void gemv8_copy_tile(const QueryParams& p, char* lds_bytes, int c0,
                                                int tid, int nthreads) {
    for (int i = tid; i < kGemvTileChunks * 256; i += nthreads) {
        const int key = i & 255, c = i >> 8;
        const int cL = c >> 4, td = (c >> 2) & 3, e = c & 3;
        float v = 0.0f;
        if (c0 + c < p.C) v = p.LUT[(size_t)(c0 + c) * 256 + key];
        *reinterpret_cast<float*>(lds_bytes + gemv8_slot_offset(cL, td, e) + key * 256) = v;
    }
}

// MAXT = largest workgroup the instantiation may be launched with: 1024 threads leave 128 VGPRs
// per lane (4 planes then keep 2 steps of keys in flight per wave instead of 4), 512 leave 256.
template <int Q, bool FUSED, int MAXT>
__device__ __forceinline__ void gemv8_body(const QueryParams& p, const int wg) {
    extern __shared__ __align__(16) float lds[];
    char* const lds_bytes = reinterpret_cast<char*>(lds);
    float* const yacc = lds + kGemvTileBytes / 4;  // [rows_per_wg], used when a workgroup walks > 1 tile

    const int task = (wg & 7) * p.tasks_per_xcd + (wg >> 3);
    if (task >= p.ntasks) return;
    const int sp = task % p.splits;
    const int rb = task / p.splits;
    // Row range.  With xcd_skew > 0 (throughput mode, whole grid = 8 x tasks_per_xcd workgroups,
    // no chunk split) the workgroups of even XCDs take rows_per_wg + skew rows and those of odd
    // XCDs rows_per_wg - skew: measured on MI355X, odd XCDs stream from HBM 6-7 % slower than
    // even ones, and the hardware binds workgroup i to XCD i & 7.
    int r0 = rb * p.rows_per_wg;
    int r1 = min(p.m, r0 + p.rows_per_wg);
    if (p.xcd_skew > 0) {
        const int x = wg & 7, j = wg >> 3;
        const int mine = p.rows_per_wg + ((x & 1) ? -p.xcd_skew : p.xcd_skew);
        // XCDs before x: (x + 1) / 2 even ones and x / 2 odd ones
        const int before = p.tasks_per_xcd * (x * p.rows_per_wg + (((x + 1) >> 1) - (x >> 1)) * p.xcd_skew);
        r0 = min(p.m, before + j * mine);
        r1 = min(p.m, r0 + mine);
    }
    const int tile0 = sp * p.tps;
    const int tile1 = min(p.tiles, tile0 + p.tps);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    // The lookups address LDS absolutely (see lds_read_abs): fixed at compile time by this
    // kernel having no static LDS.  Should that ever change, leave Y untouched rather than
    // read wrong tables.
    if (lds_address_of(lds) != 0u) return;

    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    const int L = lane & 7;
    const int rsub = lane >> 3;  // row group inside the wave
    const int rho = rsub & 3;    // rotation: the 4 row groups of a 32-lane half get distinct values

    // v_perm_b32 operands: S0 = key dword (bytes 4..7 of the pair), S1 = base (bytes 0..3).
    // result byte 0 <- base byte 0, byte 1 <- key byte (te + rho) & 3, byte 2 <- base byte 2.
    uint32_t sel[4], base_lo[4], base_hi[4];
#pragma unroll
    for (int te = 0; te < 4; ++te) {
        const int e = (te + rho) & 3;
        sel[te] = 0x0c020000u | ((uint32_t)(4 + e) << 8);
        base_lo[te] = (uint32_t)((L + 8 * e) * 4);
        base_hi[te] = base_lo[te] | 0x10000u;
    }

    auto lookup16 = [&](const u32x4& k) -> float {
        const uint32_t w[4] = {k.x, k.y, k.z, k.w};
        float a0, a1;
#pragma unroll
        for (int td = 0; td < 4; ++td) {
#pragma unroll
            for (int te = 0; te < 4; ++te) {
                const uint32_t b = (td & 2) ? base_hi[te] : base_lo[te];
                const uint32_t addr = __builtin_amdgcn_perm(w[td], b, sel[te]);
                const float v = lds_read_abs(addr + (td & 1) * 128);
                if (td == 0 && te < 2) { if (te) a1 = v; else a0 = v; }
                else if (te & 1) a1 += v;
                else a0 += v;
            }
        }
        return a0 + a1;
    };

    const uint32_t stride_bytes = (uint32_t)p.stride_dw * 4u;
    const int nrows = r1 - r0;
    if (nrows <= 0) return;  // (uneven XCD shares can leave the last workgroups without rows)

    if (p.row_mode == 1) {
        // ---- latency mode: one tile per workgroup, one step of 8 rows per wave at a time.  The
        // first step's keys are requested before the tables are built.
        const int tile = tile0;
        const bool have_keys = (uint32_t)(tile * 128 + L * 16) < stride_bytes;
        const int nsteps = (nrows + 7) >> 3;
        // unconditional, from clamped addresses (a step or row past the end: the workgroup's first
        // row; a lane past the end of the row: its start), so that the compiler can count the
        // requests in flight; such lanes meet zero tables, such rows are not stored
        auto load_step = [&](int s, u32x4 (&k)[Q], float (&al)[Q]) {
            int row = 8 * s + rsub;
            if (s >= nsteps || row >= nrows) row = 0;
            const uint32_t seg = have_keys ? (uint32_t)(tile * 128 + 16 * L) : 0u;
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                const size_t kr = (size_t)i * p.m + r0 + row;
                k[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(
                    reinterpret_cast<const char*>(p.K) + kr * stride_bytes + seg));
                al[i] = p.alpha[kr];
            }
        };
        u32x4 k[Q], kn[Q];
        float al[Q], aln[Q];
        // the tile's inputs, then the first step of keys, are requested before the tables are
        // built; the build waits for the inputs alone
        const bool x_first = FUSED && nthreads == 1024 && x_rows_vectorizable(p) && p.table_fill == 0;
        float xf[8];
        if (x_first) gemv8_job_x_ahead(p, tile * kGemvTileChunks, tid, xf);
        load_step(wave, k, al);
        if constexpr (FUSED) {
            if (x_first) gemv8_job_build(p, lds_bytes, tile * kGemvTileChunks, tid, xf);
            else gemv8_build_tile(p, lds_bytes, tile * kGemvTileChunks, tid, nthreads);
        } else {
            gemv8_copy_tile(p, lds_bytes, tile * kGemvTileChunks, tid, nthreads);
        }
        __syncthreads();
        for (int s = wave; s < nsteps; s += nwaves) {
            load_step(s + nwaves, kn, aln);
            float y = 0.0f;
#pragma unroll
            for (int i = 0; i < Q; ++i) y = fmaf(al[i], lookup16(k[i]), y);
            y = reduce8(y);
            const int row = 8 * s + rsub;
            if (L == 0 && row < nrows) p.out[(size_t)sp * p.m + r0 + row] = y;
#pragma unroll
            for (int i = 0; i < Q; ++i) { k[i] = kn[i]; al[i] = aln[i]; }
        }
        return;
    }

    // ---- throughput mode.  Rows are handled in blocks of 64: in step t (0..7) row group g of
    // the wave reads row 8*g + t of the block, and the lane with L == t keeps the row's sum, so
    // that after the 8 steps lane j holds row j of the block: alpha and Y are accessed coalesced.
    // Block b of a tile goes to wave b mod nwaves; every wave runs the same number of block
    // iterations per tile (blocks that do not exist are skipped, their loads read one cache line).
    // All loads are issued unconditionally, from addresses clamped into the row block: with loads
    // behind per-lane conditions the compiler cannot count the requests in flight and drains them
    // (s_waitcnt vmcnt(0)) where it should wait for the oldest only.  So the ring of PD steps per
    // wave really stays in flight, runs on across tile boundaries, and the next tile's inputs are
    // fetched a tile ahead.
    const int nblk = (nrows + 63) >> 6;
    const int iters = (nblk + nwaves - 1) / nwaves;  // block iterations per wave and tile, >= 1
    // PD * Q KiB in flight per wave.  About 4 KiB per wave (64 KiB per CU) is the optimum: measured
    // with two planes, a ring of 4 steps is 3-6 % slower than one of 2 from 64 to 512 MiB of keys and
    // one of 8 is 15-30 % slower (requests queue in the memory system); with one plane 4 beats 2.
    constexpr int PD = Q == 1 ? 4 : 2;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const char* kbase[Q];
    const char* abase[Q];
#pragma unroll
    for (int i = 0; i < Q; ++i) {
        kbase[i] = reinterpret_cast<const char*>(p.K) + ((size_t)i * p.m + r0) * stride_bytes;
        abase[i] = reinterpret_cast<const char*>(p.alpha + (size_t)i * p.m + r0);
    }
    float* const obase = p.out + (size_t)sp * p.m + r0;
    const uint32_t last_row = (uint32_t)(nrows - 1);
    auto load_iter = [&](int tile, int bk, int t, u32x4 (&k)[Q]) {
        const bool there = bk < nblk && tile < tile1;  // the same for the whole wave
        const uint32_t row = min((uint32_t)(64 * bk + 8 * rsub + t), last_row);
        const uint32_t seg = min((uint32_t)(tile * 128 + L * 16), stride_bytes - 16u);
        const uint32_t voff = there ? row * stride_bytes + seg : 0u;
#pragma unroll
        for (int i = 0; i < Q; ++i)
            k[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kbase[i] + voff));
    };
    const bool x_ahead = FUSED && nthreads == 1024 && x_rows_vectorizable(p);
    float xa[8];
    if (x_ahead) gemv8_job_x_ahead(p, tile0 * kGemvTileChunks, tid, xa);
    auto build = [&](int tile) {
        if constexpr (FUSED) {
            if (p.table_fill == 1) {  // Algorithm 1's order (needs all 1024 jobs: 512 do the work)
                for (int job = tid; job < 1024; job += nthreads) {
                    float x[8];
                    if (x_ahead) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) x[j] = xa[j];
                    } else {
                        load_chunk8(p.X, p.n, 1, 0, tile * kGemvTileChunks + gemv8_job_chunk(job), x_rows_vectorizable(p), x);
                    }
                    gemv8_job_build_dp(p, lds_bytes, tile * kGemvTileChunks, job, x);
                }
            } else if (x_ahead) gemv8_job_build(p, lds_bytes, tile * kGemvTileChunks, tid, xa);
            else gemv8_build_tile(p, lds_bytes, tile * kGemvTileChunks, tid, nthreads);
            if (x_ahead && tile + 1 < tile1) gemv8_job_x_ahead(p, (tile + 1) * kGemvTileChunks, tid, xa);
        } else {
            gemv8_copy_tile(p, lds_bytes, tile * kGemvTileChunks, tid, nthreads);
        }
    };

    // Start-up: one step of keys per wave and the first tile's inputs are requested, the tables
    // are built, then the rest of the ring is requested.  (A CU's address unit takes about 20 clocks
    // per 128-bit wave load: the whole ring first would put the table build 2 us behind it.)
    u32x4 buf[PD][Q];
    BIQ_STAMP(p, 0);
    load_iter(tile0, wave_u, 0, buf[0]);
    BIQ_STAMP(p, 1);
    build(tile0);
    __syncthreads();
    BIQ_STAMP(p, 2);
#pragma unroll
    for (int s = 1; s < PD; ++s) load_iter(tile0, wave_u, s, buf[s]);

    for (int tile = tile0; tile < tile1; ++tile) {
        int it = 0;
        do {
            // The four waves that share a SIMD (w, w + 4, w + 8, w + 12) are served oldest first:
            // with equal shares the first ends 5 us before the last (measured at 4096 rows per
            // workgroup) and idles.  The issue priority rotates among them from block to block.
            switch (((wave_u >> 2) + it) & 3) {
                case 0: __builtin_amdgcn_s_setprio(0); break;
                case 1: __builtin_amdgcn_s_setprio(1); break;
                case 2: __builtin_amdgcn_s_setprio(2); break;
                default: __builtin_amdgcn_s_setprio(3); break;
            }
            const int bk = wave_u + it * nwaves;
            const bool last = it + 1 >= iters;
            const int next_bk = last ? wave_u : bk + nwaves;
            const int next_tile = last ? tile + 1 : tile;
            const int row_l = 64 * bk + lane;  // the row this lane finishes, relative to r0
            float al[Q], keep[Q];
#pragma unroll
            for (int i = 0; i < Q; ++i) {
                al[i] = *reinterpret_cast<const float*>(abase[i] + 4u * min((uint32_t)row_l, last_row));
                keep[i] = 0.0f;
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (bk < nblk) {  // the same for the whole wave
#pragma unroll
                    for (int i = 0; i < Q; ++i) {
                        const float sum = reduce8(lookup16(buf[t % PD][i]));
                        keep[i] = (L == t) ? sum : keep[i];
                    }
                }
                if (t + PD < 8) load_iter(tile, bk, t + PD, buf[t % PD]);
                else load_iter(next_tile, next_bk, t + PD - 8, buf[t % PD]);
            }
            if (bk < nblk) {
                float y = 0.0f;
#pragma unroll
                for (int i = 0; i < Q; ++i) y = fmaf(al[i], keep[i], y);
                if (tile != tile0) y += yacc[row_l];
                if (tile + 1 < tile1) yacc[row_l] = y;
                else if (row_l < nrows) obase[row_l] = y;
            }
        } while (++it < iters);
        if (tile + 1 < tile1) {
            BIQ_STAMP(p, 3);
            __syncthreads();  // every wave is done with these tables
            BIQ_STAMP(p, 4);
            build(tile + 1);
            __syncthreads();
            BIQ_STAMP(p, 5);
        }
    }
    BIQ_STAMP(p, 6);
}

template <int Q, bool FUSED, int MAXT = 1024>
__global__ __launch_bounds__(MAXT) void gemv8_kernel(const QueryParams p) {
    gemv8_body<Q, FUSED, MAXT>(p, blockIdx.x);
}

}  // namespace biq
