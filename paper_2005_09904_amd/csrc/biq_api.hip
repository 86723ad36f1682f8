// C ABI of libbiq (see include/biq.h): argument checks, launch planning, launches.
#include "biq.h"

#include <hip/hip_runtime.h>

#include "biq_launch.h"
// kernel headers: only their geometry constants are used here (no kernel is instantiated in this file)
#include "biq_gemv8.h"
#include "biq_gemm8x2.h"
#include "biq_gemv8h.h"
#include "biq_gemm8x2h.h"
#include "biq_query_wide.h"
#include "biq_quantize.h"
#include "biq_grouped.h"

namespace {

using namespace biq;

// gfx950 (MI355X) limits the planner is written for.
constexpr int kLdsTableBudget = 128 * 1024;  // tables of one tile (leaves room for 1 WG/CU extras)
constexpr int kNumCu = 256;
constexpr int kNumXcd = 8;

enum KernelId { KERNEL_GENERIC = 0, KERNEL_GEMV8 = 1, KERNEL_GEMM8X2 = 2, KERNEL_UNPACK_MFMA = 3, KERNEL_GEMV8H = 4, KERNEL_GEMM8X2H = 5, KERNEL_WIDE = 6, KERNEL_COUNT };

inline bool shape_ok(int m, int n, int q, int batch, int mu) {
    if (m < 1 || n < 1 || q < 1 || batch < 1) return false;
    if (mu < 1 || mu > kMaxMu) return false;
    if ((long long)m * q >= (1ll << 31)) return false;
    return true;
}

inline int unit_keys(int mu) {
    switch (mu) {
        case 10: return KeyUnit<10>::UK; case 9: return KeyUnit<9>::UK;
        case 8: return KeyUnit<8>::UK; case 7: return KeyUnit<7>::UK; case 6: return KeyUnit<6>::UK;
        case 5: return KeyUnit<5>::UK; case 4: return KeyUnit<4>::UK; case 3: return KeyUnit<3>::UK;
        case 2: return KeyUnit<2>::UK; default: return KeyUnit<1>::UK;
    }
}

inline int ceil_div(int a, int b) { return (int)(((long long)a + b - 1) / b); }
inline long long ceil_div_ll(long long a, long long b) { return (a + b - 1) / b; }
// rows per workgroup from a 64-bit estimate: rounded up to a multiple of `step`, at least `lo`, and
// never beyond what the 32-bit plan field holds (more rows than m are pointless anyway)
inline int rows_from(long long want, int step, int lo, int m) {
    long long r = ceil_div_ll(want, step) * step;
    const long long cap = ceil_div_ll(m, step) * step;
    if (r > cap) r = cap;
    if (r < lo) r = lo;
    return (int)r;
}
inline int ilog2(int v) { int l = 0; while ((1 << (l + 1)) <= v) ++l; return l; }

// 16-byte pieces of prepared input per key group (16 MFMA steps): column tiles x terms x 64 lanes
inline long long unpack_group_pieces(int batch_tile, int terms) { return 16ll * (batch_tile / 32) * terms * 64; }

// Unpack-MFMA plans: workgroups of 4 waves, key groups (32 key bytes of a row) instead of LUT tiles.
bool plan_finish_unpack(biq_plan& pl, int m, int n, int q, int batch) {
    if (q > 4 || pl.threads != kUnpackThreads) return false;
    if (pl.batch_tile != 32 && pl.batch_tile != 64) return false;
    if (pl.chunks_per_tile != kUnpackGroupBytes) return false;
    if (pl.wave_splits == 0) pl.wave_splits = 1;
    if (pl.input_terms == 0) pl.input_terms = 3;     // exact split unless the caller asks for two terms
    if (pl.input_terms != 2 && pl.input_terms != 3) return false;
    const int ws = pl.wave_splits;
    if (ws != 1 && ws != 2 && ws != 4) return false;
    // (4 / ws) waves side by side x r row tiles of 32 rows per plane, at most 4 row tiles per wave
    const int per_r = (4 / ws) * 32;
    if (pl.rows_per_wg % per_r) return false;
    const int r = pl.rows_per_wg / per_r;
    if ((r != 1 && r != 2 && r != 4) || q * r > 4) return false;
    if (ws == 4 && q * r * (pl.batch_tile / 32) == 8) return false;  // would not fit the register file
    if (pl.row_mode != 0 || pl.xcd_skew != 0 || pl.tiles_per_split < 1) return false;
    const int groups = (int)((biq_key_row_stride(n) + kUnpackGroupBytes - 1) / kUnpackGroupBytes);
    if (pl.tiles_per_split > groups) pl.tiles_per_split = groups;
    pl.chunk_splits = (groups + pl.tiles_per_split - 1) / pl.tiles_per_split;
    pl.row_blocks = (m + pl.rows_per_wg - 1) / pl.rows_per_wg;
    pl.batch_tiles = (batch + pl.batch_tile - 1) / pl.batch_tile;
    pl.lds_bytes = ws == 1 ? 24 * 1024 : 96 * 1024;   // partial sums of the wave groups, transpose patches (UnpackGeom::LDS_BYTES)
    const long long tasks = (long long)pl.row_blocks * pl.chunk_splits * pl.batch_tiles;
    if (tasks > (1ll << 30)) return false;
    // prepared input: 2 bytes per term and (padded column, padded element)
    const long long xf = (long long)pl.batch_tiles * pl.chunk_splits * pl.tiles_per_split *
                         unpack_group_pieces(pl.batch_tile, pl.input_terms) * 16;
    if (xf > (1ll << 40)) return false;
    return true;
}

inline int plan_lds_bytes(const biq_plan& pl, int mu) {
    if (pl.kernel == KERNEL_GEMV8)
        return kGemvTileBytes +
               (pl.tiles_per_split > 1 ? ((pl.rows_per_wg + pl.xcd_skew + 63) / 64) * 64 * 4 : 0);
    if (pl.kernel == KERNEL_GEMV8H)
        return kGemvHalfTileBytes + (pl.tiles_per_split > 1 ? ((pl.rows_per_wg + 3) / 4) * 16 : 0);
    if (pl.kernel == KERNEL_GEMM8X2H) return kGemmHalfTileBytes;
    if (pl.kernel == KERNEL_WIDE) return 128 * 1024;
    if (pl.kernel == KERNEL_GEMM8X2)
        return kGemmTileBytes + (pl.tiles_per_split > 1 ? ((pl.rows_per_wg + 63) / 64) * 64 * 8 : 0);
    long long b = (long long)pl.chunks_per_tile * (1 << mu) * pl.batch_tile * 4;
    if (pl.tiles_per_split > 1) b += (long long)pl.rows_per_wg * pl.batch_tile * 4;
    return b > (1ll << 30) ? (1 << 30) : (int)b;
}

// Completes the derived fields and checks a plan against the shape and device limits.
bool plan_finish(biq_plan& pl, int m, int n, int q, int batch, int mu) {
    const int UK = unit_keys(mu);
    const int C = ceil_div(n, mu);
    if (pl.kernel < 0 || pl.kernel >= KERNEL_COUNT) return false;
    if (pl.kernel == KERNEL_UNPACK_MFMA) return plan_finish_unpack(pl, m, n, q, batch);
    if (pl.wave_splits != 0 || pl.input_terms != 0) return false;  // unpack_mfma only
    if (pl.table_fill != 0 && !(pl.table_fill == 1 && pl.kernel == KERNEL_GEMV8 && pl.row_mode == 0)) return false;
    if (pl.threads < 64 || pl.threads > 1024 || pl.threads % 64) return false;
    if (pl.kernel == KERNEL_GEMV8) {
        // mu = 8, one input vector, at most 4 planes; one 128-chunk tile per workgroup
        if (mu != 8 || batch != 1 || q > 4) return false;
        if (pl.chunks_per_tile != kGemvTileChunks || pl.batch_tile != 1) return false;
        // 32-bit byte offsets inside a workgroup's row block
        if ((long long)pl.rows_per_wg * (long long)biq_key_row_stride(n) >= (1ll << 31)) return false;
    }
    if (pl.kernel == KERNEL_GEMV8H) {
        // mu = 8, one input vector, at most 4 planes; 256-chunk tiles of half tables, latency mode
        // only; row_mode 1 can walk several tiles (row sums carried in LDS beside the tables)
        if (mu != 8 || batch != 1 || q > 4) return false;
        if (pl.chunks_per_tile != kGemvHalfTileChunks || pl.batch_tile != 1) return false;
        if (pl.row_mode != 1 && pl.row_mode != 2) return false;
        if (pl.tiles_per_split != 1 && (pl.row_mode != 1 || pl.rows_per_wg > 4096)) return false;
    }
    if (pl.kernel == KERNEL_WIDE) {
        // mu <= 6; one tile of 32 key units per workgroup, batch tile fixed by mu (tables fill 128 KiB)
        if (mu > 6 || pl.chunks_per_tile != 32 * UK) return false;
        if (pl.batch_tile != (128 * 1024) / (32 * UK * (1 << mu) * 4)) return false;
        if (pl.row_mode != 0 || pl.tiles_per_split != 1) return false;
    }
    if (pl.kernel == KERNEL_GEMM8X2H) {
        // mu = 8, at most 4 planes; one 128-chunk tile of half tables for two input vectors per
        // workgroup, latency mode only
        if (mu != 8 || q > 4) return false;
        if (pl.chunks_per_tile != kGemmHalfTileChunks || pl.batch_tile != 2) return false;
        if (pl.row_mode != 1 || pl.tiles_per_split != 1) return false;
    }
    if (pl.kernel == KERNEL_GEMM8X2) {
        // mu = 8, at most 4 planes; 64-chunk tiles of two input vectors
        if (mu != 8 || q > 4) return false;
        if (pl.chunks_per_tile != kGemmTileChunks || pl.batch_tile != kGemmBT) return false;
        if ((long long)pl.rows_per_wg * (long long)biq_key_row_stride(n) >= (1ll << 31)) return false;
    }
    if (pl.batch_tile != 1 && pl.batch_tile != 2 && pl.batch_tile != 4 && pl.batch_tile != 8) return false;
    if (pl.chunks_per_tile < UK || pl.chunks_per_tile % UK) return false;
    const int G = pl.chunks_per_tile / UK;
    if (G > 64 || (G & (G - 1))) return false;
    if (pl.rows_per_wg < 1 || pl.tiles_per_split < 1) return false;
    const int tiles = ceil_div(C, pl.chunks_per_tile);
    if (pl.tiles_per_split > tiles) pl.tiles_per_split = tiles;
    if (pl.row_mode != 0 &&
        !(pl.row_mode == 1 && pl.kernel != KERNEL_GENERIC && (pl.tiles_per_split == 1 || pl.kernel == KERNEL_GEMV8H)) &&
        !(pl.row_mode == 2 && pl.kernel == KERNEL_GEMV8H))
        return false;
    if (pl.xcd_skew != 0) {
        // only the GEMV kernel's throughput mode, whole grid = 8 equal XCD shares, no chunk split
        if (pl.kernel != KERNEL_GEMV8 || pl.row_mode != 0 || pl.xcd_skew < 0) return false;
        if (pl.xcd_skew >= pl.rows_per_wg || ceil_div(m, pl.rows_per_wg) % kNumXcd != 0) return false;
        if (ceil_div(tiles, pl.tiles_per_split) != 1) return false;
        // (even XCDs hold rows_per_wg + xcd_skew rows in LDS: counted in lds_bytes below)
    }
    pl.chunk_splits = ceil_div(tiles, pl.tiles_per_split);
    pl.row_blocks = ceil_div(m, pl.rows_per_wg);
    pl.batch_tiles = ceil_div(batch, pl.batch_tile);
    pl.lds_bytes = plan_lds_bytes(pl, mu);
    if (pl.lds_bytes > kLdsPerCu) return false;
    const long long tasks = (long long)pl.row_blocks * pl.chunk_splits * pl.batch_tiles;
    if (tasks > (1ll << 30)) return false;
    return true;
}

// Where the lookup tables stop paying off (the crossover of Sec. IV-B / Fig. 10): estimated
// run times of both paths from rates measured on MI355X.  Table lookups: about 13e12 lookups/s
// for the conflict-free kernels (mu = 8, mu <= 5, mu = 6 up to 4 input vectors); 6.5e12 for the
// generic one, which also streams keys at no more than about 0.25 TB/s; plus 6 us of launch
// and table build.  Unpack + MFMA with the exact split: 2 * 3 flop per weight and padded input
// vector (three bf16 terms) at 1.45e15 flop/s, plus 10 us (input split, launches, combining
// partial sums).
bool unpack_mfma_is_faster(int m, int n, int q, int batch, int mu) {
    const double weights = (double)q * m * n;
    const double lookups = weights / mu * batch;
    const bool tuned = mu == 8 || mu <= 5 || (mu == 6 && batch <= 4);
    double t_lut = lookups / (tuned ? 13e12 : 6.5e12);
    if (!tuned && t_lut < weights / 8 / 0.25e12) t_lut = weights / 8 / 0.25e12;
    t_lut += 6e-6;
    const double padded = (double)((batch + 31) / 32) * 32;
    const double t_mfma = 10e-6 + 6.0 * weights * padded / 1.45e15;
    return t_mfma < t_lut;
}

// The mapping of the unpack + MFMA kernel - column tile (32 or 64 input vectors), row tiles per
// wave and plane (r), wave groups along the contraction inside a workgroup (ws; partial sums
// added in LDS) and workgroups along the contraction (S; partial sums through the workspace and
// a second kernel) - is the candidate with the lowest estimated time.  The estimate: MFMAs per
// wave x 33 clk at 2.1 GHz (measured rate of back-to-back MFMAs under load) x an issue-overhead
// factor per accumulator shape (smallest for 4 x 2 tiles, more for fewer, where key expansion
// and fragment loads are shared by fewer MFMAs) x rounds of workgroups over the 256 CUs, plus
// fixed costs per launch, accumulator tile and round, the input split (per byte of padded X)
// and the second kernel.  The constants (one set per number of input terms) are least-squares
// fits to sweeps of 16 layer shapes x all valid mappings, on which the estimate's choice was the
// fastest or within 5 % of it.
struct UnpackCost {
    double shape8, shape6, shape4x1, shape3x1, shape2x2, shape2x1, shape1x2, shape1x1;
    double fix, per_tile, per_round, split_per_mb, second_kernel, second_per_mb, per_wave_group;
};
const UnpackCost kUnpackCost3 = {1.13, 1.16, 1.19, 1.22, 1.22, 1.30, 1.45, 1.65, 9.0, 0.25, 0.0, 0.0, 3.5, 0.4, 0.6};
const UnpackCost kUnpackCost2 = {1.20, 1.20, 1.36, 1.29, 1.42, 1.67, 2.10, 2.27, 5.3, 1.0, 1.1, 1.65, 2.45, 0.1, 0.0};

bool plan_unpack(biq_plan& pl, int m, int n, int q, int batch, int mu, int terms) {
    if (q > 4 || (terms != 2 && terms != 3)) return false;
    const UnpackCost& c = terms == 3 ? kUnpackCost3 : kUnpackCost2;
    pl = biq_plan{};
    pl.kernel = KERNEL_UNPACK_MFMA;
    pl.threads = kUnpackThreads;
    pl.chunks_per_tile = kUnpackGroupBytes;
    pl.input_terms = terms;
    const int groups = (int)((biq_key_row_stride(n) + kUnpackGroupBytes - 1) / kUnpackGroupBytes);
    double best = 1e30;
    for (int bt = 32; bt <= 64; bt += 32)
        for (int ws = 1; ws <= 4; ws *= 2)
            for (int r = 1; r <= 4; r *= 2)
                for (int S = 1; S <= 16; S *= 2) {
                    const int ct = bt / 32, rt = q * r;
                    if (rt > 4 || S * ws > groups) continue;
                    if (ws == 4 && rt * ct == 8) continue;   // would not fit the register file
                    const int rows = (4 / ws) * 32 * r;
                    const long long wgs = (long long)ceil_div(m, rows) * ceil_div(batch, bt) * S;
                    if (wgs > 4ll * kNumCu && S > 1) continue;
                    const int gpw = ceil_div(ceil_div(groups, S), ws);   // key groups per wave
                    const double shape = rt * ct == 8 ? c.shape8 : rt * ct == 6 ? c.shape6 : rt == 4 ? c.shape4x1
                                       : rt == 3 ? c.shape3x1 : (rt == 2 && ct == 2) ? c.shape2x2
                                       : rt == 2 ? c.shape2x1 : ct == 2 ? c.shape1x2 : c.shape1x1;
                    const double rounds = (double)ceil_div_ll(wgs, kNumCu);
                    const double bpad_mb = (double)ceil_div(batch, bt) * bt * 4 / 1e6;   // MB per element of a vector
                    double t = (double)terms * rt * ct * gpw * 16 * 33 * shape / 2100.0 * rounds;
                    t += c.fix + c.per_tile * rt * ct * rounds + c.per_round * (rounds - 1.0) + c.split_per_mb * bpad_mb * n;
                    if (S > 1) t += c.second_kernel + c.second_per_mb * (S + 1.0) * bpad_mb * m;
                    if (ws > 1) t += c.per_wave_group * (ws - 1) * rt * ct / 4;
                    if (t < best) {
                        best = t;
                        pl.batch_tile = bt;
                        pl.wave_splits = ws;
                        pl.rows_per_wg = rows;
                        pl.tiles_per_split = ceil_div(groups, S);
                    }
                }
    return plan_finish(pl, m, n, q, batch, mu);
}

// Default mapping.  Algorithm 2 leaves the tile sizes open; the choices here are:
//  - batch tile: as many input vectors as one lookup can serve with a single wide LDS read
//  - tile width: the largest power-of-two number of key units whose tables fit the LDS budget
//  - chunk splits: bounded so that the partial sums written stay below about twice the
//    bytes the method has to move anyway
//  - rows per workgroup: enough workgroups to fill the 256 CUs several times over
bool plan_generic(biq_plan& pl, int m, int n, int q, int batch, int mu);

bool plan_tuned(biq_plan& pl, int m, int n, int q, int batch, int mu, bool tables_given) {
    const int UK = unit_keys(mu);
    const int C = ceil_div(n, mu);
    const int E = 1 << mu;
    pl = biq_plan{};
    if (!tables_given && q <= 4 && unpack_mfma_is_faster(m, n, q, batch, mu)) {
        // Many input vectors: the contraction is compute bound and the matrix cores beat the
        // table lookups (the crossover of Sec. IV-B / Fig. 10); exact input split.
        return plan_unpack(pl, m, n, q, batch, mu, 3);
    }
    if (mu == 8 && batch == 1 && q <= 4) {
        // GEMV: workgroups of 1024 threads, 128-chunk tiles, one workgroup per CU when the
        // rows allow it (every further round of workgroups pays the table build again).  With
        // >= 512 rows per CU a workgroup walks all tiles of its rows (no partial sums: measured
        // equal to or faster than a split from there on); otherwise the tiles are split over
        // workgroups as well and the partials are summed by a second small kernel.
        pl.kernel = KERNEL_GEMV8;
        pl.threads = 1024;
        pl.chunks_per_tile = kGemvTileChunks;
        pl.batch_tile = 1;
        const int tiles = ceil_div(C, kGemvTileChunks);
        if (ceil_div(m, 512) >= kNumCu) {
            pl.tiles_per_split = tiles;
            int rows = ceil_div(ceil_div(m, kNumCu), 64) * 64;
            pl.rows_per_wg = rows > 8192 ? 8192 : rows;
            // Odd XCDs stream slower than even ones, by an amount that differs from box to box and
            // grows with the run time (in-kernel time stamps, back-to-back launches, equal shares:
            // workgroups on odd XCDs end 6 % later on one box and 13 % on another with 4096 rows
            // each, 0-7 % with 1024 rows): rows are moved from the odd to the even XCDs, 4.5 % of a
            // workgroup's share from 4096 rows on, 3 % from 2048, in units of 32 rows.
            if (ceil_div(m, pl.rows_per_wg) % kNumXcd == 0 && pl.rows_per_wg >= 2048) {
                const int permille = pl.rows_per_wg >= 4096 ? 45 : 30;
                pl.xcd_skew = ((pl.rows_per_wg * permille / 1000 + 16) / 32) * 32;
                if (tiles > 1 && pl.rows_per_wg + pl.xcd_skew > 8192) pl.xcd_skew = 0;
            }
        } else if (C > kGemvTileChunks && (long long)m * ceil_div(C, kGemvHalfTileChunks) <= 512ll * kNumCu) {
            // small and mid-size (up to where a workgroup of the full-table kernel gets 512 rows and
            // walks all its tiles), wider than one full-table tile: half tables (256 chunks per
            // workgroup), so that rows up to n = 2048 need no split and no second kernel.  One workgroup per CU if the
            // rows allow it (a second round of workgroups pays the table build again), at least
            // 8 rows each; 4 rows per wave step, at most 4 steps per wave.
            pl.kernel = KERNEL_GEMV8H;
            pl.chunks_per_tile = kGemvHalfTileChunks;
            pl.tiles_per_split = 1;
            pl.row_mode = 1;
            const int tiles_h = ceil_div(C, kGemvHalfTileChunks);
            if (tiles_h == 2 || tiles_h == 3) {
                // two or three tiles: a workgroup walks them (a table build of 1.3 us each) rather
                // than sharing the row with other workgroups, which costs a second dispatch (2.5 us
                // and more) for the sum of the partial results
                pl.tiles_per_split = tiles_h;
                pl.rows_per_wg = rows_from(ceil_div(m, kNumCu), 4, 8, m);
            } else {
                pl.rows_per_wg = rows_from(ceil_div_ll((long long)m * tiles_h, kNumCu), 4, 8, m);
                // up to one row per wave: 64 lanes per row instead of 16 (4 lookups per lane and plane)
                if (pl.rows_per_wg <= 16) pl.row_mode = 2;
            }
        } else if ((long long)m * tiles <= 4ll * 128 * kNumCu) {
            // small: latency mode, 8 rows per wave step, at most 4 steps per wave
            pl.tiles_per_split = 1;
            pl.row_mode = 1;
            pl.rows_per_wg = rows_from(ceil_div_ll((long long)m * tiles, kNumCu), 8, 8, m);
        } else {
            pl.tiles_per_split = 1;
            const int rows = rows_from(ceil_div_ll((long long)m * tiles, kNumCu), 64, 64, m);
            pl.rows_per_wg = rows > 8192 ? 8192 : rows;
        }
        return plan_finish(pl, m, n, q, batch, mu);
    }
    if (mu == 8 && batch >= 2 && q <= 4 && C > kGemmTileChunks &&
        (long long)m * ceil_div(C, kGemmHalfTileChunks) * ceil_div(batch, 2) <= 512ll * kNumCu) {
        // Small batched calls wider than one full-table tile: half tables (128 chunks x 2 input
        // vectors per workgroup) halve the number of row splits; up to n = 1024 there is none and
        // no second kernel.  One workgroup per CU if the rows allow it, at least 8 rows each;
        // 8 rows per wave step, at most 4 steps per wave.
        pl.kernel = KERNEL_GEMM8X2H;
        pl.threads = 1024;
        pl.chunks_per_tile = kGemmHalfTileChunks;
        pl.batch_tile = 2;
        pl.tiles_per_split = 1;
        pl.row_mode = 1;
        const long long units = (long long)m * ceil_div(C, kGemmHalfTileChunks) * ceil_div(batch, 2);
        pl.rows_per_wg = rows_from(ceil_div_ll(units, kNumCu), 8, 8, m);
        return plan_finish(pl, m, n, q, batch, mu);
    }
    if (mu == 8 && batch >= 2 && q <= 4) {
        // Batched: workgroups of 1024 threads over (row block, chunk split, pair of input
        // vectors).  Rows per workgroup as many as the LDS row accumulators hold (4096), so that
        // a table build is amortised over many lookups; tiles are split over workgroups only as
        // far as needed to give every CU a workgroup; if that is still not enough, rows shrink.
        pl.kernel = KERNEL_GEMM8X2;
        pl.threads = 1024;
        pl.chunks_per_tile = kGemmTileChunks;
        pl.batch_tile = kGemmBT;
        const int tiles = ceil_div(C, kGemmTileChunks);
        const int T = ceil_div(batch, kGemmBT);
        int rows = ceil_div(m, 64) * 64;
        if (rows > 4096) rows = 4096;
        const long long RT = (long long)ceil_div(m, rows) * T;
        int S = 1;
        if (RT < kNumCu) {
            S = (int)ceil_div_ll(kNumCu, RT);
            if (S > tiles) S = tiles;
        }
        pl.tiles_per_split = ceil_div(tiles, S);
        S = ceil_div(tiles, pl.tiles_per_split);
        if (RT * S < kNumCu) {
            const int r2 = rows_from(ceil_div_ll((long long)m * T * S, kNumCu), 64, 64, m);
            if (r2 < rows) rows = r2;
        }
        if (pl.tiles_per_split == 1 && rows <= 4 * 256) {
            // few rows per workgroup: latency mode, 16 rows per wave step, at most 4 steps per wave
            pl.row_mode = 1;
            rows = ceil_div(rows, 256) * 256;
        }
        pl.rows_per_wg = rows;
        return plan_finish(pl, m, n, q, batch, mu);
    }
    if ((mu <= 5 || (mu == 6 && batch <= 4)) && 2 * C >= 32 * UK) {
        // Narrow keys, rows at least half a tile wide: 32 lanes per row, conflict-free gathers.
        // (mu = 6 holds one input vector per pass only and re-reads the keys per vector: measured
        // faster than the generic kernel up to 4 input vectors, slower from 16 on.)
        // One tile per workgroup (wider rows are split, partial sums through the workspace); one
        // workgroup per CU (the tables fill the LDS: a second round of workgroups would only
        // build tables again), at least 32 rows (one step of the 16 waves) each.
        pl.kernel = KERNEL_WIDE;
        pl.threads = 1024;
        pl.chunks_per_tile = 32 * UK;
        pl.batch_tile = (128 * 1024) / (32 * UK * E * 4);
        pl.tiles_per_split = 1;
        const long long units = (long long)m * ceil_div(C, pl.chunks_per_tile) * ceil_div(batch, pl.batch_tile);
        const int rows = rows_from(ceil_div_ll(units, kNumCu), 32, 32, m);
        pl.rows_per_wg = rows > (1 << 20) ? (1 << 20) : rows;
        return plan_finish(pl, m, n, q, batch, mu);
    }
    return plan_generic(pl, m, n, q, batch, mu);
}

// The generic kernel: any mu, any q.
bool plan_generic(biq_plan& pl, int m, int n, int q, int batch, int mu) {
    const int UK = unit_keys(mu);
    const int C = ceil_div(n, mu);
    const int E = 1 << mu;
    pl = biq_plan{};
    pl.kernel = KERNEL_GENERIC;
    pl.batch_tile = batch >= 5 ? 8 : batch >= 3 ? 4 : batch;
    // one key unit's tables must fit the LDS budget (mu = 9, 10: 64 KiB per unit and input vector)
    while (pl.batch_tile > 1 && (long long)UK * E * pl.batch_tile * 4 > kLdsTableBudget) pl.batch_tile /= 2;
    // widest tile: G units, G a power of two, tables within the budget, no wider than the row
    int G = 1;
    while (G < 64 && (long long)(2 * G) * UK * E * pl.batch_tile * 4 <= kLdsTableBudget &&
           G * UK < C)
        G *= 2;
    pl.chunks_per_tile = G * UK;
    const int tiles = ceil_div(C, pl.chunks_per_tile);
    pl.threads = 512;
    const int groups = pl.threads / G;
    const int batch_tiles = ceil_div(batch, pl.batch_tile);
    // chunk splits
    const long long algo_bytes = (long long)q * m * ((n + 7) / 8) + 4ll * q * m + 4ll * n * batch +
                                 4ll * m * batch;
    long long max_splits = (2 * algo_bytes) / (4ll * m * batch);
    if (max_splits < 1) max_splits = 1;
    int splits = tiles < max_splits ? tiles : (int)max_splits;
    pl.tiles_per_split = ceil_div(tiles, splits);
    splits = ceil_div(tiles, pl.tiles_per_split);
    // rows per workgroup: aim at 2 workgroups per CU (every workgroup builds its own tables, and
    // with the tables filling most of the LDS only one is resident per CU anyway; measured: 8 per
    // CU was up to 2.7x slower on small-batch calls) while each keeps >= 1 row iteration
    const long long row_iters = ceil_div(m, groups);
    const long long want_wgs = 2ll * kNumCu;
    long long k = (row_iters * splits * batch_tiles) / want_wgs;
    if (k < 1) k = 1;
    if (k > 64) k = 64;
    if (pl.tiles_per_split > 1) {
        // row accumulators share the LDS with the tables
        const long long table_bytes = (long long)pl.chunks_per_tile * E * pl.batch_tile * 4;
        const long long fit = (kLdsPerCu - table_bytes) / (4ll * pl.batch_tile * groups);
        if (k > fit) k = fit < 1 ? 1 : fit;
    }
    pl.rows_per_wg = (int)(k * groups);
    return plan_finish(pl, m, n, q, batch, mu);
}

// The library's plan for a shape.  Should the tuned choice not pass plan_finish (a shape outside
// what its kernel's 32-bit offsets cover), the generic kernel takes the call; false if that
// fails too (the caller reports BIQ_EUNSUPPORTED, sizes read as 0).
bool plan_default(biq_plan& pl, int m, int n, int q, int batch, int mu, bool tables_given = false) {
    if (plan_tuned(pl, m, n, q, batch, mu, tables_given)) return true;
    return plan_generic(pl, m, n, q, batch, mu);
}

// Bytes of the prepared-input area at the start of the workspace (unpack-MFMA plans only): the
// B fragments, then one scaling exponent per padded input vector (two terms) or one count of
// non-zero terms per MFMA step and column tile (three).
size_t plan_xfrag_bytes(const biq_plan& pl) {
    const size_t b = (size_t)pl.batch_tiles * pl.chunk_splits * pl.tiles_per_split *
                     (size_t)unpack_group_pieces(pl.batch_tile, pl.input_terms) * 16;
    return (b + 255) & ~(size_t)255;
}
size_t plan_xf_bytes(const biq_plan& pl) {
    if (pl.kernel != KERNEL_UNPACK_MFMA) return 0;
    const size_t e = pl.input_terms == 2
                         ? (size_t)pl.batch_tiles * pl.batch_tile * sizeof(int)
                         : (size_t)pl.batch_tiles * pl.chunk_splits * pl.tiles_per_split * 16 * (pl.batch_tile / 32) *
                               sizeof(int);
    return plan_xfrag_bytes(pl) + ((e + 255) & ~(size_t)255);
}

size_t plan_workspace(const biq_plan& pl, int m, int batch) {
    return plan_xf_bytes(pl) +
           (pl.chunk_splits > 1 ? (size_t)pl.chunk_splits * batch * m * sizeof(float) : 0);
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Kernel parameters of a lookup-table plan.
void fill_query_params(QueryParams& qp, const biq_plan& pl, const uint8_t* K, const float* alpha, const float* X,
                       const float* LUT, float* out, int m, int n, int q, int batch, int mu) {
    qp.K = reinterpret_cast<const uint32_t*>(K);
    qp.alpha = alpha;
    qp.X = X;
    qp.LUT = LUT;
    qp.out = out;
    qp.m = m; qp.n = n; qp.q = q; qp.batch = batch;
    qp.stride_dw = (int)(biq_key_row_stride(n) / 4);
    qp.C = ceil_div(n, mu);
    qp.CT = pl.chunks_per_tile;
    qp.G = pl.chunks_per_tile / unit_keys(mu);
    qp.log2G = ilog2(qp.G);
    qp.tiles = ceil_div(qp.C, qp.CT);
    qp.tps = pl.tiles_per_split;
    qp.splits = pl.chunk_splits;
    qp.rows_per_wg = pl.rows_per_wg;
    qp.row_blocks = pl.row_blocks;
    qp.batch_tiles = pl.batch_tiles;
    qp.ntasks = pl.row_blocks * pl.chunk_splits * pl.batch_tiles;
    qp.tasks_per_xcd = ceil_div(qp.ntasks, kNumXcd);
    qp.row_mode = pl.row_mode;
    qp.xcd_skew = pl.xcd_skew;
    qp.table_fill = pl.table_fill;
}

// Plan of one problem of a grouped launch: mu = 8, at most 4 planes, a single dispatch without
// workspace (rows no wider than one tile), and only `cus` CUs' worth of workgroups, since the
// other problems of the group fill the rest of the chip.  false: the shape needs biq_gemm.
bool plan_grouped(biq_plan& pl, int& kind, int m, int n, int q, int batch, int mu, int cus) {
    if (mu != 8 || q > 4) return false;
    const int C = ceil_div(n, 8);
    pl = biq_plan{};
    pl.threads = 1024;
    pl.tiles_per_split = 1;
    pl.row_mode = 1;
    if (batch == 1 && C <= kGemvTileChunks) {
        kind = GROUP_GEMV8;
        pl.kernel = KERNEL_GEMV8;
        pl.chunks_per_tile = kGemvTileChunks;
        pl.batch_tile = 1;
        pl.rows_per_wg = rows_from(ceil_div_ll(m, cus), 8, 8, m);
    } else if (batch == 1 && C <= kGemvHalfTileChunks) {
        kind = GROUP_GEMV8H;
        pl.kernel = KERNEL_GEMV8H;
        pl.chunks_per_tile = kGemvHalfTileChunks;
        pl.batch_tile = 1;
        pl.rows_per_wg = rows_from(ceil_div_ll(m, cus), 4, 8, m);
    } else if (batch >= 2 && C <= kGemmHalfTileChunks) {
        kind = GROUP_GEMM8X2H;
        pl.kernel = KERNEL_GEMM8X2H;
        pl.chunks_per_tile = kGemmHalfTileChunks;
        pl.batch_tile = 2;
        pl.rows_per_wg = rows_from(ceil_div_ll((long long)m * ceil_div(batch, 2), cus), 8, 8, m);
    } else {
        return false;
    }
    return plan_finish(pl, m, n, q, batch, mu) && pl.chunk_splits == 1;
}

// Large-batch path: split X into 16-bit terms in MFMA operand order (workspace), contract, and
// sum the partial results when the key groups were split over workgroups.
biq_status run_unpack_mfma(const biq_plan& pl, const uint8_t* K, const float* alpha, const float* X,
                           float* Y, int m, int n, int q, int batch, void* workspace, hipStream_t s) {
    const int CT = pl.batch_tile / 32;
    const int groups = (int)((biq_key_row_stride(n) + kUnpackGroupBytes - 1) / kUnpackGroupBytes);
    const int steps = groups * 16;  // MFMA steps along a row
    mfma_u32x4* Xf = reinterpret_cast<mfma_u32x4*>(workspace);
    int* colexp = reinterpret_cast<int*>(reinterpret_cast<char*>(workspace) + plan_xfrag_bytes(pl));
    float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + plan_xf_bytes(pl));

    if (launch_xsplit(pl.input_terms, CT, X, Xf, colexp, n, batch, steps, pl.batch_tiles * pl.batch_tile, s) !=
        hipSuccess)
        return BIQ_EHIP;

    UnpackParams up{};
    up.K = K;
    up.alpha = alpha;
    up.Xf = Xf;
    up.colexp = colexp;
    up.nterms = colexp;   // the same area: exponents (two terms) or term counts (three)
    up.out = pl.chunk_splits > 1 ? partial : Y;
    up.m = m;
    up.batch = batch;
    up.stride_bytes = (uint32_t)biq_key_row_stride(n);
    up.groups = groups;
    up.gps = pl.tiles_per_split;
    up.splits = pl.chunk_splits;
    up.row_blocks = pl.row_blocks;
    up.col_groups = pl.batch_tiles;
    up.ntasks = pl.row_blocks * pl.chunk_splits * pl.batch_tiles;
    up.tasks_per_xcd = ceil_div(up.ntasks, kNumXcd);
    const int grid = up.tasks_per_xcd * kNumXcd;
    const int rpw = pl.rows_per_wg / ((4 / pl.wave_splits) * 32);
    const hipError_t e = launch_unpack(pl.input_terms, q, rpw, CT, pl.wave_splits, up, grid, pl.lds_bytes, s);
    if (e != hipSuccess) return BIQ_EHIP;
    if (pl.chunk_splits > 1) {
        const long long count = (long long)batch * m;
        if (launch_reduce_splits(partial, Y, count, pl.chunk_splits, s) != hipSuccess) return BIQ_EHIP;
    }
    return BIQ_OK;
}

biq_status run_query(bool fused, const uint8_t* K, const float* alpha, const float* X,
                     const float* LUT, float* Y, int m, int n, int q, int batch, int mu,
                     const biq_plan* user_plan, void* workspace, size_t workspace_bytes,
                     void* stream) {
    if (!shape_ok(m, n, q, batch, mu)) return BIQ_EINVAL;
    if (!K || !alpha || !Y || (fused ? !X : !LUT)) return BIQ_EINVAL;
    if (!aligned(K, 16) || !aligned(alpha, 4) || !aligned(Y, 4) || !aligned(fused ? X : LUT, 4))
        return BIQ_EINVAL;
    biq_plan pl;
    if (user_plan) {
        pl = *user_plan;
        if (!plan_finish(pl, m, n, q, batch, mu)) return BIQ_EINVAL;
    } else {
        if (!plan_default(pl, m, n, q, batch, mu, !fused)) return BIQ_EUNSUPPORTED;
    }
    if (pl.kernel == KERNEL_UNPACK_MFMA && !fused) return BIQ_EINVAL;  // that kernel reads X, not tables
    if (pl.table_fill != 0 && !fused) return BIQ_EINVAL;               // a build method needs tables to build
    const size_t need = plan_workspace(pl, m, batch);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return BIQ_EWORKSPACE;
        if (!aligned(workspace, 16)) return BIQ_EINVAL;
    }
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (pl.kernel == KERNEL_UNPACK_MFMA)
        return run_unpack_mfma(pl, K, alpha, X, Y, m, n, q, batch, workspace, s);

    QueryParams qp{};
    fill_query_params(qp, pl, K, alpha, X, LUT, pl.chunk_splits > 1 ? reinterpret_cast<float*>(workspace) : Y, m, n, q,
                      batch, mu);
#ifdef BIQ_TRACE
    if (fused) qp.LUT = reinterpret_cast<const float*>(workspace);  // time stamps of a trace build go here
#endif
    const int grid = qp.tasks_per_xcd * kNumXcd;

    hipError_t e;
    if (pl.kernel == KERNEL_GEMV8) e = launch_gemv8(fused, q, qp, grid, pl.threads, pl.lds_bytes, s);
    else if (pl.kernel == KERNEL_GEMV8H) e = launch_gemv8h(fused, q, qp, grid, pl.threads, pl.lds_bytes, s);
    else if (pl.kernel == KERNEL_WIDE) e = launch_wide(fused, mu, qp, grid, pl.threads, pl.lds_bytes, s);
    else if (pl.kernel == KERNEL_GEMM8X2H) e = launch_gemm8x2h(fused, q, qp, grid, pl.threads, pl.lds_bytes, s);
    else if (pl.kernel == KERNEL_GEMM8X2) e = launch_gemm8x2(fused, q, qp, grid, pl.threads, pl.lds_bytes, s);
    else e = launch_query_generic(fused, mu, pl.batch_tile, qp, grid, pl.threads, pl.lds_bytes, s);
    if (e != hipSuccess) return BIQ_EHIP;
    if (pl.chunk_splits > 1) {
        const long long count = (long long)batch * m;
        if (launch_reduce_splits(reinterpret_cast<const float*>(workspace), Y, count, pl.chunk_splits, s) !=
            hipSuccess)
            return BIQ_EHIP;
    }
    return BIQ_OK;
}

template <typename KEY>
biq_status unpack_keys_any(const uint8_t* K, KEY* keys, int m, int n, int q, int mu, void* stream) {
    if (!shape_ok(m, n, q, 1, mu) || !K || !keys) return BIQ_EINVAL;
    if (!aligned(K, 16) || !aligned(keys, sizeof(KEY))) return BIQ_EINVAL;
    if (mu > 8 * (int)sizeof(KEY)) return BIQ_EUNSUPPORTED;  // key does not fit the output type
    const long long key_rows = (long long)q * m;
    const int stride_dw = (int)(biq_key_row_stride(n) / 4);
    const int C = ceil_div(n, mu);
    const hipError_t e = launch_unpack_keys(mu, sizeof(KEY) == 2, reinterpret_cast<const uint32_t*>(K), keys,
                                            key_rows, C, stride_dw, reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? BIQ_OK : BIQ_EHIP;
}

// ---- the allocation-free entry point's scratch buffer -------------------------------------
// Workspace of biq_gemm_noalloc: device memory that belongs to the library's code object, one
// copy per GPU, held until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; the device address is looked up once per device and kept.
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_addr[kMaxDevices];  // device address of `scratch` on each device, 0 = not looked up yet

// Device address of the current device's copy of `scratch`.
hipError_t scratch_address(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = __atomic_load_n(&g_scratch_addr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        __atomic_store_n(&g_scratch_addr[dev], p, __ATOMIC_RELEASE);  // racing first calls store the same value
    }
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" {

const char* biq_status_str(biq_status status) {
    switch (status) {
        case BIQ_OK: return "ok";
        case BIQ_EINVAL: return "invalid argument";
        case BIQ_EUNSUPPORTED: return "unsupported request";
        case BIQ_EWORKSPACE: return "workspace too small";
        case BIQ_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

int biq_version(void) { return 100; }

size_t biq_key_row_stride(int n) { return n < 1 ? 0 : (size_t)((n + 127) / 128) * 16; }

size_t biq_packed_bytes(int m, int n, int q) {
    if (m < 1 || n < 1 || q < 1) return 0;
    return (size_t)q * m * biq_key_row_stride(n);
}

size_t biq_num_chunks(int n, int mu) {
    if (n < 1 || mu < 1 || mu > kMaxMu) return 0;
    return (size_t)((n + mu - 1) / mu);
}

size_t biq_lut_bytes(int n, int batch, int mu) {
    if (n < 1 || batch < 1 || mu < 1 || mu > kMaxMu) return 0;
    return biq_num_chunks(n, mu) * ((size_t)1 << mu) * batch * sizeof(float);
}

biq_status biq_plan_get(int m, int n, int q, int batch, int mu, biq_plan* plan) {
    if (!plan || !shape_ok(m, n, q, batch, mu)) return BIQ_EINVAL;
    return plan_default(*plan, m, n, q, batch, mu) ? BIQ_OK : BIQ_EUNSUPPORTED;
}

biq_status biq_plan_get_lut(int m, int n, int q, int batch, int mu, biq_plan* plan) {
    if (!plan || !shape_ok(m, n, q, batch, mu)) return BIQ_EINVAL;
    return plan_default(*plan, m, n, q, batch, mu, true) ? BIQ_OK : BIQ_EUNSUPPORTED;
}

biq_status biq_plan_get_mfma(int m, int n, int q, int batch, int mu, int input_terms, biq_plan* plan) {
    if (!plan || !shape_ok(m, n, q, batch, mu)) return BIQ_EINVAL;
    if (input_terms != 2 && input_terms != 3) return BIQ_EINVAL;
    if (q > 4) return BIQ_EUNSUPPORTED;
    return plan_unpack(*plan, m, n, q, batch, mu, input_terms) ? BIQ_OK : BIQ_EUNSUPPORTED;
}

biq_status biq_plan_check(int m, int n, int q, int batch, int mu, biq_plan* plan) {
    if (!plan || !shape_ok(m, n, q, batch, mu)) return BIQ_EINVAL;
    return plan_finish(*plan, m, n, q, batch, mu) ? BIQ_OK : BIQ_EINVAL;
}

size_t biq_plan_workspace_bytes(const biq_plan* plan, int m, int batch) {
    if (!plan || m < 1 || batch < 1) return 0;
    return plan_workspace(*plan, m, batch);
}

size_t biq_workspace_bytes(int m, int n, int q, int batch, int mu) {
    if (!shape_ok(m, n, q, batch, mu)) return 0;
    // the larger of what biq_gemm's and biq_query's default plans need
    biq_plan pl;
    if (!plan_default(pl, m, n, q, batch, mu, false)) return 0;
    const size_t a = plan_workspace(pl, m, batch);
    if (!plan_default(pl, m, n, q, batch, mu, true)) return 0;
    const size_t b = plan_workspace(pl, m, batch);
    return a > b ? a : b;
}

const char* biq_kernel_name(int kernel) {
    switch (kernel) {
        case KERNEL_GENERIC: return "query_generic";
        case KERNEL_GEMV8: return "gemv8";
        case KERNEL_GEMM8X2: return "gemm8x2";
        case KERNEL_UNPACK_MFMA: return "unpack_mfma";
        case KERNEL_GEMV8H: return "gemv8_half";
        case KERNEL_GEMM8X2H: return "gemm8x2_half";
        case KERNEL_WIDE: return "query_wide";
    }
    return "unknown";
}

biq_status biq_pack(const int8_t* B, uint8_t* K, int m, int n, int q, int mu, void* stream) {
    if (!shape_ok(m, n, q, 1, mu) || !B || !K) return BIQ_EINVAL;
    if (!aligned(K, 16)) return BIQ_EINVAL;
    const long long key_rows = (long long)q * m;
    const int stride_dw = (int)(biq_key_row_stride(n) / 4);
    const long long total = key_rows * stride_dw;
    if (total > (1ll << 38)) return BIQ_EUNSUPPORTED;
    const hipError_t e = launch_pack(B, reinterpret_cast<uint32_t*>(K), key_rows, n, stride_dw,
                                     reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? BIQ_OK : BIQ_EHIP;
}

biq_status biq_quantize(const float* W, uint8_t* K, float* alpha, int m, int n, int q, void* stream) {
    if (!shape_ok(m, n, q, 1, 8) || !W || !K || !alpha) return BIQ_EINVAL;
    if (!aligned(K, 16) || !aligned(W, 4) || !aligned(alpha, 4)) return BIQ_EINVAL;
    if (n > kQuantMaxN) return BIQ_EUNSUPPORTED;  // a row's residual is kept in the registers of one workgroup
    const int stride_dw = (int)(biq_key_row_stride(n) / 4);
    const hipError_t e = launch_quantize(W, reinterpret_cast<uint32_t*>(K), alpha, m, n, q, stride_dw,
                                         reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? BIQ_OK : BIQ_EHIP;
}

biq_status biq_unpack_keys(const uint8_t* K, uint8_t* keys, int m, int n, int q, int mu, void* stream) {
    return unpack_keys_any<uint8_t>(K, keys, m, n, q, mu, stream);
}

biq_status biq_unpack_keys16(const uint8_t* K, uint16_t* keys, int m, int n, int q, int mu, void* stream) {
    return unpack_keys_any<uint16_t>(K, keys, m, n, q, mu, stream);
}

biq_status biq_build_lut(const float* X, float* LUT, int n, int batch, int mu, void* stream) {
    if (!shape_ok(1, n, 1, batch, mu) || !X || !LUT) return BIQ_EINVAL;
    if (!aligned(X, 4) || !aligned(LUT, 4)) return BIQ_EINVAL;
    const hipError_t e = launch_build_lut(mu, X, LUT, n, batch, ceil_div(n, mu),
                                          reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? BIQ_OK : BIQ_EHIP;
}

biq_status biq_query(const uint8_t* K, const float* alpha, const float* LUT, float* Y, int m, int n,
                     int q, int batch, int mu, void* workspace, size_t workspace_bytes, void* stream) {
    return run_query(false, K, alpha, nullptr, LUT, Y, m, n, q, batch, mu, nullptr, workspace,
                     workspace_bytes, stream);
}

biq_status biq_gemm(const uint8_t* K, const float* alpha, const float* X, float* Y, int m, int n,
                    int q, int batch, int mu, void* workspace, size_t workspace_bytes, void* stream) {
    return run_query(true, K, alpha, X, nullptr, Y, m, n, q, batch, mu, nullptr, workspace,
                     workspace_bytes, stream);
}

biq_status biq_gemm_ex(const uint8_t* K, const float* alpha, const float* X, float* Y, int m, int n,
                       int q, int batch, int mu, const biq_plan* plan, void* workspace,
                       size_t workspace_bytes, void* stream) {
    if (!plan) return BIQ_EINVAL;
    return run_query(true, K, alpha, X, nullptr, Y, m, n, q, batch, mu, plan, workspace,
                     workspace_bytes, stream);
}

biq_status biq_init(void) {
    void* p = nullptr;
    return scratch_address(&p) == hipSuccess ? BIQ_OK : BIQ_EHIP;
}

size_t biq_noalloc_scratch_bytes(void) { return kScratchBytes; }

biq_status biq_gemm_noalloc(const uint8_t* K, const float* alpha, const float* X, float* Y, int m, int n,
                            int q, int batch, int mu, void* stream) {
    if (!shape_ok(m, n, q, batch, mu)) return BIQ_EINVAL;
    biq_plan pl;
    if (!plan_default(pl, m, n, q, batch, mu, false)) return BIQ_EUNSUPPORTED;
    const size_t need = plan_workspace(pl, m, batch);
    if (need > kScratchBytes) return BIQ_EWORKSPACE;  // beyond the fixed buffer: use biq_gemm with a workspace
    void* ws = nullptr;
    if (need > 0 && scratch_address(&ws) != hipSuccess) return BIQ_EHIP;
    // Every kernel writes the part of the workspace it later reads (split input, partial sums) in
    // full before reading it, so what an earlier call left there does not matter and nothing is
    // cleared.
    return run_query(true, K, alpha, X, nullptr, Y, m, n, q, batch, mu, &pl, ws, need, stream);
}

biq_status biq_gemm_grouped(const biq_problem* problems, int count, int mu, void* stream) {
    if (!problems || count < 1) return BIQ_EINVAL;
    for (int i = 0; i < count; ++i) {
        const biq_problem& pr = problems[i];
        if (!shape_ok(pr.m, pr.n, pr.q, pr.batch, mu)) return BIQ_EINVAL;
        if (!pr.K || !pr.alpha || !pr.X || !pr.Y) return BIQ_EINVAL;
        if (!aligned(pr.K, 16) || !aligned(pr.alpha, 4) || !aligned(pr.X, 4) || !aligned(pr.Y, 4)) return BIQ_EINVAL;
    }
    // every problem gets its share of the CUs; all are planned before anything is launched
    const int cus = count >= kNumCu ? 1 : kNumCu / count;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // first pass (launch = false) only checks that every problem has a single-dispatch plan
    for (int pass = 0; pass < 2; ++pass) {
        int i = 0;
        while (i < count) {
            GroupParams g{};
            int kind = -1, q = 0, lds = 0, grid = 0;
            while (i < count && g.count < kGroupMax) {
                const biq_problem& pr = problems[i];
                biq_plan pl;
                int k = -1;
                if (!plan_grouped(pl, k, pr.m, pr.n, pr.q, pr.batch, mu, cus)) return BIQ_EUNSUPPORTED;
                if (g.count > 0 && (k != kind || pr.q != q)) break;  // next dispatch
                kind = k;
                q = pr.q;
                if (pl.lds_bytes > lds) lds = pl.lds_bytes;
                QueryParams& qp = g.p[g.count];
                fill_query_params(qp, pl, pr.K, pr.alpha, pr.X, nullptr, pr.Y, pr.m, pr.n, pr.q, pr.batch, mu);
                g.first_wg[g.count] = grid;
                grid += qp.tasks_per_xcd * kNumXcd;
                ++g.count;
                ++i;
            }
            g.first_wg[g.count] = grid;
            if (pass == 1 && launch_grouped(kind, q, g, grid, lds, s) != hipSuccess) return BIQ_EHIP;
        }
    }
    return BIQ_OK;
}

biq_status biq_lstm_cell(const uint8_t* K, const float* alpha, const float* bias, const float* X,
                         const float* C_prev, float* H_out, float* C_out, int hidden, int n, int q, int batch,
                         int mu, void* stream) {
    if (hidden < 1 || hidden > (1 << 28)) return BIQ_EINVAL;
    const int m = 4 * hidden;
    if (!shape_ok(m, n, q, batch, mu)) return BIQ_EINVAL;
    if (!K || !alpha || !bias || !X || !C_prev || !H_out || !C_out) return BIQ_EINVAL;
    if (!aligned(K, 16) || !aligned(alpha, 4) || !aligned(bias, 4) || !aligned(X, 4) || !aligned(C_prev, 4) ||
        !aligned(H_out, 4) || !aligned(C_out, 4))
        return BIQ_EINVAL;
    if (mu != 8 || q > 4) return BIQ_EUNSUPPORTED;
    const int C = ceil_div(n, 8);
    biq_plan pl{};
    pl.threads = 1024;
    pl.tiles_per_split = 1;
    pl.row_mode = 1;
    int units;  // hidden units per workgroup: one workgroup per CU if the units allow it
    if (batch == 1 && C <= kGemvHalfTileChunks) {
        pl.kernel = KERNEL_GEMV8H;
        pl.chunks_per_tile = kGemvHalfTileChunks;
        pl.batch_tile = 1;
        units = ceil_div(hidden, kNumCu);
    } else if (batch >= 2 && C <= kGemmHalfTileChunks) {
        pl.kernel = KERNEL_GEMM8X2H;
        pl.chunks_per_tile = kGemmHalfTileChunks;
        pl.batch_tile = 2;
        units = 2 * (int)ceil_div_ll((long long)hidden * ceil_div(batch, 2), 2ll * kNumCu);  // two per wave step
    } else {
        return BIQ_EUNSUPPORTED;  // rows wider than one half-table tile: biq_gemm, then the cell update by the caller
    }
    if (units < 1) units = 1;
    pl.rows_per_wg = 4 * units;
    if (!plan_finish(pl, m, n, q, batch, mu) || pl.chunk_splits != 1) return BIQ_EUNSUPPORTED;
    QueryParams qp{};
    fill_query_params(qp, pl, K, alpha, X, nullptr, H_out, m, n, q, batch, mu);
    // workgroups are laid out over hidden units, not gate rows
    qp.row_blocks = ceil_div(hidden, units);
    qp.ntasks = qp.row_blocks * qp.batch_tiles;
    qp.tasks_per_xcd = ceil_div(qp.ntasks, kNumXcd);
    qp.bias = bias;
    qp.c_prev = C_prev;
    qp.c_out = C_out;
    qp.hidden = hidden;
    const int grid = qp.tasks_per_xcd * kNumXcd;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const hipError_t e = pl.kernel == KERNEL_GEMV8H ? launch_lstm8h(q, qp, grid, pl.threads, pl.lds_bytes, s)
                                                    : launch_lstm8x2h(q, qp, grid, pl.threads, pl.lds_bytes, s);
    return e == hipSuccess ? BIQ_OK : BIQ_EHIP;
}

}  // extern "C"
