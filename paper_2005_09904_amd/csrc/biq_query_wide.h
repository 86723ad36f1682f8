// LUT query for mu <= 6: conflict-free gathers for narrow keys.
//
// The generic kernel (biq_kernels.h) keeps tables as [chunk][key][batch tile] and gathers with
// wide reads, which collide on LDS banks at random (keys decide the bank).  Here the 32 lanes
// of an LDS half-wave all work on the SAME row, lane L on the L-th key unit (a run of whole
// dwords holding UK whole keys, see biq_common.h), and the table entry of (key position s in the
// unit, key k, input vector v, unit L) lives at byte
//       k * (UK/2 * BT * 256) + ((s >> 1) * BT + v) * 256 + (s & 1) * 128 + L * 4
// (the key in the high bits: everything else of a lookup's address is a per-lane constant plus an
// immediate offset of the read), so the bank is L whatever the keys are: every ds_read_b32 of a half-wave is conflict-free
// (the arrangement idea of Fig. 8 with the lane's unit as the interleaving index).  A tile is
// 32 units = 32*UK chunks and fills 128 KiB with BT = 2 (mu 4), 1 (mu 5, 6) or 4 (mu <= 3)
// input vectors.  Per key: one bit-field extract, one shift-add for the address, BT reads.
// One tile per workgroup; a row wider than a tile is split over workgroups (partial sums).
#pragma once

#include "biq_gemv8h.h"

namespace biq {

template <int MU> struct WideGeom {
    static constexpr int E = 1 << MU;
    static constexpr int UD = KeyUnit<MU>::UD, UK = KeyUnit<MU>::UK;
    static constexpr int CT = 32 * UK;                         // chunks per tile
    static constexpr int BT = (128 * 1024) / (CT * E * 4);     // input vectors per pass
    static constexpr int LDS_BYTES = CT * E * BT * 4;          // 131072
    static_assert(BT >= 1 && LDS_BYTES == 128 * 1024, "tile must fill 128 KiB");
};

template <int MU, int BT>
__device__ __forceinline__ uint32_t wide_slot(int s, int key, int v, int L) {
    constexpr int KB = KeyUnit<MU>::UK / 2 * BT * 256;   // bytes per key value
    return (uint32_t)(key * KB + ((s >> 1) * BT + v) * 256 + (s & 1) * 128 + L * 4);
}

// Lookups of key positions T .. UK-1 of one unit: acc[v] += table[s][key_s][v][L].  lane_even /
// lane_odd = L * 4 (+ 128): the per-lane part of the address for even / odd key positions; the
// rest, ((s >> 1) * BT + v) * 256, is an immediate offset of the read.
template <int MU, int BT, int T>
__device__ __forceinline__ void wide_lookup(const uint32_t (&w)[KeyUnit<MU>::UD], uint32_t lane_even,
                                            uint32_t lane_odd, float (&acc)[BT]) {
    if constexpr (T < KeyUnit<MU>::UK) {
        constexpr uint32_t KB = (uint32_t)(KeyUnit<MU>::UK / 2 * BT * 256);
        const uint32_t key = unit_key<MU, T>(w);
        const uint32_t addr = key * KB + ((T & 1) ? lane_odd : lane_even);
#pragma unroll
        for (int v = 0; v < BT; ++v) acc[v] += lds_read_abs(addr + (uint32_t)(((T >> 1) * BT + v) * 256));
        wide_lookup<MU, BT, T + 1>(w, lane_even, lane_odd, acc);
    }
}

template <int MU, bool FUSED>
__global__ __launch_bounds__(1024) void query_wide_kernel(const QueryParams p) {
    using G = WideGeom<MU>;
    constexpr int E = G::E, UD = G::UD, UK = G::UK, CT = G::CT, BT = G::BT;
    extern __shared__ __align__(16) float lds[];
    char* const lds_bytes = reinterpret_cast<char*>(lds);

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
    const int tile = sp;  // one tile per split
    const int c0 = tile * CT;

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    // lookups address LDS absolutely (see lds_read_abs)
    if (lds_address_of(lds) != 0u) return;

    // ---- tables of chunks [c0, c0 + CT) for input vectors b0 .. b0 + BT - 1 ----------------------
    if constexpr (FUSED) {
        constexpr int HG = (MU > 4) ? (1 << (MU - 4)) : 1;   // groups of 16 keys per table
        constexpr int LN = (MU > 4) ? 16 : E;                // keys per group
        for (int job = tid; job < CT * BT * HG; job += nthreads) {
            const int L = job & 31;                          // consecutive threads: consecutive banks
            int r = job >> 5;
            const int s = r % UK; r /= UK;
            const int v = r % BT;
            const int h = r / BT;
            if (b0 + v >= p.batch) continue;   // no such input vector: its entries are read but never used
            float ent[16];
            chunk_table16<MU>(p.X, p.n, p.batch, b0 + v, c0 + L * UK + s, (uint32_t)h, ent);
            constexpr int KB = UK / 2 * BT * 256;
            char* dst = lds_bytes + wide_slot<MU, BT>(s, h * 16, v, L);
#pragma unroll
            for (int l = 0; l < LN; ++l) *reinterpret_cast<float*>(dst + l * KB) = ent[l];
        }
    } else {
        for (int i = tid; i < CT * E * BT; i += nthreads) {
            const int L = i & 31;
            int r = i >> 5;
            const int v = r % BT; r /= BT;
            const int key = r % E;
            const int s = r / E;
            const int c = c0 + L * UK + s;
            float val = 0.0f;
            if (c < p.C && b0 + v < p.batch) val = p.LUT[((size_t)c * E + key) * p.batch + b0 + v];
            *reinterpret_cast<float*>(lds_bytes + wide_slot<MU, BT>(s, key, v, L)) = val;
        }
    }
    __syncthreads();

    // ---- rows: a half-wave per row, lane L on unit L; (row step, plane) pairs walked with the
    // next pair's keys already requested ---------------------------------------------------------
    const int lane = tid & 63;
    const int L = lane & 31;
    const int half = lane >> 5;
    const int wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    const uint32_t lane_even = (uint32_t)(L * 4);
    const uint32_t lane_odd = lane_even + 128u;
    const int dw0 = tile * 32 * UD + L * UD;     // this lane's unit inside a packed row
    const int nrows = r1 - r0;
    const int nsteps = (nrows + 1) >> 1;         // steps of 2 rows per wave

    auto load_pair = [&](int step, int plane, uint32_t (&w)[UD], float& al) {
        const int row = 2 * step + half;
#pragma unroll
        for (int d = 0; d < UD; ++d) w[d] = 0u;
        al = 0.0f;
        if (step < nsteps && row < nrows) {
            const size_t kr = (size_t)plane * p.m + r0 + row;
            load_unit<UD>(p.K + kr * p.stride_dw, dw0, p.stride_dw, w);
            al = p.alpha[kr];
        }
    };

    uint32_t w[UD], wn[UD];
    float al, aln;
    int step = wave, plane = 0;
    load_pair(step, plane, w, al);
    float y[BT];
#pragma unroll
    for (int v = 0; v < BT; ++v) y[v] = 0.0f;
    while (step < nsteps) {
        int nstep = step, nplane = plane + 1;
        if (nplane == p.q) { nplane = 0; nstep = step + nwaves; }
        load_pair(nstep, nplane, wn, aln);
        float acc[BT];
#pragma unroll
        for (int v = 0; v < BT; ++v) acc[v] = 0.0f;
        wide_lookup<MU, BT, 0>(w, lane_even, lane_odd, acc);
#pragma unroll
        for (int v = 0; v < BT; ++v) y[v] = fmaf(al, acc[v], y[v]);
        if (nplane == 0) {
            // last plane of this row step: sum over the 32 lanes of the half-wave and store
            const int row = 2 * step + half;
#pragma unroll
            for (int v = 0; v < BT; ++v) {
                float t = reduce16(y[v]);
                t += __shfl_xor(t, 16, 64);
                if (L == 0 && row < nrows && b0 + v < p.batch)
                    p.out[((size_t)sp * p.batch + b0 + v) * p.m + r0 + row] = t;
                y[v] = 0.0f;
            }
        }
#pragma unroll
        for (int d = 0; d < UD; ++d) w[d] = wn[d];
        al = aln;
        step = nstep;
        plane = nplane;
    }
}

}  // namespace biq
