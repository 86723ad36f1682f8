/*
 * biq.h - C ABI of libbiq: the BiQGEMM lookup-table matrix multiply
 * (arxiv 2005.09904) as hand-written HIP kernels for AMD gfx950 (MI355X).
 *
 *     Y = sum_{i=1..q} alpha_i o (B_i . X)            (paper Eq. 2)
 *
 * with B_i in {-1,+1}^(m x n) (binary-coding quantised weights, Sec. II-B),
 * X real n x batch, alpha_i in R^m.  The product is never formed from unpacked
 * weights: each row's signs are packed into mu-bit keys (Sec. III-B), every
 * mu-element chunk of every input vector gets a table of all 2^mu signed
 * partial sums q = M_mu . x (Sec. III-B, Algorithm 1), and the keys index
 * those tables (Algorithm 2).
 *
 * Notation (the paper's): m output size, n input size, batch = b, q = number of
 * bit-planes (beta_w), mu = LUT-unit, C = ceil(n / mu) chunks per row.
 *
 * General rules
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or keeps device memory (workspace is passed in).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; calls return without synchronising.
 *   - Output buffers are overwritten, never accumulated into.  Buffers must
 *     not overlap.
 *   - 1 <= mu <= 10, q >= 1, m, n, batch >= 1; m*q and n below 2^31.  Any
 *     m, n, batch is accepted: there is no "multiple of the tile" requirement.
 *   - Errors are returned as a negative biq_status; nothing aborts or throws
 *     across this boundary.  On an error no kernel has been launched unless
 *     the status is BIQ_EHIP.
 *   - Inputs are assumed finite; behaviour on NaN/Inf is unspecified.
 *   - Threads: every function may be called from several host threads at once.  The library
 *     keeps no state between calls apart from per-device one-time set-up (the opt-in to large
 *     LDS per kernel, the address of the biq_gemm_noalloc buffer), which is idempotent: two
 *     threads racing through it do the same work twice and store the same values.  Calls use
 *     the calling thread's current device.  What the caller must keep apart is the memory:
 *     two calls whose workspace or output buffers overlap (and any two biq_gemm_noalloc calls
 *     on one GPU) must not be in flight at the same time, whatever threads or streams issue them.
 *   - Beyond the paper's problem statement (pack, build tables, query; m, n, q, batch, mu):
 *     biq_query takes a workspace like biq_gemm (wide rows are split over workgroups in both),
 *     mu goes up to 10 (keys of 9 and 10 bits are served by the generic kernel;
 *     biq_unpack_keys16 returns them), and biq_plan_*, biq_gemm_ex, biq_gemm_grouped,
 *     biq_lstm_cell, biq_quantize and biq_gemm_noalloc are additions.
 *
 * Data layouts
 *   B      int8   [q][m][n]            +1 / -1 (bit = (B > 0); other values are
 *                                      not checked on the device)
 *   K      uint8  [q][m][stride]       packed signs: bit (j mod 8) of byte
 *                                      (j / 8) of a row is 1 iff B[.., j] = +1
 *                                      (element j <-> bit j, LSB first, as in
 *                                      Algorithms 1 and 3); stride =
 *                                      biq_key_row_stride(n) = ceil(n/128)*16
 *                                      bytes, padding bits are 0.  The key of
 *                                      chunk c for LUT-unit mu is the bit field
 *                                      [mu*c, mu*c + mu) of the row, so one
 *                                      packed matrix serves every mu; for
 *                                      mu = 8 byte c IS key c.  Planes are
 *                                      concatenated vertically (Sec. III-B).
 *   alpha  float  [q][m]               one scale per output row per plane
 *   X      float  [batch][n]           each input vector contiguous
 *   LUT    float  [C][2^mu][batch]     entries of one key adjacent across the
 *                                      batch (the arrangement of Fig. 8)
 *   Y      float  [batch][m]
 *   K must be 16-byte aligned; float buffers 4-byte aligned.
 */
#ifndef BIQ_H_
#define BIQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BIQ_OK = 0,
    BIQ_EINVAL = -1,       /* null pointer, size out of range, misaligned buffer      */
    BIQ_EUNSUPPORTED = -2, /* valid request this build cannot serve                   */
    BIQ_EWORKSPACE = -3,   /* workspace smaller than biq_workspace_bytes()            */
    BIQ_EHIP = -4          /* the HIP runtime reported an error (launch, attribute)   */
} biq_status;

/* Static, NUL-terminated description of a status; never freed. */
const char* biq_status_str(biq_status status);

/* Library version as major*10000 + minor*100 + patch. */
int biq_version(void);

/* ---- sizes (pure host arithmetic, no device access; 0 on invalid arguments) ---- */

/* Bytes between packed rows: ceil(n/128)*16. */
size_t biq_key_row_stride(int n);
/* Bytes of the packed matrix K: q*m*stride.  With n a multiple of 128 this is
 * q*m*n/8, the weight footprint of Table II. */
size_t biq_packed_bytes(int m, int n, int q);
/* C = ceil(n/mu). */
size_t biq_num_chunks(int n, int mu);
/* Bytes of the full table set: C * 2^mu * batch * 4 (Eq. 6 counts its entries). */
size_t biq_lut_bytes(int n, int batch, int mu);
/* Workspace biq_gemm / biq_query need for this shape (may be 0). */
size_t biq_workspace_bytes(int m, int n, int q, int batch, int mu);

/*
 * How a call is mapped on the GPU.  Algorithm 2 leaves tile width/height free
 * (Sec. III-B); biq_plan_get reports the choice the library makes, biq_gemm_ex
 * accepts a caller-supplied one (for tuning sweeps).
 */
typedef struct {
    int kernel;          /* kernel family (biq_kernel_name): 0 query_generic (any mu, q),
                            1 gemv8 (mu 8, batch 1, q <= 4), 2 gemm8x2 (mu 8, q <= 4, two input
                            vectors per pass), 3 unpack_mfma (any mu, q <= 4, matrix cores),
                            4 gemv8_half / 5 gemm8x2_half (as 1 / 2 with half tables: 256 /
                            128 chunks per tile, row_mode 1 and tiles_per_split 1 only),
                            6 query_wide (mu <= 6, any q: 32 key units per tile, batch_tile 4 / 2 /
                            1 for mu <= 3 / 4 / 5-6, tiles_per_split 1)                      */
    int threads;         /* threads per workgroup                                         */
    int chunks_per_tile; /* chunks whose tables one workgroup holds in LDS at a time
                            (unpack_mfma kernel: 32, the key bytes of a row per key group;
                            "tile" below then means key group)                            */
    int batch_tile;      /* input vectors served by one workgroup                         */
    int chunk_splits;    /* workgroups sharing one row block along n (partials if > 1)    */
    int tiles_per_split; /* LUT tiles each of those workgroups walks through              */
    int rows_per_wg;     /* output rows per workgroup                                     */
    int row_blocks;      /* ceil(m / rows_per_wg)                                         */
    int batch_tiles;     /* ceil(batch / batch_tile)                                      */
    int lds_bytes;       /* dynamic LDS per workgroup                                     */
    int row_mode;        /* mu = 8 kernels: 0 = a wave works through blocks of 64 rows
                            (throughput), 1 = one step of rows per wave at a time, keys
                            requested before the tables are built (latency; needs
                            tiles_per_split = 1), 2 = gemv8_half only: one row per wave at a
                            time, its 64 lanes on the row's 64 key dwords (few rows per
                            workgroup)                                                     */
    int xcd_skew;        /* GEMV kernel, row_mode 0, no chunk split, row_blocks a multiple of 8:
                            workgroups on even XCDs take rows_per_wg + xcd_skew rows, those on
                            odd XCDs rows_per_wg - xcd_skew (odd XCDs stream slower)        */
    int wave_splits;     /* unpack_mfma kernel: 1, 2 or 4 groups of waves inside a workgroup, each
                            contracting its own part of the workgroup's key groups; their partial
                            sums are added in LDS (0 is read as 1).  rows_per_wg is then
                            (4 / wave_splits) * 32 * r with r row tiles per wave and plane,
                            r in {1, 2, 4}, q * r <= 4                                       */
    int table_fill;      /* GEMV kernel, fused tables: 0 = every entry from the chunk's pair sums (a direct,
                            GEMM-like fill), 1 = the order of Algorithm 1: a block's first entry, then
                            each further entry of the lower half from an earlier one by adding 2 x_t,
                            the upper half by negation.  Same tables up to rounding; kept selectable
                            so that the two build methods Sec. III-B weighs can be timed against each
                            other (the default, 0, is the faster one here)                       */
    int input_terms;     /* unpack_mfma kernel: 16-bit terms every fp32 input is split into for the matrix
                            cores.  3 (0 is read as 3; what the library chooses): three bf16 terms, an
                            exact split - the result is that of an fp32 evaluation of Eq. 2 up to the
                            order of the additions; terms that are zero for all input vectors of a
                            workgroup over a wave's whole part of the row are skipped, so inputs holding
                            fp16 (bf16) values cost two thirds (one third) of the matrix instructions,
                            with the same bits out.  2: every input vector scaled by a power of two (its
                            largest magnitude in [2^14, 2^15)) and split into two fp16 terms rounded to
                            nearest, 22 significand bits: a third fewer matrix instructions for an input
                            rounding of 2^-22 relative per element (2^-39 of the vector's largest
                            magnitude where the second term is subnormal), the scaling undone on
                            output; a second term that is zero for all input vectors of a workgroup
                            (inputs holding fp16 values) is skipped; an input vector holding Inf or NaN gives non-finite outputs for that
                            vector.  Only on request                                              */
    int reserved[1];
} biq_plan;

biq_status biq_plan_get(int m, int n, int q, int batch, int mu, biq_plan* plan);
/* The library's choice among the lookup-table kernels only (Algorithm 2 proper): what biq_query
 * runs, and what biq_gemm runs below the batch size from which it switches to unpacking the
 * keys into the matrix cores (the large-batch regime of Sec. IV-B where a plain GEMM on
 * unpacked weights wins). */
biq_status biq_plan_get_lut(int m, int n, int q, int batch, int mu, biq_plan* plan);
/* The library's mapping of the unpack_mfma kernel for a shape (q <= 4, else BIQ_EUNSUPPORTED),
 * whichever side of the crossover the shape is on, for input_terms = 3 or 2 (see biq_plan):
 * how a caller asks for the two-term variant, or times the matrix-core path below the
 * crossover.  For biq_gemm_ex. */
biq_status biq_plan_get_mfma(int m, int n, int q, int batch, int mu, int input_terms, biq_plan* plan);
/* Validates a caller-filled plan (kernel, threads, chunks_per_tile, batch_tile,
 * tiles_per_split, rows_per_wg) against the shape and the device limits and fills in the
 * derived fields (chunk_splits, row_blocks, batch_tiles, lds_bytes). */
biq_status biq_plan_check(int m, int n, int q, int batch, int mu, biq_plan* plan);
/* Workspace a checked plan needs. */
size_t biq_plan_workspace_bytes(const biq_plan* plan, int m, int batch);
const char* biq_kernel_name(int kernel);

/* ---- operations ---- */

/*
 * Key packing (Sec. III-B: mu consecutive binary weights of a row become the
 * integer key; the weights are fixed at inference time, so K is produced once, ahead of the
 * multiplies).  B device int8 [q][m][n] -> K device
 * uint8 [q][m][stride].  The byte format does not depend on mu (see above); mu is
 * validated only.  Bit = (B > 0).
 */
biq_status biq_pack(const int8_t* B, uint8_t* K, int m, int n, int q, int mu, void* stream);

/*
 * Binary-coding quantisation of a weight matrix (Sec. II-B, Eq. 1), row by row:
 * W[r] ~ sum_i alpha[i][r] * B_i[r], B_i in {-1,+1}.  The paper names the heuristic only
 * ("greedy approximation"); implemented is the greedy residual method that Eq. 1 implies: with
 * r = W[r] at the start, for i = 1..q: B_i = sign(r) (sign(0) = +1), alpha_i = mean|r|,
 * r <- r - alpha_i B_i; every step is the exact minimiser of Eq. 1 for q = 1 on the residual.
 * W device float [m][n] (row-major) -> K device uint8 [q][m][stride] (packed signs, padding 0)
 * and alpha device float [q][m], ready for biq_gemm.  fp32 arithmetic, sums in a fixed order
 * (deterministic).  n <= 32768 (BIQ_EUNSUPPORTED beyond); m * q < 2^31.
 */
biq_status biq_quantize(const float* W, uint8_t* K, float* alpha, int m, int n, int q, void* stream);

/*
 * The table indices exactly as the query kernels extract them from K:
 * keys device uint8 [q][m][C], keys[i][r][c] = bit field [mu*c, mu*c+mu) of
 * packed row (i, r).  For checking indices bit for bit against a reference.
 */
biq_status biq_unpack_keys(const uint8_t* K, uint8_t* keys, int m, int n, int q, int mu, void* stream);
/* The same with 16-bit indices, for every mu (biq_unpack_keys returns BIQ_EUNSUPPORTED for mu > 8:
 * the key does not fit a byte).  keys device uint16 [q][m][C], 2-byte aligned. */
biq_status biq_unpack_keys16(const uint8_t* K, uint16_t* keys, int m, int n, int q, int mu, void* stream);

/*
 * Table construction (Sec. III-B, q_alpha^beta = M_mu . x_alpha^beta; Algorithm 1):
 * LUT[c][k][a] = sum_j s_j(k) * X[a][mu*c + j], s_j(k) = +1 if bit j of k is set
 * else -1, elements past column n count as 0.  fp32.  LUT[c][~k][a] = -LUT[c][k][a]
 * holds bit for bit.  X device [batch][n] -> LUT device [C][2^mu][batch].
 */
biq_status biq_build_lut(const float* X, float* LUT, int n, int batch, int mu, void* stream);

/*
 * Query (Algorithm 2 lines 4-6 + Eq. 2): Y[a][r] = sum_i alpha[i][r] *
 * sum_c LUT[c][key(i,r,c)][a], with the tables read from device memory.
 * workspace: device, >= biq_workspace_bytes(...) bytes, 16-byte aligned (may be
 * NULL when that size is 0); contents undefined afterwards.
 */
biq_status biq_query(const uint8_t* K, const float* alpha, const float* LUT, float* Y,
                     int m, int n, int q, int batch, int mu,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * The fused multiply (Algorithm 2 as a whole + Eq. 2): tables are built on the
 * fly in LDS from X and never written to device memory (Sec. III-B builds them per
 * tile in fast memory instead of fetching them from DRAM), keys are streamed once,
 * partial sums are combined in a fixed order (deterministic: same inputs, same bits).
 *
 * For many input vectors (see biq_plan_get / biq_plan_get_lut) the default plan is the
 * unpack_mfma kernel instead: the "GEMM with unpacking" alternative of Sec. IV-B
 * (Algorithm 3), with the sign bits expanded to +-1 in registers and contracted on the
 * matrix cores against X split exactly into three bf16 terms; fp32 accumulation, same
 * tolerance, same determinism.  (biq_plan_get_mfma + biq_gemm_ex give the faster two-term
 * variant, see biq_plan.input_terms.)  It uses the first part of the workspace for the split X.
 */
biq_status biq_gemm(const uint8_t* K, const float* alpha, const float* X, float* Y,
                    int m, int n, int q, int batch, int mu,
                    void* workspace, size_t workspace_bytes, void* stream);

/* biq_gemm with a caller-supplied plan; BIQ_EINVAL if the plan is inconsistent
 * with the shape or exceeds device limits. */
biq_status biq_gemm_ex(const uint8_t* K, const float* alpha, const float* X, float* Y,
                       int m, int n, int q, int batch, int mu, const biq_plan* plan,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Several independent small multiplies in one dispatch.  A small layer costs one dependent
 * dispatch plus one table build whatever its size (Table IV's batch-1 column is flat from 512^2
 * to 4096^2 for the same reason); layers that do not depend on each other - the sub-layers of a
 * Transformer block, the gate or direction matrices of LSTM layers (Sec. II-C) - share that cost
 * here.  problems: HOST array of `count` descriptors (read during the call only) holding device
 * pointers with the layouts and alignments of biq_gemm; shapes, plane counts and batch sizes may
 * differ.  Consecutive problems that map to the same kernel family and plane count go into one
 * dispatch (at most 16 per dispatch), so a list of equal layers is exactly one dispatch.
 * No workspace, no allocation.  Each result equals biq_gemm's on the same problem up to the order of
 * the additions (same tolerance; bit-identical when the plans agree).
 * Served: mu = 8, q <= 4 and rows no wider than one tile of tables (batch 1: n <= 2048, batch >= 2:
 * n <= 1024); BIQ_EUNSUPPORTED otherwise, and then nothing has been launched.
 */
typedef struct {
    const uint8_t* K;    /* [q][m][stride] */
    const float* alpha;  /* [q][m] */
    const float* X;      /* [batch][n] */
    float* Y;            /* [batch][m] */
    int m, n, q, batch;
} biq_problem;
biq_status biq_gemm_grouped(const biq_problem* problems, int count, int mu, void* stream);

/*
 * One step of an LSTM cell whose four gate matrices are binary-coding quantised (Sec. II-C: LSTM
 * layers are among the method's targets) and stacked into one matrix of m = 4 * hidden rows, gates in
 * the order input, forget, cell candidate, output.  One dispatch: the lookup-table multiply of
 * biq_gemm with the cell update as its epilogue,
 *     z = W [x_t ; h_(t-1)] + bias,  c' = sigma(z_f) c + sigma(z_i) tanh(z_g),  h' = sigma(z_o) tanh(c').
 * K, alpha as for biq_gemm with m = 4 * hidden; bias device float [4 * hidden]; X device float [batch][n]
 * holds [x_t ; h_(t-1)] per input vector (n = input size + hidden: the input and the recurrent matrix
 * are the column blocks of the stacked matrix); C_prev, H_out, C_out device float [batch][hidden].
 * fp32 throughout (expf / tanhf of the device library).  Served: mu = 8, q <= 4, batch 1 with
 * n <= 2048 or batch >= 2 with n <= 1024; BIQ_EUNSUPPORTED otherwise (use biq_gemm and apply the
 * cell update separately).
 */
biq_status biq_lstm_cell(const uint8_t* K, const float* alpha, const float* bias, const float* X,
                         const float* C_prev, float* H_out, float* C_out, int hidden, int n, int q, int batch,
                         int mu, void* stream);

/*
 * biq_gemm for callers that cannot allocate or hand over device memory for a workspace: code
 * whose launches are being captured into a HIP graph, serving loops with a fixed memory plan,
 * harnesses that forbid hipMalloc.  Same arguments, plan, kernels and results (bit for bit) as
 * biq_gemm, but the workspace is a fixed buffer of biq_noalloc_scratch_bytes() = 32 MiB of device
 * memory inside the library's own code object (one copy per GPU, held until the process ends).
 * Nothing is allocated or freed, by the library or by the runtime on its behalf.
 *   - BIQ_EWORKSPACE if biq_workspace_bytes(m, n, q, batch, mu) exceeds that size (no kernel is
 *     launched; all five benchmark configurations fit): use biq_gemm with a caller workspace.
 *   - Every call on one GPU uses that GPU's single buffer: calls that may overlap in time on one
 *     GPU (different streams, different host threads) race on it and must be serialised by the
 *     caller.  Calls on different GPUs are independent.  The buffer's contents after a call are
 *     undefined; no call relies on what an earlier one left there.
 *   - biq_init() looks the buffer's device address up for the current device (once per device;
 *     no allocation).  Calling it is optional - biq_gemm_noalloc does the same on its first call
 *     on a device - but a caller about to start a graph capture should call it beforehand.
 */
biq_status biq_init(void);
size_t biq_noalloc_scratch_bytes(void);
biq_status biq_gemm_noalloc(const uint8_t* K, const float* alpha, const float* X, float* Y,
                            int m, int n, int q, int batch, int mu, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BIQ_H_ */
