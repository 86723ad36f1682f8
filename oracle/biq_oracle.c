/*
 * CPU oracle for the BiQGEMM lookup-table matrix multiply.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded C in fp64, written
 * from the paper (arxiv 2005.09904) so that a reader can check it against the
 * text by eye.  It shares no code, header, table or constant with the GPU
 * library and is never called by the product path; only tests, the smoke check
 * and the benchmark's cpu_baseline leg load it.
 *
 * Notation follows the paper: m = output size, n = input size, b = batch,
 * q = number of bit-planes (beta_w), mu = LUT-unit, C = ceil(n / mu) chunks.
 *
 * Readings taken where the paper is silent or garbled (each is also listed in
 * the design notes of this repository):
 *   - bit order inside a key: element j of a chunk is bit j (value 2^j),
 *     +1 <-> bit 1, -1 <-> bit 0.  Follows Algorithm 1 (index 2^(i-1)+j adds
 *     2*x_(i-1)) and Algorithm 3 (w_i = ((x >> i) & 1) * 2 - 1); agrees with
 *     the printed example {-1,1,1,-1} -> 6 (Sec. III-B).
 *   - Algorithm 1's first loop is read as r_0 = -(x_0 + ... + x_(mu-1)), the
 *     entry of key 0 (all signs -1); as printed (r_0 = +sum) the later
 *     "+ 2 x_(i-1)" steps would not give +-1 combinations.
 *   - n not a multiple of mu: the last chunk is padded with x = 0 and key
 *     bits 0; padding bits of a packed row are 0.
 *   - alpha is one fp32 scalar per output row per plane: alpha[q][m] (Eq. 2).
 *   - X is stored [b][n], Y is stored [b][m] (each input vector contiguous,
 *     Definition 2's column-wise traversal of the n-by-b matrix).
 *   - planes are concatenated vertically (Sec. III-B, Fig. of multi-bit
 *     weights): keys[q][m][C], B[q][m][n].
 *
 * Every function returns 0 on success, a negative number on invalid input.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define BIQO_OK 0
#define BIQO_EINVAL (-1)
#define BIQO_EVALUE (-2) /* an element of B is not +1 or -1 */
#define BIQO_ENOMEM (-3)

/* C = ceil(n / mu): number of mu-element chunks of an input vector (Sec. III-B:
 * 0 <= beta < n/mu, extended to a ragged tail). */
long biqo_num_chunks(long n, int mu) { return (n + mu - 1) / mu; }

/* Bytes of one packed row: the n sign bits, padded with zero bits to a
 * multiple of 128 bits. */
long biqo_row_stride_bytes(long n) { return ((n + 127) / 128) * 16; }

/* Table II's weight footprint for q-bit binary coding: q*m*n bits. */
long biqo_packed_bits(long m, long n, int q) { return (long)q * m * n; }

static int check_dims(long m, long n, int q, long b, int mu) {
    if (m < 1 || n < 1 || q < 1 || b < 1) return BIQO_EINVAL;
    if (mu < 1 || mu > 16) return BIQO_EINVAL;
    return BIQO_OK;
}

/*
 * Key matrix K (Sec. III-B, Fig. "retrieving partial results"): for plane i,
 * row r, chunk c the mu consecutive signs B_i[r, mu*c .. mu*c+mu-1] become the
 * integer sum_j [B = +1] * 2^j.  keys is [q][m][C], one uint16 per key.
 */
int biqo_pack_keys(const int8_t* B, long m, long n, int q, int mu, uint16_t* keys) {
    if (!B || !keys || check_dims(m, n, q, 1, mu)) return BIQO_EINVAL;
    long C = biqo_num_chunks(n, mu);
    for (int i = 0; i < q; ++i)
        for (long r = 0; r < m; ++r)
            for (long c = 0; c < C; ++c) {
                unsigned key = 0;
                for (int j = 0; j < mu; ++j) {
                    long col = c * mu + j;
                    if (col >= n) break; /* ragged tail: missing bits are 0 */
                    int8_t s = B[((long)i * m + r) * n + col];
                    if (s != 1 && s != -1) return BIQO_EVALUE;
                    if (s == 1) key |= 1u << j;
                }
                keys[((long)i * m + r) * C + c] = (uint16_t)key;
            }
    return BIQO_OK;
}

/*
 * The same signs as a byte stream: bit (col mod 8) of byte (col / 8) of a row
 * is 1 iff B = +1; rows are biqo_row_stride_bytes(n) apart, plane-major
 * [q][m][stride].  For mu = 8 byte c of a row is the key of chunk c.
 */
int biqo_pack_bitmap(const int8_t* B, long m, long n, int q, uint8_t* out) {
    if (!B || !out || check_dims(m, n, q, 1, 1)) return BIQO_EINVAL;
    long stride = biqo_row_stride_bytes(n);
    memset(out, 0, (size_t)q * m * stride);
    for (int i = 0; i < q; ++i)
        for (long r = 0; r < m; ++r)
            for (long col = 0; col < n; ++col) {
                int8_t s = B[((long)i * m + r) * n + col];
                if (s != 1 && s != -1) return BIQO_EVALUE;
                if (s == 1) out[((long)i * m + r) * stride + col / 8] |= (uint8_t)(1u << (col % 8));
            }
    return BIQO_OK;
}

/* Reads the keys of LUT-unit mu back out of a packed byte stream: key bit j of
 * chunk c is stream bit mu*c + j (0 past column n). */
int biqo_keys_from_bitmap(const uint8_t* bitmap, long m, long n, int q, int mu, uint16_t* keys) {
    if (!bitmap || !keys || check_dims(m, n, q, 1, mu)) return BIQO_EINVAL;
    long stride = biqo_row_stride_bytes(n);
    long C = biqo_num_chunks(n, mu);
    for (long kr = 0; kr < (long)q * m; ++kr)
        for (long c = 0; c < C; ++c) {
            unsigned key = 0;
            for (int j = 0; j < mu; ++j) {
                long col = c * mu + j;
                if (col >= n) break;
                if ((bitmap[kr * stride + col / 8] >> (col % 8)) & 1u) key |= 1u << j;
            }
            keys[kr * C + c] = (uint16_t)key;
        }
    return BIQO_OK;
}

/*
 * One lookup table by its definition q = M_mu . x (Sec. III-B, the equation
 * defining q_alpha^beta; Definition 5 for M_mu): entry k is the sum over j of
 * s_j(k) * x_j with s_j(k) = +1 if bit j of k is set, else -1.
 */
void biqo_lut_enum(const double* x, int mu, double* table) {
    for (unsigned k = 0; k < (1u << mu); ++k) {
        double acc = 0.0;
        for (int j = 0; j < mu; ++j) acc += ((k >> j) & 1u) ? x[j] : -x[j];
        table[k] = acc;
    }
}

/*
 * The same table by Algorithm 1 (dynamic programming), in the reading stated
 * at the top of this file.  Returns the number of arithmetic operations it
 * performed, which Eq. 6 states as 2^mu + mu - 1 per table.
 */
long biqo_lut_dp(const double* x, int mu, double* r) {
    const long half = 1L << (mu - 1);
    const long last = (1L << mu) - 1;
    long ops = 0;
    /* Key 0 has every sign negative: -(x_0 + ... + x_(mu-1)), mu operations. */
    double total = 0.0;
    for (int j = 0; j < mu; ++j) total += x[j];
    ops += mu - 1;             /* the first term of a sum is a move, not an addition */
    r[0] = -total; ++ops;
    /* Every other key of the lower half (top bit clear) is an already known key plus one more
     * set bit: with t the highest set bit of k, the key k - 2^t has the same signs except
     * for x_t, which flips from - to +, i.e. the sum grows by 2 x_t.  Keys in increasing
     * order, so k - 2^t < k is always there already.  One operation each. */
    int t = 0;
    for (long k = 1; k < half; ++k) {
        if (k == (2L << t)) ++t;                 /* k reached the next power of two */
        r[k] = r[k - (1L << t)] + 2.0 * x[t];
        ++ops;
    }
    /* The upper half needs no arithmetic on x: complementing a key negates every sign. */
    for (long k = half; k <= last; ++k) { r[k] = -r[last - k]; ++ops; }
    return ops;
}

/*
 * All tables of an input matrix (Sec. III-B): Q[c][k][a] for chunk c, key k,
 * input vector a; X is [b][n] fp32, Q is [C][2^mu][b] fp64.
 */
int biqo_build_lut(const float* X, long n, long b, int mu, double* Q) {
    if (!X || !Q || check_dims(1, n, 1, b, mu)) return BIQO_EINVAL;
    long C = biqo_num_chunks(n, mu);
    long E = 1L << mu;
    double xs[16], table[1 << 16];
    for (long c = 0; c < C; ++c)
        for (long a = 0; a < b; ++a) {
            for (int j = 0; j < mu; ++j) {
                long col = c * mu + j;
                xs[j] = col < n ? (double)X[a * n + col] : 0.0;
            }
            biqo_lut_enum(xs, mu, table);
            for (long k = 0; k < E; ++k) Q[(c * E + k) * b + a] = table[k];
        }
    return BIQO_OK;
}

/*
 * Eq. 2 written out: W = sum_i alpha_i B_i reconstructed explicitly (one row
 * at a time), then Y = W X.  fp64 throughout.  If rows != NULL only the nrows
 * listed output rows are computed and Y is [b][nrows]; otherwise Y is [b][m].
 */
int biqo_gemm_dense_rows(const int8_t* B, const float* alpha, const float* X, long m, long n, int q,
                         long b, const int64_t* rows, long nrows, double* Y) {
    if (!B || !alpha || !X || !Y || check_dims(m, n, q, b, 1)) return BIQO_EINVAL;
    long nout = rows ? nrows : m;
    double* w = (double*)malloc((size_t)n * sizeof(double));
    if (!w) return BIQO_ENOMEM;
    for (long o = 0; o < nout; ++o) {
        long r = rows ? (long)rows[o] : o;
        if (r < 0 || r >= m) { free(w); return BIQO_EINVAL; }
        for (long j = 0; j < n; ++j) w[j] = 0.0;
        for (int i = 0; i < q; ++i) {
            double a = (double)alpha[(long)i * m + r];
            for (long j = 0; j < n; ++j) {
                int8_t s = B[((long)i * m + r) * n + j];
                if (s != 1 && s != -1) { free(w); return BIQO_EVALUE; }
                w[j] += a * (double)s;
            }
        }
        for (long c = 0; c < b; ++c) {
            double acc = 0.0;
            for (long j = 0; j < n; ++j) acc += w[j] * (double)X[c * n + j];
            Y[c * nout + o] = acc;
        }
    }
    free(w);
    return BIQO_OK;
}

int biqo_gemm_dense(const int8_t* B, const float* alpha, const float* X, long m, long n, int q,
                    long b, double* Y) {
    return biqo_gemm_dense_rows(B, alpha, X, m, n, q, b, NULL, 0, Y);
}

/*
 * The method itself, Algorithm 2 without tiling: build every table, then for
 * each plane, row and input vector accumulate Q[c][K[i][r][c]][a] over the
 * chunks, scale the plane's sum by alpha_i[r] and add the planes (Eq. 2 and
 * the multi-bit paragraph of Sec. III-B).  keys is [q][m][C]; Y is [b][m].
 */
int biqo_gemm_lut(const uint16_t* keys, const float* alpha, const float* X, long m, long n, int q,
                  long b, int mu, double* Y) {
    if (!keys || !alpha || !X || !Y || check_dims(m, n, q, b, mu)) return BIQO_EINVAL;
    long C = biqo_num_chunks(n, mu);
    long E = 1L << mu;
    double* Q = (double*)malloc((size_t)C * E * b * sizeof(double));
    if (!Q) return BIQO_ENOMEM;
    int rc = biqo_build_lut(X, n, b, mu, Q);
    if (rc) { free(Q); return rc; }
    for (long a = 0; a < b; ++a)
        for (long r = 0; r < m; ++r) {
            double y = 0.0;
            for (int i = 0; i < q; ++i) {
                double p = 0.0;
                for (long c = 0; c < C; ++c) {
                    unsigned k = keys[((long)i * m + r) * C + c];
                    if (k >= (unsigned long)E) { free(Q); return BIQO_EINVAL; }
                    p += Q[(c * E + k) * b + a];
                }
                y += (double)alpha[(long)i * m + r] * p;
            }
            Y[a * m + r] = y;
        }
    free(Q);
    return BIQO_OK;
}

/*
 * Binary-coding quantisation of a matrix, row by row (Sec. II-B, Eq. 1):
 * w ~ sum_{i=1..q} alpha_i b_i with b_i in {-1,+1}^n, one alpha per row and plane.
 * The paper names the heuristic only ("greedy approximation"); the procedure here is the greedy
 * one that Eq. 1 itself suggests, one plane at a time on the residual r (r = w at the start):
 *     b_i = sign(r)      (for fixed alpha > 0 this minimises ||r - alpha b||^2 element by element;
 *                         sign(0) is taken as +1)
 *     alpha_i = (r . b_i) / n = mean |r|        (least squares in alpha for that b)
 *     r <- r - alpha_i b_i
 * so that every step is the exact minimiser of Eq. 1 for q = 1 applied to the residual, and
 * ||r_new||^2 = ||r||^2 - n alpha_i^2.
 * W float [m][n]; B int8 [q][m][n]; alpha double [q][m]; R (may be NULL) double [q][m][n] receives
 * the residual each plane's signs were taken from (its magnitude tells how firm a sign is).
 */
int biqo_quantize_greedy(const float* W, long m, long n, int q, int8_t* B, double* alpha, double* R) {
    if (!W || !B || !alpha || m < 1 || n < 1 || q < 1) return BIQO_EINVAL;
    double* r = (double*)malloc((size_t)n * sizeof(double));
    if (!r) return BIQO_ENOMEM;
    for (long row = 0; row < m; ++row) {
        for (long j = 0; j < n; ++j) r[j] = (double)W[row * n + j];
        for (int i = 0; i < q; ++i) {
            double sum_abs = 0.0;
            for (long j = 0; j < n; ++j) sum_abs += r[j] < 0.0 ? -r[j] : r[j];
            const double a = sum_abs / (double)n;
            alpha[(long)i * m + row] = a;
            for (long j = 0; j < n; ++j) {
                const int8_t b = r[j] < 0.0 ? -1 : 1;
                B[((long)i * m + row) * n + j] = b;
                if (R) R[((long)i * m + row) * n + j] = r[j];
                r[j] -= a * (double)b;
            }
        }
    }
    free(r);
    return BIQO_OK;
}

/*
 * One step of an LSTM cell whose four gate matrices are binary-coding quantised and stacked into
 * one weight matrix of 4H rows (Sec. II-C names LSTM layers as a target of the method and gives
 * their shapes; the cell itself is the textbook one, gates in the order input, forget, cell
 * candidate, output: rows [0,H), [H,2H), [2H,3H), [3H,4H)).  The layer's input is the
 * concatenation [x_t ; h_(t-1)] of length n, given as X [b][n]; the recurrent and the input
 * matrix are the column blocks of the stacked matrix.
 *     z = W [x ; h] + bias          (W = sum_i alpha_i B_i, Eq. 2; z has 4H entries)
 *     i = sigma(z_i), f = sigma(z_f), g = tanh(z_g), o = sigma(z_o)
 *     c' = f * c + i * g,   h' = o * tanh(c')
 * B int8 [q][4H][n], alpha float [q][4H], bias float [4H], X float [b][n], C_prev float [b][H];
 * H_out, C_out double [b][H].  fp64 throughout.
 */
static double biqo_sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

int biqo_lstm_cell(const int8_t* B, const float* alpha, const float* bias, const float* X,
                   const float* C_prev, long H, long n, int q, long b, double* H_out, double* C_out) {
    if (!B || !alpha || !bias || !X || !C_prev || !H_out || !C_out || H < 1) return BIQO_EINVAL;
    long m = 4 * H;
    double* Z = (double*)malloc((size_t)b * m * sizeof(double));
    if (!Z) return BIQO_ENOMEM;
    int rc = biqo_gemm_dense(B, alpha, X, m, n, q, b, Z); /* Z [b][4H] */
    if (rc) { free(Z); return rc; }
    for (long a = 0; a < b; ++a)
        for (long j = 0; j < H; ++j) {
            double zi = Z[a * m + j] + (double)bias[j];
            double zf = Z[a * m + H + j] + (double)bias[H + j];
            double zg = Z[a * m + 2 * H + j] + (double)bias[2 * H + j];
            double zo = Z[a * m + 3 * H + j] + (double)bias[3 * H + j];
            double c = biqo_sigmoid(zf) * (double)C_prev[a * H + j] + biqo_sigmoid(zi) * tanh(zg);
            C_out[a * H + j] = c;
            H_out[a * H + j] = biqo_sigmoid(zo) * tanh(c);
        }
    free(Z);
    return BIQO_OK;
}
