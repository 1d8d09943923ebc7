/*
 * CPU oracle for the Low-bit Module and the partition-local GNN layer of
 * "Sylvie" (arXiv 2303.01277).  TEST INFRASTRUCTURE ONLY: the tests, the smoke
 * check and the benchmark's cpu_baseline leg are the only callers.  The product
 * (the HIP library) shares no code with this file and never calls it.
 *
 * Everything is written as the plain definition: scalar loops, one element at a
 * time, no blocking, no fusion.  Sums that the method defines over real numbers
 * (aggregation, dense transform) are accumulated in double and rounded to float
 * once; steps whose single-precision arithmetic decides an integer (the
 * stochastic-rounding comparison) or whose order is part of the definition (the
 * backward "integrate" accumulation) are done in float exactly as stated below.
 * Build with -O2 -ffp-contract=off (no fast-math) so every float operation is
 * one IEEE-754 binary32 operation.
 *
 * "parity unpinned": the constants of the counter hash below.  The paper only
 * says "with probability"; any hash that passes the uniformity / independence /
 * unbiasedness tests is a correct reading, so no external value pins them.
 *
 * OpenMP `parallel for` over independent rows only; results do not depend on
 * the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Counter-based random bits for the stochastic rounding of Sec. 3.2, Eq. 4. */
/* Keyed on (seed, stream, wire row, column); 24 uniform bits per element.   */
/* ------------------------------------------------------------------------- */

#define ORC_M1 0xce6e1acdu
#define ORC_M2 0x6d3cb3a7u
#define ORC_COL_STRIDE 0x9e3779b9u /* odd: floor(2^32 / golden ratio) */
#define ORC_DOMAIN 0x53594c56u     /* "SYLV" */

static uint32_t orc_mix(uint32_t x)
{
    x ^= x >> 16;
    x *= ORC_M1;
    x ^= x >> 15;
    x *= ORC_M2;
    x ^= x >> 16;
    return x;
}

/* Key of one call: folds the 64-bit seed and the 32-bit stream id. */
uint32_t orc_call_key(uint64_t seed, uint32_t stream)
{
    uint32_t k = orc_mix((uint32_t)(seed & 0xffffffffu) ^ ORC_DOMAIN);
    k = orc_mix(k ^ (uint32_t)(seed >> 32));
    k = orc_mix(k ^ stream);
    return k;
}

/* Key of one wire row. */
static uint32_t orc_row_key(uint32_t call_key, uint32_t row)
{
    return orc_mix(call_key ^ row);
}

/* 24 random bits of element (row, col): the top 24 bits of the second product. */
static uint32_t orc_elem_u24(uint32_t row_key, uint32_t col)
{
    uint32_t x = row_key + col * ORC_COL_STRIDE;
    x ^= x >> 16;
    x *= ORC_M1;
    x ^= x >> 16;
    x *= ORC_M2;
    return x >> 8;
}

/* Exposed for the statistical tests: the 24-bit integer behind u = k * 2^-24. */
uint32_t orc_uniform24(uint64_t seed, uint32_t stream, uint32_t row, uint32_t col)
{
    return orc_elem_u24(orc_row_key(orc_call_key(seed, stream), row), col);
}

/* ------------------------------------------------------------------------- */
/* Quantizer (Sec. 3.2 "Quantizer", Eq. 3 and Eq. 4 with b = 1, B = 1) and     */
/* the scale / zero-point side channel (Sec. 3.2 "Communicator").              */
/* ------------------------------------------------------------------------- */

int64_t orc_words_per_row(int32_t d) { return ((int64_t)d + 63) / 64; }

/*
 * For wire row i = 0..n_rows-1 the source row is idx[i] (idx != NULL) or
 * row_offset + i (idx == NULL) of the row-major matrix src (leading dim ld).
 * wire_row0 is added to i where i keys the random draws, so that a window of a
 * longer exchange can be recomputed on its own (0 for a whole exchange).
 *
 *   mn = min_c r_c, mx = max_c r_c, each then "+ 0.0f" (turns -0 into +0)
 *   zero = mn,  scale = mx - mn            (B = 1, so (max-min)/B is the range)
 *   u    = k * 2^-24, k the 24 random bits of (seed, stream, i, c)
 *   bit  = [ fl(u * scale) < fl(r_c - mn) ]
 *
 * Eq. 3 normalises h to hbar = (h - min)/(max - min) in [0, 1]; Eq. 4 rounds hbar
 * up with probability hbar - floor(hbar), i.e. to 1 with probability hbar.  With
 * u uniform on [0,1), "u < hbar" has exactly that probability; multiplying both
 * sides by the range avoids the division and leaves a constant row (range 0)
 * with all bits 0 and no special case.
 *
 * Packing: bit j (least significant = 0) of word k of a row is column 64k + j;
 * ceil(d/64) words per row; bits of columns >= d are 0.
 */
void orc_quantize_1bit(const float *src, int64_t ld, int32_t d, const int32_t *idx,
                       int64_t row_offset, int64_t n_rows, uint64_t seed, uint32_t stream,
                       int64_t wire_row0, uint64_t *packed, float *scale, float *zero)
{
    const int64_t W = orc_words_per_row(d);
    const uint32_t ck = orc_call_key(seed, stream);
    const float two_m24 = 1.0f / 16777216.0f;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t srow = idx ? (int64_t)idx[i] : row_offset + i;
        const float *r = src + srow * ld;
        float mn = r[0], mx = r[0];
        for (int32_t c = 1; c < d; ++c) {
            if (r[c] < mn) mn = r[c];
            if (r[c] > mx) mx = r[c];
        }
        mn = mn + 0.0f;
        mx = mx + 0.0f;
        const float sc = mx - mn;
        zero[i] = mn;
        scale[i] = sc;
        const uint32_t rk = orc_row_key(ck, (uint32_t)(wire_row0 + i));
        for (int64_t k = 0; k < W; ++k) packed[i * W + k] = 0;
        for (int32_t c = 0; c < d; ++c) {
            const float u = (float)orc_elem_u24(rk, (uint32_t)c) * two_m24;
            const float lhs = u * sc;
            const float rhs = r[c] - mn;
            if (lhs < rhs) packed[i * W + (c >> 6)] |= (uint64_t)1 << (c & 63);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Dequantizer (Sec. 3.2 "Dequantizer", Eq. 5 with B = 1).                     */
/* ------------------------------------------------------------------------- */

static float orc_deq(const uint64_t *prow, float sc, float zp, int32_t c)
{
    const int bit = (int)((prow[c >> 6] >> (c & 63)) & 1u);
    /* (max-min) * hhat / B + min: hhat is 0 or 1, so one float addition at most */
    return bit ? zp + sc : zp;
}

/* Forward: received row i overwrites row row_offset + i of dst (Alg. 1: the
 * recovered rows are appended below the inner rows, "concatenate"). */
void orc_dequantize_1bit_fwd(const uint64_t *packed, const float *scale, const float *zero,
                             int64_t n_rows, int32_t d, float *dst, int64_t ld,
                             int64_t row_offset)
{
    const int64_t W = orc_words_per_row(d);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        float *o = dst + (row_offset + i) * ld;
        for (int32_t c = 0; c < d; ++c) o[c] = orc_deq(packed + i * W, scale[i], zero[i], c);
    }
}

/* Backward: J[dst_row[i]] += dequantized row i (Alg. 2 "integrate feature
 * gradients").  Several wire rows may name one destination; the additions are
 * single-precision and happen in ascending wire-row order. */
void orc_dequantize_1bit_bwd(const uint64_t *packed, const float *scale, const float *zero,
                             int64_t n_rows, int32_t d, float *J, int64_t ld,
                             const int32_t *dst_row)
{
    const int64_t W = orc_words_per_row(d);
    for (int64_t i = 0; i < n_rows; ++i) {
        float *o = J + (int64_t)dst_row[i] * ld;
        for (int32_t c = 0; c < d; ++c) {
            const float v = orc_deq(packed + i * W, scale[i], zero[i], c);
            o[c] = o[c] + v;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* b-bit quantizer / dequantizer: Eq. 3, Eq. 4 and Eq. 5 for b in {1, 2, 4, 8}, */
/* B = 2^b - 1 bins (Sec. 3.2; the bit-width study of Sec. 4.3).               */
/* ------------------------------------------------------------------------- */

int64_t orc_words_per_row_bits(int32_t d, int32_t bits) { return ((int64_t)d * bits + 63) / 64; }

/*
 * Row selection, extrema, random draws and the metadata convention are those of
 * orc_quantize_1bit.  Per row, in single precision, one IEEE operation each:
 *
 *   range = mx - mn,  zero = mn,  scale = range / B           (Sec. 3.2 "Communicator":
 *                                                              scale is the ratio of the range to B)
 *   g     = 2^64 if range < 2^-60, else 1                      (exact rescaling that keeps the
 *                                                              reciprocal below finite)
 *   inv   = B / (range * g)   if range > 0, else 0
 * and per element
 *   t  = ((r_c - mn) * g) * inv,  then t = min(t, B)           (Eq. 3: hbar in [0, B])
 *   q  = floor(t) + [ u < t - floor(t) ],  u = k * 2^-24        (Eq. 4: up with probability frac(hbar))
 *
 * t - floor(t) is exact, so the comparison with u involves no rounding.  The clamp
 * covers the one case where rounding of inv pushes the arg-max element above B.
 * A constant row has inv = 0, hence all codes 0.
 *
 * Packing: 64/b codes per 64-bit word; the code of column c sits in bits
 * [b (c mod 64/b), b (c mod 64/b) + b) of word c / (64/b); unused high codes are 0.
 */
void orc_quantize_bbit(const float *src, int64_t ld, int32_t d, const int32_t *idx,
                       int64_t row_offset, int64_t n_rows, int32_t bits, uint64_t seed,
                       uint32_t stream, int64_t wire_row0, uint64_t *packed, float *scale,
                       float *zero)
{
    const int64_t W = orc_words_per_row_bits(d, bits);
    const int32_t per = 64 / bits;
    const uint32_t ck = orc_call_key(seed, stream);
    const float two_m24 = 1.0f / 16777216.0f;
    const float Bf = (float)((1 << bits) - 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t srow = idx ? (int64_t)idx[i] : row_offset + i;
        const float *r = src + srow * ld;
        float mn = r[0], mx = r[0];
        for (int32_t c = 1; c < d; ++c) {
            if (r[c] < mn) mn = r[c];
            if (r[c] > mx) mx = r[c];
        }
        mn = mn + 0.0f;
        mx = mx + 0.0f;
        const float range = mx - mn;
        zero[i] = mn;
        scale[i] = range / Bf;
        float g = 1.0f;
        if (range < 0x1p-60f) g = 0x1p64f;
        float inv = 0.0f;
        if (range > 0.0f) inv = Bf / (range * g);
        const uint32_t rk = orc_row_key(ck, (uint32_t)(wire_row0 + i));
        for (int64_t k = 0; k < W; ++k) packed[i * W + k] = 0;
        for (int32_t c = 0; c < d; ++c) {
            const float u = (float)orc_elem_u24(rk, (uint32_t)c) * two_m24;
            const float diff = r[c] - mn;
            const float scaled = diff * g;
            float t = scaled * inv;
            if (t > Bf) t = Bf;
            const float fl = floorf(t);
            const float fr = t - fl;
            uint64_t q = (uint64_t)fl;
            if (u < fr) q += 1;
            packed[i * W + c / per] |= q << (bits * (c % per));
        }
    }
}

/* Eq. 5: (max - min) * q / B + min, evaluated as fl(fl(scale * q) + zero). */
static float orc_deq_bbit(const uint64_t *prow, float sc, float zp, int32_t bits, int32_t c)
{
    const int32_t per = 64 / bits;
    const uint64_t q = (prow[c / per] >> (bits * (c % per))) & (((uint64_t)1 << bits) - 1);
    const float step = sc * (float)q;
    return step + zp;
}

void orc_dequantize_bbit_fwd(const uint64_t *packed, const float *scale, const float *zero,
                             int64_t n_rows, int32_t d, int32_t bits, float *dst, int64_t ld,
                             int64_t row_offset)
{
    const int64_t W = orc_words_per_row_bits(d, bits);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        float *o = dst + (row_offset + i) * ld;
        for (int32_t c = 0; c < d; ++c)
            o[c] = orc_deq_bbit(packed + i * W, scale[i], zero[i], bits, c);
    }
}

/* Backward integrate, as orc_dequantize_1bit_bwd: ascending wire-row order. */
void orc_dequantize_bbit_bwd(const uint64_t *packed, const float *scale, const float *zero,
                             int64_t n_rows, int32_t d, int32_t bits, float *J, int64_t ld,
                             const int32_t *dst_row)
{
    const int64_t W = orc_words_per_row_bits(d, bits);
    for (int64_t i = 0; i < n_rows; ++i) {
        float *o = J + (int64_t)dst_row[i] * ld;
        for (int32_t c = 0; c < d; ++c) {
            const float v = orc_deq_bbit(packed + i * W, scale[i], zero[i], bits, c);
            o[c] = o[c] + v;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Half-precision wire (the FP16 point of the bit-width study, Sec. 4.3): each  */
/* element is rounded to IEEE binary16, nearest-even; no side channel.          */
/* ------------------------------------------------------------------------- */

/* binary32 -> binary16, round to nearest, ties to even; overflow gives infinity. */
static uint16_t orc_f32_to_f16(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    const uint32_t mag = x & 0x7fffffffu;
    if (mag >= 0x7f800000u) /* infinity or NaN */
        return (uint16_t)(sign | 0x7c00u | (mag > 0x7f800000u ? 0x200u : 0u));
    const int32_t e = (int32_t)(mag >> 23) - 127; /* unbiased exponent of a normal input */
    if (e >= 16) return (uint16_t)(sign | 0x7c00u); /* >= 2^16: beyond the largest half */
    if (e >= -14) {
        /* normal half: keep 10 fraction bits, round on the 13 dropped ones */
        uint32_t h = ((uint32_t)(e + 15) << 10) | ((mag >> 13) & 0x3ffu);
        const uint32_t rest = mag & 0x1fffu;
        if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h += 1; /* may carry into the exponent: correct */
        return (uint16_t)(sign | h);
    }
    if (e < -25) return sign; /* below half of the smallest subnormal: zero */
    /* subnormal half: value = m * 2^-24, m = round(|f| * 2^24) */
    const uint32_t sig = (mag & 0x7fffffu) | 0x800000u; /* 24-bit significand, |f| = sig * 2^(e-23) */
    const int32_t shift = -e - 1;                       /* m = sig >> shift, shift in [14, 24] */
    uint32_t m = sig >> shift;
    const uint32_t rest = sig & (((uint32_t)1 << shift) - 1);
    const uint32_t half = (uint32_t)1 << (shift - 1);
    if (rest > half || (rest == half && (m & 1u))) m += 1;
    return (uint16_t)(sign | m);
}

static float orc_f16_to_f32(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
    float v;
    if (e == 0) {
        v = (float)m * 0x1p-24f;
    } else if (e == 31) {
        const uint32_t x = 0x7f800000u | (m << 13);
        memcpy(&v, &x, 4);
    } else {
        const uint32_t x = ((e + 112u) << 23) | (m << 13);
        memcpy(&v, &x, 4);
    }
    uint32_t x;
    memcpy(&x, &v, 4);
    x |= sign;
    memcpy(&v, &x, 4);
    return v;
}

int64_t orc_words_per_row_fp16(int32_t d) { return ((int64_t)d + 3) / 4; }

/* Wire row i: the d halves of the selected source row, then zero halves up to a
 * multiple of four (rows are whole 64-bit words). */
void orc_convert_fp16(const float *src, int64_t ld, int32_t d, const int32_t *idx,
                      int64_t row_offset, int64_t n_rows, uint16_t *wire)
{
    const int64_t dp = 4 * orc_words_per_row_fp16(d);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t srow = idx ? (int64_t)idx[i] : row_offset + i;
        for (int64_t c = 0; c < dp; ++c)
            wire[i * dp + c] = c < d ? orc_f32_to_f16(src[srow * ld + c]) : 0;
    }
}

void orc_recover_fp16_fwd(const uint16_t *wire, int64_t n_rows, int32_t d, float *dst,
                          int64_t ld, int64_t row_offset)
{
    const int64_t dp = 4 * orc_words_per_row_fp16(d);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i)
        for (int32_t c = 0; c < d; ++c)
            dst[(row_offset + i) * ld + c] = orc_f16_to_f32(wire[i * dp + c]);
}

void orc_recover_fp16_bwd(const uint16_t *wire, int64_t n_rows, int32_t d, float *J, int64_t ld,
                          const int32_t *dst_row)
{
    const int64_t dp = 4 * orc_words_per_row_fp16(d);
    for (int64_t i = 0; i < n_rows; ++i) {
        float *o = J + (int64_t)dst_row[i] * ld;
        for (int32_t c = 0; c < d; ++c) o[c] = o[c] + orc_f16_to_f32(wire[i * dp + c]);
    }
}

/* ------------------------------------------------------------------------- */
/* Normalised operators (Sec. 3.4: A_hat = D^-1/2 (A + I) D^-1/2 for GCN;       */
/* mean over neighbours for GraphSAGE, Eq. 1 with rho = mean).                  */
/* ------------------------------------------------------------------------- */

/*
 * GCN rows of one partition.  Input: adjacency (rowptr, col) of the n_in inner
 * rows without self loops, columns ascending; deg[r] = degree of local row r in
 * the whole graph (self loop not counted).  Output CSR has the self loop (r, r)
 * inserted in column order and weights 1/sqrt((deg_r+1)(deg_c+1)), evaluated in
 * double and rounded to float.  out_rowptr has n_in+1 entries; out_col/out_w
 * need nnz + n_in entries.
 */
void orc_gcn_operator(const int64_t *rowptr, const int32_t *col, const int32_t *deg,
                      int64_t n_in, int64_t *out_rowptr, int32_t *out_col, float *out_w)
{
    for (int64_t r = 0; r <= n_in; ++r) out_rowptr[r] = rowptr[r] + r;
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t r = 0; r < n_in; ++r) {
        int64_t o = out_rowptr[r];
        const double dr = (double)deg[r] + 1.0;
        int placed = 0;
        for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e) {
            if (!placed && (int64_t)col[e] > r) {
                out_col[o] = (int32_t)r;
                out_w[o] = (float)(1.0 / sqrt(dr * dr));
                ++o;
                placed = 1;
            }
            out_col[o] = col[e];
            out_w[o] = (float)(1.0 / sqrt(dr * ((double)deg[col[e]] + 1.0)));
            ++o;
        }
        if (!placed) {
            out_col[o] = (int32_t)r;
            out_w[o] = (float)(1.0 / sqrt(dr * dr));
        }
    }
}

/* GraphSAGE mean: weight of every entry of row r is 1/len(r) (in double, rounded). */
void orc_mean_weights(const int64_t *rowptr, int64_t n_in, float *out_w)
{
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t r = 0; r < n_in; ++r) {
        const int64_t len = rowptr[r + 1] - rowptr[r];
        for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e) out_w[e] = (float)(1.0 / (double)len);
    }
}

/* ------------------------------------------------------------------------- */
/* Neighbour aggregation (Eq. 1; Alg. 1 "update embeddings", the A * Htilde     */
/* product) and its transpose (Alg. 2 "compute feature gradients").             */
/* ------------------------------------------------------------------------- */

/* Z[v][c] = sum_e w_e * X[col_e][c] over the entries e of row v; double sum,
 * one rounding.  If S != NULL also S[v][c] = sum_e |w_e * X[col_e][c]| (the
 * magnitude the tolerance of a float re-implementation is measured against). */
void orc_aggregate_fwd(const int64_t *rowptr, const int32_t *col, const float *w,
                       int64_t n_rows, const float *X, int64_t ldx, int32_t d, float *Z,
                       int64_t ldz, float *S, int64_t lds)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n_rows; ++v) {
        for (int32_t c = 0; c < d; ++c) {
            double acc = 0.0, mag = 0.0;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                const double t = (double)w[e] * (double)X[(int64_t)col[e] * ldx + c];
                acc += t;
                mag += fabs(t);
            }
            Z[v * ldz + c] = (float)acc;
            if (S) S[v * lds + c] = (float)mag;
        }
    }
}

/* dX[u][c] = sum over entries (v, u) of w_vu * dZ[v][c], for every local row
 * u in [0, n_cols): scattered straight from the forward CSR into a double
 * buffer, rounded once at the end.  S as above (may be NULL). */
int orc_aggregate_bwd(const int64_t *rowptr, const int32_t *col, const float *w, int64_t n_rows,
                      int64_t n_cols, const float *dZ, int64_t ldz, int32_t d, float *dX,
                      int64_t ldx, float *S, int64_t lds)
{
    double *acc = (double *)calloc((size_t)n_cols * (size_t)d, sizeof(double));
    double *mag = S ? (double *)calloc((size_t)n_cols * (size_t)d, sizeof(double)) : NULL;
    if (!acc || (S && !mag)) {
        free(acc);
        free(mag);
        return -1;
    }
    for (int64_t v = 0; v < n_rows; ++v) {
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const int64_t u = col[e];
            for (int32_t c = 0; c < d; ++c) {
                const double t = (double)w[e] * (double)dZ[v * ldz + c];
                acc[u * d + c] += t;
                if (mag) mag[u * d + c] += fabs(t);
            }
        }
    }
    for (int64_t u = 0; u < n_cols; ++u)
        for (int32_t c = 0; c < d; ++c) {
            dX[u * ldx + c] = (float)acc[u * d + c];
            if (S) S[u * lds + c] = (float)mag[u * d + c];
        }
    free(acc);
    free(mag);
    return 0;
}

/* The same transpose product, but only for the n_sel output rows listed in
 * sel (ascending, distinct): one pass over the forward CSR, for checks at sizes
 * where the full double buffer would not fit.  out / S are [n_sel][d]. */
void orc_aggregate_bwd_rows(const int64_t *rowptr, const int32_t *col, const float *w,
                            int64_t n_rows, const float *dZ, int64_t ldz, int32_t d,
                            const int32_t *sel, int64_t n_sel, float *out, float *S)
{
    double *acc = (double *)calloc((size_t)n_sel * (size_t)d * 2, sizeof(double));
    double *mag = acc + (size_t)n_sel * (size_t)d;
    for (int64_t v = 0; v < n_rows; ++v) {
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            /* binary search for col[e] in sel */
            int64_t lo = 0, hi = n_sel;
            while (lo < hi) {
                const int64_t mid = (lo + hi) / 2;
                if (sel[mid] < col[e]) lo = mid + 1; else hi = mid;
            }
            if (lo == n_sel || sel[lo] != col[e]) continue;
            for (int32_t c = 0; c < d; ++c) {
                const double t = (double)w[e] * (double)dZ[v * ldz + c];
                acc[lo * d + c] += t;
                mag[lo * d + c] += fabs(t);
            }
        }
    }
    for (int64_t i = 0; i < n_sel * d; ++i) {
        out[i] = (float)acc[i];
        if (S) S[i] = (float)mag[i];
    }
    free(acc);
}

/* ------------------------------------------------------------------------- */
/* Dense transform (Eq. 2; Alg. 1 H = sigma(Z W); Alg. 2 weight and feature     */
/* gradients).  sigma = ReLU.  The left operand may be two column blocks side   */
/* by side, [A1 | A2] (GraphSAGE: own embedding next to the neighbour mean);    */
/* pass k2 = 0 for a single block.  W is (k1+k2) x h row-major.                 */
/* ------------------------------------------------------------------------- */

/* P = [A1|A2] W (double sum, one rounding); H = relu ? max(P, 0) : P.
 * P_out and S (sum of |terms|) may be NULL. */
void orc_transform_fwd(const float *A1, int64_t ld1, int32_t k1, const float *A2, int64_t ld2,
                       int32_t k2, const float *Wm, int32_t h, int64_t n, int relu, float *H,
                       int64_t ldh, float *P_out, float *S)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int32_t j = 0; j < h; ++j) {
            double acc = 0.0, mag = 0.0;
            for (int32_t k = 0; k < k1; ++k) {
                const double t = (double)A1[i * ld1 + k] * (double)Wm[(int64_t)k * h + j];
                acc += t;
                mag += fabs(t);
            }
            for (int32_t k = 0; k < k2; ++k) {
                const double t = (double)A2[i * ld2 + k] * (double)Wm[(int64_t)(k1 + k) * h + j];
                acc += t;
                mag += fabs(t);
            }
            const float p = (float)acc;
            if (P_out) P_out[i * h + j] = p;
            if (S) S[i * h + j] = (float)mag;
            H[i * ldh + j] = (relu && !(p > 0.0f)) ? 0.0f : p;
        }
    }
}

/* Backward of the transform.  M = J o [H > 0] when relu (H is the forward
 * output, so H > 0 exactly where the pre-activation was > 0), else M = J.
 *   G  = [A1|A2]^T M          ((k1+k2) x h, double sums)          if G  != NULL
 *   dA = M W^T                (n x (k1+k2), written as two blocks dA1 | dA2
 *                              with leading dims ldd1, ldd2)       if dA1 != NULL
 * SG / SdA1 / SdA2: sums of |terms|, dense ((k1+k2) x h, n x k1, n x k2; may be NULL). */
void orc_transform_bwd(const float *A1, int64_t ld1, int32_t k1, const float *A2, int64_t ld2,
                       int32_t k2, const float *Wm, int32_t h, int64_t n, int relu,
                       const float *H, int64_t ldh, const float *J, int64_t ldj, float *G,
                       float *SG, float *dA1, int64_t ldd1, float *dA2, int64_t ldd2,
                       float *SdA1, float *SdA2)
{
    const int32_t K = k1 + k2;
    if (G) {
#pragma omp parallel for schedule(static)
        for (int32_t k = 0; k < K; ++k) {
            for (int32_t j = 0; j < h; ++j) {
                double acc = 0.0, mag = 0.0;
                for (int64_t i = 0; i < n; ++i) {
                    const float m = (relu && !(H[i * ldh + j] > 0.0f)) ? 0.0f : J[i * ldj + j];
                    const float a = k < k1 ? A1[i * ld1 + k] : A2[i * ld2 + (k - k1)];
                    const double t = (double)a * (double)m;
                    acc += t;
                    mag += fabs(t);
                }
                G[(int64_t)k * h + j] = (float)acc;
                if (SG) SG[(int64_t)k * h + j] = (float)mag;
            }
        }
    }
    if (dA1) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            for (int32_t k = 0; k < K; ++k) {
                double acc = 0.0, mag = 0.0;
                for (int32_t j = 0; j < h; ++j) {
                    const float m = (relu && !(H[i * ldh + j] > 0.0f)) ? 0.0f : J[i * ldj + j];
                    const double t = (double)m * (double)Wm[(int64_t)k * h + j];
                    acc += t;
                    mag += fabs(t);
                }
                if (k < k1) {
                    dA1[i * ldd1 + k] = (float)acc;
                    if (SdA1) SdA1[i * k1 + k] = (float)mag;
                } else {
                    dA2[i * ldd2 + (k - k1)] = (float)acc;
                    if (SdA2) SdA2[i * k2 + (k - k1)] = (float)mag;
                }
            }
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Attention aggregator (the GAT model of Sec. 2.1 / Sec. 4; the paper cites   */
/* the model and gives no formulas, so these are the cited model's):             */
/*   P = Htilde W,  s_dst[v] = P_v . a_dst,  s_src[u] = P_u . a_src               */
/*   e_vu = leaky_relu(s_dst[v] + s_src[u]),  alpha_v. = softmax_u e_vu           */
/*   z_v = sum_u alpha_vu P_u   (the aggregation of Eq. 1 with learned weights)   */
/* over the entries (v, u) of the local operator pattern (self loop included).    */
/* Sums in double, results rounded to float once.                                */
/* ------------------------------------------------------------------------- */

/* out[i] = P_i . a for i < n. */
void orc_row_dot(const float *P, int64_t ld, int64_t n, int32_t F, const float *a, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int32_t c = 0; c < F; ++c) acc += (double)P[i * ld + c] * (double)a[c];
        out[i] = (float)acc;
    }
}

static double orc_lrelu(double x, double slope) { return x > 0.0 ? x : slope * x; }

/* alpha[e] for every entry e of rows 0 .. n_rows-1 (softmax over each row's entries). */
void orc_edge_softmax_fwd(const int64_t *rowptr, const int32_t *col, int64_t n_rows,
                          const float *s_dst, const float *s_src, float slope, float *alpha)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n_rows; ++v) {
        const int64_t e0 = rowptr[v], e1 = rowptr[v + 1];
        if (e0 == e1) continue;
        double mx = -INFINITY;
        for (int64_t e = e0; e < e1; ++e) {
            const double x = orc_lrelu((double)s_dst[v] + (double)s_src[col[e]], slope);
            if (x > mx) mx = x;
        }
        double sum = 0.0;
        for (int64_t e = e0; e < e1; ++e)
            sum += exp(orc_lrelu((double)s_dst[v] + (double)s_src[col[e]], slope) - mx);
        for (int64_t e = e0; e < e1; ++e)
            alpha[e] = (float)(exp(orc_lrelu((double)s_dst[v] + (double)s_src[col[e]], slope) - mx) / sum);
    }
}

/* out[e] = A_v . B_u for every entry e = (v, u): the gradient of z_v = sum alpha_vu P_u with
 * respect to alpha_vu is dZ_v . P_u.  S (optional): sum of |terms|. */
void orc_sddmm(const int64_t *rowptr, const int32_t *col, int64_t n_rows, const float *A,
               int64_t lda, const float *Bm, int64_t ldb, int32_t F, float *out, float *S)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n_rows; ++v)
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            double acc = 0.0, mag = 0.0;
            for (int32_t c = 0; c < F; ++c) {
                const double t = (double)A[v * lda + c] * (double)Bm[(int64_t)col[e] * ldb + c];
                acc += t;
                mag += fabs(t);
            }
            out[e] = (float)acc;
            if (S) S[e] = (float)mag;
        }
}

/* Backward of the edge softmax and of the leaky ReLU in front of it:
 *   g_e  = alpha_e (dalpha_e - sum_{w in row} alpha_w dalpha_w)
 *   de_e = g_e * (s_dst[v] + s_src[u] > 0 ? 1 : slope)
 * S (optional): |alpha_e dalpha_e| + alpha_e sum_w |alpha_w dalpha_w|, times the same factor. */
void orc_edge_softmax_bwd(const int64_t *rowptr, const int32_t *col, int64_t n_rows,
                          const float *alpha, const float *dalpha, const float *s_dst,
                          const float *s_src, float slope, float *de, float *S)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n_rows; ++v) {
        double dot = 0.0, mag = 0.0;
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const double t = (double)alpha[e] * (double)dalpha[e];
            dot += t;
            mag += fabs(t);
        }
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            const double raw = (double)s_dst[v] + (double)s_src[col[e]];
            const double f = raw > 0.0 ? 1.0 : (double)slope;
            const double t = (double)alpha[e] * (double)dalpha[e];
            de[e] = (float)((t - (double)alpha[e] * dot) * f);
            if (S) S[e] = (float)((fabs(t) + (double)alpha[e] * mag) * fabs(f));
        }
    }
}

/* out[v] = sum of vals over the entries of row v (S optional: sum of |vals|). */
void orc_segment_sum(const int64_t *rowptr, int64_t n_rows, const float *vals, float *out, float *S)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t v = 0; v < n_rows; ++v) {
        double acc = 0.0, mag = 0.0;
        for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            acc += (double)vals[e];
            mag += fabs((double)vals[e]);
        }
        out[v] = (float)acc;
        if (S) S[v] = (float)mag;
    }
}

/* out[u] = sum of vals[e] over the entries e with col[e] = u (scatter form, from the
 * forward pattern, so that the transposed pattern of the product is itself checked). */
void orc_column_sum(const int64_t *rowptr, const int32_t *col, int64_t n_rows, int64_t n_cols,
                    const float *vals, float *out, float *S)
{
    double *acc = (double *)calloc((size_t)n_cols * 2, sizeof(double));
    double *mag = acc + n_cols;
    for (int64_t e = 0; e < rowptr[n_rows]; ++e) {
        acc[col[e]] += (double)vals[e];
        mag[col[e]] += fabs((double)vals[e]);
    }
    for (int64_t u = 0; u < n_cols; ++u) {
        out[u] = (float)acc[u];
        if (S) S[u] = (float)mag[u];
    }
    free(acc);
}

/* X[i][c] = fl(X[i][c] + fl(s[i] * a[c])) for i < n: the part of dP that comes through the
 * attention scores (single precision, two operations per element). */
void orc_rank1_add(float *X, int64_t ld, int64_t n, int32_t F, const float *s, const float *a)
{
    for (int64_t i = 0; i < n; ++i)
        for (int32_t c = 0; c < F; ++c) {
            const float t = s[i] * a[c];
            X[i * ld + c] = X[i * ld + c] + t;
        }
}

/* ------------------------------------------------------------------------- */
/* Loss, gradient synchronisation and model update (Alg. 1 last line; Alg. 2    */
/* J^(L) = gradient of the loss, G = AllReduce(G_n), W_t = W_{t-1} - eta G).    */
/* ------------------------------------------------------------------------- */

/*
 * Softmax cross-entropy over the labelled rows, averaged over `count` rows (the number
 * of labelled nodes of the WHOLE graph, so that partition sums add up to the
 * unpartitioned loss):
 *   p_ic = exp(H_ic - max_c H_ic) / sum_c exp(H_ic - max_c H_ic)
 *   loss = -(1/count) sum_{i labelled} log p_{i, y_i}
 *   J_ic = (p_ic - [c == y_i]) / count for labelled rows, 0 for the others (label < 0).
 * Everything in double; J is rounded to float once.  SJ (optional) receives
 * (p_ic + [c == y_i]) / count, the magnitude the tolerance is taken against.
 * Returns the loss contribution of these rows.
 */
double orc_softmax_xent(const float *H, int64_t ldh, int64_t n, int32_t C, const int32_t *label,
                        double count, float *J, int64_t ldj, float *SJ)
{
    double loss = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const float *h = H + i * ldh;
        float *j = J + i * ldj;
        const int32_t y = label[i];
        if (y < 0) {
            for (int32_t c = 0; c < C; ++c) {
                j[c] = 0.0f;
                if (SJ) SJ[i * C + c] = 0.0f;
            }
            continue;
        }
        double mx = h[0];
        for (int32_t c = 1; c < C; ++c)
            if (h[c] > mx) mx = h[c];
        double sum = 0.0;
        for (int32_t c = 0; c < C; ++c) sum += exp((double)h[c] - mx);
        loss -= ((double)h[y] - mx) - log(sum);
        for (int32_t c = 0; c < C; ++c) {
            const double p = exp((double)h[c] - mx) / sum;
            const double onehot = c == y ? 1.0 : 0.0;
            j[c] = (float)((p - onehot) / count);
            if (SJ) SJ[i * C + c] = (float)((p + onehot) / count);
        }
    }
    return loss / count;
}

/* Gradient synchronisation of one process that holds every partition: dst = the sum of
 * the n_src arrays, added in ascending order in single precision (dst may be srcs[0]). */
void orc_sum_gradients(float *dst, const float *const *srcs, int32_t n_src, int64_t elems)
{
    for (int64_t e = 0; e < elems; ++e) {
        float s = srcs[0][e];
        for (int32_t k = 1; k < n_src; ++k) s = s + srcs[k][e];
        dst[e] = s;
    }
}

/* Plain SGD: W = fl(W - fl(eta * G)), single precision, two operations per element. */
void orc_sgd_update(float *W, const float *G, int64_t elems, float eta)
{
    for (int64_t e = 0; e < elems; ++e) {
        const float step = eta * G[e];
        W[e] = W[e] - step;
    }
}

/* ------------------------------------------------------------------------- */
/* Graph Engine set-up (Sec. 3.2; Alg. 1, the lines before the epoch loop):      */
/* HALO node set, send / receive sets, local numbering, transposed operator.     */
/* Sequential loops in the order of the definitions; integers only.              */
/* ------------------------------------------------------------------------- */

/*
 * V_HALO,n = { v in G_n : v not in V_n }: the nodes that the adjacency of the
 * partition's inner rows names and the partition does not own, in ascending
 * global id.  owner[g] = partition of node g; (rowptr, gcol) = adjacency of the
 * n_in inner rows in global ids.  Also numbers the partition's local rows:
 * pos[g] = rank of g among the partition's own nodes (ascending id) for an inner
 * node, n_in + rank in V_HALO,n for a halo node, -1 for every other node.
 * Returns |V_HALO,n|; *n_inner receives |V_n|.
 */
int64_t orc_halo_set(const int64_t *rowptr, const int32_t *gcol, int64_t n_in,
                     const int32_t *owner, int64_t n_nodes, int32_t part, int32_t *pos,
                     int32_t *halo_gid, int64_t *n_inner)
{
    int64_t inner = 0, halo = 0;
    for (int64_t g = 0; g < n_nodes; ++g) pos[g] = -1;
    for (int64_t e = 0; e < rowptr[n_in]; ++e)
        if (owner[gcol[e]] != part) pos[gcol[e]] = -2;          /* named, not owned */
    for (int64_t g = 0; g < n_nodes; ++g)
        if (owner[g] == part) ++inner;
    for (int64_t g = 0, r = 0; g < n_nodes; ++g) {
        if (owner[g] == part) pos[g] = (int32_t)r++;
        else if (pos[g] == -2) {
            halo_gid[halo] = (int32_t)g;
            pos[g] = (int32_t)(inner + halo);
            ++halo;
        }
    }
    *n_inner = inner;
    return halo;
}

/* Local column of every adjacency entry: col[e] = pos[gcol[e]]. */
void orc_relabel_columns(const int32_t *gcol, int64_t nnz, const int32_t *pos, int32_t *col)
{
    for (int64_t e = 0; e < nnz; ++e) col[e] = pos[gcol[e]];
}

/* row_of[g] = rank of node g among the nodes of its own partition (ascending id): its row
 * in the owner's inner block.  part_ptr[k] = number of nodes owned by partitions < k. */
void orc_rows_in_owner(const int32_t *owner, int64_t n_nodes, int32_t n_parts, int32_t *row_of,
                       int64_t *part_ptr)
{
    for (int32_t k = 0; k <= n_parts; ++k) part_ptr[k] = 0;
    for (int64_t g = 0; g < n_nodes; ++g) {
        row_of[g] = (int32_t)part_ptr[owner[g] + 1];
        ++part_ptr[owner[g] + 1];
    }
    for (int32_t k = 0; k < n_parts; ++k) part_ptr[k + 1] += part_ptr[k];
}

/*
 * R_k = V_HALO,n intersected with V_k, for k = 0 .. n_parts-1, each in ascending id:
 * R_halo lists the halo rows j (indices into halo_gid) of R_0, R_1, ... one after the
 * other, R_ptr[k] .. R_ptr[k+1] delimits R_k, and R_row[i] = row of that node in its
 * owner's inner block, i.e. the row the owner has to send.
 */
void orc_recv_sets(const int32_t *halo_gid, int64_t n_halo, const int32_t *owner,
                   const int32_t *row_of, int32_t n_parts, int64_t *R_ptr, int32_t *R_halo,
                   int32_t *R_row)
{
    int64_t o = 0;
    for (int32_t k = 0; k < n_parts; ++k) {
        R_ptr[k] = o;
        for (int64_t j = 0; j < n_halo; ++j)
            if (owner[halo_gid[j]] == k) {
                R_halo[o] = (int32_t)j;
                R_row[o] = row_of[halo_gid[j]];
                ++o;
            }
    }
    R_ptr[n_parts] = o;
}

/*
 * S_k = V_n intersected with V_HALO,k for one peer k: the inner rows of partition `part`
 * that peer k's halo set names, in ascending id.  peer_halo = V_HALO,k (ascending).
 * Returns |S_k|.
 */
int64_t orc_send_set(const int32_t *peer_halo, int64_t n_peer_halo, const int32_t *owner,
                     const int32_t *row_of, int32_t part, int32_t *S_row)
{
    int64_t o = 0;
    for (int64_t j = 0; j < n_peer_halo; ++j)
        if (owner[peer_halo[j]] == part) S_row[o++] = row_of[peer_halo[j]];
    return o;
}

/*
 * Transposed operator as a CSR of its own: row c of the transpose lists the entries
 * (r, c) of the operator in ascending r (the order a row-by-row sweep meets them).
 * colT[i] = r, wT[i] = w of that entry, perm[i] = its index in the operator.
 * w / wT may be NULL.
 */
void orc_transpose_csr(const int64_t *rowptr, const int32_t *col, const float *w, int64_t n_rows,
                       int64_t n_cols, int64_t *rowptrT, int32_t *colT, float *wT, int64_t *perm)
{
    for (int64_t c = 0; c <= n_cols; ++c) rowptrT[c] = 0;
    for (int64_t e = 0; e < rowptr[n_rows]; ++e) ++rowptrT[col[e] + 1];
    for (int64_t c = 0; c < n_cols; ++c) rowptrT[c + 1] += rowptrT[c];
    int64_t *next = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_cols > 0 ? n_cols : 1));
    for (int64_t c = 0; c < n_cols; ++c) next[c] = rowptrT[c];
    for (int64_t r = 0; r < n_rows; ++r)
        for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e) {
            const int64_t o = next[col[e]]++;
            colT[o] = (int32_t)r;
            if (w) wT[o] = w[e];
            perm[o] = e;
        }
    free(next);
}

/*
 * Wire rows grouped by destination row for the backward accumulate (Alg. 2, "integrate
 * gradients"): destination r receives wire rows seg_rows[seg_ptr[r] .. seg_ptr[r+1]),
 * ascending.  One segment per destination row 0 .. n_dst-1, empty ones included.
 */
void orc_scatter_segments(const int32_t *dst_row, int64_t n, int64_t n_dst, int64_t *seg_ptr,
                          int32_t *seg_rows)
{
    for (int64_t r = 0; r <= n_dst; ++r) seg_ptr[r] = 0;
    for (int64_t i = 0; i < n; ++i) ++seg_ptr[dst_row[i] + 1];
    for (int64_t r = 0; r < n_dst; ++r) seg_ptr[r + 1] += seg_ptr[r];
    int64_t *next = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_dst > 0 ? n_dst : 1));
    for (int64_t r = 0; r < n_dst; ++r) next[r] = seg_ptr[r];
    for (int64_t i = 0; i < n; ++i) seg_rows[next[dst_row[i]]++] = (int32_t)i;
    free(next);
}

/* Threads the row loops may use from now on (timing with one thread vs all cores; */
/* results do not depend on it: rows are independent and the draws are counter-based). */
void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
