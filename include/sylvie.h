/*
 * sylvie.h -- C ABI of the MI355X (gfx950) hot path of Sylvie's per-layer boundary
 * exchange on one graph partition (arXiv 2303.01277): the Low-bit Module
 * (1-bit quantizer / dequantizer, Sec. 3.2, Eq. 3-5) and the partition-local
 * layer it feeds (CSR neighbour aggregation and dense transform, Alg. 1 / Alg. 2).
 *
 * Conventions (all entry points)
 *   - Every pointer is DEVICE memory owned by the caller unless the parameter
 *     says "host".  The library never allocates, frees or keeps a pointer (one exception,
 *     switched on by the caller: sylvie_seed_offset_source).
 *   - Matrices are row-major float32; `ld_*` is the distance between rows in
 *     elements (>= the number of columns used).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.  Buffers must
 *     stay valid and unaliased (except where stated) until that work is done.
 *   - Return value: SYLVIE_OK or a negative SYLVIE_ERR_* code; nothing is
 *     enqueued when an error is returned.  sylvie_last_error() gives a
 *     thread-local text for the last failing call.
 *   - Sizes of zero rows are valid no-ops.  Inputs must be finite with
 *     |x| < 2^126; row indices must be in range (not checked on the device).
 *   - Debug mode: with the environment variable SYLVIE_VALIDATE set to 1, the quantizers, the
 *     backward dequantizer and the aggregations first check those preconditions on the device
 *     (quantizer source rows finite and below 2^126, gather indices >= 0; CSR row pointers
 *     ascending, columns >= 0 and, for sylvie_aggregate_csr_fwd_wire, below n_dense + n_wire
 *     with every dense column before every wire column of its row; segment tables ascending
 *     with wire rows in range).  Such a call WAITS for `stream`, and returns
 *     SYLVIE_ERR_INVALID_ARG without enqueueing its work when a check fails.  Upper bounds are
 *     only checked where the call states the row count of the array an index points into.
 *
 * Wire format of one exchange of n_rows rows of width d (Sec. 3.2, "1-bit
 * integers" plus the scale / zero-point side channel): one contiguous array
 *   wire : uint64 [n_rows][W + 1], W = ceil(d/64), little-endian
 *     words 0..W-1 : the bits; bit j (LSB = 0) of word k is column 64k + j; bits of
 *                    columns >= d are 0
 *     word W       : the error-compensation pair of the row, scale in bits 0..31
 *                    and zero-point in bits 32..63, both float32:
 *                    scale = max - min (B = 2^1 - 1 = 1), zero = min (-0 stored as +0)
 * so one row (and one message to a peer) is a single contiguous run of bytes.  Every 1-bit
 * entry point takes the row stride of the array it reads or writes as `ld_wire` (64-bit
 * words; 0 means W + 1, rows back to back): a resident wire may keep its rows further
 * apart than they travel, e.g. at 8 words so that no row straddles a cache line.  Words
 * W + 1 .. ld_wire - 1 of a row are never read or written.
 */
#ifndef SYLVIE_H
#define SYLVIE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SYLVIE_OK 0
#define SYLVIE_ERR_INVALID_ARG (-1)
#define SYLVIE_ERR_BAD_ALIGNMENT (-2)
#define SYLVIE_ERR_HIP (-3)
#define SYLVIE_ERR_UNIMPLEMENTED (-4)
#define SYLVIE_ERR_WORKSPACE (-5)

/* Library version, major*10000 + minor*100 + patch. */
int32_t sylvie_version(void);
/* Static text for a status code. */
const char *sylvie_status_string(int32_t status);
/* Thread-local detail of the last error returned on this thread ("" if none). */
const char *sylvie_last_error(void);

/*
 * Seed offset in device memory, for launches recorded in a HIP graph.  The quantizing entry
 * points take their seed by value, so a recorded launch would draw the same bits on every
 * replay.  After sylvie_seed_offset_source(p), p a DEVICE pointer to one uint64, every quantizing
 * call made by this thread (sylvie_quantize_1bit_*, sylvie_quantize_bbit_*,
 * sylvie_aggregate_csr_bwd_quantize*) uses the seed `seed + *p` (wrapping), with *p read by the
 * kernel when it runs: advance *p between replays (any kernel or copy on the same stream) and
 * each replay is the call with the next seed, bit for bit what the call with that seed passed
 * by value writes.  p must stay valid while such work is pending; NULL (the initial state)
 * turns the offset off.  This is the one pointer the library keeps between calls; it is
 * thread-local, like the error text.
 */
int32_t sylvie_seed_offset_source(const uint64_t *offset);

/* uint64 words of one wire row: ceil(d / 64) + 1 (the smallest ld_wire). */
int64_t sylvie_wire_row_words(int32_t d);

/*
 * Quantizer, forward direction (Alg. 1, "quantize([H(S_1), ..., H(S_N)])"; Eq. 3-4).
 *
 * Wire row i (0 <= i < n_rows) is source row idx[i] of `src` when idx != NULL,
 * else source row row_offset + i.  Per row, in float32:
 *     mn = min_c r_c, mx = max_c r_c (each + 0.0f);  zero = mn;  scale = mx - mn
 *     u  = k / 2^24, k = 24 random bits of (seed, stream_id, i, c)
 *     bit(i, c) = [ fl(u * scale) < fl(r_c - mn) ]
 * which rounds the normalised value (r_c - mn)/(mx - mn) of Eq. 3 up to 1 with
 * probability equal to that value (Eq. 4, b = 1) and gives all-zero bits for a
 * constant row.  The random bits are a counter hash of the four keys; the same
 * keys always give the same bits.  `stream_id` separates layers and directions
 * (the callers here use 2*layer + direction).
 *
 *   src        [*, ld_src] float32, d <= ld_src, 1 <= d <= 65536
 *   idx        int32 [n_rows] or NULL; duplicates allowed
 *   n_rows     0 <= n_rows < 2^31
 *   wire_out   uint64 [n_rows][ld_wire], 8-byte aligned; a row's ceil(d/64) + 1 words
 *              come first, the rest of the row is not touched
 *   ld_wire    64-bit words from one wire row to the next; 0 = ceil(d/64) + 1 (packed).
 *              A receiver may keep its wire rows at a wider stride than they travel at:
 *              with 8 words (64 bytes) for d = 256 a row never straddles a 128-byte line,
 *              which is what the aggregation that gathers wire rows pays for per reference.
 */
int32_t sylvie_quantize_1bit_fwd(const float *src, int64_t ld_src, int32_t d,
                                 const int32_t *idx, int64_t row_offset, int64_t n_rows,
                                 uint64_t seed, uint32_t stream_id, uint64_t *wire_out,
                                 int64_t ld_wire, void *stream);

/*
 * Quantizer, backward direction (Alg. 2, "quantize([J(R_1), ..., J(R_N)])").
 * Same operation and arguments; the rows are feature gradients.  The usual call
 * passes the gradient of the halo block: idx = NULL, row_offset = number of
 * inner rows.
 */
int32_t sylvie_quantize_1bit_bwd(const float *src, int64_t ld_src, int32_t d,
                                 const int32_t *idx, int64_t row_offset, int64_t n_rows,
                                 uint64_t seed, uint32_t stream_id, uint64_t *wire_out,
                                 int64_t ld_wire, void *stream);

/*
 * Dequantizer, forward direction (Eq. 5; Alg. 1 "dequantize" + "concatenate"):
 *     dst[row_offset + i][c] = bit(i, c) ? fl(zero_i + scale_i) : zero_i,  c < d.
 * Writing at row_offset = number of inner rows places the recovered rows directly
 * below the inner rows, which is the concatenation.  Columns >= d of dst are not
 * touched.
 */
int32_t sylvie_dequantize_1bit_fwd(const uint64_t *wire, int64_t ld_wire, int64_t n_rows, int32_t d,
                                   float *dst, int64_t ld_dst, int64_t row_offset, void *stream);

/*
 * Dequantizer, backward direction (Eq. 5; Alg. 2 "integrate feature gradients",
 * J = J + R~): received gradient rows are added into the rows of `dst` they
 * belong to.  Several wire rows may belong to one destination row, so the caller
 * passes the wire rows grouped by destination:
 *     for k in [0, n_dst_rows):  r = dst_ids[k]
 *         acc = dst[r][:]
 *         for j in [seg_ptr[k], seg_ptr[k+1]):  acc = fl(acc + deq(seg_rows[j])[:])
 *         dst[r][:] = acc
 * With seg_rows ascending inside each group this equals "for i ascending:
 * dst[dst_row[i]] += deq(i)" bit for bit, with no atomics.
 *
 *   seg_ptr   int64 [n_dst_rows + 1], seg_ptr[0] = 0, seg_ptr[n_dst_rows] <= n_rows
 *   seg_rows  int32 [seg_ptr[n_dst_rows]], wire row indices in [0, n_rows)
 *   dst_ids   int32 [n_dst_rows], distinct rows of dst
 */
int32_t sylvie_dequantize_1bit_bwd(const uint64_t *wire, int64_t ld_wire, int64_t n_rows, int32_t d,
                                   float *dst, int64_t ld_dst, const int64_t *seg_ptr,
                                   const int32_t *seg_rows, int64_t n_dst_rows,
                                   const int32_t *dst_ids, void *stream);

/*
 * b-bit Low-bit Module (Sec. 3.2, Eq. 3-5 with B = 2^b - 1 bins; the bit-width study of
 * Sec. 4.3, which also has a half-precision and a full-precision point).  `bits` is 1, 2, 4 or
 * 8 for b-bit stochastic rounding, 16 for IEEE binary16 (round to nearest even, no side channel,
 * seed ignored), or 32 for the vanilla exchange: the float rows themselves, unchanged (seed
 * ignored).  bits = 1 is exactly the 1-bit entry points above.
 *
 * Arithmetic for bits in {2, 4, 8}, single precision, one operation each:
 *   mn, mx as for 1 bit;  range = mx - mn;  zero = mn;  scale = range / B;
 *   g = 2^64 if range < 2^-60 else 1;  inv = B / (range * g), 0 for a constant row;
 *   t = min(((x - mn) * g) * inv, B);  q = floor(t) + [k * 2^-24 < t - floor(t)]
 * with k the 24-bit draw of (seed, stream_id, wire row i, column c), the same draws as
 * the 1-bit quantizer.  Recovered value (Eq. 5): fl(fl(scale * q) + zero).
 *
 * Wire row for bits in {2, 4, 8}: uint64 [ceil(d * bits / 64) + 1]; the code of column
 * c is bits [bits * (c mod 64/bits), + bits) of word c / (64/bits), unused high codes
 * are 0; the last word is scale | zero << 32 as for 1 bit.  Wire row for bits = 16:
 * uint64 [ceil(d / 4)] holding d binary16 values in column order, zero padded; for bits = 32:
 * uint64 [ceil(d / 2)] holding the d floats, zero padded.
 * sylvie_wire_row_words_bits returns that word count (0 for an invalid argument).
 *
 * All other arguments, row selection, destinations, ordering and error behaviour are
 * those of the 1-bit entry points of the same direction.
 */
size_t sylvie_wire_row_words_bits(int32_t d, int32_t bits);
int32_t sylvie_quantize_bbit_fwd(const float *src, int64_t ld_src, int32_t d, const int32_t *idx,
                                 int64_t row_offset, int64_t n_rows, int32_t bits, uint64_t seed,
                                 uint32_t stream_id, uint64_t *wire_out, void *stream);
int32_t sylvie_quantize_bbit_bwd(const float *src, int64_t ld_src, int32_t d, const int32_t *idx,
                                 int64_t row_offset, int64_t n_rows, int32_t bits, uint64_t seed,
                                 uint32_t stream_id, uint64_t *wire_out, void *stream);
int32_t sylvie_dequantize_bbit_fwd(const uint64_t *wire, int64_t n_rows, int32_t d, int32_t bits,
                                   float *dst, int64_t ld_dst, int64_t row_offset, void *stream);
int32_t sylvie_dequantize_bbit_bwd(const uint64_t *wire, int64_t n_rows, int32_t d, int32_t bits,
                                   float *dst, int64_t ld_dst, const int64_t *seg_ptr,
                                   const int32_t *seg_rows, int64_t n_dst_rows,
                                   const int32_t *dst_ids, void *stream);

/*
 * Neighbour aggregation, forward (Eq. 1; Alg. 1, the product A_n * H~ with A_n
 * the normalised local adjacency, Sec. 3.4):
 *     Y[v][c] = row_scale[v] * sum_{e in [rowptr[v], rowptr[v+1])}
 *                                  w[e] * col_scale[col[e]] * X[col[e]][c]
 * for v < n_rows, c < d; a NULL w / row_scale / col_scale counts as all ones.
 * float32 accumulation in a fixed order (results are reproducible run to run).
 * If `addend` != NULL, rows v < addend_rows get Y[v][c] += addend[v][c]
 * (GraphSAGE backward: the gradient of a node's own embedding).
 *
 * Rows longer than `chunk` entries are split into ceil(len/chunk) tasks whose
 * partial sums go through `workspace` and are added in task order.  The caller
 * lists those rows (built once per graph from rowptr):
 *   long_rows  int32 [n_long]   rows with len > chunk, ascending
 *   long_ptr   int64 [n_long+1] prefix sum of ceil(len/chunk) over long_rows
 *   n_tasks    = long_ptr[n_long] (host value)
 *   workspace  float32 [n_tasks][d] (workspace_bytes >= n_tasks*d*4), 16-byte aligned
 * With n_long = 0 these may be NULL / 0 and every row is summed by one wavefront.
 * chunk must be a positive multiple of 64.
 *
 * Processing order (optional, every aggregation entry point takes it): row_order int32
 * [n_rows], a permutation of [0, n_rows); wavefront i of the launch sums row
 * row_begin + row_order[i] (row_begin = 0 where the call has no such argument).  NULL = rows
 * in index order.  Results do not depend on it bit for bit - every row is still summed by one
 * wavefront (or its tasks) in entry order - only the traffic between the caches and memory
 * does: rows handed out longest first reach a higher hit rate in the L2s on power-law
 * graphs (sylvie_graph_rows_by_length builds that order).
 *
 *   rowptr int64 [n_rows+1]; col int32 [nnz] in [0, rows of X)
 */
int32_t sylvie_aggregate_csr_fwd(const int64_t *rowptr, const int32_t *col, const float *w,
                                 const float *row_scale, const float *col_scale,
                                 int64_t n_rows, const float *X, int64_t ld_x, int32_t d,
                                 float *Y, int64_t ld_y, const float *addend,
                                 int64_t ld_addend, int64_t addend_rows, const int32_t *row_order, int32_t chunk,
                                 const int32_t *long_rows, const int64_t *long_ptr,
                                 int64_t n_long, int64_t n_tasks, float *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * sylvie_aggregate_csr_fwd for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same operation, same kernels, same results bit for bit; the partial sums of the
 * long rows' tasks go to a scratch array that is part of the library's device image
 * (SYLVIE_STATIC_SCRATCH_BYTES per GPU, resident until the process ends) instead of a caller
 * workspace.  The call allocates and frees nothing.
 *   - n_tasks * d * 4 must not exceed SYLVIE_STATIC_SCRATCH_BYTES: SYLVIE_ERR_WORKSPACE
 *     otherwise (nothing is enqueued).  With n_long = 0 the scratch is not used.
 *   - The scratch needs no clearing: every task writes its whole partial row before the
 *     reduction reads it, and nothing else is read.  It keeps the last call's contents.
 *   - All calls on one GPU share that GPU's array: two calls whose work overlaps in time on the
 *     same GPU (different streams) race.  Calls on one stream are ordered and safe.
 *   - The device address of the array is looked up on the first call on each device (the
 *     device current at the call, which must be the stream's).
 * Other arguments as in sylvie_aggregate_csr_fwd.
 */
#define SYLVIE_STATIC_SCRATCH_BYTES (16ull << 20)
int32_t sylvie_aggregate_csr_fwd_noalloc(const int64_t *rowptr, const int32_t *col, const float *w,
                                         const float *row_scale, const float *col_scale,
                                         int64_t n_rows, const float *X, int64_t ld_x, int32_t d,
                                         float *Y, int64_t ld_y, const float *addend,
                                         int64_t ld_addend, int64_t addend_rows, const int32_t *row_order, int32_t chunk,
                                         const int32_t *long_rows, const int64_t *long_ptr,
                                         int64_t n_long, int64_t n_tasks, void *stream);

/*
 * Neighbour aggregation, forward, reading the halo rows straight from the wire
 * (Alg. 1 "dequantize" + "concatenate" + the product A_n * H~ in one pass; Eq. 5
 * is applied to each gathered element): the same result as
 * sylvie_dequantize_1bit_fwd into rows n_dense.. of X followed by
 * sylvie_aggregate_csr_fwd, without ever materialising the dequantized rows.
 *     column c <  n_dense : row c of X (float32, as above)
 *     column c >= n_dense : wire row c - n_dense of `wire`, width d
 * Inside every CSR row all columns < n_dense must precede all columns >= n_dense
 * (true when columns are ascending).  n_wire = number of wire rows (0: plain X).
 * Other arguments as in sylvie_aggregate_csr_fwd (no addend).
 */
int32_t sylvie_aggregate_csr_fwd_wire(const int64_t *rowptr, const int32_t *col, const float *w,
                                      const float *row_scale, const float *col_scale,
                                      int64_t n_rows, const float *X, int64_t ld_x, int32_t d,
                                      int64_t n_dense, const uint64_t *wire, int64_t ld_wire,
                                      int64_t n_wire, float *Y, int64_t ld_y, const int32_t *row_order, int32_t chunk,
                                      const int32_t *long_rows,
                                      const int64_t *long_ptr, int64_t n_long, int64_t n_tasks,
                                      float *workspace, size_t workspace_bytes, void *stream);

/*
 * Neighbour aggregation, backward (Alg. 2, the product A_n^T * (J o sigma') W^T,
 * here its sparse factor): the same operation applied to the CSR of the
 * transposed operator, whose rows are ALL local rows (inner and halo) and whose
 * columns are the inner rows, so that dX = A^T dY.  The halo block of dX is what
 * the backward quantizer sends.  Arguments as in the forward call.
 */
int32_t sylvie_aggregate_csr_bwd(const int64_t *rowptrT, const int32_t *colT, const float *wT,
                                 const float *row_scale, const float *col_scale,
                                 int64_t n_rowsT, const float *dY, int64_t ld_dy, int32_t d,
                                 float *dX, int64_t ld_dx, const float *addend,
                                 int64_t ld_addend, int64_t addend_rows, const int32_t *row_order, int32_t chunk,
                                 const int32_t *long_rows, const int64_t *long_ptr,
                                 int64_t n_long, int64_t n_tasks, float *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * Neighbour aggregation, backward, halo block, quantized on the spot (Alg. 2 "compute
 * feature gradients" restricted to the rows that are sent, fused with "quantize"):
 * the same wire as sylvie_aggregate_csr_bwd into a float block followed by
 * sylvie_quantize_1bit_bwd of that block (idx = NULL), bit for bit, but the float
 * rows never reach memory.  Rows row_begin .. row_begin + n_rows - 1 of the
 * transposed operator are computed; wire row i is row row_begin + i and takes the
 * random draws of wire row i.  rowptrT is indexed by the absolute row; long_rows
 * holds absolute rows inside the range.  d <= 2048.
 *   wire_out uint64 [n_rows][ceil(d/64) + 1]
 */
int32_t sylvie_aggregate_csr_bwd_quantize(const int64_t *rowptrT, const int32_t *colT,
                                          const float *wT, const float *row_scale,
                                          const float *col_scale, int64_t row_begin,
                                          int64_t n_rows, const float *dY, int64_t ld_dy,
                                          int32_t d, uint64_t seed, uint32_t stream_id,
                                          uint64_t *wire_out, int64_t ld_wire, const int32_t *row_order, int32_t chunk,
                                          const int32_t *long_rows, const int64_t *long_ptr,
                                          int64_t n_long, int64_t n_tasks, float *workspace,
                                          size_t workspace_bytes, void *stream);

/*
 * Neighbour aggregation, backward, inner block, with the received gradients added
 * (Alg. 2 "compute feature gradients" fused with "dequantize" and "integrate"):
 *     dX[v] = (A^T dY)[v] (+ addend[v]) , then for j in [seg_ptr[v - row_begin],
 *     seg_ptr[v - row_begin + 1]):  dX[v] = fl(dX[v] + deq(wire row seg_rows[j]))
 * for rows v = row_begin .. row_begin + n_rows - 1: the same values as
 * sylvie_aggregate_csr_bwd followed by sylvie_dequantize_1bit_bwd, bit for bit, with
 * one store per row.
 *   seg_ptr  int64 [n_rows + 1] (every row has an entry; empty segments allowed)
 *   seg_rows int32 [seg_ptr[n_rows]] wire rows, ascending inside a segment
 */
int32_t sylvie_aggregate_csr_bwd_integrate(const int64_t *rowptrT, const int32_t *colT,
                                           const float *wT, const float *row_scale,
                                           const float *col_scale, int64_t row_begin,
                                           int64_t n_rows, const float *dY, int64_t ld_dy,
                                           int32_t d, float *dX, int64_t ld_dx,
                                           const float *addend, int64_t ld_addend,
                                           int64_t addend_rows, const uint64_t *wire,
                                           int64_t ld_wire, int64_t n_wire, const int64_t *seg_ptr,
                                           const int32_t *seg_rows, const int32_t *row_order, int32_t chunk,
                                           const int32_t *long_rows, const int64_t *long_ptr,
                                           int64_t n_long, int64_t n_tasks, float *workspace,
                                           size_t workspace_bytes, void *stream);

/*
 * The three fused aggregation calls above for the wider wires of the bit-width study (Sec. 4.3;
 * Eq. 3-5 with B = 2^bits - 1): `bits` is 1, 2, 4, 8 (1 = the calls above) or 16 (the study's
 * half-precision point: binary16 rows, no rounding draws, no metadata word) and `wire` /
 * `wire_out` hold rows in the format of sylvie_quantize_bbit_* (ceil(d bits / 64) code words and
 * the scale | zero word, or ceil(d / 4) words of halves; ld_wire = words from one row to the
 * next, 0 = packed).
 *   - sylvie_aggregate_csr_fwd_wire_bbit: a gathered halo element is fl(fl(scale q) + zero)
 *     (Eq. 5), then weighted and summed as every other element; the same result as
 *     sylvie_dequantize_bbit_fwd followed by sylvie_aggregate_csr_fwd up to the order of the
 *     single-precision additions.
 *   - sylvie_aggregate_csr_bwd_quantize_bbit: the same wire, bit for bit, as
 *     sylvie_aggregate_csr_bwd followed by sylvie_quantize_bbit_bwd of the row block.
 *   - sylvie_aggregate_csr_bwd_integrate_bbit: the same rows, bit for bit, as
 *     sylvie_aggregate_csr_bwd followed by sylvie_dequantize_bbit_bwd.
 * For bits > 1 the float rows must be 16-byte aligned with d and the leading dimensions
 * multiples of 4 (SYLVIE_ERR_UNIMPLEMENTED otherwise: use the separate calls).
 */
int32_t sylvie_aggregate_csr_fwd_wire_bbit(const int64_t *rowptr, const int32_t *col, const float *w,
                                           const float *row_scale, const float *col_scale,
                                           int64_t n_rows, const float *X, int64_t ld_x, int32_t d,
                                           int32_t bits, int64_t n_dense, const uint64_t *wire,
                                           int64_t ld_wire, int64_t n_wire, float *Y, int64_t ld_y,
                                           const int32_t *row_order, int32_t chunk,
                                           const int32_t *long_rows, const int64_t *long_ptr,
                                           int64_t n_long, int64_t n_tasks, float *workspace,
                                           size_t workspace_bytes, void *stream);
int32_t sylvie_aggregate_csr_bwd_quantize_bbit(const int64_t *rowptrT, const int32_t *colT,
                                               const float *wT, const float *row_scale,
                                               const float *col_scale, int64_t row_begin,
                                               int64_t n_rows, const float *dY, int64_t ld_dy,
                                               int32_t d, int32_t bits, uint64_t seed,
                                               uint32_t stream_id, uint64_t *wire_out, int64_t ld_wire,
                                               const int32_t *row_order, int32_t chunk,
                                               const int32_t *long_rows, const int64_t *long_ptr,
                                               int64_t n_long, int64_t n_tasks, float *workspace,
                                               size_t workspace_bytes, void *stream);
int32_t sylvie_aggregate_csr_bwd_integrate_bbit(const int64_t *rowptrT, const int32_t *colT,
                                                const float *wT, const float *row_scale,
                                                const float *col_scale, int64_t row_begin,
                                                int64_t n_rows, const float *dY, int64_t ld_dy,
                                                int32_t d, int32_t bits, float *dX, int64_t ld_dx,
                                                const float *addend, int64_t ld_addend,
                                                int64_t addend_rows, const uint64_t *wire,
                                                int64_t ld_wire, int64_t n_wire,
                                                const int64_t *seg_ptr, const int32_t *seg_rows,
                                                const int32_t *row_order, int32_t chunk,
                                                const int32_t *long_rows, const int64_t *long_ptr,
                                                int64_t n_long, int64_t n_tasks, float *workspace,
                                                size_t workspace_bytes, void *stream);

/*
 * Dense transform, forward (Eq. 2; Alg. 1 "update embeddings", H = sigma(Z W)):
 *     P = [A1 | A2] * W,   H = relu ? max(P, 0) : P
 * A1 is n x k1 (ld_a1), A2 is n x k2 (ld_a2) or NULL with k2 = 0 (GraphSAGE puts a
 * node's own embedding next to the neighbour mean); W is (k1+k2) x h, row-major,
 * contiguous; H is n x h (ld_h).  float32 inputs, float32 MFMA accumulation.
 * k1, k2 and h must be multiples of 4 and all pointers 16-byte aligned.
 */
int32_t sylvie_transform_fwd(const float *A1, int64_t ld_a1, int32_t k1, const float *A2,
                             int64_t ld_a2, int32_t k2, const float *W, int32_t h, int64_t n,
                             int32_t relu, float *H, int64_t ld_h, void *stream);

/* Bytes of workspace sylvie_transform_bwd needs for the weight gradient. */
size_t sylvie_transform_bwd_workspace_bytes(int32_t k1, int32_t k2, int32_t h, int64_t n);

/*
 * Dense transform, backward (Alg. 2 "compute weight gradients" and the dense
 * factor of "compute feature gradients"):
 *     M  = relu ? J o [H > 0] : J            (H is the forward output)
 *     G  = [A1 | A2]^T * M     ((k1+k2) x h, contiguous)        if G   != NULL
 *     dA = M * W^T             (n x (k1+k2), written as the two blocks
 *                               dA1 (ld_da1) and dA2 (ld_da2))    if dA1 != NULL
 * The weight gradient is summed over row slabs through `workspace`
 * (sylvie_transform_bwd_workspace_bytes) in a fixed order.
 */
int32_t sylvie_transform_bwd(const float *A1, int64_t ld_a1, int32_t k1, const float *A2,
                             int64_t ld_a2, int32_t k2, const float *W, int32_t h, int64_t n,
                             int32_t relu, const float *H, int64_t ld_h, const float *J,
                             int64_t ld_j, float *G, float *dA1, int64_t ld_da1, float *dA2,
                             int64_t ld_da2, float *workspace, size_t workspace_bytes,
                             void *stream);

/*
 * Loss and its gradient (Alg. 1, last line: L = Loss(softmax(H^(L)), Y); Alg. 2:
 * J^(L) = dL/dH^(L)).  Softmax cross-entropy over the labelled rows, divided by `count`,
 * the number of labelled nodes of the whole graph (so partition losses and gradients add
 * up to the unpartitioned ones):
 *     p = softmax(H[i][0 .. n_classes)),  loss_i = -log p[label[i]] / count,
 *     J[i][c] = (p[c] - [c == label[i]]) / count;   label[i] < 0: row unlabelled, J row = 0.
 * Single precision.  loss_rows float [n] is scratch that receives loss_i; loss_out double
 * [1] (device memory) receives their sum, added in double in a fixed order.
 */
int32_t sylvie_softmax_xent(const float *H, int64_t ld_h, int64_t n, int32_t n_classes,
                            const int32_t *label, double count, float *J, int64_t ld_j,
                            float *loss_rows, double *loss_out, void *stream);

/*
 * Gradient synchronisation inside one process (Alg. 2, G = AllReduce(G_n), for partitions
 * that share a GPU): dst[e] = ((srcs[0][e] + srcs[1][e]) + ...) in single precision, in
 * that order.  srcs is a HOST array of n_src (1..16) device pointers; dst may be srcs[0].
 */
int32_t sylvie_sum_gradients(float *dst, const float *const *srcs, int32_t n_src, int64_t elems,
                             void *stream);

/* Model update (Alg. 2, W_t = W_{t-1} - eta G): W[e] = fl(W[e] - fl(eta * G[e])). */
int32_t sylvie_sgd_update(float *W, const float *G, int64_t elems, float eta, void *stream);

/*
 * Attention aggregator: the GAT model of the evaluation (Sec. 4), i.e. Eq. 1 with learned
 * edge weights.  The paper cites the model without formulas; these are the cited model's:
 *     P = H~ W,  s_dst[v] = P_v . a_dst,  s_src[u] = P_u . a_src,
 *     alpha_v. = softmax over the entries (v, u) of row v of leaky_relu(s_dst[v] + s_src[u]),
 *     z_v = sum_u alpha_vu P_u       (sylvie_aggregate_csr_fwd with w = alpha)
 * and backward
 *     dalpha_vu = dZ_v . P_u (sylvie_sddmm),  g = alpha (dalpha - sum_row alpha dalpha),
 *     de = g * (s_dst[v] + s_src[u] > 0 ? 1 : slope)            (sylvie_edge_softmax_bwd),
 *     ds_dst = row sums of de, ds_src = column sums of de        (sylvie_segment_sum on the
 *     operator and, after sylvie_permute_f32, on its transpose),
 *     dP = A^T(alpha) dZ + ds_src (x) a_src + ds_dst (x) a_dst   (sylvie_aggregate_csr_bwd,
 *     sylvie_rank1_add).
 *
 * Piece table (built at set-up, shared by these calls): every row's entries are cut into
 * pieces of at most `chunk` consecutive entries, one wavefront per piece; rows without
 * entries have no piece.
 *     piece_ptr int64 [n_pieces + 1]  entry offsets, ascending, piece k = [piece_ptr[k], piece_ptr[k+1])
 *     piece_row int32 [n_pieces]      row of piece k
 *     row_piece int64 [n_rows + 1]    pieces of row v = [row_piece[v], row_piece[v+1])
 * Row-wide quantities are reduced per piece and joined per row in piece order (no atomics).
 * `col` is the operator's column array (entry e of the CSR the pieces were cut from).
 * Workspaces are caller-owned device memory: sylvie_edge_softmax_workspace_bytes for the two
 * softmax calls (the backward needs (n_pieces + n_rows) floats, which is less),
 * n_pieces floats for sylvie_segment_sum.
 */
int32_t sylvie_row_dot(const float *P, int64_t ld_p, int64_t n, int32_t F, const float *a, float *out,
                       void *stream);
size_t sylvie_edge_softmax_workspace_bytes(int64_t n_pieces, int64_t n_rows);
int32_t sylvie_edge_softmax_fwd(const int64_t *piece_ptr, const int32_t *piece_row,
                                const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                const int32_t *col, const float *s_dst, const float *s_src, float slope,
                                float *alpha, void *workspace, size_t workspace_bytes, void *stream);
int32_t sylvie_sddmm(const int64_t *piece_ptr, const int32_t *piece_row, const int64_t *row_piece,
                     int64_t n_pieces, int64_t n_rows, const int32_t *col, const float *A, int64_t ld_a,
                     const float *B, int64_t ld_b, int32_t F, float *out, void *stream);
int32_t sylvie_edge_softmax_bwd(const int64_t *piece_ptr, const int32_t *piece_row,
                                const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                const int32_t *col, const float *alpha, const float *dalpha,
                                const float *s_dst, const float *s_src, float slope, float *de,
                                void *workspace, size_t workspace_bytes, void *stream);
int32_t sylvie_segment_sum(const int64_t *piece_ptr, const int32_t *piece_row, const int64_t *row_piece,
                           int64_t n_pieces, int64_t n_rows, const float *vals, float *out,
                           void *workspace, size_t workspace_bytes, void *stream);
/* out[c] = sum_{i < n} s[i] * X[i][c], c < F: the gradients of the attention vectors
 * (da_dst = sum_v ds_dst[v] P_v, da_src = sum_u ds_src[u] P_u).  The order of the additions is
 * fixed (slabs of 2048 rows, sixteen interleaved partial sums per slab, slabs joined in
 * ascending order), so results repeat bit for bit.  Workspace: see the size query. */
size_t sylvie_scaled_column_sum_workspace_bytes(int64_t n, int32_t F);
int32_t sylvie_scaled_column_sum(const float *X, int64_t ld_x, int64_t n, int32_t F, const float *s,
                                 float *out, void *workspace, size_t workspace_bytes, void *stream);
/* out[i] = in[perm[i]], i < n (edge values from operator order into transposed-operator order). */
int32_t sylvie_permute_f32(const float *in, const int64_t *perm, int64_t n, float *out, void *stream);
/* X[i][c] = fl(X[i][c] + fl(s[i] * a[c])), i < n, c < F. */
int32_t sylvie_rank1_add(float *X, int64_t ld_x, int64_t n, int32_t F, const float *s, const float *a,
                         void *stream);
/* H = max(Z, 0);  dZ = H > 0 ? J : 0 (the activation sits after the aggregation in this model). */
int32_t sylvie_relu_fwd(const float *Z, int64_t ld_z, int64_t n, int32_t F, float *H, int64_t ld_h,
                        void *stream);
int32_t sylvie_relu_bwd(const float *H, int64_t ld_h, const float *J, int64_t ld_j, int64_t n, int32_t F,
                        float *dZ, int64_t ld_dz, void *stream);

/*
 * The same attention aggregator (GAT, Sec. 4) for `heads` = K attention heads at once.  The
 * heads share the projection column-wise: head k owns columns [k F, (k+1) F) of P and of the
 * attention vectors a_dst / a_src (each K F long).  Per-node arrays hold a node's K values side
 * by side (s_dst, ds_dst: [n_rows][K]; s_src: [number of columns][K]), per-entry arrays an
 * entry's K values (alpha, dalpha, de: [entries][K]), so an entry's column index and its
 * node's scores are fetched once for all heads.  Per head the arithmetic and its order are
 * those of the single-head calls above, which are these with K = 1: results agree bit for bit
 * with K single-head calls on the head's own slices (tested).
 *
 * K is 1, 2, 4 or 8 (sylvie_row_dot_heads, sylvie_sddmm_heads and sylvie_scaled_column_sum_heads:
 * any K); per-node and per-entry arrays of a K-head call must be 4 K-byte aligned
 * (SYLVIE_ERR_BAD_ALIGNMENT otherwise).
 *
 *   sylvie_row_dot_heads           out[i][k] = P[i][k F .. (k+1) F) . a[k F .. (k+1) F), i < n; with a2
 *                                  (may be NULL) also out2[i][k] with a2 for i < n2, from the same
 *                                  pass over P (s_dst over the inner rows and s_src over all rows)
 *   sylvie_edge_softmax_fwd_heads  alpha[e][k]; workspace sylvie_edge_softmax_heads_workspace_bytes
 *   sylvie_sddmm_heads             out[e][k] = A_v[k F ..) . B_u[k F ..) for entry e = (v, u)
 *   sylvie_edge_softmax_bwd_heads  de[e][k]; if ds_dst is not NULL also ds_dst[v][k] = the row sums
 *                                  of de (what sylvie_segment_sum_heads would return, bit for bit);
 *                                  workspace (n_pieces + n_rows) K floats, 4 K-byte aligned
 *   sylvie_segment_sum_heads       out[v][k] = sum over the entries e of row v of vals[i_e][k],
 *                                  i_e = e, or index[e] when `index` (int64 [entries]) is given:
 *                                  with the pieces of the TRANSPOSED operator and the
 *                                  transposition's entry map as index these are the column sums of
 *                                  values left in forward entry order (ds_src from de);
 *                                  workspace n_pieces K floats
 *   sylvie_scaled_column_sum_heads out[c] = sum_{i < n} s[i][c / (F / K)] X[i][c], c < F (F = all
 *                                  K heads' columns here); with s2 (may be NULL) also out2 from s2
 *                                  over i < n2 in the same pass over X; each sum has the value and
 *                                  bits it has alone.  Workspace: the single-head query for
 *                                  max(n, n2) rows, twice that with s2
 */
int32_t sylvie_row_dot_heads(const float *P, int64_t ld_p, int64_t n, int32_t F, int32_t heads,
                             const float *a, float *out, const float *a2, int64_t n2, float *out2,
                             void *stream);
size_t sylvie_edge_softmax_heads_workspace_bytes(int64_t n_pieces, int64_t n_rows, int32_t heads);
int32_t sylvie_edge_softmax_fwd_heads(const int64_t *piece_ptr, const int32_t *piece_row,
                                      const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                      const int32_t *col, const float *s_dst, const float *s_src,
                                      int32_t heads, float slope, float *alpha, void *workspace,
                                      size_t workspace_bytes, void *stream);
int32_t sylvie_sddmm_heads(const int64_t *piece_ptr, const int32_t *piece_row, const int64_t *row_piece,
                           int64_t n_pieces, int64_t n_rows, const int32_t *col, const float *A,
                           int64_t ld_a, const float *B, int64_t ld_b, int32_t F, int32_t heads,
                           float *out, void *stream);
int32_t sylvie_edge_softmax_bwd_heads(const int64_t *piece_ptr, const int32_t *piece_row,
                                      const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                      const int32_t *col, const float *alpha, const float *dalpha,
                                      const float *s_dst, const float *s_src, int32_t heads, float slope,
                                      float *de, float *ds_dst, void *workspace, size_t workspace_bytes,
                                      void *stream);
int32_t sylvie_segment_sum_heads(const int64_t *piece_ptr, const int32_t *piece_row,
                                 const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                 const float *vals, const int64_t *index, int32_t heads, float *out,
                                 void *workspace, size_t workspace_bytes, void *stream);
int32_t sylvie_scaled_column_sum_heads(const float *X, int64_t ld_x, int64_t n, int32_t F, int32_t heads,
                                       const float *s, float *out, const float *s2, int64_t n2,
                                       float *out2, void *workspace, size_t workspace_bytes,
                                       void *stream);

/*
 * Aggregation of the attention model (GAT, Sec. 4; Eq. 1 with learned edge weights), all heads
 * in one launch:
 *     Y[v][c] = act( sum_e w[i_e][c / F] X[col_e][c]  +  s1[v][c / F] a1[c]  +  s2[v][c / F] a2[c] )
 * over the entries e of row v of the CSR (rowptr, col); F = d / heads; i_e = e, or w_index[e]
 * when w_index (int64 [entries]) is given.  Forward: w = alpha, Y = Z (relu != 0: Y = max(Z, 0),
 * the hidden layers' activation).  Backward: (rowptr, col) is the transposed operator, w still
 * alpha in forward entry order, w_index the transposition's entry map, X = dZ, and the two
 * rank-1 terms add the gradient that reaches P through the scores (s1 = ds_src [n1][heads] with
 * a1 = a_src on rows [0, n1), s2 = ds_dst with a2 = a_dst on rows [0, n2)); each term is a
 * single-precision product and add, term 1 first, as two sylvie_rank1_add calls would do.
 * Either term may be NULL.  heads is 1 .. 8 and divides d; the sums are accumulated entry by
 * entry in ascending order with one FMA per element; long rows, chunk, the task plan and the
 * workspace (n_tasks * d floats, 16-byte aligned) are those of sylvie_aggregate_csr_fwd.
 * SYLVIE_ERR_UNIMPLEMENTED if d is wider than one launch covers (2048 columns for 16-byte
 * aligned rows whose F is a multiple of 4).
 */
/* X[i][c] = fl(fl(X[i][c] + fl(s1[i][c / (F / K)] a1[c])) + fl(s2[i][c / (F / K)] a2[c])): the two
 * rank-1 terms of the attention backward (dP += ds_src (x) a_src + ds_dst (x) a_dst) for K heads in
 * one pass, term 1 on rows [0, n1), term 2 on rows [0, n2); F = all heads' columns; either term
 * may be NULL.  Equal bit for bit to sylvie_rank1_add per head and term, term 1 first. */
int32_t sylvie_rank1_add_heads(float *X, int64_t ld_x, int32_t F, int32_t heads, const float *s1,
                               const float *a1, int64_t n1, const float *s2, const float *a2, int64_t n2,
                               void *stream);

int32_t sylvie_aggregate_csr_attention(const int64_t *rowptr, const int32_t *col, const float *w,
                                       const int64_t *w_index, int32_t heads, int64_t n_rows,
                                       const float *X, int64_t ld_x, int32_t d, float *Y, int64_t ld_y,
                                       const float *s1, const float *a1, int64_t n1, const float *s2,
                                       const float *a2, int64_t n2, int32_t relu, int32_t chunk,
                                       const int32_t *long_rows, const int64_t *long_ptr, int64_t n_long,
                                       int64_t n_tasks, float *workspace, size_t workspace_bytes,
                                       void *stream);

/*
 * The transposed aggregation of the attention backward together with the sampled product of the
 * softmax backward (GAT, Sec. 4): over the rows u of the transposed operator (rowptr, col),
 *     Y[u][c]        = sum_e w[i_e][c / F] X[col_e][c]                    (dP without its rank-1 terms)
 *     dalpha[i_e][k] = X[col_e][k F .. (k+1) F) . B[u][k F .. (k+1) F)    (dalpha_vu = dZ_v . P_u)
 * with X = dZ, B = P and i_e = w_index[e] (the forward entry of transposed entry e; i_e = e when
 * w_index is NULL).  The wavefront of row u gathers the rows dZ_v once for both results; the
 * product is what sylvie_sddmm_heads computes over the forward pattern, entry by entry, with the
 * additions of a dot product in another order (four adjacent columns per lane, then the lanes of
 * the head pairwise).  Every entry of dalpha named by the pattern is written, once.  Follow it
 * with sylvie_edge_softmax_bwd_heads and sylvie_rank1_add_heads.
 * Shapes: d <= 256 and F = d / heads one of 16, 32, 64, 128, 256 (ask
 * sylvie_aggregate_csr_attention_sddmm_supported, which returns 1 or 0; otherwise
 * SYLVIE_ERR_UNIMPLEMENTED); rows of X, Y and B 16-byte aligned with leading dimensions that are
 * multiples of 4.  Long rows, chunk, plan and workspace as for sylvie_aggregate_csr_attention.
 */
int32_t sylvie_aggregate_csr_attention_sddmm_supported(int32_t d, int32_t heads);
int32_t sylvie_aggregate_csr_attention_sddmm(const int64_t *rowptr, const int32_t *col, const float *w,
                                             const int64_t *w_index, int32_t heads, int64_t n_rows,
                                             const float *X, int64_t ld_x, int32_t d, float *Y,
                                             int64_t ld_y, const float *B, int64_t ld_b, float *dalpha,
                                             int32_t chunk, const int32_t *long_rows,
                                             const int64_t *long_ptr, int64_t n_long, int64_t n_tasks,
                                             float *workspace, size_t workspace_bytes, void *stream);

/*
 * Graph Engine set-up on the device (Sec. 3.2; Alg. 1, the lines before the epoch loop).
 * Not on the per-layer path: each call waits for `stream` before it returns, because it
 * reports counts and the result of the kernels' own range checks (a bad id gives
 * SYLVIE_ERR_INVALID_ARG, never an out-of-range access).  All arrays are device memory
 * unless named *_host; ids and rows are int32, pointers into arrays int64; item counts must
 * stay below 2^31 - 4096.  Workspace: caller-owned device memory of at least
 * sylvie_graph_workspace_bytes(n) bytes, n = the largest item count of the call (stated per
 * call); contents are scratch.
 */
size_t sylvie_graph_workspace_bytes(int64_t n);

/*
 * V_HALO,n = { v in G_n : v not in V_n } and the local numbering of partition `part`.
 * gcol int32 [nnz]: global neighbour ids of the partition's inner rows (any order);
 * owner int32 [n_nodes]: partition of every node.  Writes pos int32 [n_nodes]: the row of
 * node g in this partition = its rank among the partition's own nodes (ascending id), or
 * n_in + its rank in V_HALO,n, or -1 for a node the partition neither owns nor names; and
 * halo_gid int32 [<= halo_capacity]: V_HALO,n ascending.  counts_host int64 [2] (host)
 * receives |V_n| and |V_HALO,n|.  Fails if |V_n| != n_in or the halo set exceeds the capacity
 * (counts_host is valid then, so the caller can retry with room).  Workspace n = n_nodes.
 */
int32_t sylvie_graph_local_index(const int32_t *gcol, int64_t nnz, int64_t n_in, const int32_t *owner,
                                 int64_t n_nodes, int32_t part, int32_t *pos, int32_t *halo_gid,
                                 int64_t halo_capacity, int64_t *counts_host, void *workspace,
                                 size_t workspace_bytes, void *stream);

/* col[e] = pos[gcol[e]]: the adjacency in local rows.  Fails if an entry names a node with
 * pos < 0.  Workspace: 256 bytes. */
int32_t sylvie_graph_relabel_columns(const int32_t *gcol, int64_t nnz, const int32_t *pos, int64_t n_nodes,
                                     int32_t *col, void *workspace, size_t workspace_bytes, void *stream);

/* row_of[g] = rank of node g among the nodes of owner[g], ascending id (its row in the
 * owner's inner block); part_ptr int64 [n_parts + 1]: nodes owned by partitions < k.
 * Workspace n = n_nodes. */
int32_t sylvie_graph_rows_in_owner(const int32_t *owner, int64_t n_nodes, int32_t n_parts, int32_t *row_of,
                                   int64_t *part_ptr, void *workspace, size_t workspace_bytes, void *stream);

/*
 * R_k = V_HALO,n intersected with V_k for every partition k (Alg. 1, the receive sets):
 * R_halo int32 [n_halo] lists the halo rows j (indices into halo_gid) of R_0, R_1, ... one
 * after the other, each ascending; R_ptr int64 [n_parts + 1] delimits them; R_row[i] =
 * row_of[halo_gid[R_halo[i]]], the row the owner sends.  The send set S_k of partition n
 * toward k (V_n intersected with V_HALO,k) is the slice [R_ptr[n], R_ptr[n+1]) of R_row as
 * computed for partition k: nothing further is computed for it.  Workspace n = n_halo.
 */
int32_t sylvie_graph_recv_sets(const int32_t *halo_gid, int64_t n_halo, const int32_t *owner,
                               const int32_t *row_of, int64_t n_nodes, int32_t n_parts, int64_t *R_ptr,
                               int32_t *R_halo, int32_t *R_row, void *workspace, size_t workspace_bytes,
                               void *stream);

/*
 * The transposed operator as a CSR of its own (Alg. 2 aggregates with it): row c lists the
 * entries (r, c) of the operator in ascending entry order (ascending r).  rowptrT int64
 * [n_cols + 1], colT int32 [nnz] = r, wT = w of the entry (w and wT both NULL: no weights),
 * perm int64 [nnz] | NULL = index of the entry in the operator (valuesT = values[perm]).
 * nnz must equal rowptr[n_rows]; columns of a row need not ascend.  Workspace n = nnz.
 */
int32_t sylvie_graph_transpose_csr(const int64_t *rowptr, const int32_t *col, const float *w, int64_t n_rows,
                                   int64_t n_cols, int64_t nnz, int64_t *rowptrT, int32_t *colT, float *wT,
                                   int64_t *perm, void *workspace, size_t workspace_bytes, void *stream);

/* Wire rows grouped by destination row for the backward accumulate: destination r receives
 * wire rows seg_rows[seg_ptr[r] .. seg_ptr[r+1]), ascending; seg_ptr int64 [n_dst + 1].
 * Workspace n = n. */
int32_t sylvie_graph_scatter_segments(const int32_t *dst_row, int64_t n, int64_t n_dst, int64_t *seg_ptr,
                                      int32_t *seg_rows, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The normalised operator of a partition (Sec. 3.4: A_n = D^-1/2 (A + I) D^-1/2 restricted to
 * the partition's inner rows; Eq. 1's aggregation weights for GCN).  rowptr / col: adjacency of
 * the n_in inner rows over all n_cols local rows, no self loops, columns ascending; deg int32
 * [n_cols]: degree of every local row in the WHOLE graph, self loop not counted.  Writes
 * rowptr_out int64 [n_in + 1] (= rowptr[r] + r), col_out int32 and w_out float [nnz + n_in]:
 * every row with its self loop (r, r) merged in column order and
 * w = 1 / sqrt((deg_r + 1)(deg_c + 1)) evaluated in double precision, rounded once to float.
 * Fails on a column outside [0, n_cols) or a self loop in the input.  Workspace: 256 bytes.
 */
int32_t sylvie_graph_gcn_operator(const int64_t *rowptr, const int32_t *col, const int32_t *deg, int64_t n_in,
                                  int64_t n_cols, int64_t nnz, int64_t *rowptr_out, int32_t *col_out, float *w_out,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* GraphSAGE mean aggregator (Sec. 2.1 / Sec. 4): w_out[e] = 1 / len(row of e), evaluated in
 * double precision, rounded once to float.  Workspace: 256 bytes. */
int32_t sylvie_graph_mean_weights(const int64_t *rowptr, int64_t n_rows, int64_t nnz, float *w_out, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Launch plans of the aggregation kernels (no counterpart in the paper: how this library cuts
 * the work of Eq. 1).  All three wait for `stream`.  Workspace n = n_rows.
 *
 * sylvie_graph_long_row_plan: the rows of [row_begin, row_begin + n_rows) longer than `chunk`
 * entries, ascending, as absolute row indices in long_rows int32 [<= capacity], and long_ptr
 * int64 [n_long + 1] = prefix sum of ceil(len / chunk) over them (what the aggregation calls take);
 * counts_host int64 [2] (host) receives n_long and n_tasks.  Fails if n_long > capacity
 * (counts_host is valid then).  nnz / chunk + 1 is always room enough.
 *
 * sylvie_graph_piece_table: every row cut into pieces of at most `chunk` consecutive entries
 * (the attention kernels' work units): row_piece int64 [n_rows + 1], piece_ptr int64
 * [n_pieces + 1], piece_row int32 [n_pieces] as described above; n_pieces_host (host) receives
 * the count; capacity = room in piece_row (piece_ptr has one more).  n_rows + nnz / chunk is
 * always room enough.
 *
 * sylvie_graph_rows_by_length: order int32 [n_rows] = the rows of the range, longest first,
 * ties in index order, as indices relative to row_begin: a row_order argument of the
 * aggregation calls.
 */
int32_t sylvie_graph_long_row_plan(const int64_t *rowptr, int64_t row_begin, int64_t n_rows, int32_t chunk,
                                   int32_t *long_rows, int64_t *long_ptr, int64_t capacity, int64_t *counts_host,
                                   void *workspace, size_t workspace_bytes, void *stream);
int32_t sylvie_graph_piece_table(const int64_t *rowptr, int64_t n_rows, int32_t chunk, int64_t *row_piece,
                                 int64_t *piece_ptr, int32_t *piece_row, int64_t capacity, int64_t *n_pieces_host,
                                 void *workspace, size_t workspace_bytes, void *stream);
int32_t sylvie_graph_rows_by_length(const int64_t *rowptr, int64_t row_begin, int64_t n_rows, int32_t *order,
                                    void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SYLVIE_H */
