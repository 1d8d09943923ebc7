// Attention aggregator (the GAT model evaluated in Sec. 4; Eq. 1 with learned edge
// weights): scores, edge softmax, the product that differentiates it, and their backward.
//   s_dst[v] = P_v . a_dst, s_src[u] = P_u . a_src
//   e_vu = leaky_relu(s_dst[v] + s_src[u]); alpha_v. = softmax over the entries of row v
//   backward: dalpha_vu = dZ_v . P_u; g = alpha (dalpha - sum_row alpha dalpha);
//             de = g * leaky_relu'(.); ds_dst = row sums of de, ds_src = column sums of de
// The weighted sums themselves (Z = sum alpha P_u and its transpose) are the ordinary CSR
// aggregation kernels with alpha as the edge weights.
//
// Work unit of every kernel here: one PIECE, walked by a wavefront (the sampled product, whose
// lanes split the columns) or by a group of 16 lanes (the per-entry scalar kernels: most rows
// have a few dozen entries, so four pieces share a wavefront).  A piece is a run of at most
// `chunk` consecutive entries of one row; rows up to `chunk` entries are one piece, longer
// rows (hubs) several, so that no wavefront walks a 100 000-entry row alone.  The piece table
// is built at set-up: piece_ptr[k] .. piece_ptr[k+1] are the entries of piece k, piece_row[k]
// its row, row_piece[v] .. row_piece[v+1] the pieces of row v.  Row-wide quantities (softmax
// maximum and denominator, row sums) are first reduced per piece, then joined per row in
// piece order: fixed order, no atomics.
#include "common.hpp"

namespace sylvie {

constexpr int kGatWavesPerBlock = 4;

struct Pieces {
    const int64_t *piece_ptr;   // [n_pieces + 1] entry offsets
    const int32_t *piece_row;   // [n_pieces]
    const int64_t *row_piece;   // [n_rows + 1]
    int64_t n_pieces;
    int64_t n_rows;
};

__device__ __forceinline__ float gat_wave_max(float v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const float o = __shfl_xor(v, s);
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ float gat_wave_sum(float v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
    return v;
}
__device__ __forceinline__ float lrelu(float x, float slope) { return x > 0.0f ? x : slope * x; }

// Sum over the 16 lanes of a DPP row, left in every lane of the row.
__device__ __forceinline__ float row16_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));  // row_mirror
    return v;
}

__device__ __forceinline__ float row16_max(float v)
{
    float o;
    o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
    v = o > v ? o : v;
    o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
    v = o > v ? o : v;
    o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
    v = o > v ? o : v;
    o = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));
    v = o > v ? o : v;
    return v;
}

constexpr int kGroup = 16;                                         // lanes per piece
constexpr int kPiecesPerBlock = kGatWavesPerBlock * kWave / kGroup;

// Piece of this 16-lane group, or -1 past the end (the whole group leaves together).
__device__ __forceinline__ int64_t group_piece(const Pieces &pc)
{
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kPiecesPerBlock + static_cast<int>(threadIdx.x) / kGroup;
    return k < pc.n_pieces ? k : -1;
}

// ---- row dot products ---------------------------------------------------------------

// 16 lanes per row, four rows per wavefront.  VEC = 4: 16-byte loads (ld, F multiples of 4,
// 16-byte aligned base); VEC = 1: element by element.
template <int VEC>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void row_dot_kernel(
    const float *__restrict__ P, int64_t ld, int64_t n, int F, const float *__restrict__ a,
    float *__restrict__ out)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kPiecesPerBlock + static_cast<int>(threadIdx.x) / kGroup;
    if (i >= n) return;
    const float *row = P + i * ld;
    float acc = 0.0f;
    if constexpr (VEC == 4) {
        for (int c = g * 4; c < F; c += kGroup * 4) {
            const float4 x = *reinterpret_cast<const float4 *>(row + c);
            const float4 y = *reinterpret_cast<const float4 *>(a + c);
            acc = fmaf(x.x, y.x, acc);
            acc = fmaf(x.y, y.y, acc);
            acc = fmaf(x.z, y.z, acc);
            acc = fmaf(x.w, y.w, acc);
        }
    } else {
        for (int c = g; c < F; c += kGroup) acc = fmaf(row[c], a[c], acc);
    }
    acc = row16_sum(acc);
    if (g == 0) out[i] = acc;
}

// ---- edge softmax, forward ------------------------------------------------------------

// Per piece: maximum m and sum of exp(x - m) of its scores x = leaky_relu(s_dst + s_src), in one
// sweep (a lane rescales its running sum whenever its maximum grows; the 16 lanes are joined
// the same way).  The scores are left in `score` so that the last step need not gather again.
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void softmax_piece_stats_kernel(
    Pieces pc, const int32_t *__restrict__ col, const float *__restrict__ s_dst,
    const float *__restrict__ s_src, float slope, float2 *__restrict__ piece_stats, float *__restrict__ score)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    const float sd = s_dst[pc.piece_row[k]];
    float m = -__builtin_inff(), s = 0.0f;
    for (int64_t e = e0 + g; e < e1; e += kGroup) {
        const float x = lrelu(sd + s_src[col[e]], slope);
        score[e] = x;
        if (x > m) {
            s = s * __expf(m - x) + 1.0f;
            m = x;
        } else {
            s += __expf(x - m);
        }
    }
    const float M = row16_max(m);                   // finite: a piece has at least one entry
    s = row16_sum(s * __expf(m - M));               // a lane without entries holds s = 0, m = -inf
    if (g == 0) piece_stats[k] = make_float2(M, s);
}

// Per row: join the pieces in order: m = max m_k, s = sum s_k exp(m_k - m).
__global__ void softmax_row_stats_kernel(Pieces pc, const float2 *__restrict__ piece_stats,
                                         float2 *__restrict__ row_stats)
{
    const int64_t v = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (v >= pc.n_rows) return;
    const int64_t k0 = pc.row_piece[v], k1 = pc.row_piece[v + 1];
    float m = -__builtin_inff();
    for (int64_t k = k0; k < k1; ++k) m = piece_stats[k].x > m ? piece_stats[k].x : m;
    float s = 0.0f;
    for (int64_t k = k0; k < k1; ++k) s += piece_stats[k].y * __expf(piece_stats[k].x - m);
    row_stats[v] = make_float2(m, s);
}

// alpha = exp(score - m_row) / s_row, in place over the scores.
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void softmax_alpha_kernel(
    Pieces pc, const float2 *__restrict__ row_stats, float *__restrict__ alpha)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    const float2 st = row_stats[pc.piece_row[k]];
    const float inv = 1.0f / st.y;
    for (int64_t e = e0 + g; e < e1; e += kGroup) alpha[e] = __expf(alpha[e] - st.x) * inv;
}

// ---- sampled dense-dense product: out[e] = A_v . B_u ----------------------------------------

// 16 lanes per entry, four entries at a time per wavefront.  VEC = 4: lane g of a group holds
// the 4-column pieces g, g + 16, ... of A_v in registers (PP of them, F <= 64 PP) and loads the
// same pieces of B_u; VEC = 1: any F, both rows are read element by element.
template <int VEC, int PP>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void sddmm_kernel(
    Pieces pc, const int32_t *__restrict__ col, const float *__restrict__ A, int64_t lda,
    const float *__restrict__ Bm, int64_t ldb, int F, float *__restrict__ out)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kGatWavesPerBlock + wave;
    if (k >= pc.n_pieces) return;
    const int64_t e0 = uniform(pc.piece_ptr[k]), e1 = uniform(pc.piece_ptr[k + 1]);
    const float *arow = A + static_cast<int64_t>(uniform(pc.piece_row[k])) * lda;
    const int g = lane & 15, grp = lane >> 4;
    if constexpr (VEC == 4) {
        float4 av[PP];
        int coff[PP];
#pragma unroll
        for (int p = 0; p < PP; ++p) {
            const int c = (g + 16 * p) * 4;
            coff[p] = c < F ? c : -1;
            av[p] = c < F ? *reinterpret_cast<const float4 *>(arow + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        // sixteen entries per step: four independent gathers per lane are in flight
        for (int64_t e = e0; e < e1; e += 16) {
            float4 b[4][PP];
            int64_t me[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                me[u] = e + 4 * u + grp;
                const float *brow = Bm + static_cast<int64_t>(col[me[u] < e1 ? me[u] : e0]) * ldb;
#pragma unroll
                for (int p = 0; p < PP; ++p)
                    b[u][p] = coff[p] >= 0 ? *reinterpret_cast<const float4 *>(brow + coff[p])
                                           : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float acc = 0.0f;
#pragma unroll
                for (int p = 0; p < PP; ++p) {
                    acc = fmaf(av[p].x, b[u][p].x, acc);
                    acc = fmaf(av[p].y, b[u][p].y, acc);
                    acc = fmaf(av[p].z, b[u][p].z, acc);
                    acc = fmaf(av[p].w, b[u][p].w, acc);
                }
                acc = row16_sum(acc);
                if (me[u] < e1 && g == 0) out[me[u]] = acc;
            }
        }
    } else {
        for (int64_t e = e0; e < e1; e += 4) {
            const int64_t me = e + grp;
            const bool on = me < e1;
            const float *brow = Bm + static_cast<int64_t>(col[on ? me : e0]) * ldb;
            float acc = 0.0f;
            for (int c = g; c < F; c += 16) acc = fmaf(arow[c], brow[c], acc);
            acc = row16_sum(acc);
            if (on && g == 0) out[me] = acc;
        }
    }
}

// ---- row sums of per-entry values ---------------------------------------------------------

// WEIGHTED: sum of a[e] * b[e] (the softmax backward's row term); otherwise sum of a[e].
template <bool WEIGHTED>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void piece_sum_kernel(
    Pieces pc, const float *__restrict__ a, const float *__restrict__ b, float *__restrict__ piece_sum)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    float s = 0.0f;
    for (int64_t e = e0 + g; e < e1; e += kGroup) s += WEIGHTED ? a[e] * b[e] : a[e];
    s = row16_sum(s);
    if (g == 0) piece_sum[k] = s;
}

__global__ void row_sum_kernel(Pieces pc, const float *__restrict__ piece_sum, float *__restrict__ out)
{
    const int64_t v = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (v >= pc.n_rows) return;
    float s = 0.0f;
    for (int64_t k = pc.row_piece[v]; k < pc.row_piece[v + 1]; ++k) s += piece_sum[k];
    out[v] = s;
}

// ---- edge softmax, backward ---------------------------------------------------------------

__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void softmax_bwd_kernel(
    Pieces pc, const int32_t *__restrict__ col, const float *__restrict__ alpha,
    const float *__restrict__ dalpha, const float *__restrict__ s_dst,
    const float *__restrict__ s_src, float slope, const float *__restrict__ row_dot,
    float *__restrict__ de)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    const int v = pc.piece_row[k];
    const float sd = s_dst[v], dot = row_dot[v];
    for (int64_t e = e0 + g; e < e1; e += kGroup) {
        const float f = sd + s_src[col[e]] > 0.0f ? 1.0f : slope;
        de[e] = (alpha[e] * dalpha[e] - alpha[e] * dot) * f;
    }
}

// ---- out[c] = sum_i s[i] X[i][c]: gradients of the attention vectors -----------------------

constexpr int kColSumRows = 2048;     // rows per slab

// Slab z of rows -> part[z][0..F).  Wave w of the block takes rows r0 + w, r0 + w + 4, ... of the
// slab, lane l columns l, l + 64, ...; four independent chains per lane (rows 16 apart) keep
// loads in flight.  Chains, then waves, are joined in a fixed order.
__global__ __launch_bounds__(256) void scaled_column_sum_slab_kernel(
    const float *__restrict__ X, int64_t ld, int64_t n, int F, const float *__restrict__ s,
    float *__restrict__ part)
{
    __shared__ float red[4][kWave];
    const int wave = static_cast<int>(threadIdx.x) / kWave, lane = lane_id();
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * kColSumRows;
    const int64_t r1 = r0 + kColSumRows < n ? r0 + kColSumRows : n;
    for (int c0 = 0; c0 < F; c0 += kWave) {
        const int c = c0 + lane;
        float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
        if (c < F) {
            int64_t i = r0 + wave;
            for (; i + 12 < r1; i += 16) {
                a0 = fmaf(s[i], X[i * ld + c], a0);
                a1 = fmaf(s[i + 4], X[(i + 4) * ld + c], a1);
                a2 = fmaf(s[i + 8], X[(i + 8) * ld + c], a2);
                a3 = fmaf(s[i + 12], X[(i + 12) * ld + c], a3);
            }
            for (; i < r1; i += 4) a0 = fmaf(s[i], X[i * ld + c], a0);
        }
        red[wave][lane] = (a0 + a1) + (a2 + a3);
        __syncthreads();
        if (wave == 0 && c < F)
            part[static_cast<int64_t>(blockIdx.x) * F + c] =
                ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
        __syncthreads();
    }
}

// out[c] = sum over the slabs of part[z][c].  One block per 64 columns: wave w adds slabs
// w, w + 4, ... in four chains (slabs 16 apart), chains then waves are joined in a fixed order.
__global__ __launch_bounds__(256) void scaled_column_sum_join_kernel(const float *__restrict__ part, int64_t n_slabs,
                                                                    int F, float *__restrict__ out)
{
    __shared__ float red[4][kWave];
    const int wave = static_cast<int>(threadIdx.x) / kWave, lane = lane_id();
    const int c = static_cast<int>(blockIdx.x) * kWave + lane;
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    if (c < F) {
        int64_t z = wave;
        for (; z + 12 < n_slabs; z += 16) {
            a0 += part[z * F + c];
            a1 += part[(z + 4) * F + c];
            a2 += part[(z + 8) * F + c];
            a3 += part[(z + 12) * F + c];
        }
        for (; z < n_slabs; z += 4) a0 += part[z * F + c];
    }
    red[wave][lane] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (wave == 0 && c < F) out[c] = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
}

// ---- small element-wise pieces ------------------------------------------------------------

__global__ void permute_kernel(const float *__restrict__ in, const int64_t *__restrict__ perm, int64_t n,
                               float *__restrict__ out)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) out[i] = in[perm[i]];
}

// X[i][c] = X[i][c] + s[i] * a[c] (two single-precision operations), one thread per element.
__global__ void rank1_add_kernel(float *__restrict__ X, int64_t ld, int64_t n, int F,
                                 const float *__restrict__ s, const float *__restrict__ a)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t >= n * F) return;
    const int64_t i = t / F;
    const int c = static_cast<int>(t - i * F);
    const float step = s[i] * a[c];
    X[i * ld + c] = X[i * ld + c] + step;
}

// FWD: out = max(in, 0); otherwise out = gate > 0 ? in : 0.
template <bool FWD>
__global__ void relu_kernel(const float *__restrict__ in, int64_t ld_in, const float *__restrict__ gate,
                            int64_t ld_gate, int64_t n, int F, float *__restrict__ out, int64_t ld_out)
{
    const int64_t t = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t >= n * F) return;
    const int64_t i = t / F;
    const int c = static_cast<int>(t - i * F);
    const float x = in[i * ld_in + c];
    if constexpr (FWD) out[i * ld_out + c] = x > 0.0f ? x : 0.0f;
    else out[i * ld_out + c] = gate[i * ld_gate + c] > 0.0f ? x : 0.0f;
}

// ---- host side ----------------------------------------------------------------------------

static int32_t check_pieces(const char *name, const int64_t *piece_ptr, const int32_t *piece_row,
                            const int64_t *row_piece, int64_t n_pieces, int64_t n_rows)
{
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31) || n_pieces < 0 || n_pieces >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: row / piece count out of range", name);
    // rows without entries have no piece, so n_pieces may be below n_rows
    if ((n_pieces > 0 && (!piece_ptr || !piece_row)) || (n_rows > 0 && !row_piece))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null piece table", name);
    if (n_pieces > 0 && (!aligned(piece_ptr, 8) || !aligned(piece_row, 4) || !aligned(row_piece, 8)))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned piece table", name);
    return SYLVIE_OK;
}

static dim3 piece_grid(int64_t n_pieces)
{
    return dim3(static_cast<unsigned>((n_pieces + kGatWavesPerBlock - 1) / kGatWavesPerBlock));
}
static dim3 group_grid(int64_t n_pieces)       // kernels that walk a piece with 16 lanes
{
    return dim3(static_cast<unsigned>((n_pieces + kPiecesPerBlock - 1) / kPiecesPerBlock));
}

}  // namespace sylvie

extern "C" int32_t sylvie_row_dot(const float *P, int64_t ld_p, int64_t n, int32_t F, const float *a,
                                  float *out, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_row_dot";
    if (n < 0 || n >= (int64_t(1) << 31) || F < 1 || F > 65536 || ld_p < F)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (n == 0) return SYLVIE_OK;
    if (!P || !a || !out) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    const bool v4 = F % 4 == 0 && ld_p % 4 == 0 && aligned(P, 16) && aligned(a, 16);
    if (v4)
        hipLaunchKernelGGL(row_dot_kernel<4>, group_grid(n), dim3(kGatWavesPerBlock * kWave), 0,
                           static_cast<hipStream_t>(stream), P, ld_p, n, F, a, out);
    else
        hipLaunchKernelGGL(row_dot_kernel<1>, group_grid(n), dim3(kGatWavesPerBlock * kWave), 0,
                           static_cast<hipStream_t>(stream), P, ld_p, n, F, a, out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" size_t sylvie_edge_softmax_workspace_bytes(int64_t n_pieces, int64_t n_rows)
{
    if (n_pieces < 0 || n_rows < 0) return 0;
    return static_cast<size_t>(n_pieces + n_rows) * sizeof(float2);
}

extern "C" int32_t sylvie_edge_softmax_fwd(const int64_t *piece_ptr, const int32_t *piece_row,
                                           const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                           const int32_t *col, const float *s_dst, const float *s_src,
                                           float slope, float *alpha, void *workspace,
                                           size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_edge_softmax_fwd";
    const int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    if (n_pieces == 0 || n_rows == 0) return SYLVIE_OK;
    if (!col || !s_dst || !s_src || !alpha) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_edge_softmax_workspace_bytes(n_pieces, n_rows) ||
        !aligned(workspace, 8))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small or misaligned", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    float2 *piece_stats = static_cast<float2 *>(workspace);
    float2 *row_stats = piece_stats + n_pieces;
    const dim3 block(kGatWavesPerBlock * kWave);
    hipLaunchKernelGGL(softmax_piece_stats_kernel, group_grid(n_pieces), block, 0, st, pc, col, s_dst, s_src,
                       slope, piece_stats, alpha);
    hipLaunchKernelGGL(softmax_row_stats_kernel, dim3(static_cast<unsigned>((n_rows + 255) / 256)), dim3(256),
                       0, st, pc, piece_stats, row_stats);
    hipLaunchKernelGGL(softmax_alpha_kernel, group_grid(n_pieces), block, 0, st, pc, row_stats, alpha);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_sddmm(const int64_t *piece_ptr, const int32_t *piece_row,
                                const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                const int32_t *col, const float *A, int64_t ld_a, const float *Bm,
                                int64_t ld_b, int32_t F, float *out, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_sddmm";
    const int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    if (F < 1 || F > 65536 || ld_a < F || ld_b < F) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad widths", name);
    if (n_pieces == 0) return SYLVIE_OK;
    if (!col || !A || !Bm || !out) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    const dim3 block(kGatWavesPerBlock * kWave);
    const bool v4 = F % 4 == 0 && ld_a % 4 == 0 && ld_b % 4 == 0 && aligned(A, 16) && aligned(Bm, 16);
#define SYLVIE_SDDMM(V, PPV) \
    hipLaunchKernelGGL((sddmm_kernel<V, PPV>), piece_grid(n_pieces), block, 0, st, pc, col, A, ld_a, Bm, ld_b, F, out)
    if (v4 && F <= 64) SYLVIE_SDDMM(4, 1);
    else if (v4 && F <= 128) SYLVIE_SDDMM(4, 2);
    else if (v4 && F <= 256) SYLVIE_SDDMM(4, 4);
    else if (v4 && F <= 512) SYLVIE_SDDMM(4, 8);
    else SYLVIE_SDDMM(1, 1);
#undef SYLVIE_SDDMM
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_segment_sum(const int64_t *piece_ptr, const int32_t *piece_row,
                                      const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                      const float *vals, float *out, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_segment_sum";
    const int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    if (n_rows == 0) return SYLVIE_OK;
    if (!out || (n_pieces > 0 && !vals)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (n_pieces > 0 && (!workspace || workspace_bytes < static_cast<size_t>(n_pieces) * sizeof(float)))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace below n_pieces floats", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    float *ps = static_cast<float *>(workspace);
    if (n_pieces > 0)
        hipLaunchKernelGGL(piece_sum_kernel<false>, group_grid(n_pieces), dim3(kGatWavesPerBlock * kWave), 0, st,
                           pc, vals, nullptr, ps);
    hipLaunchKernelGGL(row_sum_kernel, dim3(static_cast<unsigned>((n_rows + 255) / 256)), dim3(256), 0, st, pc,
                       ps, out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_edge_softmax_bwd(const int64_t *piece_ptr, const int32_t *piece_row,
                                           const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                           const int32_t *col, const float *alpha, const float *dalpha,
                                           const float *s_dst, const float *s_src, float slope,
                                           float *de, void *workspace, size_t workspace_bytes,
                                           void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_edge_softmax_bwd";
    const int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    if (n_pieces == 0 || n_rows == 0) return SYLVIE_OK;
    if (!col || !alpha || !dalpha || !s_dst || !s_src || !de)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < static_cast<size_t>(n_pieces + n_rows) * sizeof(float))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace below n_pieces + n_rows floats", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    float *ps = static_cast<float *>(workspace);
    float *row_dot = ps + n_pieces;
    const dim3 block(kGatWavesPerBlock * kWave);
    hipLaunchKernelGGL(piece_sum_kernel<true>, group_grid(n_pieces), block, 0, st, pc, alpha, dalpha, ps);
    hipLaunchKernelGGL(row_sum_kernel, dim3(static_cast<unsigned>((n_rows + 255) / 256)), dim3(256), 0, st, pc,
                       ps, row_dot);
    hipLaunchKernelGGL(softmax_bwd_kernel, group_grid(n_pieces), block, 0, st, pc, col, alpha, dalpha, s_dst,
                       s_src, slope, row_dot, de);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" size_t sylvie_scaled_column_sum_workspace_bytes(int64_t n, int32_t F)
{
    if (n < 0 || F < 1) return 0;
    return static_cast<size_t>((n + sylvie::kColSumRows - 1) / sylvie::kColSumRows) * static_cast<size_t>(F) *
           sizeof(float);
}

extern "C" int32_t sylvie_scaled_column_sum(const float *X, int64_t ld_x, int64_t n, int32_t F,
                                            const float *s, float *out, void *workspace,
                                            size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_scaled_column_sum";
    if (n < 0 || n >= (int64_t(1) << 31) || F < 1 || F > 65536 || ld_x < F)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!out) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null output", name);
    if (n > 0 && (!X || !s)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    const int64_t slabs = (n + kColSumRows - 1) / kColSumRows;
    if (slabs > 0 && (!workspace || workspace_bytes < sylvie_scaled_column_sum_workspace_bytes(n, F)))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(workspace);
    if (slabs > 0)
        hipLaunchKernelGGL(scaled_column_sum_slab_kernel, dim3(static_cast<unsigned>(slabs)), dim3(256), 0, st, X,
                           ld_x, n, F, s, part);
    hipLaunchKernelGGL(scaled_column_sum_join_kernel, dim3((F + kWave - 1) / kWave), dim3(256), 0, st, part, slabs, F, out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_permute_f32(const float *in, const int64_t *perm, int64_t n, float *out,
                                      void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_permute_f32";
    if (n < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative size", name);
    if (n == 0) return SYLVIE_OK;
    if (!in || !perm || !out) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    hipLaunchKernelGGL(permute_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), in, perm, n, out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_rank1_add(float *X, int64_t ld_x, int64_t n, int32_t F, const float *s,
                                    const float *a, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_rank1_add";
    if (n < 0 || n >= (int64_t(1) << 31) || F < 1 || F > 65536 || ld_x < F)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (n == 0) return SYLVIE_OK;
    if (!X || !s || !a) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    const int64_t total = n * F;
    hipLaunchKernelGGL(rank1_add_kernel, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), X, ld_x, n, F, s, a);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

static int32_t relu_common(const char *name, bool fwd, const float *in, int64_t ld_in, const float *gate,
                           int64_t ld_gate, int64_t n, int32_t F, float *out, int64_t ld_out, void *stream)
{
    using namespace sylvie;
    if (n < 0 || n >= (int64_t(1) << 31) || F < 1 || F > 65536 || ld_in < F || ld_out < F ||
        (!fwd && ld_gate < F))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (n == 0) return SYLVIE_OK;
    if (!in || !out || (!fwd && !gate)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    const int64_t total = n * F;
    const dim3 grid(static_cast<unsigned>((total + 255) / 256));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (fwd) hipLaunchKernelGGL(relu_kernel<true>, grid, dim3(256), 0, st, in, ld_in, gate, ld_gate, n, F, out, ld_out);
    else hipLaunchKernelGGL(relu_kernel<false>, grid, dim3(256), 0, st, in, ld_in, gate, ld_gate, n, F, out, ld_out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_relu_fwd(const float *Z, int64_t ld_z, int64_t n, int32_t F, float *H,
                                   int64_t ld_h, void *stream)
{
    return relu_common("sylvie_relu_fwd", true, Z, ld_z, nullptr, 0, n, F, H, ld_h, stream);
}

extern "C" int32_t sylvie_relu_bwd(const float *H, int64_t ld_h, const float *J, int64_t ld_j, int64_t n,
                                   int32_t F, float *dZ, int64_t ld_dz, void *stream)
{
    return relu_common("sylvie_relu_bwd", false, J, ld_j, H, ld_h, n, F, dZ, ld_dz, stream);
}
