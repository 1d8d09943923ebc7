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
#include <initializer_list>

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

// 16 lanes per (row, head), four of them per wavefront: out[i][k] = P[i][k F .. (k+1) F) . a[k F ..)
// for i < n and, when a2 is given, out2[i][k] with a2 for i < n2 from the same loads of P.
// VEC = 4: 16-byte loads (ld, F multiples of 4, 16-byte aligned bases); VEC = 1: element by element.
template <int VEC>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void row_dot_kernel(
    const float *__restrict__ P, int64_t ld, int64_t n, int F, int K, const float *__restrict__ a,
    float *__restrict__ out, const float *__restrict__ a2, int64_t n2, float *__restrict__ out2)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t u = static_cast<int64_t>(blockIdx.x) * kPiecesPerBlock + static_cast<int>(threadIdx.x) / kGroup;
    const int64_t rows = n > n2 ? n : n2;
    if (u >= rows * K) return;
    const int64_t i = u / K;
    const int k = static_cast<int>(u - i * K);
    const float *row = P + i * ld + k * F;
    const float *av = a + k * F;
    const float *bv = a2 ? a2 + k * F : av;
    float acc = 0.0f, acc2 = 0.0f;
    if constexpr (VEC == 4) {
        for (int c = g * 4; c < F; c += kGroup * 4) {
            const float4 x = *reinterpret_cast<const float4 *>(row + c);
            const float4 y = *reinterpret_cast<const float4 *>(av + c);
            const float4 z = *reinterpret_cast<const float4 *>(bv + c);
            acc = fmaf(x.x, y.x, acc);
            acc = fmaf(x.y, y.y, acc);
            acc = fmaf(x.z, y.z, acc);
            acc = fmaf(x.w, y.w, acc);
            acc2 = fmaf(x.x, z.x, acc2);
            acc2 = fmaf(x.y, z.y, acc2);
            acc2 = fmaf(x.z, z.z, acc2);
            acc2 = fmaf(x.w, z.w, acc2);
        }
    } else {
        for (int c = g; c < F; c += kGroup) {
            acc = fmaf(row[c], av[c], acc);
            acc2 = fmaf(row[c], bv[c], acc2);
        }
    }
    acc = row16_sum(acc);
    acc2 = row16_sum(acc2);
    if (g == 0 && i < n) out[u] = acc;
    if (g == 0 && a2 && i < n2) out2[u] = acc2;
}

// ---- K adjacent floats (the heads of one entry or of one node) as one access ------------------

template <int K>
struct HeadVec { typedef float type __attribute__((ext_vector_type(K))); };
template <>
struct HeadVec<1> { typedef float type; };
template <int K>
__device__ __forceinline__ void load_heads(float (&o)[K], const float *p)
{
    typedef typename HeadVec<K>::type V;
    const V v = *reinterpret_cast<const V *>(p);
    __builtin_memcpy(o, &v, sizeof(V));
}
template <int K>
__device__ __forceinline__ void store_heads(float *p, const float (&o)[K])
{
    typedef typename HeadVec<K>::type V;
    V v;
    __builtin_memcpy(&v, o, sizeof(V));
    *reinterpret_cast<V *>(p) = v;
}

// ---- edge softmax, forward ------------------------------------------------------------
// Per-entry arrays hold the K heads of an entry side by side ([entries][K]), per-node arrays
// the K heads of a node ([nodes][K]): an entry's column index and its node's scores are
// fetched once for all heads.

// Per piece and head: maximum m and sum of exp(x - m) of its scores x = leaky_relu(s_dst + s_src),
// in one sweep (a lane rescales its running sum whenever its maximum grows; the 16 lanes are
// joined the same way).  The scores are left in `score` so that the last step need not gather again.
template <int K>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void softmax_piece_stats_kernel(
    Pieces pc, const int32_t *__restrict__ col, const float *__restrict__ s_dst,
    const float *__restrict__ s_src, float slope, float2 *__restrict__ piece_stats, float *__restrict__ score)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    float sd[K], m[K], s[K];
    load_heads<K>(sd, s_dst + static_cast<int64_t>(pc.piece_row[k]) * K);
#pragma unroll
    for (int h = 0; h < K; ++h) { m[h] = -__builtin_inff(); s[h] = 0.0f; }
    for (int64_t e = e0 + g; e < e1; e += kGroup) {
        float ss[K], x[K];
        load_heads<K>(ss, s_src + static_cast<int64_t>(col[e]) * K);
#pragma unroll
        for (int h = 0; h < K; ++h) {
            x[h] = lrelu(sd[h] + ss[h], slope);
            if (x[h] > m[h]) {
                s[h] = s[h] * __expf(m[h] - x[h]) + 1.0f;
                m[h] = x[h];
            } else {
                s[h] += __expf(x[h] - m[h]);
            }
        }
        store_heads<K>(score + e * K, x);
    }
#pragma unroll
    for (int h = 0; h < K; ++h) {
        const float M = row16_max(m[h]);                    // finite: a piece has at least one entry
        const float t = row16_sum(s[h] * __expf(m[h] - M)); // a lane without entries holds s = 0, m = -inf
        if (g == 0) piece_stats[k * K + h] = make_float2(M, t);
    }
}

// Per row and head: join the pieces in order: m = max m_k, s = sum s_k exp(m_k - m).
__global__ void softmax_row_stats_kernel(Pieces pc, int K, const float2 *__restrict__ piece_stats,
                                         float2 *__restrict__ row_stats)
{
    const int64_t u = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (u >= pc.n_rows * K) return;
    const int64_t v = u / K;
    const int h = static_cast<int>(u - v * K);
    const int64_t k0 = pc.row_piece[v], k1 = pc.row_piece[v + 1];
    float m = -__builtin_inff();
    for (int64_t k = k0; k < k1; ++k) m = piece_stats[k * K + h].x > m ? piece_stats[k * K + h].x : m;
    float s = 0.0f;
    for (int64_t k = k0; k < k1; ++k) s += piece_stats[k * K + h].y * __expf(piece_stats[k * K + h].x - m);
    row_stats[u] = make_float2(m, s);
}

// alpha = exp(score - m_row) / s_row, in place over the scores.
template <int K>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void softmax_alpha_kernel(
    Pieces pc, const float2 *__restrict__ row_stats, float *__restrict__ alpha)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    float mx[K], inv[K];
#pragma unroll
    for (int h = 0; h < K; ++h) {
        const float2 st = row_stats[static_cast<int64_t>(pc.piece_row[k]) * K + h];
        mx[h] = st.x;
        inv[h] = 1.0f / st.y;
    }
    for (int64_t e = e0 + g; e < e1; e += kGroup) {
        float x[K];
        load_heads<K>(x, alpha + e * K);
#pragma unroll
        for (int h = 0; h < K; ++h) x[h] = __expf(x[h] - mx[h]) * inv[h];
        store_heads<K>(alpha + e * K, x);
    }
}

// ---- sampled dense-dense product: out[e][h] = A_v[h F ..) . B_u[h F ..) ---------------------

// 16 lanes per entry, four entries at a time per wavefront; a wavefront walks one piece.  Lane g
// of a group holds, per head, the 4-column pieces g, g + 16, ... of the head's slice of A_v in
// registers (PP of them, F <= 64 PP) and loads the same pieces of B_u: the whole gathered row
// for all K heads, so that the entry's column index is read once.
template <int K, int PP>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void sddmm_kernel(
    Pieces pc, const int32_t *__restrict__ col, const float *__restrict__ A, int64_t lda,
    const float *__restrict__ Bm, int64_t ldb, int F, float *__restrict__ out)
{
    constexpr int U = K * PP <= 4 ? 4 : (K * PP <= 8 ? 2 : 1);     // gathered rows in flight per group
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kGatWavesPerBlock + wave;
    if (k >= pc.n_pieces) return;
    const int64_t e0 = uniform(pc.piece_ptr[k]), e1 = uniform(pc.piece_ptr[k + 1]);
    const float *arow = A + static_cast<int64_t>(uniform(pc.piece_row[k])) * lda;
    const int g = lane & 15, grp = lane >> 4;
    float4 av[K][PP];
    int coff[PP];
#pragma unroll
    for (int p = 0; p < PP; ++p) {
        const int c = (g + 16 * p) * 4;
        coff[p] = c < F ? c : -1;
#pragma unroll
        for (int h = 0; h < K; ++h)
            av[h][p] = c < F ? *reinterpret_cast<const float4 *>(arow + h * F + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int64_t e = e0; e < e1; e += 4 * U) {
        float4 b[U][K][PP];
        int64_t me[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            me[u] = e + 4 * u + grp;
            const float *brow = Bm + static_cast<int64_t>(col[me[u] < e1 ? me[u] : e0]) * ldb;
#pragma unroll
            for (int h = 0; h < K; ++h)
#pragma unroll
                for (int p = 0; p < PP; ++p)
                    b[u][h][p] = coff[p] >= 0 ? *reinterpret_cast<const float4 *>(brow + h * F + coff[p])
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float r[K];
#pragma unroll
            for (int h = 0; h < K; ++h) {
                float acc = 0.0f;
#pragma unroll
                for (int p = 0; p < PP; ++p) {
                    acc = fmaf(av[h][p].x, b[u][h][p].x, acc);
                    acc = fmaf(av[h][p].y, b[u][h][p].y, acc);
                    acc = fmaf(av[h][p].z, b[u][h][p].z, acc);
                    acc = fmaf(av[h][p].w, b[u][h][p].w, acc);
                }
                r[h] = row16_sum(acc);
            }
            if (me[u] < e1 && g == 0) store_heads<K>(out + me[u] * K, r);
        }
    }
}

// Any F, K and alignment: both rows are read element by element.
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void sddmm_plain_kernel(
    Pieces pc, const int32_t *__restrict__ col, const float *__restrict__ A, int64_t lda,
    const float *__restrict__ Bm, int64_t ldb, int F, int K, float *__restrict__ out)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kGatWavesPerBlock + wave;
    if (k >= pc.n_pieces) return;
    const int64_t e0 = uniform(pc.piece_ptr[k]), e1 = uniform(pc.piece_ptr[k + 1]);
    const float *arow = A + static_cast<int64_t>(uniform(pc.piece_row[k])) * lda;
    const int g = lane & 15, grp = lane >> 4;
    for (int64_t e = e0; e < e1; e += 4) {
        const int64_t me = e + grp;
        const bool on = me < e1;
        const float *brow = Bm + static_cast<int64_t>(col[on ? me : e0]) * ldb;
        for (int h = 0; h < K; ++h) {
            float acc = 0.0f;
            for (int c = g; c < F; c += 16) acc = fmaf(arow[h * F + c], brow[h * F + c], acc);
            acc = row16_sum(acc);
            if (on && g == 0) out[me * K + h] = acc;
        }
    }
}

// ---- row sums of per-entry values ---------------------------------------------------------

// Per piece and head.  WEIGHTED: sum of a[e] * b[e] (the softmax backward's row term); otherwise
// the sum of a[i_e], i_e = e or index[e] (the entry map of a transposition: column sums through
// the transposed operator's pieces, with the values left in the forward order).
template <bool WEIGHTED, int K>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void piece_sum_kernel(
    Pieces pc, const float *__restrict__ a, const float *__restrict__ b, const int64_t *__restrict__ index,
    float *__restrict__ piece_sum)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    float s[K];
#pragma unroll
    for (int h = 0; h < K; ++h) s[h] = 0.0f;
    for (int64_t e = e0 + g; e < e1; e += kGroup) {
        const int64_t ie = index ? index[e] : e;
        float x[K];
        load_heads<K>(x, a + ie * K);
        if constexpr (WEIGHTED) {
            float y[K];
            load_heads<K>(y, b + ie * K);
#pragma unroll
            for (int h = 0; h < K; ++h) s[h] += x[h] * y[h];
        } else {
#pragma unroll
            for (int h = 0; h < K; ++h) s[h] += x[h];
        }
    }
#pragma unroll
    for (int h = 0; h < K; ++h) {
        const float t = row16_sum(s[h]);
        if (g == 0) piece_sum[k * K + h] = t;
    }
}

__global__ void row_sum_kernel(Pieces pc, int K, const float *__restrict__ piece_sum, float *__restrict__ out)
{
    const int64_t u = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (u >= pc.n_rows * K) return;
    const int64_t v = u / K;
    const int h = static_cast<int>(u - v * K);
    float s = 0.0f;
    for (int64_t k = pc.row_piece[v]; k < pc.row_piece[v + 1]; ++k) s += piece_sum[k * K + h];
    out[u] = s;
}

// ---- edge softmax, backward ---------------------------------------------------------------

// de = alpha (dalpha - row term) leaky_relu'(.), and, when piece_de is given, the piece's sum of
// de per head in the order piece_sum_kernel would take (their row sums are the score gradients
// of the destination side).
template <int K>
__global__ __launch_bounds__(kGatWavesPerBlock *kWave) void softmax_bwd_kernel(
    Pieces pc, const int32_t *__restrict__ col, const float *__restrict__ alpha,
    const float *__restrict__ dalpha, const float *__restrict__ s_dst,
    const float *__restrict__ s_src, float slope, const float *__restrict__ row_dot,
    float *__restrict__ de, float *__restrict__ piece_de)
{
    const int g = static_cast<int>(threadIdx.x) & (kGroup - 1);
    const int64_t k = group_piece(pc);
    if (k < 0) return;
    const int64_t e0 = pc.piece_ptr[k], e1 = pc.piece_ptr[k + 1];
    const int64_t v = pc.piece_row[k];
    float sd[K], dot[K], sum[K];
    load_heads<K>(sd, s_dst + v * K);
    load_heads<K>(dot, row_dot + v * K);
#pragma unroll
    for (int h = 0; h < K; ++h) sum[h] = 0.0f;
    for (int64_t e = e0 + g; e < e1; e += kGroup) {
        float ss[K], al[K], da[K], o[K];
        load_heads<K>(ss, s_src + static_cast<int64_t>(col[e]) * K);
        load_heads<K>(al, alpha + e * K);
        load_heads<K>(da, dalpha + e * K);
#pragma unroll
        for (int h = 0; h < K; ++h) {
            const float f = sd[h] + ss[h] > 0.0f ? 1.0f : slope;
            o[h] = (al[h] * da[h] - al[h] * dot[h]) * f;
            sum[h] += o[h];
        }
        store_heads<K>(de + e * K, o);
    }
    if (piece_de) {
#pragma unroll
        for (int h = 0; h < K; ++h) {
            const float t = row16_sum(sum[h]);
            if (g == 0) piece_de[k * K + h] = t;
        }
    }
}

// ---- out[c] = sum_i s[i][c / Fh] X[i][c]: gradients of the attention vectors ----------------

constexpr int kColSumRows = 2048;     // rows per slab

// Slab z of rows, block y of 64 VEC columns -> part[z][.].  Wave w of the block takes the rows
// r0 + w, r0 + w + 4, ... of the slab, lane l the VEC adjacent columns (64 y + l) VEC ..; a lane
// keeps four independent chains, chain q the rows r0 + w + 4 q + 16 j (loads in flight).  Chains,
// then waves, are joined in a fixed order, so a column's sum depends only on the slab's rows.
// s holds K values per row, a column uses the one of its head c / Fh (VEC divides Fh).  With
// s2: a second sum over rows [0, n2) into part2 from the same loads of X; each of the two keeps
// the order it has alone.
template <int VEC>
__global__ __launch_bounds__(256) void scaled_column_sum_slab_kernel(
    const float *__restrict__ X, int64_t ld, int F, int Fh, int K, const float *__restrict__ s1, int64_t n1,
    float *__restrict__ part1, const float *__restrict__ s2, int64_t n2, float *__restrict__ part2)
{
    __shared__ float red[2][4][kWave * VEC];
    const int wave = static_cast<int>(threadIdx.x) / kWave, lane = lane_id();
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * kColSumRows;
    const int64_t e1 = r0 + kColSumRows < n1 ? r0 + kColSumRows : n1;      // end of the slab for sum 1
    const int64_t e2 = s2 ? (r0 + kColSumRows < n2 ? r0 + kColSumRows : n2) : e1;   // no s2: sum 2 is never stored
    const int64_t both = e1 < e2 ? e1 : e2, any = e1 > e2 ? e1 : e2;
    const int c = (static_cast<int>(blockIdx.y) * kWave + lane) * VEC;
    float a[4][VEC], b[4][VEC];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int t = 0; t < VEC; ++t) a[q][t] = b[q][t] = 0.0f;
    if (c < F) {
        const int hk = c / Fh;
        const float *sa = s1 + hk, *sb = s2 ? s2 + hk : s1 + hk;
        int64_t i = r0 + wave;
        for (; i + 12 < both; i += 16) {         // all four rows feed both sums
            float x[4][VEC];
#pragma unroll
            for (int q = 0; q < 4; ++q) load_vec<VEC>(x[q], X + (i + 4 * q) * ld + c);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float u = sa[(i + 4 * q) * K], v = sb[(i + 4 * q) * K];
#pragma unroll
                for (int t = 0; t < VEC; ++t) {
                    a[q][t] = fmaf(u, x[q][t], a[q][t]);
                    b[q][t] = fmaf(v, x[q][t], b[q][t]);
                }
            }
        }
        for (; i < any; i += 16) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t r = i + 4 * q;
                if (r < any) {
                    float x[VEC];
                    load_vec<VEC>(x, X + r * ld + c);
                    if (r < e1) {
                        const float u = sa[r * K];
#pragma unroll
                        for (int t = 0; t < VEC; ++t) a[q][t] = fmaf(u, x[t], a[q][t]);
                    }
                    if (r < e2) {
                        const float v = sb[r * K];
#pragma unroll
                        for (int t = 0; t < VEC; ++t) b[q][t] = fmaf(v, x[t], b[q][t]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
        red[0][wave][lane * VEC + t] = (a[0][t] + a[1][t]) + (a[2][t] + a[3][t]);
        red[1][wave][lane * VEC + t] = (b[0][t] + b[1][t]) + (b[2][t] + b[3][t]);
    }
    __syncthreads();
    // 64 VEC columns of two sums: thread t takes column t (and t + 256, ...) of each
    for (int j = static_cast<int>(threadIdx.x); j < 2 * kWave * VEC; j += 256) {
        const int which = j / (kWave * VEC), cl = j - which * (kWave * VEC);
        const int cc = static_cast<int>(blockIdx.y) * kWave * VEC + cl;
        if (cc < F && (which == 0 || s2)) {
            float *part = which ? part2 : part1;
            part[static_cast<int64_t>(blockIdx.x) * F + cc] =
                ((red[which][0][cl] + red[which][1][cl]) + red[which][2][cl]) + red[which][3][cl];
        }
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

// The two rank-1 terms of the attention backward in one pass over X, K heads side by side:
// X[i][c] = fl(fl(X[i][c] + fl(s1[i][c / Fh] a1[c])) + fl(s2[i][c / Fh] a2[c])), term 1 on rows
// [0, n1), term 2 on rows [0, n2).  One thread per VEC adjacent columns (VEC divides Fh).
template <int VEC>
__global__ void rank1_pair_kernel(float *__restrict__ X, int64_t ld, int64_t rows, int F, int Fh, int K,
                                  const float *__restrict__ s1, const float *__restrict__ a1, int64_t n1,
                                  const float *__restrict__ s2, const float *__restrict__ a2, int64_t n2)
{
    const int per_row = F / VEC;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t >= rows * per_row) return;
    const int64_t i = t / per_row;
    const int c = static_cast<int>(t - i * per_row) * VEC;
    const int hk = c / Fh;
    float x[VEC];
    stream_load<VEC>(x, X + i * ld + c);
    if (s1 && i < n1) {
        const float u = s1[i * K + hk];
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
            const float step = u * a1[c + q];
            x[q] = x[q] + step;
        }
    }
    if (s2 && i < n2) {
        const float u = s2[i * K + hk];
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
            const float step = u * a2[c + q];
            x[q] = x[q] + step;
        }
    }
    stream_store<VEC>(X + i * ld + c, x);
}

// FWD: out = max(in, 0); otherwise out = gate > 0 ? in : 0.  One thread per VEC adjacent columns;
// every operand is read or written once, with the streaming hint.
template <bool FWD, int VEC>
__global__ void relu_kernel(const float *__restrict__ in, int64_t ld_in, const float *__restrict__ gate,
                            int64_t ld_gate, int64_t n, int F, float *__restrict__ out, int64_t ld_out)
{
    const int per_row = F / VEC;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (t >= n * per_row) return;
    const int64_t i = t / per_row;
    const int c = static_cast<int>(t - i * per_row) * VEC;
    float x[VEC];
    stream_load<VEC>(x, in + i * ld_in + c);
    if constexpr (FWD) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) x[q] = x[q] > 0.0f ? x[q] : 0.0f;
    } else {
        float g[VEC];
        stream_load<VEC>(g, gate + i * ld_gate + c);
#pragma unroll
        for (int q = 0; q < VEC; ++q) x[q] = g[q] > 0.0f ? x[q] : 0.0f;
    }
    stream_store<VEC>(out + i * ld_out + c, x);
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

// Entry points with a `heads` argument serve K = 1, 2, 4 or 8 heads whose per-entry and per-node
// values sit side by side; such arrays are read K floats at a time.
static int32_t check_heads(const char *name, int32_t heads, std::initializer_list<const void *> arrays)
{
    if (heads != 1 && heads != 2 && heads != 4 && heads != 8)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: heads must be 1, 2, 4 or 8 (got %d)", name, heads);
    for (const void *p : arrays)
        if (p && !aligned(p, 4 * static_cast<size_t>(heads)))
            return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: per-entry / per-node arrays need %d-byte alignment", name,
                        4 * heads);
    return SYLVIE_OK;
}

#define SYLVIE_BY_HEADS(heads, CALL) \
    do {                             \
        if ((heads) == 1) { CALL(1); } \
        else if ((heads) == 2) { CALL(2); } \
        else if ((heads) == 4) { CALL(4); } \
        else { CALL(8); }            \
    } while (0)

static dim3 unit_grid(int64_t units) { return dim3(static_cast<unsigned>((units + 255) / 256)); }

}  // namespace sylvie

extern "C" int32_t sylvie_row_dot_heads(const float *P, int64_t ld_p, int64_t n, int32_t F, int32_t heads,
                                        const float *a, float *out, const float *a2, int64_t n2, float *out2,
                                        void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_row_dot_heads";
    if (heads < 1 || heads > 65536) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad heads", name);
    if (!a2) n2 = 0;
    const int64_t rows = n > n2 ? n : n2;
    if (n < 0 || n2 < 0 || rows * heads >= (int64_t(1) << 31) || F < 1 || F > 65536 ||
        ld_p < static_cast<int64_t>(F) * heads)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (rows == 0) return SYLVIE_OK;
    if (!P || !a || (n > 0 && !out) || (a2 && n2 > 0 && !out2))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    const bool v4 = F % 4 == 0 && ld_p % 4 == 0 && aligned(P, 16) && aligned(a, 16) && (!a2 || aligned(a2, 16));
    const dim3 grid = group_grid(rows * heads), block(kGatWavesPerBlock * kWave);
    if (v4)
        hipLaunchKernelGGL(row_dot_kernel<4>, grid, block, 0, static_cast<hipStream_t>(stream), P, ld_p, n, F,
                           heads, a, out, a2, n2, out2);
    else
        hipLaunchKernelGGL(row_dot_kernel<1>, grid, block, 0, static_cast<hipStream_t>(stream), P, ld_p, n, F,
                           heads, a, out, a2, n2, out2);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_row_dot(const float *P, int64_t ld_p, int64_t n, int32_t F, const float *a,
                                  float *out, void *stream)
{
    return sylvie_row_dot_heads(P, ld_p, n, F, 1, a, out, nullptr, 0, nullptr, stream);
}

extern "C" size_t sylvie_edge_softmax_heads_workspace_bytes(int64_t n_pieces, int64_t n_rows, int32_t heads)
{
    if (n_pieces < 0 || n_rows < 0 || heads < 1) return 0;
    return static_cast<size_t>(n_pieces + n_rows) * static_cast<size_t>(heads) * sizeof(float2);
}

extern "C" size_t sylvie_edge_softmax_workspace_bytes(int64_t n_pieces, int64_t n_rows)
{
    return sylvie_edge_softmax_heads_workspace_bytes(n_pieces, n_rows, 1);
}

extern "C" int32_t sylvie_edge_softmax_fwd_heads(const int64_t *piece_ptr, const int32_t *piece_row,
                                                 const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                                 const int32_t *col, const float *s_dst, const float *s_src,
                                                 int32_t heads, float slope, float *alpha, void *workspace,
                                                 size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_edge_softmax_fwd_heads";
    int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    rc = check_heads(name, heads, {s_dst, s_src, alpha});
    if (rc != SYLVIE_OK) return rc;
    if (n_pieces == 0 || n_rows == 0) return SYLVIE_OK;
    if (!col || !s_dst || !s_src || !alpha) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_edge_softmax_heads_workspace_bytes(n_pieces, n_rows, heads) ||
        !aligned(workspace, 8))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small or misaligned", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    float2 *piece_stats = static_cast<float2 *>(workspace);
    float2 *row_stats = piece_stats + n_pieces * heads;
    const dim3 block(kGatWavesPerBlock * kWave);
#define SYLVIE_STATS(KV) \
    hipLaunchKernelGGL(softmax_piece_stats_kernel<KV>, group_grid(n_pieces), block, 0, st, pc, col, s_dst, s_src, \
                       slope, piece_stats, alpha)
    SYLVIE_BY_HEADS(heads, SYLVIE_STATS);
#undef SYLVIE_STATS
    hipLaunchKernelGGL(softmax_row_stats_kernel, unit_grid(n_rows * heads), dim3(256), 0, st, pc, heads, piece_stats,
                       row_stats);
#define SYLVIE_ALPHA(KV) \
    hipLaunchKernelGGL(softmax_alpha_kernel<KV>, group_grid(n_pieces), block, 0, st, pc, row_stats, alpha)
    SYLVIE_BY_HEADS(heads, SYLVIE_ALPHA);
#undef SYLVIE_ALPHA
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_edge_softmax_fwd(const int64_t *piece_ptr, const int32_t *piece_row,
                                           const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                           const int32_t *col, const float *s_dst, const float *s_src,
                                           float slope, float *alpha, void *workspace,
                                           size_t workspace_bytes, void *stream)
{
    return sylvie_edge_softmax_fwd_heads(piece_ptr, piece_row, row_piece, n_pieces, n_rows, col, s_dst, s_src, 1,
                                         slope, alpha, workspace, workspace_bytes, stream);
}

extern "C" int32_t sylvie_sddmm_heads(const int64_t *piece_ptr, const int32_t *piece_row,
                                      const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                      const int32_t *col, const float *A, int64_t ld_a, const float *Bm,
                                      int64_t ld_b, int32_t F, int32_t heads, float *out, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_sddmm_heads";
    const int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    if (heads < 1 || heads > 64) return fail(SYLVIE_ERR_INVALID_ARG, "%s: heads must be 1 .. 64", name);
    const int64_t width = static_cast<int64_t>(F) * heads;
    if (F < 1 || F > 65536 || ld_a < width || ld_b < width)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad widths", name);
    if (n_pieces == 0) return SYLVIE_OK;
    if (!col || !A || !Bm || !out) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    const dim3 block(kGatWavesPerBlock * kWave);
    const bool v4 = F % 4 == 0 && ld_a % 4 == 0 && ld_b % 4 == 0 && aligned(A, 16) && aligned(Bm, 16) &&
                    aligned(out, 4 * static_cast<size_t>(heads));
    const int pp = F <= 64 ? 1 : F <= 128 ? 2 : F <= 256 ? 4 : F <= 512 ? 8 : 0;
    bool done = false;
#define SYLVIE_SDDMM(KV, PPV)                                                                              \
    if (!done && heads == KV && pp == PPV) {                                                               \
        hipLaunchKernelGGL((sddmm_kernel<KV, PPV>), piece_grid(n_pieces), block, 0, st, pc, col, A, ld_a, Bm, \
                           ld_b, F, out);                                                                  \
        done = true;                                                                                       \
    }
    if (v4) {
        SYLVIE_SDDMM(1, 1) SYLVIE_SDDMM(1, 2) SYLVIE_SDDMM(1, 4) SYLVIE_SDDMM(1, 8)
        SYLVIE_SDDMM(2, 1) SYLVIE_SDDMM(2, 2) SYLVIE_SDDMM(2, 4) SYLVIE_SDDMM(2, 8)
        SYLVIE_SDDMM(4, 1) SYLVIE_SDDMM(4, 2) SYLVIE_SDDMM(4, 4)
        SYLVIE_SDDMM(8, 1) SYLVIE_SDDMM(8, 2)
    }
#undef SYLVIE_SDDMM
    if (!done)
        hipLaunchKernelGGL(sddmm_plain_kernel, piece_grid(n_pieces), block, 0, st, pc, col, A, ld_a, Bm, ld_b, F,
                           heads, out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_sddmm(const int64_t *piece_ptr, const int32_t *piece_row,
                                const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                const int32_t *col, const float *A, int64_t ld_a, const float *Bm,
                                int64_t ld_b, int32_t F, float *out, void *stream)
{
    return sylvie_sddmm_heads(piece_ptr, piece_row, row_piece, n_pieces, n_rows, col, A, ld_a, Bm, ld_b, F, 1, out,
                              stream);
}

extern "C" int32_t sylvie_segment_sum_heads(const int64_t *piece_ptr, const int32_t *piece_row,
                                            const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                            const float *vals, const int64_t *index, int32_t heads, float *out,
                                            void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_segment_sum_heads";
    int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    rc = check_heads(name, heads, {vals});
    if (rc != SYLVIE_OK) return rc;
    if (n_rows == 0) return SYLVIE_OK;
    if (!out || (n_pieces > 0 && !vals)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (index && !aligned(index, 8)) return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned index", name);
    if (n_pieces > 0 &&
        (!workspace || workspace_bytes < static_cast<size_t>(n_pieces) * static_cast<size_t>(heads) * sizeof(float)))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace below n_pieces * heads floats", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    float *ps = static_cast<float *>(workspace);
    const dim3 block(kGatWavesPerBlock * kWave);
    if (n_pieces > 0) {
#define SYLVIE_PSUM(KV) \
    hipLaunchKernelGGL((piece_sum_kernel<false, KV>), group_grid(n_pieces), block, 0, st, pc, vals, nullptr, index, ps)
        SYLVIE_BY_HEADS(heads, SYLVIE_PSUM);
#undef SYLVIE_PSUM
    }
    hipLaunchKernelGGL(row_sum_kernel, unit_grid(n_rows * heads), dim3(256), 0, st, pc, heads, ps, out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_segment_sum(const int64_t *piece_ptr, const int32_t *piece_row,
                                      const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                      const float *vals, float *out, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    return sylvie_segment_sum_heads(piece_ptr, piece_row, row_piece, n_pieces, n_rows, vals, nullptr, 1, out,
                                    workspace, workspace_bytes, stream);
}

extern "C" int32_t sylvie_edge_softmax_bwd_heads(const int64_t *piece_ptr, const int32_t *piece_row,
                                                 const int64_t *row_piece, int64_t n_pieces, int64_t n_rows,
                                                 const int32_t *col, const float *alpha, const float *dalpha,
                                                 const float *s_dst, const float *s_src, int32_t heads,
                                                 float slope, float *de, float *ds_dst, void *workspace,
                                                 size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_edge_softmax_bwd_heads";
    int32_t rc = check_pieces(name, piece_ptr, piece_row, row_piece, n_pieces, n_rows);
    if (rc != SYLVIE_OK) return rc;
    rc = check_heads(name, heads, {alpha, dalpha, s_dst, s_src, de, workspace});
    if (rc != SYLVIE_OK) return rc;
    if (n_rows == 0) return SYLVIE_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Pieces pc{piece_ptr, piece_row, row_piece, n_pieces, n_rows};
    if (n_pieces == 0) {
        // rows without entries: their score gradients are zero
        if (ds_dst)
            hipLaunchKernelGGL(row_sum_kernel, unit_grid(n_rows * heads), dim3(256), 0, st, pc, heads, nullptr, ds_dst);
        SYLVIE_HIP_LAUNCH_CHECK(name);
        return SYLVIE_OK;
    }
    if (!col || !alpha || !dalpha || !s_dst || !s_src || !de)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    // the row part of the workspace starts n_pieces * heads floats in and is read `heads` floats at a time
    if (!workspace ||
        workspace_bytes < static_cast<size_t>(n_pieces + n_rows) * static_cast<size_t>(heads) * sizeof(float))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace below (n_pieces + n_rows) * heads floats", name);
    float *ps = static_cast<float *>(workspace);
    float *row_dot = ps + n_pieces * heads;
    const dim3 block(kGatWavesPerBlock * kWave);
#define SYLVIE_PSUM(KV) \
    hipLaunchKernelGGL((piece_sum_kernel<true, KV>), group_grid(n_pieces), block, 0, st, pc, alpha, dalpha, nullptr, ps)
    SYLVIE_BY_HEADS(heads, SYLVIE_PSUM);
#undef SYLVIE_PSUM
    hipLaunchKernelGGL(row_sum_kernel, unit_grid(n_rows * heads), dim3(256), 0, st, pc, heads, ps, row_dot);
    float *piece_de = ds_dst ? ps : nullptr;       // the piece sums above have been consumed by then
#define SYLVIE_SBWD(KV) \
    hipLaunchKernelGGL(softmax_bwd_kernel<KV>, group_grid(n_pieces), block, 0, st, pc, col, alpha, dalpha, s_dst, \
                       s_src, slope, row_dot, de, piece_de)
    SYLVIE_BY_HEADS(heads, SYLVIE_SBWD);
#undef SYLVIE_SBWD
    if (ds_dst)
        hipLaunchKernelGGL(row_sum_kernel, unit_grid(n_rows * heads), dim3(256), 0, st, pc, heads, ps, ds_dst);
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
    return sylvie_edge_softmax_bwd_heads(piece_ptr, piece_row, row_piece, n_pieces, n_rows, col, alpha, dalpha,
                                         s_dst, s_src, 1, slope, de, nullptr, workspace, workspace_bytes, stream);
}

extern "C" size_t sylvie_scaled_column_sum_workspace_bytes(int64_t n, int32_t F)
{
    if (n < 0 || F < 1) return 0;
    return static_cast<size_t>((n + sylvie::kColSumRows - 1) / sylvie::kColSumRows) * static_cast<size_t>(F) *
           sizeof(float);
}

extern "C" int32_t sylvie_scaled_column_sum_heads(const float *X, int64_t ld_x, int64_t n, int32_t F,
                                                  int32_t heads, const float *s, float *out, const float *s2,
                                                  int64_t n2, float *out2, void *workspace,
                                                  size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_scaled_column_sum_heads";
    if (!s2) n2 = 0;
    const int64_t rows = n > n2 ? n : n2;
    if (n < 0 || n2 < 0 || rows >= (int64_t(1) << 31) || F < 1 || F > 65536 || ld_x < F)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (heads < 1 || F % heads != 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: heads must divide F (got %d, F = %d)", name, heads, F);
    if (!out || (s2 && !out2)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null output", name);
    if (rows > 0 && (!X || (n > 0 && !s))) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    const int64_t slabs = (rows + kColSumRows - 1) / kColSumRows;
    const size_t one = sylvie_scaled_column_sum_workspace_bytes(rows, F);
    if (slabs > 0 && (!workspace || workspace_bytes < (s2 ? 2 * one : one)))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *part = static_cast<float *>(workspace);
    float *part2 = s2 ? part + slabs * F : nullptr;
    const int Fh = F / heads;
    if (slabs > 0) {
        const bool v4 = Fh % 4 == 0 && ld_x % 4 == 0 && aligned(X, 16);
        if (v4)
            hipLaunchKernelGGL(scaled_column_sum_slab_kernel<4>,
                               dim3(static_cast<unsigned>(slabs), (F + 4 * kWave - 1) / (4 * kWave)), dim3(256), 0,
                               st, X, ld_x, F, Fh, heads, s, n, part, s2, n2, part2);
        else
            hipLaunchKernelGGL(scaled_column_sum_slab_kernel<1>,
                               dim3(static_cast<unsigned>(slabs), (F + kWave - 1) / kWave), dim3(256), 0, st, X,
                               ld_x, F, Fh, heads, s, n, part, s2, n2, part2);
    }
    const dim3 jg((F + kWave - 1) / kWave);
    hipLaunchKernelGGL(scaled_column_sum_join_kernel, jg, dim3(256), 0, st, part, slabs, F, out);
    if (s2) hipLaunchKernelGGL(scaled_column_sum_join_kernel, jg, dim3(256), 0, st, part2, slabs, F, out2);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_scaled_column_sum(const float *X, int64_t ld_x, int64_t n, int32_t F,
                                            const float *s, float *out, void *workspace,
                                            size_t workspace_bytes, void *stream)
{
    return sylvie_scaled_column_sum_heads(X, ld_x, n, F, 1, s, out, nullptr, 0, nullptr, workspace,
                                          workspace_bytes, stream);
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

extern "C" int32_t sylvie_rank1_add_heads(float *X, int64_t ld_x, int32_t F, int32_t heads, const float *s1,
                                          const float *a1, int64_t n1, const float *s2, const float *a2,
                                          int64_t n2, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_rank1_add_heads";
    if (!s1) n1 = 0;
    if (!s2) n2 = 0;
    const int64_t rows = n1 > n2 ? n1 : n2;
    if (n1 < 0 || n2 < 0 || rows >= (int64_t(1) << 31) || F < 1 || F > 65536 || ld_x < F)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (heads < 1 || F % heads != 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: heads must divide F (got %d, F = %d)", name, heads, F);
    if (rows == 0) return SYLVIE_OK;
    if (!X || (s1 && !a1) || (s2 && !a2)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    const int Fh = F / heads;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (rows * static_cast<int64_t>(F) >= (int64_t(1) << 39))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: too many elements", name);
    if (Fh % 4 == 0 && ld_x % 4 == 0 && aligned(X, 16)) {
        const int64_t total = rows * (F / 4);
        hipLaunchKernelGGL(rank1_pair_kernel<4>, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st,
                           X, ld_x, rows, F, Fh, heads, s1, a1, n1, s2, a2, n2);
    } else {
        const int64_t total = rows * F;
        hipLaunchKernelGGL(rank1_pair_kernel<1>, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256), 0, st,
                           X, ld_x, rows, F, Fh, heads, s1, a1, n1, s2, a2, n2);
    }
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
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool v4 = F % 4 == 0 && ld_in % 4 == 0 && ld_out % 4 == 0 && aligned(in, 16) && aligned(out, 16) &&
                    (fwd || (ld_gate % 4 == 0 && aligned(gate, 16)));
    const int64_t total = n * (v4 ? F / 4 : F);
    const dim3 grid(static_cast<unsigned>((total + 255) / 256));
#define SYLVIE_RELU(FWDV, V) \
    hipLaunchKernelGGL((relu_kernel<FWDV, V>), grid, dim3(256), 0, st, in, ld_in, gate, ld_gate, n, F, out, ld_out)
    if (fwd && v4) SYLVIE_RELU(true, 4);
    else if (fwd) SYLVIE_RELU(true, 1);
    else if (v4) SYLVIE_RELU(false, 4);
    else SYLVIE_RELU(false, 1);
#undef SYLVIE_RELU
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
