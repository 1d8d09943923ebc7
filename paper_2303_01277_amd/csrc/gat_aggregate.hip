// Aggregation of the attention model (the GAT evaluated in Sec. 4; Eq. 1 with learned edge
// weights), all heads in one launch:
//   Y[v][c] = act( sum_e alpha[i_e][c / F] X[col_e][c]  +  s1[v][c / F] a1[c]  +  s2[v][c / F] a2[c] )
// over the entries e of row v, with `heads` weights per entry stored side by side
// (alpha[i][0 .. heads)), F = d / heads columns per head, i_e = e or w_index[e].  Forward it is
// Z = sum alpha P_u (act = relu on the hidden layers); backward, through the transposed
// operator, it is dP = alpha^T dZ plus the two rank-1 terms that carry the gradient of the
// scores (s1 = summed score gradients of the source side, s2 of the destination side, a1 / a2
// the attention vectors), with the weights still in the forward operator's entry order and
// `w_index` the transposition's entry map.
//
// Shape of the work: as in the plain CSR aggregation, one wavefront per row, lane L holds VEC
// adjacent columns per pass (a gathered row is one contiguous run per pass), long rows are cut
// into tasks of `chunk` entries whose partial sums a second kernel adds in task order.  What
// differs is the weight: it depends on the lane's head, so the lanes that own the 64 entries
// of a batch put the entries' weights into a wave-private LDS table and every lane reads the
// weight of its own head from there.
//
// The backward launch can also produce the sampled product of the softmax backward,
// dalpha[i_e][k] = dZ_v[k F ..) . P_u[k F ..) for entry e = (u, v) of the transposed operator:
// the wavefront of row u gathers dZ_v for the aggregation anyway, so it keeps its own row P_u in
// registers, multiplies, and reduces over the lanes of each head -- the product costs no gather
// of its own (it would fetch a whole row of P per entry otherwise).
#include "common.hpp"
#include "validate.hpp"

namespace sylvie {

constexpr int kAttWavesPerBlock = 2;
constexpr int kMaxHeads = 8;

struct AttArgs {
    const int64_t *rowptr;
    const int32_t *col;
    const float *w;             // [entries][heads]
    const int64_t *w_index;     // optional: entry e reads w[w_index[e]][.]
    int heads;
    int head_cols;              // F = d / heads
    int w_vec;                  // floats per load of an entry's weights (4, 2 or 1)
    int64_t n_rows;
    const float *X;
    int64_t ld_x;
    int d;
    float *Y;
    int64_t ld_y;
    const float *s1, *a1;       // optional rank-1 term on rows [0, n1): s1[v][head] * a1[c]
    int64_t n1;
    const float *s2, *a2;       // the same on rows [0, n2), added after the first
    int64_t n2;
    int relu;
    int chunk;                  // 0: never split
    const int32_t *long_rows;
    const int64_t *long_ptr;
    int64_t n_long;
    float *workspace;
    // sampled product: sdd_out[i_e][head] = X[col_e][head's columns] . B[v][head's columns]
    const float *B;
    int64_t ld_b;
    float *sdd_out;
};

// Sum over the L lanes of an aligned lane group (L a power of two), left in every lane of it.
template <int L>
__device__ __forceinline__ float lane_group_sum(float v)
{
    if constexpr (L >= 2) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    if constexpr (L >= 4) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    if constexpr (L >= 8) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    if constexpr (L >= 16) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true)); // row_mirror
    if constexpr (L >= 32) v += __shfl_xor(v, 16);
    if constexpr (L >= 64) v += __shfl_xor(v, 32);
    return v;
}

// acc[p][t] += sum over entries [e0, e1) of w[i_e][head of the column] * X[col_e][column(p, t)]
// SDD = lanes per head (0: no sampled product; otherwise P = 1 and a head's columns are the VEC
// columns of SDD adjacent lanes): the entries' products with the row's own slice `own` of B go
// through the second LDS table `tab` ([slot][head]) and leave as one store per entry by the lane
// that owns the entry.
template <int VEC, int P, int SDD>
__device__ __forceinline__ void attention_gather(float (&acc)[P][VEC], int64_t e0, int64_t e1,
                                                 const AttArgs &a, int lane, float *wl,
                                                 [[maybe_unused]] const float (&own)[VEC],
                                                 [[maybe_unused]] float *tab)
{
    static_assert(SDD == 0 || P == 1, "the sampled product needs the whole row in one pass");
    constexpr int U = (P >= 4) ? 2 : (8 / P);  // gathers in flight
    const int K = a.heads;
    // column offsets of this lane; lanes past the row width re-read its last vector (never
    // stored) so that no load needs a predicate
    int coff[P], head[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int cc = (p * 64 + lane) * VEC;
        coff[p] = cc < a.d ? cc : a.d - VEC;
        head[p] = coff[p] / a.head_cols;
    }
    for (int64_t base = e0; base < e1; base += 64) {
        const int cnt = static_cast<int>(e1 - base < 64 ? e1 - base : 64);
        int my_c = 0;
        [[maybe_unused]] int64_t my_we = 0;
        wave_lds_sync();        // the previous batch's weights have been read
        if (lane < cnt) {
            my_c = a.col[base + lane];
            const int64_t we = a.w_index ? a.w_index[base + lane] : base + lane;
            my_we = we;
            const float *wp = a.w + we * K;
            float *mine = wl + lane * K;
            if (a.w_vec == 4) {
                for (int k = 0; k < K; k += 4)
                    *reinterpret_cast<float4 *>(mine + k) = *reinterpret_cast<const float4 *>(wp + k);
            } else if (a.w_vec == 2) {
                for (int k = 0; k < K; k += 2)
                    *reinterpret_cast<float2 *>(mine + k) = *reinterpret_cast<const float2 *>(wp + k);
            } else {
                for (int k = 0; k < K; ++k) mine[k] = wp[k];
            }
        }
        wave_lds_sync();        // every lane reads the weights of every entry below
        // address of the lane's own gathered row, computed once on the vector unit; an entry's
        // row is then addressed by two lane reads
        const uintptr_t my_xrow = reinterpret_cast<uintptr_t>(a.X + static_cast<int64_t>(my_c) * a.ld_x);
        const int my_xlo = static_cast<int>(static_cast<uint32_t>(my_xrow));
        const int my_xhi = static_cast<int>(static_cast<uint32_t>(my_xrow >> 32));
        auto xrow_of_slot = [&](int slot) -> const float * {
            const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(my_xlo, slot));
            const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(my_xhi, slot));
            return reinterpret_cast<const float *>((static_cast<uint64_t>(hi) << 32) | lo);
        };
        int j = 0;
        for (; j + U <= cnt; j += U) {
            float x[U][P][VEC];
            float wv[U][P];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float *xr = xrow_of_slot(j + u);
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    load_vec_at<VEC>(x[u][p], xr, static_cast<uint32_t>(coff[p]) * 4u);
                    wv[u][p] = wl[(j + u) * K + head[p]];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int p = 0; p < P; ++p)
#pragma unroll
                    for (int t = 0; t < VEC; ++t) acc[p][t] = fmaf(wv[u][p], x[u][p][t], acc[p][t]);
            if constexpr (SDD > 0) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float dot = 0.0f;
#pragma unroll
                    for (int t = 0; t < VEC; ++t) dot = fmaf(x[u][0][t], own[t], dot);
                    dot = lane_group_sum<SDD>(dot);
                    if ((lane & (SDD - 1)) == 0 && lane * VEC < a.d) tab[(j + u) * K + head[0]] = dot;
                }
            }
        }
        for (; j < cnt; ++j) {
            const float *xr = xrow_of_slot(j);
            float x[P][VEC];
            float wv[P];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                load_vec_at<VEC>(x[p], xr, static_cast<uint32_t>(coff[p]) * 4u);
                wv[p] = wl[j * K + head[p]];
            }
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int t = 0; t < VEC; ++t) acc[p][t] = fmaf(wv[p], x[p][t], acc[p][t]);
            if constexpr (SDD > 0) {
                float dot = 0.0f;
#pragma unroll
                for (int t = 0; t < VEC; ++t) dot = fmaf(x[0][t], own[t], dot);
                dot = lane_group_sum<SDD>(dot);
                if ((lane & (SDD - 1)) == 0 && lane * VEC < a.d) tab[j * K + head[0]] = dot;
            }
        }
        if constexpr (SDD > 0) {
            wave_lds_sync();    // the products of the batch are in the table
            if (lane < cnt) {
                float *op = a.sdd_out + my_we * K;
                const float *mine = tab + lane * K;
                if (a.w_vec == 4) {
                    for (int k = 0; k < K; k += 4)
                        *reinterpret_cast<float4 *>(op + k) = *reinterpret_cast<const float4 *>(mine + k);
                } else if (a.w_vec == 2) {
                    for (int k = 0; k < K; k += 2)
                        *reinterpret_cast<float2 *>(op + k) = *reinterpret_cast<const float2 *>(mine + k);
                } else {
                    for (int k = 0; k < K; ++k) op[k] = mine[k];
                }
            }
        }
    }
}

// The finished sums of row v, columns cc .. cc + VEC - 1: rank-1 terms (each a product and an
// add in single precision, in the order 1, 2), then the activation.
template <int VEC>
__device__ __forceinline__ void attention_tail(const AttArgs &a, int64_t v, int cc, float (&o)[VEC])
{
    const int hk = cc / a.head_cols;
    if (a.s1 && v < a.n1) {
        const float s = a.s1[v * a.heads + hk];
#pragma unroll
        for (int t = 0; t < VEC; ++t) {
            const float step = s * a.a1[cc + t];
            o[t] = o[t] + step;
        }
    }
    if (a.s2 && v < a.n2) {
        const float s = a.s2[v * a.heads + hk];
#pragma unroll
        for (int t = 0; t < VEC; ++t) {
            const float step = s * a.a2[cc + t];
            o[t] = o[t] + step;
        }
    }
    if (a.relu) {
#pragma unroll
        for (int t = 0; t < VEC; ++t) o[t] = o[t] > 0.0f ? o[t] : 0.0f;
    }
}

// The first workgroups take the tasks of the long rows (they start first, so the heaviest rows
// never trail the launch); every later wavefront takes one ordinary row and skips the long ones.
template <int VEC, int P, int SDD>
__global__ __launch_bounds__(kAttWavesPerBlock *kWave) void attention_gather_kernel(AttArgs a, int64_t n_tasks)
{
    __shared__ __align__(16) float wtab[kAttWavesPerBlock][64 * kMaxHeads];
    __shared__ __align__(16) float ptab[kAttWavesPerBlock][SDD > 0 ? 64 * kMaxHeads : 4];
    // the row's own slice of B for the sampled product
    float own[VEC];
#pragma unroll
    for (int t = 0; t < VEC; ++t) own[t] = 0.0f;
    auto load_own = [&](int64_t v) {
        if constexpr (SDD > 0) {
            const int cc = lane_id() * VEC;
            if (cc < a.d) load_vec<VEC>(own, a.B + v * a.ld_b + cc);
        }
    };
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t task_blocks = (n_tasks + kAttWavesPerBlock - 1) / kAttWavesPerBlock;
    float acc[P][VEC];
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int t = 0; t < VEC; ++t) acc[p][t] = 0.0f;

    if (static_cast<int64_t>(blockIdx.x) < task_blocks) {
        const int64_t t = static_cast<int64_t>(blockIdx.x) * kAttWavesPerBlock + wave;
        if (t >= n_tasks) return;
        // long row that owns task t: last i with long_ptr[i] <= t
        int64_t lo = 0, hi = a.n_long;
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (a.long_ptr[mid] <= t) lo = mid; else hi = mid;
        }
        lo = uniform(lo);
        const int64_t v = a.long_rows[lo];
        const int64_t piece = t - a.long_ptr[lo];
        const int64_t r0 = uniform(a.rowptr[v]);
        const int64_t r1 = uniform(a.rowptr[v + 1]);
        const int64_t e0 = r0 + piece * a.chunk;
        const int64_t e1 = e0 + a.chunk < r1 ? e0 + a.chunk : r1;
        load_own(v);
        attention_gather<VEC, P, SDD>(acc, e0, e1, a, lane, wtab[wave], own, ptab[wave]);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int cc = (p * 64 + lane) * VEC;
            if (cc < a.d) store_vec<VEC>(a.workspace + t * a.d + cc, acc[p]);
        }
        return;
    }

    const int64_t v = (static_cast<int64_t>(blockIdx.x) - task_blocks) * kAttWavesPerBlock + wave;
    if (v >= a.n_rows) return;
    const int64_t e0 = uniform(a.rowptr[v]);
    const int64_t e1 = uniform(a.rowptr[v + 1]);
    if (a.chunk > 0 && e1 - e0 > a.chunk) return;
    load_own(v);
    attention_gather<VEC, P, SDD>(acc, e0, e1, a, lane, wtab[wave], own, ptab[wave]);
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int cc = (p * 64 + lane) * VEC;
        if (cc < a.d) {
            attention_tail<VEC>(a, v, cc, acc[p]);
            stream_store<VEC>(a.Y + v * a.ld_y + cc, acc[p]);   // written once, read by a later launch
        }
    }
}

// One wavefront per long row: add its partial sums in task order, finish the row.
template <int VEC>
__global__ __launch_bounds__(kAttWavesPerBlock *kWave) void attention_reduce_kernel(AttArgs a)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kAttWavesPerBlock + wave;
    if (i >= a.n_long) return;
    const int64_t v = a.long_rows[i];
    const int64_t t0 = a.long_ptr[i], t1 = a.long_ptr[i + 1];
    for (int cc = lane * VEC; cc < a.d; cc += 64 * VEC) {
        float acc[VEC];
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] = 0.0f;
        for (int64_t t = t0; t < t1; ++t) {
            float part[VEC];
            load_vec<VEC>(part, a.workspace + t * a.d + cc);
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] += part[q];
        }
        attention_tail<VEC>(a, v, cc, acc);
        stream_store<VEC>(a.Y + v * a.ld_y + cc, acc);
    }
}

template <int VEC, int P, int SDD = 0>
static void attention_launch(const AttArgs &a, int64_t n_tasks, hipStream_t st)
{
    const int64_t nt = a.n_long > 0 ? n_tasks : 0;
    const int64_t blocks = (nt + kAttWavesPerBlock - 1) / kAttWavesPerBlock +
                           (a.n_rows + kAttWavesPerBlock - 1) / kAttWavesPerBlock;
    const dim3 block(kAttWavesPerBlock * kWave);
    hipLaunchKernelGGL((attention_gather_kernel<VEC, P, SDD>), dim3(static_cast<unsigned>(blocks)), block, 0, st, a, nt);
    if (a.n_long > 0) {
        const dim3 rg(static_cast<unsigned>((a.n_long + kAttWavesPerBlock - 1) / kAttWavesPerBlock));
        hipLaunchKernelGGL((attention_reduce_kernel<VEC>), rg, block, 0, st, a);
    }
}

template <int VEC>
static bool attention_launch_vec(const AttArgs &a, int64_t n_tasks, hipStream_t st)
{
    const int lanes = (a.d + VEC - 1) / VEC;
    if (lanes <= 64) attention_launch<VEC, 1>(a, n_tasks, st);
    else if (lanes <= 128) attention_launch<VEC, 2>(a, n_tasks, st);
    else if (lanes <= 192) attention_launch<VEC, 3>(a, n_tasks, st);
    else if (lanes <= 256) attention_launch<VEC, 4>(a, n_tasks, st);
    else if (lanes <= 384) attention_launch<VEC, 6>(a, n_tasks, st);
    else if (lanes <= 512) attention_launch<VEC, 8>(a, n_tasks, st);
    else return false;
    return true;
}

// Lanes per head for the launch that also forms the sampled product, or 0 if the shape has no
// such launch: four columns per lane, the whole row in one pass, heads on aligned lane groups.
static int sampled_product_lanes(int d, int heads)
{
    if (d % heads != 0 || d > 256) return 0;
    const int F = d / heads;
    for (int lanes = 4; lanes <= 64; lanes *= 2)
        if (F == 4 * lanes) return lanes;
    return 0;
}

static int32_t attention_call(const char *name, const int64_t *rowptr, const int32_t *col, const float *w,
                              const int64_t *w_index, int32_t heads, int64_t n_rows, const float *X,
                              int64_t ld_x, int32_t d, float *Y, int64_t ld_y, const float *s1, const float *a1,
                              int64_t n1, const float *s2, const float *a2, int64_t n2, int32_t relu,
                              const float *Bm, int64_t ld_b, float *sdd_out, int32_t chunk,
                              const int32_t *long_rows, const int64_t *long_ptr, int64_t n_long, int64_t n_tasks,
                              float *workspace, size_t workspace_bytes, void *stream)
{
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_rows %lld out of range", name, (long long)n_rows);
    if (d < 1 || d > 65536) return fail(SYLVIE_ERR_INVALID_ARG, "%s: d %d out of range", name, d);
    if (heads < 1 || heads > kMaxHeads || d % heads != 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: heads must be 1 .. %d and divide d (got %d, d = %d)", name,
                    kMaxHeads, heads, d);
    if (ld_x < d || ld_y < d) return fail(SYLVIE_ERR_INVALID_ARG, "%s: leading dimension < d", name);
    if (n_long < 0 || n_tasks < 0 || n1 < 0 || n2 < 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative count", name);
    const int sdd = sdd_out ? sampled_product_lanes(d, heads) : 0;
    if (sdd_out) {
        if (!Bm || ld_b < d) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad second operand", name);
        if (sdd == 0)
            return fail(SYLVIE_ERR_UNIMPLEMENTED,
                        "%s: d = %d with %d heads has no launch that also forms the sampled product (needs "
                        "d <= 256 and d / heads = 16, 32, 64, 128 or 256); call sylvie_sddmm_heads", name, d, heads);
        if (!aligned(X, 16) || !aligned(Y, 16) || !aligned(Bm, 16) || ld_x % 4 || ld_y % 4 || ld_b % 4 ||
            !aligned(sdd_out, 4))
            return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: the sampled product needs 16-byte aligned rows", name);
    }
    if (n_rows == 0) return SYLVIE_OK;
    if (!rowptr || !col || !w || !X || !Y) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if ((s1 && !a1) || (s2 && !a2))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: a rank-1 term needs both of its vectors", name);
    if (!aligned(rowptr, 8) || !aligned(col, 4) || !aligned(w, 4) || !aligned(X, 4) || !aligned(Y, 4) ||
        (w_index && !aligned(w_index, 8)))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned pointer", name);
    if (n_long > 0) {
        if (chunk <= 0 || chunk % 64 != 0)
            return fail(SYLVIE_ERR_INVALID_ARG, "%s: chunk must be a positive multiple of 64", name);
        if (!long_rows || !long_ptr || !workspace)
            return fail(SYLVIE_ERR_INVALID_ARG, "%s: long-row plan has null pointers", name);
        if (n_tasks < n_long || n_tasks >= (int64_t(1) << 31))
            return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_tasks out of range", name);
        if (workspace_bytes < static_cast<size_t>(n_tasks) * static_cast<size_t>(d) * 4)
            return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace %zu B < %zu B", name, workspace_bytes,
                        static_cast<size_t>(n_tasks) * static_cast<size_t>(d) * 4);
        if (!aligned(workspace, 16))
            return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: workspace needs 16-byte alignment", name);
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (validate_enabled()) {
        Validator v(name, st);
        v.csr(rowptr, col, 0, n_rows, -1, -1);
        const int32_t rc = v.finish();
        if (rc != SYLVIE_OK) return rc;
    }
    AttArgs a;
    a.rowptr = rowptr; a.col = col; a.w = w; a.w_index = w_index; a.heads = heads; a.head_cols = d / heads;
    // an entry's weights, and its sampled products, move `w_vec` floats at a time
    const bool v4 = heads % 4 == 0 && aligned(w, 16) && (!sdd_out || aligned(sdd_out, 16));
    const bool v2 = heads % 2 == 0 && aligned(w, 8) && (!sdd_out || aligned(sdd_out, 8));
    a.w_vec = v4 ? 4 : v2 ? 2 : 1;
    a.n_rows = n_rows; a.X = X; a.ld_x = ld_x; a.d = d; a.Y = Y; a.ld_y = ld_y;
    a.s1 = s1; a.a1 = a1; a.n1 = n1; a.s2 = s2; a.a2 = a2; a.n2 = n2; a.relu = relu != 0;
    a.chunk = n_long > 0 ? chunk : 0;
    a.long_rows = long_rows; a.long_ptr = long_ptr; a.n_long = n_long; a.workspace = workspace;
    a.B = Bm; a.ld_b = ld_b; a.sdd_out = sdd_out;
    if (sdd) {
        if (sdd == 4) attention_launch<4, 1, 4>(a, n_tasks, st);
        else if (sdd == 8) attention_launch<4, 1, 8>(a, n_tasks, st);
        else if (sdd == 16) attention_launch<4, 1, 16>(a, n_tasks, st);
        else if (sdd == 32) attention_launch<4, 1, 32>(a, n_tasks, st);
        else attention_launch<4, 1, 64>(a, n_tasks, st);
        SYLVIE_HIP_LAUNCH_CHECK(name);
        return SYLVIE_OK;
    }
    // a lane's VEC adjacent columns belong to one head
    const int F = a.head_cols;
    const bool a16 = aligned(X, 16) && aligned(Y, 16) && ld_x % 4 == 0 && ld_y % 4 == 0 && F % 4 == 0;
    const bool a8 = aligned(X, 8) && aligned(Y, 8) && ld_x % 2 == 0 && ld_y % 2 == 0 && F % 2 == 0;
    bool ok;
    if (a16) ok = attention_launch_vec<4>(a, n_tasks, st);
    else if (a8) ok = attention_launch_vec<2>(a, n_tasks, st);
    else ok = attention_launch_vec<1>(a, n_tasks, st);
    if (!ok)
        return fail(SYLVIE_ERR_UNIMPLEMENTED,
                    "%s: d = %d is wider than one launch covers at this alignment (2048 / 1024 / 512 "
                    "columns for 16 / 8 / 4-byte aligned rows); split the heads across calls", name, d);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

}  // namespace sylvie

extern "C" int32_t sylvie_aggregate_csr_attention(
    const int64_t *rowptr, const int32_t *col, const float *w, const int64_t *w_index, int32_t heads,
    int64_t n_rows, const float *X, int64_t ld_x, int32_t d, float *Y, int64_t ld_y, const float *s1,
    const float *a1, int64_t n1, const float *s2, const float *a2, int64_t n2, int32_t relu,
    int32_t chunk, const int32_t *long_rows, const int64_t *long_ptr, int64_t n_long, int64_t n_tasks,
    float *workspace, size_t workspace_bytes, void *stream)
{
    return sylvie::attention_call("sylvie_aggregate_csr_attention", rowptr, col, w, w_index, heads, n_rows, X,
                                  ld_x, d, Y, ld_y, s1, a1, n1, s2, a2, n2, relu, nullptr, 0, nullptr, chunk,
                                  long_rows, long_ptr, n_long, n_tasks, workspace, workspace_bytes, stream);
}

extern "C" int32_t sylvie_aggregate_csr_attention_sddmm(
    const int64_t *rowptr, const int32_t *col, const float *w, const int64_t *w_index, int32_t heads,
    int64_t n_rows, const float *X, int64_t ld_x, int32_t d, float *Y, int64_t ld_y, const float *B,
    int64_t ld_b, float *dalpha, int32_t chunk, const int32_t *long_rows, const int64_t *long_ptr,
    int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes, void *stream)
{
    const char *name = "sylvie_aggregate_csr_attention_sddmm";
    if (!dalpha) return sylvie::fail(SYLVIE_ERR_INVALID_ARG, "%s: null output", name);
    return sylvie::attention_call(name, rowptr, col, w, w_index, heads, n_rows, X, ld_x, d, Y, ld_y, nullptr,
                                  nullptr, 0, nullptr, nullptr, 0, 0, B, ld_b, dalpha, chunk, long_rows, long_ptr,
                                  n_long, n_tasks, workspace, workspace_bytes, stream);
}

extern "C" int32_t sylvie_aggregate_csr_attention_sddmm_supported(int32_t d, int32_t heads)
{
    if (d < 1 || heads < 1 || heads > sylvie::kMaxHeads) return 0;
    return sylvie::sampled_product_lanes(d, heads) > 0 ? 1 : 0;
}
