// Dense feature transform of a GNN layer on the matrix cores (Eq. 2; Alg. 1
// H = sigma(Z W); Alg. 2 weight gradient G = Z^T M and feature gradient
// dZ = M W^T with M = J o sigma'(.)), float32 in, float32 MFMA accumulate.
//
// One 256-thread workgroup (4 wavefronts) computes a 128 x 128 output tile; each
// wavefront owns a 64 x 64 quarter as 2 x 2 blocks of v_mfma_f32_32x32x2_f32.
// Operand tiles (16 deep) go global -> registers -> LDS, stored [k][m] / [k][n] so
// that the 32 lanes feeding one MFMA operand read 32 consecutive floats.  The
// next tile's global loads are in flight while the current one is multiplied.
// ReLU, the ReLU mask of the backward pass and the [A1 | A2] column split of
// GraphSAGE are applied on the fly in the loaders / the epilogue.
#include "common.hpp"

namespace sylvie {

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int NI = BK / 8;        // 4-element fetches per thread per operand tile
constexpr int KCT = BK / 4;       // threads that share one row of a k-contiguous tile
constexpr int kPadXC = 128;      // row stride of a tile filled along x (16-byte rows)
constexpr int kPadKC = 130;      // row stride of a tile filled along k (spreads banks)
constexpr int kGemmThreads = 256;

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Left operand [A1 | A2]: n rows, k1 + k2 columns.
struct CatA {
    const float *A1; int64_t ld1; int k1;
    const float *A2; int64_t ld2; int k2;
    int64_t n;
};
// M = relu ? J o [H > 0] : J, n x h.
struct MaskedJ {
    const float *J; int64_t ldj;
    const float *H; int64_t ldh;
    int relu; int h; int64_t n;
};

// ---- 4-element fetches along the contiguous axis (zero outside the matrix) ----

template <int V>
__device__ __forceinline__ void fetch4(float (&o)[4], const float *p, int valid)
{
    // valid = number of in-range elements among the 4 (V == 4: 0 or 4)
    if constexpr (V == 4) {
        if (valid > 0) {
            const float4 v = *reinterpret_cast<const float4 *>(p);
            o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
        } else {
            o[0] = o[1] = o[2] = o[3] = 0.0f;
        }
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = t < valid ? p[t] : 0.0f;
    }
}

// [A1|A2](row, k .. k+3)
template <int V>
__device__ __forceinline__ void cat_row4(float (&o)[4], const CatA &a, int64_t row, int k)
{
    const int K = a.k1 + a.k2;
    if (row >= a.n || k >= K) { o[0] = o[1] = o[2] = o[3] = 0.0f; return; }
    if constexpr (V == 4) {
        const float *p = k < a.k1 ? a.A1 + row * a.ld1 + k : a.A2 + row * a.ld2 + (k - a.k1);
        fetch4<4>(o, p, 4);
    } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int kk = k + t;
            o[t] = kk >= K ? 0.0f
                           : (kk < a.k1 ? a.A1[row * a.ld1 + kk] : a.A2[row * a.ld2 + (kk - a.k1)]);
        }
    }
}

// M(row, j .. j+3)
template <int V>
__device__ __forceinline__ void masked4(float (&o)[4], const MaskedJ &m, int64_t row, int j)
{
    if (row >= m.n || j >= m.h) { o[0] = o[1] = o[2] = o[3] = 0.0f; return; }
    const int valid = m.h - j < 4 ? m.h - j : 4;
    fetch4<V>(o, m.J + row * m.ldj + j, valid);
    if (m.relu) {
        float hv[4];
        fetch4<V>(hv, m.H + row * m.ldh + j, valid);
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = hv[t] > 0.0f ? o[t] : 0.0f;
    }
}

// ---- LDS tile fill patterns ----------------------------------------------------
// XC: the 4 fetched elements run along x (tile columns): thread -> (k = t/32 + 8 i, x = 4 (t%32))
// KC: the 4 fetched elements run along k (tile rows):    thread -> (x = t/KCT + (256/KCT) i,
//                                                                   k = 4 (t%KCT)),  i < NI

__device__ __forceinline__ void put_xc(float *T, int i, const float (&v)[4])
{
    const int t = threadIdx.x;
    float *p = T + (t / 32 + 8 * i) * kPadXC + 4 * (t % 32);
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void put_kc(float *T, int i, const float (&v)[4])
{
    const int t = threadIdx.x;
    float *p = T + (4 * (t % KCT)) * kPadKC + (t / KCT + (256 / KCT) * i);
#pragma unroll
    for (int q = 0; q < 4; ++q) p[q * kPadKC] = v[q];
}

// 64 x 64 quarter of the block tile: 8 k-steps of 2, 2 x 2 MFMA blocks each.  The
// operands of step k+1 are read from LDS before the MFMAs of step k are issued, so
// the LDS latency hides behind the matrix pipe.
template <int PADA, int PADB>
__device__ __forceinline__ void mma_tile(floatx16 (&acc)[2][2], const float *As, const float *Bs,
                                         int wm, int wn, int lane)
{
    const int l32 = lane & 31, kh = lane >> 5;
    const float *pa = As + kh * PADA + wm + l32;
    const float *pb = Bs + kh * PADB + wn + l32;
    float a[2][2], b[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[0][i] = pa[i * 32];
#pragma unroll
    for (int j = 0; j < 2; ++j) b[0][j] = pb[j * 32];
#pragma unroll
    for (int s = 0; s < BK / 2; ++s) {
        const int cur = s & 1, nxt = cur ^ 1;
        if (s + 1 < BK / 2) {
#pragma unroll
            for (int i = 0; i < 2; ++i) a[nxt][i] = pa[(2 * s + 2) * PADA + i * 32];
#pragma unroll
            for (int j = 0; j < 2; ++j) b[nxt][j] = pb[(2 * s + 2) * PADB + j * 32];
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the reads above ahead of the MFMAs below
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
    }
}

// Element r of lane's accumulator block sits at row 8 (r/4) + 4 (lane/32) + r%4,
// column lane%32 of the 32 x 32 block.
__device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r / 4) + 4 * (lane >> 5) + (r & 3); }

// ---- forward: H = relu?([A1|A2] W) ----------------------------------------------

template <int V>
__global__ __launch_bounds__(kGemmThreads, 3) void transform_fwd_kernel(CatA a, const float *__restrict__ Wm,
                                                                    int h, int relu,
                                                                    float *__restrict__ H, int64_t ldh)
{
    __shared__ __align__(16) float As[BK * kPadKC];
    __shared__ __align__(16) float Bs[BK * kPadXC];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x) * BM;
    const int n0 = blockIdx.y * BN;
    const int K = a.k1 + a.k2;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    float ra[NI][4], rb[NI][4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            cat_row4<V>(ra[i], a, m0 + t / KCT + (256 / KCT) * i, k0 + 4 * (t % KCT));
            const int k = k0 + t / 32 + 8 * i, x = n0 + 4 * (t % 32);
            const int valid = (k < K && x < h) ? (h - x < 4 ? h - x : 4) : 0;
            fetch4<V>(rb[i], Wm + static_cast<int64_t>(k) * h + x, valid);
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            put_kc(As, i, ra[i]);
            put_xc(Bs, i, rb[i]);
        }
        __syncthreads();
        if (k0 + BK < K) fetch(k0 + BK);
        mma_tile<kPadKC, kPadXC>(acc, As, Bs, wm, wn, lane);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm + i * 32 + acc_row(r, lane);
                if (row < a.n && c < h) {
                    float v = acc[i][j][r];
                    if (relu) v = v > 0.0f ? v : 0.0f;
                    H[row * ldh + c] = v;
                }
            }
        }
}

// ---- backward, feature gradient: [dA1 | dA2] = M W^T -----------------------------

template <int V>
__global__ __launch_bounds__(kGemmThreads, 3) void transform_bwd_da_kernel(
    MaskedJ m, const float *__restrict__ Wm, int k1, int k2, float *__restrict__ dA1, int64_t ld1,
    float *__restrict__ dA2, int64_t ld2)
{
    __shared__ __align__(16) float As[BK * kPadKC];
    __shared__ __align__(16) float Bs[BK * kPadKC];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x) * BM;
    const int n0 = blockIdx.y * BN;                 // output column = row of W
    const int K = k1 + k2, h = m.h;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    float ra[NI][4], rb[NI][4];
    auto fetch = [&](int j0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            masked4<V>(ra[i], m, m0 + t / KCT + (256 / KCT) * i, j0 + 4 * (t % KCT));
            // B(k = j, n = kcol) = W[kcol][j]: contiguous along k
            const int kcol = n0 + t / KCT + (256 / KCT) * i, j = j0 + 4 * (t % KCT);
            const int valid = (kcol < K && j < h) ? (h - j < 4 ? h - j : 4) : 0;
            fetch4<V>(rb[i], Wm + static_cast<int64_t>(kcol) * h + j, valid);
        }
    };
    fetch(0);
    for (int j0 = 0; j0 < h; j0 += BK) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            put_kc(As, i, ra[i]);
            put_kc(Bs, i, rb[i]);
        }
        __syncthreads();
        if (j0 + BK < h) fetch(j0 + BK);
        mma_tile<kPadKC, kPadKC>(acc, As, Bs, wm, wn, lane);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + wm + i * 32 + acc_row(r, lane);
                if (row < m.n && c < K) {
                    if (c < k1) dA1[row * ld1 + c] = acc[i][j][r];
                    else dA2[row * ld2 + (c - k1)] = acc[i][j][r];
                }
            }
        }
}

// ---- backward, weight gradient: G = [A1|A2]^T M, summed over row slabs ------------

// Partial product of one slab of rows: part[slab][K][h].
template <int V>
__global__ __launch_bounds__(kGemmThreads, 3) void transform_bwd_g_kernel(CatA a, MaskedJ m,
                                                                      int64_t rows_per_slab,
                                                                      float *__restrict__ part)
{
    __shared__ __align__(16) float As[BK * kPadXC];
    __shared__ __align__(16) float Bs[BK * kPadXC];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int K = a.k1 + a.k2, h = m.h;
    const int m0 = blockIdx.x * BM;                 // row of G = column of [A1|A2]
    const int n0 = blockIdx.y * BN;                 // column of G
    const int64_t r_begin = static_cast<int64_t>(blockIdx.z) * rows_per_slab;
    const int64_t r_end = r_begin + rows_per_slab < a.n ? r_begin + rows_per_slab : a.n;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    float ra[NI][4], rb[NI][4];
    auto fetch = [&](int64_t r0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int64_t row = r0 + t / 32 + 8 * i;
            // A(m = kcol, k = row) = [A1|A2][row][kcol]: contiguous along m
            cat_row4<V>(ra[i], a, row < r_end ? row : a.n, m0 + 4 * (t % 32));
            masked4<V>(rb[i], m, row < r_end ? row : m.n, n0 + 4 * (t % 32));
        }
    };
    fetch(r_begin);
    for (int64_t r0 = r_begin; r0 < r_end; r0 += BK) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            put_xc(As, i, ra[i]);
            put_xc(Bs, i, rb[i]);
        }
        __syncthreads();
        if (r0 + BK < r_end) fetch(r0 + BK);
        mma_tile<kPadXC, kPadXC>(acc, As, Bs, wm, wn, lane);
    }
    float *out = part + static_cast<int64_t>(blockIdx.z) * K * h;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int c = n0 + wn + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm + i * 32 + acc_row(r, lane);
                if (row < K && c < h) out[static_cast<int64_t>(row) * h + c] = acc[i][j][r];
            }
        }
}

// G[e] = sum over slabs, ascending.
__global__ void transform_bwd_g_reduce_kernel(const float *__restrict__ part, int64_t elems,
                                              int n_slabs, float *__restrict__ G)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= elems) return;
    float s = 0.0f;
    for (int z = 0; z < n_slabs; ++z) s += part[z * elems + e];
    G[e] = s;
}

// Row slabs of the weight-gradient product: enough of them to fill the chip even when
// the output is a single tile, at most 256 (the partial products go through a workspace).
static int g_slabs(int64_t n)
{
    const int64_t s = (n + 511) / 512;
    return static_cast<int>(s < 1 ? 1 : (s > 256 ? 256 : s));
}

static int32_t check_common(const char *name, const float *A1, int64_t ld_a1, int32_t k1,
                            const float *A2, int64_t ld_a2, int32_t k2, const float *W, int32_t h,
                            int64_t n)
{
    if (n < 0 || n >= (int64_t(1) << 31)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: n out of range", name);
    if (k1 < 1 || k2 < 0 || h < 1 || k1 > 65536 || k2 > 65536 || h > 65536)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad widths k1=%d k2=%d h=%d", name, k1, k2, h);
    if (ld_a1 < k1 || (k2 > 0 && ld_a2 < k2))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: leading dimension too small", name);
    if (n == 0) return SYLVIE_OK;
    if (!A1 || !W || (k2 > 0 && !A2)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    return SYLVIE_OK;
}

}  // namespace sylvie

extern "C" int32_t sylvie_transform_fwd(const float *A1, int64_t ld_a1, int32_t k1,
                                        const float *A2, int64_t ld_a2, int32_t k2, const float *W,
                                        int32_t h, int64_t n, int32_t relu, float *H, int64_t ld_h,
                                        void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_transform_fwd";
    const int32_t rc = check_common(name, A1, ld_a1, k1, A2, ld_a2, k2, W, h, n);
    if (rc != SYLVIE_OK) return rc;
    if (ld_h < h) return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_h < h", name);
    if (n == 0) return SYLVIE_OK;
    if (!H) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null output", name);
    const bool v4 = k1 % 4 == 0 && k2 % 4 == 0 && h % 4 == 0 && ld_a1 % 4 == 0 &&
                    (k2 == 0 || ld_a2 % 4 == 0) && aligned(A1, 16) && aligned(W, 16) &&
                    (k2 == 0 || aligned(A2, 16));
    CatA a{A1, ld_a1, k1, A2, ld_a2, k2, n};
    const dim3 grid(static_cast<unsigned>((n + BM - 1) / BM), static_cast<unsigned>((h + BN - 1) / BN));
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (v4)
        hipLaunchKernelGGL(transform_fwd_kernel<4>, grid, dim3(kGemmThreads), 0, st, a, W, h, relu, H, ld_h);
    else
        hipLaunchKernelGGL(transform_fwd_kernel<1>, grid, dim3(kGemmThreads), 0, st, a, W, h, relu, H, ld_h);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" size_t sylvie_transform_bwd_workspace_bytes(int32_t k1, int32_t k2, int32_t h, int64_t n)
{
    return static_cast<size_t>(sylvie::g_slabs(n)) * static_cast<size_t>(k1 + k2) *
           static_cast<size_t>(h) * sizeof(float);
}

extern "C" int32_t sylvie_transform_bwd(const float *A1, int64_t ld_a1, int32_t k1,
                                        const float *A2, int64_t ld_a2, int32_t k2, const float *W,
                                        int32_t h, int64_t n, int32_t relu, const float *H,
                                        int64_t ld_h, const float *J, int64_t ld_j, float *G,
                                        float *dA1, int64_t ld_da1, float *dA2, int64_t ld_da2,
                                        float *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_transform_bwd";
    const int32_t rc = check_common(name, A1, ld_a1, k1, A2, ld_a2, k2, W, h, n);
    if (rc != SYLVIE_OK) return rc;
    if (ld_j < h || (relu && ld_h < h)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_j / ld_h < h", name);
    if (n == 0) return SYLVIE_OK;
    if (!J || (relu && !H)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null J / H", name);
    if (dA1 && (ld_da1 < k1 || (k2 > 0 && (!dA2 || ld_da2 < k2))))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad dA arguments", name);
    const size_t need = sylvie_transform_bwd_workspace_bytes(k1, k2, h, n);
    if (G && (!workspace || workspace_bytes < need))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace %zu B < %zu B", name, workspace_bytes, need);
    const bool v4 = k1 % 4 == 0 && k2 % 4 == 0 && h % 4 == 0 && ld_a1 % 4 == 0 &&
                    (k2 == 0 || ld_a2 % 4 == 0) && ld_j % 4 == 0 && (!relu || ld_h % 4 == 0) &&
                    aligned(A1, 16) && aligned(W, 16) && (k2 == 0 || aligned(A2, 16)) &&
                    aligned(J, 16) && (!relu || aligned(H, 16));
    CatA a{A1, ld_a1, k1, A2, ld_a2, k2, n};
    MaskedJ m{J, ld_j, H, ld_h, relu, h, n};
    const int K = k1 + k2;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (G) {
        const int slabs = g_slabs(n);
        int64_t rps = (n + slabs - 1) / slabs;
        rps = (rps + BK - 1) / BK * BK;
        const dim3 grid(static_cast<unsigned>((K + BM - 1) / BM), static_cast<unsigned>((h + BN - 1) / BN),
                        static_cast<unsigned>(slabs));
        if (v4)
            hipLaunchKernelGGL(transform_bwd_g_kernel<4>, grid, dim3(kGemmThreads), 0, st, a, m, rps, workspace);
        else
            hipLaunchKernelGGL(transform_bwd_g_kernel<1>, grid, dim3(kGemmThreads), 0, st, a, m, rps, workspace);
        const int64_t elems = static_cast<int64_t>(K) * h;
        hipLaunchKernelGGL(transform_bwd_g_reduce_kernel, dim3(static_cast<unsigned>((elems + 255) / 256)),
                           dim3(256), 0, st, workspace, elems, slabs, G);
    }
    if (dA1) {
        const dim3 grid(static_cast<unsigned>((n + BM - 1) / BM), static_cast<unsigned>((K + BN - 1) / BN));
        if (v4)
            hipLaunchKernelGGL(transform_bwd_da_kernel<4>, grid, dim3(kGemmThreads), 0, st, m, W, k1, k2, dA1, ld_da1, dA2, ld_da2);
        else
            hipLaunchKernelGGL(transform_bwd_da_kernel<1>, grid, dim3(kGemmThreads), 0, st, m, W, k1, k2, dA1, ld_da1, dA2, ld_da2);
    }
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}
