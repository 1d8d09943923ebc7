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
#include <algorithm>

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

// =====================================================================================
// Fast path: 16-byte aligned operands whose contraction length is a multiple of BK.
//
// What changes against the kernels above is everything around the MFMAs, which is
// what limits them: operands come in through buffer descriptors (tile base in SGPRs,
// one 32-bit lane offset computed once, the k advance in the scalar offset; rows past
// the end of the matrix fail the range check and read as zero), LDS is double
// buffered (one barrier per k-step), a k-contiguous operand keeps its global layout
// in LDS ([x][k], one 16-byte write per fetch, the four 16-byte pieces of a row
// permuted by a function of the row so that neither the fill nor the read pattern
// meets a bank twice) and is read back 16 bytes at a time,
// and full output tiles leave through buffer stores whose row offset is scalar.
//
// MFMA k-slots: the 16 k of a step are two groups of 8; in group g, step j (0..3)
// lanes 0-31 contract k = 8 g + j and lanes 32-63 k = 8 g + 4 + j, for both operands,
// so that one 16-byte LDS read feeds four MFMA steps.  A wavefront owns the 32-row
// blocks 32 half + 64 i (i = 0, 1) in each direction: blocks 64 apart are reachable
// with the immediate offsets of one two-address LDS read.
// =====================================================================================

constexpr int64_t kMaxFastLd = int64_t(1) << 22;   // 128 rows of this many floats stay below 2^31 bytes
constexpr int kTileKC = BM * BK;           // floats per [x][k] tile
constexpr int kTileXC = BK * 128;          // floats per [k][x] tile

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buf(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes, 0x00020000);
}
__device__ __forceinline__ void buf_load4(float (&o)[4], __amdgpu_buffer_rsrc_t b, uint32_t voff, uint32_t soff)
{
    typedef int i4 __attribute__((ext_vector_type(4)));
    const i4 v = __builtin_bit_cast(i4, __builtin_amdgcn_raw_buffer_load_b128(b, voff, soff, 0));
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = __int_as_float(v[q]);
}

// Fill patterns (256 threads, NI fetches of 4 floats each):
//   [x][k] tile: thread -> x = t/4 + 64 i, k = 4 (t%4)
//   [k][x] tile: thread -> k = t/32 + 8 i, x = 4 (t%32)
// [x][k] tile: row x holds its pieces q = 0..3 (k = 4 q .. 4 q + 3) at piece slot q ^ kc_perm(x).
// Eight (or sixteen) consecutive rows read the same q, four lanes fill the four q of one
// row: with this permutation both patterns cover all banks once.
__device__ __forceinline__ int kc_perm(int x) { return ((x >> 1) ^ (x >> 2)) & 3; }
__device__ __forceinline__ void put_f_kc(float *T, int i, const float (&v)[4])
{
    const int t = threadIdx.x, x = t / 4 + 64 * i;
    *reinterpret_cast<float4 *>(T + x * BK + 4 * ((t % 4) ^ kc_perm(x))) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void put_f_xc(float *T, int i, const float (&v)[4])
{
    const int t = threadIdx.x;
    *reinterpret_cast<float4 *>(T + (t / 32 + 8 * i) * 128 + 4 * (t % 32)) = make_float4(v[0], v[1], v[2], v[3]);
}

// One k-step (16 deep) of the 2 x 2 block product of a wavefront.
template <bool AKC, bool BKC>
__device__ __forceinline__ void mma_step(floatx16 (&acc)[2][2], const float *As, const float *Bs,
                                         int half_m, int half_n, int lane)
{
    const int l32 = lane & 31, kh = lane >> 5;
    const int xa = 32 * half_m + l32, xb = 32 * half_n + l32;
    [[maybe_unused]] float a4[2][2][4], b4[2][2][4];     // [group][block][step]
    if constexpr (AKC) {
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const float4 v = *reinterpret_cast<const float4 *>(As + (xa + 64 * i) * BK + 4 * ((2 * g + kh) ^ kc_perm(xa)));
                a4[g][i][0] = v.x; a4[g][i][1] = v.y; a4[g][i][2] = v.z; a4[g][i][3] = v.w;
            }
    }
    if constexpr (BKC) {
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const float4 v = *reinterpret_cast<const float4 *>(Bs + (xb + 64 * i) * BK + 4 * ((2 * g + kh) ^ kc_perm(xb)));
                b4[g][i][0] = v.x; b4[g][i][1] = v.y; b4[g][i][2] = v.z; b4[g][i][3] = v.w;
            }
    }
    // [k][x] operands: one dword per MFMA step, read one step ahead
    const float *pa = As + 4 * kh * 128 + xa;
    const float *pb = Bs + 4 * kh * 128 + xb;
    [[maybe_unused]] float a1[2][2], b1[2][2];
    if constexpr (!AKC) {
#pragma unroll
        for (int i = 0; i < 2; ++i) a1[0][i] = pa[64 * i];
    }
    if constexpr (!BKC) {
#pragma unroll
        for (int i = 0; i < 2; ++i) b1[0][i] = pb[64 * i];
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int g = s >> 2, j = s & 3, cur = s & 1, nxt = cur ^ 1;
        if (s + 1 < 8) {
            const int row = 8 * ((s + 1) >> 2) + ((s + 1) & 3);
            if constexpr (!AKC) {
#pragma unroll
                for (int i = 0; i < 2; ++i) a1[nxt][i] = pa[row * 128 + 64 * i];
            }
            if constexpr (!BKC) {
#pragma unroll
                for (int i = 0; i < 2; ++i) b1[nxt][i] = pb[row * 128 + 64 * i];
            }
        }
        if constexpr (!AKC || !BKC) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jn = 0; jn < 2; ++jn) {
                const float av = AKC ? a4[g][i][j] : a1[cur][i];
                const float bv = BKC ? b4[g][jn][j] : b1[cur][jn];
                acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][jn], 0, 0, 0);
            }
    }
}

// Row (r) of accumulator element r inside the block tile, and the block's first column.
__device__ __forceinline__ int f_row(int half_m, int i, int r, int lane)
{
    return 32 * half_m + 64 * i + 8 * (r / 4) + 4 * (lane >> 5) + (r & 3);
}
__device__ __forceinline__ int f_col(int half_n, int jn, int lane) { return 32 * half_n + 64 * jn + (lane & 31); }

// Stores one 32 x 32 accumulator block whose rows and columns are all inside the
// output: `out` starts at the block tile's (row 0, column col0) element.
template <bool RELU>
__device__ __forceinline__ void store_block(const floatx16 &acc, __amdgpu_buffer_rsrc_t out, uint32_t ld4,
                                            int row0, int col, int lane)
{
    const uint32_t o0 = static_cast<uint32_t>(row0 + 4 * (lane >> 5)) * ld4 + static_cast<uint32_t>(col) * 4u;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        float v = acc[r];
        if constexpr (RELU) asm("v_max_f32 %0, 0, %1" : "=v"(v) : "v"(v));
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), out, o0, (8 * (r / 4) + (r & 3)) * ld4, 0);
    }
}

#define SYLVIE_ZERO_ACC(acc)                                   \
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)           \
    _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_)           \
    _Pragma("unroll") for (int r_ = 0; r_ < 16; ++r_) acc[i_][j_][r_] = 0.0f

// Tile coordinates of workgroup b of a one-dimensional launch over n_major x n_minor tiles.
// Consecutive workgroups go to the chip's 8 XCDs in turn, each with an L2 of its own, and tiles
// that share an operand block (the column tiles of one row block; the tiles of one row slab)
// should meet in ONE L2 shortly after each other: workgroups b and b + 8 (same XCD, consecutive
// there) get the same `major` and consecutive `minor`.  Any n_major works (the last n_major % 8
// majors are laid out plainly); the map is a bijection of [0, n_major n_minor).
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ void xcd_tile(uint32_t b, uint32_t n_major, uint32_t n_minor, uint32_t &major,
                                         uint32_t &minor)
{
    const uint32_t group = kXcds * n_minor, full = n_major / kXcds;
    if (b < full * group) {
        const uint32_t g = b / group, r = b % group;
        major = g * kXcds + r % kXcds;
        minor = r / kXcds;
    } else {
        const uint32_t rem = n_major - full * kXcds, bb = b - full * group;
        major = full * kXcds + bb % rem;
        minor = bb / rem;
    }
}

// H = relu?([A1|A2] W); K % BK == 0, k1 % BK == 0, h % 4 == 0.
__global__ __launch_bounds__(kGemmThreads, 3) void transform_fwd_fast_kernel(CatA a, const float *__restrict__ Wm,
                                                                         int h, int relu,
                                                                         float *__restrict__ H, int64_t ldh)
{
    __shared__ __align__(16) float As[2][kTileKC];
    __shared__ __align__(16) float Bs[2][kTileXC];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    uint32_t row_blk, col_tile;
    xcd_tile(blockIdx.x, static_cast<uint32_t>((a.n + BM - 1) / BM), static_cast<uint32_t>((h + BN - 1) / BN), row_blk, col_tile);
    const int64_t m0 = static_cast<int64_t>(row_blk) * BM;
    const int n0 = static_cast<int>(col_tile) * BN;
    const int K = a.k1 + a.k2;
    const int half_m = wave >> 1, half_n = wave & 1;
    const int rows = a.n - m0 < BM ? static_cast<int>(a.n - m0) : BM;
    floatx16 acc[2][2];
    SYLVIE_ZERO_ACC(acc);

    const __amdgpu_buffer_rsrc_t buf1 =
        make_buf(a.A1 + m0 * a.ld1, (static_cast<uint32_t>(rows - 1) * static_cast<uint32_t>(a.ld1) + a.k1) * 4u);
    const __amdgpu_buffer_rsrc_t buf2 =
        a.k2 ? make_buf(a.A2 + m0 * a.ld2, (static_cast<uint32_t>(rows - 1) * static_cast<uint32_t>(a.ld2) + a.k2) * 4u)
             : buf1;
    const __amdgpu_buffer_rsrc_t bufw = make_buf(Wm, static_cast<uint32_t>(K) * h * 4u);
    uint32_t oa1[NI], oa2[NI], ob[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const uint32_t x = t / 4 + 64 * i;
        oa1[i] = (x * static_cast<uint32_t>(a.ld1) + 4 * (t % 4)) * 4u;
        oa2[i] = (x * static_cast<uint32_t>(a.ld2) + 4 * (t % 4)) * 4u;
        int c = n0 + 4 * (t % 32);
        if (c > h - 4) c = h - 4;                // feeds columns that are never stored
        ob[i] = (static_cast<uint32_t>(t / 32 + 8 * i) * h + c) * 4u;
    }
    float ra[NI][4], rb[NI][4];
    auto fetch = [&](int k0) {
        if (k0 < a.k1) {
#pragma unroll
            for (int i = 0; i < NI; ++i) buf_load4(ra[i], buf1, oa1[i], k0 * 4);
        } else {
#pragma unroll
            for (int i = 0; i < NI; ++i) buf_load4(ra[i], buf2, oa2[i], (k0 - a.k1) * 4);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) buf_load4(rb[i], bufw, ob[i], static_cast<uint32_t>(k0) * h * 4u);
    };
    auto put = [&](int b) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            put_f_kc(As[b], i, ra[i]);
            put_f_xc(Bs[b], i, rb[i]);
        }
    };
    fetch(0);
    put(0);
    __syncthreads();
    if (BK < K) fetch(BK);
    for (int k0 = 0, b = 0; k0 < K; k0 += BK, b ^= 1) {
        mma_step<true, false>(acc, As[b], Bs[b], half_m, half_n, lane);
        if (k0 + BK < K) {
            put(b ^ 1);
            if (k0 + 2 * BK < K) fetch(k0 + 2 * BK);
        }
        __syncthreads();
    }
    if (rows == BM && n0 + BN <= h) {
        const uint32_t ld4 = static_cast<uint32_t>(ldh) * 4u;
        const __amdgpu_buffer_rsrc_t out = make_buf(H + m0 * ldh + n0, (BM - 1) * ld4 + BN * 4);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jn = 0; jn < 2; ++jn) {
                if (relu) store_block<true>(acc[i][jn], out, ld4, 32 * half_m + 64 * i, f_col(half_n, jn, lane), lane);
                else store_block<false>(acc[i][jn], out, ld4, 32 * half_m + 64 * i, f_col(half_n, jn, lane), lane);
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) {
            const int c = n0 + f_col(half_n, jn, lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = m0 + f_row(half_m, i, r, lane);
                if (row < a.n && c < h) {
                    float v = acc[i][jn][r];
                    if (relu) v = v > 0.0f ? v : 0.0f;
                    H[row * ldh + c] = v;
                }
            }
        }
}

// [dA1 | dA2] = M W^T; h % BK == 0, k1 % 4 == 0.
__global__ __launch_bounds__(kGemmThreads, 3) void transform_bwd_da_fast_kernel(
    MaskedJ m, const float *__restrict__ Wm, int k1, int k2, float *__restrict__ dA1, int64_t ld1,
    float *__restrict__ dA2, int64_t ld2)
{
    __shared__ __align__(16) float As[2][kTileKC];
    __shared__ __align__(16) float Bs[2][kTileKC];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int K = k1 + k2, h = m.h;
    uint32_t row_blk, col_tile;
    xcd_tile(blockIdx.x, static_cast<uint32_t>((m.n + BM - 1) / BM), static_cast<uint32_t>((K + BN - 1) / BN), row_blk, col_tile);
    const int64_t m0 = static_cast<int64_t>(row_blk) * BM;
    const int n0 = static_cast<int>(col_tile) * BN;       // output column = row of W
    const int half_m = wave >> 1, half_n = wave & 1;
    const int rows = m.n - m0 < BM ? static_cast<int>(m.n - m0) : BM;
    const int wrows = K - n0 < BN ? K - n0 : BN;
    floatx16 acc[2][2];
    SYLVIE_ZERO_ACC(acc);

    const __amdgpu_buffer_rsrc_t bufj =
        make_buf(m.J + m0 * m.ldj, (static_cast<uint32_t>(rows - 1) * static_cast<uint32_t>(m.ldj) + h) * 4u);
    const __amdgpu_buffer_rsrc_t bufh =
        m.relu ? make_buf(m.H + m0 * m.ldh, (static_cast<uint32_t>(rows - 1) * static_cast<uint32_t>(m.ldh) + h) * 4u)
               : bufj;
    const __amdgpu_buffer_rsrc_t bufw =
        make_buf(Wm + static_cast<int64_t>(n0) * h, static_cast<uint32_t>(wrows) * h * 4u);
    uint32_t oj[NI], oh[NI], ow[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const uint32_t x = t / 4 + 64 * i;
        oj[i] = (x * static_cast<uint32_t>(m.ldj) + 4 * (t % 4)) * 4u;
        oh[i] = (x * static_cast<uint32_t>(m.ldh) + 4 * (t % 4)) * 4u;
        ow[i] = (x * static_cast<uint32_t>(h) + 4 * (t % 4)) * 4u;
    }
    float ra[NI][4], rh[NI][4], rb[NI][4];
    auto fetch = [&](int j0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) buf_load4(ra[i], bufj, oj[i], j0 * 4);
        if (m.relu) {
#pragma unroll
            for (int i = 0; i < NI; ++i) buf_load4(rh[i], bufh, oh[i], j0 * 4);
        }
#pragma unroll
        for (int i = 0; i < NI; ++i) buf_load4(rb[i], bufw, ow[i], j0 * 4);
    };
    auto put = [&](int b) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if (m.relu) {
#pragma unroll
                for (int q = 0; q < 4; ++q) ra[i][q] = rh[i][q] > 0.0f ? ra[i][q] : 0.0f;
            }
            put_f_kc(As[b], i, ra[i]);
            put_f_kc(Bs[b], i, rb[i]);
        }
    };
    fetch(0);
    put(0);
    __syncthreads();
    if (BK < h) fetch(BK);
    for (int j0 = 0, b = 0; j0 < h; j0 += BK, b ^= 1) {
        mma_step<true, true>(acc, As[b], Bs[b], half_m, half_n, lane);
        if (j0 + BK < h) {
            put(b ^ 1);
            if (j0 + 2 * BK < h) fetch(j0 + 2 * BK);
        }
        __syncthreads();
    }
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
        const int c0 = n0 + 32 * half_n + 64 * jn;          // first column of this 32-wide block
        const bool in1 = c0 + 32 <= k1, in2 = c0 >= k1 && c0 + 32 <= K;
        if (rows == BM && (in1 || in2)) {
            float *basep = in1 ? dA1 + m0 * ld1 + c0 : dA2 + m0 * ld2 + (c0 - k1);
            const uint32_t ld4 = static_cast<uint32_t>(in1 ? ld1 : ld2) * 4u;
            const __amdgpu_buffer_rsrc_t out = make_buf(basep, (BM - 1) * ld4 + 32 * 4);
#pragma unroll
            for (int i = 0; i < 2; ++i)
                store_block<false>(acc[i][jn], out, ld4, 32 * half_m + 64 * i, lane & 31, lane);
        } else {
            const int c = c0 + (lane & 31);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = m0 + f_row(half_m, i, r, lane);
                    if (row < m.n && c < K) {
                        if (c < k1) dA1[row * ld1 + c] = acc[i][jn][r];
                        else dA2[row * ld2 + (c - k1)] = acc[i][jn][r];
                    }
                }
        }
    }
}

// part[slab] = [A1|A2]^T M over one slab of rows; k1 % 128 == 0 or k2 == 0 (a tile of
// 128 operand columns lies in one of the two matrices), widths % 4 == 0.
__global__ __launch_bounds__(kGemmThreads, 3) void transform_bwd_g_fast_kernel(CatA a, MaskedJ m,
                                                                           int64_t rows_per_slab, int n_slabs,
                                                                           float *__restrict__ part)
{
    __shared__ __align__(16) float As[2][kTileXC];
    __shared__ __align__(16) float Bs[2][kTileXC];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int K = a.k1 + a.k2, h = m.h;
    const uint32_t tiles_m = static_cast<uint32_t>((K + BM - 1) / BM), tiles_n = static_cast<uint32_t>((h + BN - 1) / BN);
    uint32_t slab, tile;
    xcd_tile(blockIdx.x, static_cast<uint32_t>(n_slabs), tiles_m * tiles_n, slab, tile);
    const int m0 = static_cast<int>(tile % tiles_m) * BM;   // row of G = column of [A1|A2]
    const int n0 = static_cast<int>(tile / tiles_m) * BN;   // column of G
    const int64_t r_begin = static_cast<int64_t>(slab) * rows_per_slab;
    const int64_t r_end = r_begin + rows_per_slab < a.n ? r_begin + rows_per_slab : a.n;
    const int half_m = wave >> 1, half_n = wave & 1;
    floatx16 acc[2][2];
    SYLVIE_ZERO_ACC(acc);
    float *out = part + static_cast<int64_t>(slab) * K * h;
    const int nr = static_cast<int>(r_end - r_begin);      // rows of this slab (may be <= 0)
    if (nr > 0) {
        const bool first = m0 < a.k1;
        const float *Ap = first ? a.A1 : a.A2;
        const uint32_t lda = static_cast<uint32_t>(first ? a.ld1 : a.ld2);
        const int wa = first ? a.k1 : a.k2, ca0 = first ? m0 : m0 - a.k1;
        const __amdgpu_buffer_rsrc_t bufa = make_buf(Ap + r_begin * lda, (static_cast<uint32_t>(nr - 1) * lda + wa) * 4u);
        const __amdgpu_buffer_rsrc_t bufj =
            make_buf(m.J + r_begin * m.ldj, (static_cast<uint32_t>(nr - 1) * static_cast<uint32_t>(m.ldj) + h) * 4u);
        const __amdgpu_buffer_rsrc_t bufh =
            m.relu ? make_buf(m.H + r_begin * m.ldh, (static_cast<uint32_t>(nr - 1) * static_cast<uint32_t>(m.ldh) + h) * 4u)
                   : bufj;
        uint32_t oa[NI], oj[NI], oh[NI];
        int ca = ca0 + 4 * (t % 32), cj = n0 + 4 * (t % 32);
        if (ca > wa - 4) ca = wa - 4;               // feed rows / columns of G that are never stored
        if (cj > h - 4) cj = h - 4;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const uint32_t k = t / 32 + 8 * i;
            oa[i] = (k * lda + ca) * 4u;
            oj[i] = (k * static_cast<uint32_t>(m.ldj) + cj) * 4u;
            oh[i] = (k * static_cast<uint32_t>(m.ldh) + cj) * 4u;
        }
        const uint32_t sa = lda * 4u, sj = static_cast<uint32_t>(m.ldj) * 4u, sh = static_cast<uint32_t>(m.ldh) * 4u;
        float ra[NI][4], rh[NI][4], rb[NI][4];
        // the row advance goes into the lane offset: the range check that zeroes rows past
        // the slab looks at the lane offset only
        auto fetch = [&](int r0) {
#pragma unroll
            for (int i = 0; i < NI; ++i) buf_load4(ra[i], bufa, oa[i] + r0 * sa, 0);
#pragma unroll
            for (int i = 0; i < NI; ++i) buf_load4(rb[i], bufj, oj[i] + r0 * sj, 0);
            if (m.relu) {
#pragma unroll
                for (int i = 0; i < NI; ++i) buf_load4(rh[i], bufh, oh[i] + r0 * sh, 0);
            }
        };
        auto put = [&](int b) {
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                if (m.relu) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) rb[i][q] = rh[i][q] > 0.0f ? rb[i][q] : 0.0f;
                }
                put_f_xc(As[b], i, ra[i]);
                put_f_xc(Bs[b], i, rb[i]);
            }
        };
        fetch(0);
        put(0);
        __syncthreads();
        if (BK < nr) fetch(BK);
        for (int r0 = 0, b = 0; r0 < nr; r0 += BK, b ^= 1) {
            mma_step<false, false>(acc, As[b], Bs[b], half_m, half_n, lane);
            if (r0 + BK < nr) {
                put(b ^ 1);
                if (r0 + 2 * BK < nr) fetch(r0 + 2 * BK);
            }
            __syncthreads();
        }
    }
    if (m0 + BM <= K && n0 + BN <= h) {
        const uint32_t ld4 = static_cast<uint32_t>(h) * 4u;
        const __amdgpu_buffer_rsrc_t ob = make_buf(out + static_cast<int64_t>(m0) * h + n0, (BM - 1) * ld4 + BN * 4);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jn = 0; jn < 2; ++jn)
                store_block<false>(acc[i][jn], ob, ld4, 32 * half_m + 64 * i, f_col(half_n, jn, lane), lane);
        return;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) {
            const int c = n0 + f_col(half_n, jn, lane);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + f_row(half_m, i, r, lane);
                if (row < K && c < h) out[static_cast<int64_t>(row) * h + c] = acc[i][jn][r];
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
// Slabs of 512 rows by default; a small partition whose output has few tiles gets shorter slabs
// (down to 64 rows) until about 512 workgroups exist: with one 64 x 64 output tile and 10 000
// rows, 20 workgroups walked 512 rows each (38 us) where 155 now walk 64 (the launch is then as
// short as the other launches of such a step).
static int g_slabs(int64_t n, int K, int h)
{
    const int64_t tiles = static_cast<int64_t>((K + BM - 1) / BM) * ((h + BN - 1) / BN);
    int64_t s = (n + 511) / 512;
    const int64_t fill = (512 + tiles - 1) / tiles, shortest = n / 64;
    const int64_t more = fill < shortest ? fill : shortest;
    if (more > s) s = more;
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
    const int K = k1 + k2;
    const bool fast = v4 && K % BK == 0 && k1 % BK == 0 && ld_a1 < kMaxFastLd && ld_a2 < kMaxFastLd &&
                      ld_h < kMaxFastLd && static_cast<int64_t>(K) * h < (int64_t(1) << 29);
    if (fast)
        hipLaunchKernelGGL(transform_fwd_fast_kernel, dim3(grid.x * grid.y), dim3(kGemmThreads), 0, st, a, W, h, relu, H, ld_h);
    else if (v4)
        hipLaunchKernelGGL(transform_fwd_kernel<4>, grid, dim3(kGemmThreads), 0, st, a, W, h, relu, H, ld_h);
    else
        hipLaunchKernelGGL(transform_fwd_kernel<1>, grid, dim3(kGemmThreads), 0, st, a, W, h, relu, H, ld_h);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" size_t sylvie_transform_bwd_workspace_bytes(int32_t k1, int32_t k2, int32_t h, int64_t n)
{
    return static_cast<size_t>(sylvie::g_slabs(n, k1 + k2, h)) * static_cast<size_t>(k1 + k2) *
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
        const int slabs = g_slabs(n, K, h);
        int64_t rps = (n + slabs - 1) / slabs;
        rps = (rps + BK - 1) / BK * BK;
        const dim3 grid(static_cast<unsigned>((K + BM - 1) / BM), static_cast<unsigned>((h + BN - 1) / BN),
                        static_cast<unsigned>(slabs));
        const int64_t ldmax = std::max(std::max(ld_a1, k2 > 0 ? ld_a2 : 0), std::max(ld_j, relu ? ld_h : 0));
        const bool fast = v4 && (k2 == 0 || k1 % BM == 0) && rps * ldmax < (int64_t(1) << 29);
        if (fast)
            hipLaunchKernelGGL(transform_bwd_g_fast_kernel, dim3(grid.x * grid.y * grid.z), dim3(kGemmThreads), 0, st, a, m,
                               rps, slabs, workspace);
        else if (v4)
            hipLaunchKernelGGL(transform_bwd_g_kernel<4>, grid, dim3(kGemmThreads), 0, st, a, m, rps, workspace);
        else
            hipLaunchKernelGGL(transform_bwd_g_kernel<1>, grid, dim3(kGemmThreads), 0, st, a, m, rps, workspace);
        const int64_t elems = static_cast<int64_t>(K) * h;
        hipLaunchKernelGGL(transform_bwd_g_reduce_kernel, dim3(static_cast<unsigned>((elems + 255) / 256)),
                           dim3(256), 0, st, workspace, elems, slabs, G);
    }
    if (dA1) {
        const dim3 grid(static_cast<unsigned>((n + BM - 1) / BM), static_cast<unsigned>((K + BN - 1) / BN));
        const bool fast = v4 && h % BK == 0 && ld_j < kMaxFastLd && (!relu || ld_h < kMaxFastLd) &&
                          ld_da1 < kMaxFastLd && (k2 == 0 || ld_da2 < kMaxFastLd);
        if (fast)
            hipLaunchKernelGGL(transform_bwd_da_fast_kernel, dim3(grid.x * grid.y), dim3(kGemmThreads), 0, st, m, W, k1, k2,
                               dA1, ld_da1, dA2, ld_da2);
        else if (v4)
            hipLaunchKernelGGL(transform_bwd_da_kernel<4>, grid, dim3(kGemmThreads), 0, st, m, W, k1, k2, dA1, ld_da1, dA2, ld_da2);
        else
            hipLaunchKernelGGL(transform_bwd_da_kernel<1>, grid, dim3(kGemmThreads), 0, st, m, W, k1, k2, dA1, ld_da1, dA2, ld_da2);
    }
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}
