// Loss, gradient synchronisation and model update that close the training step
// (Alg. 1, last line: L = Loss(softmax(H^(L)), Y); Alg. 2: J^(L) = dL/dH^(L),
// G = AllReduce(G_n), W_t = W_{t-1} - eta G).  Small streaming kernels.
#include "common.hpp"

namespace sylvie {

constexpr int kTrWavesPerBlock = 4;

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) {
        const float o = __shfl_xor(v, s);
        v = o > v ? o : v;
    }
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
    return v;
}

// One wavefront per row; the row (P values per lane, column lane + 64 k) is read once and
// stays in registers.  Unlabelled rows (label < 0) get a zero gradient row and no loss.
template <int P>
__global__ __launch_bounds__(kTrWavesPerBlock *kWave) void softmax_xent_kernel(
    const float *__restrict__ H, int64_t ldh, int64_t n, int C, const int32_t *__restrict__ label,
    float inv_count, float *__restrict__ J, int64_t ldj, float *__restrict__ loss_rows)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kTrWavesPerBlock + wave;
    if (i >= n) return;
    const float *h = H + i * ldh;
    float *j = J + i * ldj;
    const int y = uniform(label[i]);
    if (y < 0) {
        for (int c = lane; c < C; c += 64) j[c] = 0.0f;
        if (lane == 0) loss_rows[i] = 0.0f;
        return;
    }
    float v[P];
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const int c = lane + 64 * k;
        v[k] = c < C ? h[c] : -__builtin_inff();
    }
    float mx = v[0];
#pragma unroll
    for (int k = 1; k < P; ++k) mx = v[k] > mx ? v[k] : mx;
    mx = wave_max(mx);
    float sum = 0.0f;
#pragma unroll
    for (int k = 0; k < P; ++k) {
        v[k] = __expf(v[k] - mx);              // exp(-inf) = 0 for the columns past C
        sum += v[k];
    }
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
    const float hy = h[y];
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const int c = lane + 64 * k;
        if (c < C) j[c] = (v[k] * inv - (c == y ? 1.0f : 0.0f)) * inv_count;
    }
    if (lane == 0) loss_rows[i] = (__logf(sum) - (hy - mx)) * inv_count;
}

// Any number of classes: the row is read three times (the re-reads hit the cache).
__global__ __launch_bounds__(kTrWavesPerBlock *kWave) void softmax_xent_wide_kernel(
    const float *__restrict__ H, int64_t ldh, int64_t n, int C, const int32_t *__restrict__ label,
    float inv_count, float *__restrict__ J, int64_t ldj, float *__restrict__ loss_rows)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kTrWavesPerBlock + wave;
    if (i >= n) return;
    const float *h = H + i * ldh;
    float *j = J + i * ldj;
    const int y = uniform(label[i]);
    if (y < 0) {
        for (int c = lane; c < C; c += 64) j[c] = 0.0f;
        if (lane == 0) loss_rows[i] = 0.0f;
        return;
    }
    float mx = -__builtin_inff();
    for (int c = lane; c < C; c += 64) mx = h[c] > mx ? h[c] : mx;
    mx = wave_max(mx);
    float sum = 0.0f;
    for (int c = lane; c < C; c += 64) sum += __expf(h[c] - mx);
    sum = wave_sum(sum);
    const float inv = 1.0f / sum;
    for (int c = lane; c < C; c += 64) {
        const float p = __expf(h[c] - mx) * inv;
        j[c] = (p - (c == y ? 1.0f : 0.0f)) * inv_count;
    }
    if (lane == 0) loss_rows[i] = (__logf(sum) - (h[y] - mx)) * inv_count;
}

// out[0] = sum of v[0..n) in double, in a fixed order: thread t owns elements t + 1024 m;
// it keeps eight running sums (m mod 8) so that eight loads are in flight, adds them
// in ascending order, and a fixed tree joins the 1024 threads.
__global__ __launch_bounds__(1024) void sum_to_double_kernel(const float *__restrict__ v, int64_t n,
                                                            double *__restrict__ out)
{
    __shared__ double part[1024];
    const int t = threadIdx.x;
    double s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int64_t e = t;
    for (; e + 7 * 1024 < n; e += 8 * 1024) {
        float x[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) x[q] = v[e + q * 1024];
#pragma unroll
        for (int q = 0; q < 8; ++q) s[q] += static_cast<double>(x[q]);
    }
    for (int q = 0; e < n; e += 1024, ++q) s[q] += static_cast<double>(v[e]);
    double tot = s[0];
#pragma unroll
    for (int q = 1; q < 8; ++q) tot += s[q];
    part[t] = tot;
    __syncthreads();
    for (int w = 512; w >= 1; w >>= 1) {
        if (t < w) part[t] += part[t + w];
        __syncthreads();
    }
    if (t == 0) out[0] = part[0];
}

constexpr int kMaxGradSources = 16;
struct GradSources {
    const float *p[kMaxGradSources];
};

__global__ void sum_gradients_kernel(float *__restrict__ dst, GradSources src, int n_src, int64_t elems)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= elems) return;
    float s = src.p[0][e];
    for (int k = 1; k < n_src; ++k) s = s + src.p[k][e];
    dst[e] = s;
}

__global__ void sgd_update_kernel(float *__restrict__ W, const float *__restrict__ G, int64_t elems,
                                  float eta)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (e >= elems) return;
    const float step = eta * G[e];
    W[e] = W[e] - step;
}

}  // namespace sylvie

extern "C" int32_t sylvie_softmax_xent(const float *H, int64_t ld_h, int64_t n, int32_t n_classes,
                                       const int32_t *label, double count, float *J, int64_t ld_j,
                                       float *loss_rows, double *loss_out, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_softmax_xent";
    if (n < 0 || n >= (int64_t(1) << 31)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: n out of range", name);
    if (n_classes < 1 || n_classes > 65536)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_classes %d out of range", name, n_classes);
    if (ld_h < n_classes || ld_j < n_classes)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: leading dimension below n_classes", name);
    if (!(count > 0.0)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: count must be positive", name);
    if (!loss_out) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null loss_out", name);
    if (!aligned(loss_out, 8)) return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: loss_out needs 8-byte alignment", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n > 0) {
        if (!H || !label || !J || !loss_rows) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
        const dim3 grid(static_cast<unsigned>((n + kTrWavesPerBlock - 1) / kTrWavesPerBlock));
        const dim3 block(kTrWavesPerBlock * kWave);
        const float ic = static_cast<float>(1.0 / count);
#define SYLVIE_XENT(P) hipLaunchKernelGGL(softmax_xent_kernel<P>, grid, block, 0, st, H, ld_h, n, n_classes, label, ic, J, ld_j, loss_rows)
        if (n_classes <= 64) SYLVIE_XENT(1);
        else if (n_classes <= 128) SYLVIE_XENT(2);
        else if (n_classes <= 256) SYLVIE_XENT(4);
        else if (n_classes <= 512) SYLVIE_XENT(8);
        else if (n_classes <= 1024) SYLVIE_XENT(16);
        else
            hipLaunchKernelGGL(softmax_xent_wide_kernel, grid, block, 0, st, H, ld_h, n, n_classes, label, ic,
                               J, ld_j, loss_rows);
#undef SYLVIE_XENT
    }
    hipLaunchKernelGGL(sum_to_double_kernel, dim3(1), dim3(1024), 0, st, loss_rows, n, loss_out);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_sum_gradients(float *dst, const float *const *srcs, int32_t n_src,
                                        int64_t elems, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_sum_gradients";
    if (n_src < 1 || n_src > kMaxGradSources)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_src must be 1..%d", name, kMaxGradSources);
    if (elems < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative size", name);
    if (elems == 0) return SYLVIE_OK;
    if (!dst || !srcs) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    GradSources g{};
    for (int k = 0; k < n_src; ++k) {
        if (!srcs[k]) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null source %d", name, k);
        g.p[k] = srcs[k];
    }
    hipLaunchKernelGGL(sum_gradients_kernel, dim3(static_cast<unsigned>((elems + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), dst, g, n_src, elems);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_sgd_update(float *W, const float *G, int64_t elems, float eta, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_sgd_update";
    if (elems < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative size", name);
    if (elems == 0) return SYLVIE_OK;
    if (!W || !G) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    hipLaunchKernelGGL(sgd_update_kernel, dim3(static_cast<unsigned>((elems + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), W, G, elems, eta);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}
