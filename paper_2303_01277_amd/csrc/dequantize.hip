// 1-bit dequantizer (Sec. 3.2 "Dequantizer", Eq. 5 with B = 1): unpack the bits
// and recover float32 rows, either overwriting the halo block (forward,
// Alg. 1 "concatenate") or adding into the rows the gradients belong to
// (backward, Alg. 2 "integrate feature gradients").
//
// One wavefront per row.  Lane L produces VEC consecutive columns per pass so the
// float stores are full-width and contiguous across the wave; the VEC bits it
// needs sit in one 64-bit word, which neighbouring lanes share through the cache.
#include "common.hpp"

namespace sylvie {

constexpr int kDqWavesPerBlock = 4;
constexpr int kDqRowsPerWave = 4;

template <int VEC>
struct VecT;
template <>
struct VecT<4> { using type = float4; };
template <>
struct VecT<2> { using type = float2; };
template <>
struct VecT<1> { using type = float; };

template <int VEC>
__device__ __forceinline__ void select_store(float *p, uint32_t bits, float lo, float hi)
{
    if constexpr (VEC == 4) {
        float4 o;
        o.x = (bits & 1u) ? hi : lo;
        o.y = (bits & 2u) ? hi : lo;
        o.z = (bits & 4u) ? hi : lo;
        o.w = (bits & 8u) ? hi : lo;
        *reinterpret_cast<float4 *>(p) = o;
    } else if constexpr (VEC == 2) {
        float2 o;
        o.x = (bits & 1u) ? hi : lo;
        o.y = (bits & 2u) ? hi : lo;
        *reinterpret_cast<float2 *>(p) = o;
    } else {
        *p = (bits & 1u) ? hi : lo;
    }
}

template <int VEC>
__global__ __launch_bounds__(kDqWavesPerBlock *kWave) void dequantize_fwd_kernel(
    const uint64_t *__restrict__ wire, int64_t n_rows, int d, float *__restrict__ dst, int64_t ld,
    int64_t row_offset)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first =
        (static_cast<int64_t>(blockIdx.x) * kDqWavesPerBlock + wave) * kDqRowsPerWave;
    const int W = (d + 63) >> 6;
#pragma unroll 1
    for (int r = 0; r < kDqRowsPerWave; ++r) {
        const int64_t i = first + r;
        if (i >= n_rows) break;
        const uint64_t *prow = wire + i * (W + 1);
        const uint64_t meta = prow[W];                      // scale | zero << 32
        const float zp = __uint_as_float(static_cast<uint32_t>(meta >> 32));
        const float hi = zp + __uint_as_float(static_cast<uint32_t>(meta));
        float *orow = dst + (row_offset + i) * ld;
        for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
            const uint64_t word = prow[c0 >> 6];
            const uint32_t bits = static_cast<uint32_t>(word >> (c0 & 63));
            select_store<VEC>(orow + c0, bits, zp, hi);
        }
    }
}

// One wavefront per destination row k: dst[dst_ids[k]] += the dequantised wire
// rows seg_rows[seg_ptr[k] .. seg_ptr[k+1]) in that order, float32.
template <int VEC>
__global__ __launch_bounds__(kDqWavesPerBlock *kWave) void dequantize_bwd_kernel(
    const uint64_t *__restrict__ wire, int d, float *__restrict__ dst, int64_t ld,
    const int64_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_rows,
    int64_t n_dst_rows, const int32_t *__restrict__ dst_ids)
{
    using V = typename VecT<VEC>::type;
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kDqWavesPerBlock + wave;
    if (k >= n_dst_rows) return;
    const int W = (d + 63) >> 6;
    const int64_t j0 = seg_ptr[k], j1 = seg_ptr[k + 1];
    if (j0 >= j1) return;
    float *orow = dst + static_cast<int64_t>(dst_ids[k]) * ld;
    for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
        V accv = *reinterpret_cast<const V *>(orow + c0);
        float acc[VEC];
        __builtin_memcpy(acc, &accv, sizeof(V));
        for (int64_t j = j0; j < j1; ++j) {
            const uint64_t *prow = wire + static_cast<int64_t>(seg_rows[j]) * (W + 1);
            const uint64_t meta = prow[W];
            const float zp = __uint_as_float(static_cast<uint32_t>(meta >> 32));
            const float hi = zp + __uint_as_float(static_cast<uint32_t>(meta));
            const uint64_t word = prow[c0 >> 6];
            const uint32_t bits = static_cast<uint32_t>(word >> (c0 & 63));
#pragma unroll
            for (int t = 0; t < VEC; ++t) acc[t] = acc[t] + (((bits >> t) & 1u) ? hi : zp);
        }
        __builtin_memcpy(&accv, acc, sizeof(V));
        *reinterpret_cast<V *>(orow + c0) = accv;
    }
}

static int pick_vec(int d, int64_t ld, const void *p)
{
    if (d % 4 == 0 && ld % 4 == 0 && aligned(p, 16)) return 4;
    if (d % 2 == 0 && ld % 2 == 0 && aligned(p, 8)) return 2;
    return 1;
}

static int32_t check_wire(const char *name, const uint64_t *wire, int64_t n_rows, int32_t d,
                          const float *dst, int64_t ld)
{
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_rows %lld out of range", name, (long long)n_rows);
    if (d < 1 || d > 65536) return fail(SYLVIE_ERR_INVALID_ARG, "%s: d %d out of range", name, d);
    if (ld < d) return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_dst %lld < d %d", name, (long long)ld, d);
    if (n_rows == 0) return SYLVIE_OK;
    if (!wire || !dst) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(wire, 8) || !aligned(dst, 4))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned pointer", name);
    return SYLVIE_OK;
}

}  // namespace sylvie

extern "C" int32_t sylvie_dequantize_1bit_fwd(const uint64_t *wire, int64_t n_rows, int32_t d,
                                              float *dst, int64_t ld_dst, int64_t row_offset,
                                              void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_dequantize_1bit_fwd";
    const int32_t rc = check_wire(name, wire, n_rows, d, dst, ld_dst);
    if (rc != SYLVIE_OK) return rc;
    if (row_offset < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative row_offset", name);
    if (n_rows == 0) return SYLVIE_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t per_block = kDqWavesPerBlock * kDqRowsPerWave;
    const dim3 grid(static_cast<unsigned>((n_rows + per_block - 1) / per_block));
    const dim3 block(kDqWavesPerBlock * kWave);
    // the vector width must also hold for the first written row
    const int vec = pick_vec(d, ld_dst, dst + row_offset * ld_dst);
    if (vec == 4)
        hipLaunchKernelGGL(dequantize_fwd_kernel<4>, grid, block, 0, st, wire, n_rows,
                           d, dst, ld_dst, row_offset);
    else if (vec == 2)
        hipLaunchKernelGGL(dequantize_fwd_kernel<2>, grid, block, 0, st, wire, n_rows,
                           d, dst, ld_dst, row_offset);
    else
        hipLaunchKernelGGL(dequantize_fwd_kernel<1>, grid, block, 0, st, wire, n_rows,
                           d, dst, ld_dst, row_offset);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_dequantize_1bit_bwd(const uint64_t *wire, int64_t n_rows, int32_t d,
                                              float *dst, int64_t ld_dst, const int64_t *seg_ptr,
                                              const int32_t *seg_rows, int64_t n_dst_rows,
                                              const int32_t *dst_ids, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_dequantize_1bit_bwd";
    const int32_t rc = check_wire(name, wire, n_rows, d, dst, ld_dst);
    if (rc != SYLVIE_OK) return rc;
    if (n_dst_rows < 0 || n_dst_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_dst_rows out of range", name);
    if (n_rows == 0 || n_dst_rows == 0) return SYLVIE_OK;
    if (!seg_ptr || !seg_rows || !dst_ids) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(seg_ptr, 8) || !aligned(seg_rows, 4) || !aligned(dst_ids, 4))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned index array", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(static_cast<unsigned>((n_dst_rows + kDqWavesPerBlock - 1) / kDqWavesPerBlock));
    const dim3 block(kDqWavesPerBlock * kWave);
    const int vec = pick_vec(d, ld_dst, dst);
    if (vec == 4)
        hipLaunchKernelGGL(dequantize_bwd_kernel<4>, grid, block, 0, st, wire, d, dst,
                           ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    else if (vec == 2)
        hipLaunchKernelGGL(dequantize_bwd_kernel<2>, grid, block, 0, st, wire, d, dst,
                           ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    else
        hipLaunchKernelGGL(dequantize_bwd_kernel<1>, grid, block, 0, st, wire, d, dst,
                           ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}
