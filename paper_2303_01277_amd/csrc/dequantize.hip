// 1-bit dequantizer (Sec. 3.2 "Dequantizer", Eq. 5 with B = 1): unpack the bits
// and recover float32 rows, either overwriting the halo block (forward,
// Alg. 1 "concatenate") or adding into the rows the gradients belong to
// (backward, Alg. 2 "integrate feature gradients").
//
// One wavefront per row.  Lane L produces VEC consecutive columns per pass so the
// float stores are full-width and contiguous across the wave; the VEC bits it
// needs sit in one 64-bit word, which neighbouring lanes share through the cache.
#include "common.hpp"
#include "validate.hpp"

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
    float o[VEC];
#pragma unroll
    for (int t = 0; t < VEC; ++t) o[t] = ((bits >> t) & 1u) ? hi : lo;
    stream_store<VEC>(p, o);            // recovered rows are written once and read by a later launch
}

// ONEPASS: d <= 64 VEC, every lane owns at most one vector of a row.  Then the loads
// of all the wave's rows (metadata word + the lane's bit word) are issued before the
// first store, so one wave keeps several rows in flight.
template <int VEC, bool ONEPASS>
__global__ __launch_bounds__(kDqWavesPerBlock *kWave) void dequantize_fwd_kernel(
    const uint64_t *__restrict__ wire, int64_t ldw, int64_t n_rows, int d, float *__restrict__ dst,
    int64_t ld, int64_t row_offset)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first =
        (static_cast<int64_t>(blockIdx.x) * kDqWavesPerBlock + wave) * kDqRowsPerWave;
    const int W = (d + 63) >> 6;
    if constexpr (ONEPASS) {
        const int c0 = lane * VEC;
        const int cw = (c0 < d ? c0 : 0) >> 6;
        uint64_t meta[kDqRowsPerWave], word[kDqRowsPerWave];
#pragma unroll
        for (int r = 0; r < kDqRowsPerWave; ++r) {
            meta[r] = 0;
            word[r] = 0;
            if (first + r < n_rows) {
                const uint64_t *prow = wire + (first + r) * ldw;
                meta[r] = prow[W];
                word[r] = prow[cw];
            }
        }
#pragma unroll
        for (int r = 0; r < kDqRowsPerWave; ++r) {
            if (first + r < n_rows && c0 < d) {
                const float zp = __uint_as_float(static_cast<uint32_t>(meta[r] >> 32));
                const float hi = zp + __uint_as_float(static_cast<uint32_t>(meta[r]));
                const uint32_t bits = static_cast<uint32_t>(word[r] >> (c0 & 63));
                select_store<VEC>(dst + (row_offset + first + r) * ld + c0, bits, zp, hi);
            }
        }
    } else {
#pragma unroll 1
        for (int r = 0; r < kDqRowsPerWave; ++r) {
            const int64_t i = first + r;
            if (i >= n_rows) break;
            const uint64_t *prow = wire + i * ldw;
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
}

constexpr int kDqDstPerWave = 4;

// dst[dst_ids[k]] += the dequantised wire rows seg_rows[seg_ptr[k] .. seg_ptr[k+1]) in
// that order, float32.  One wavefront takes kDqDstPerWave destinations and walks their
// (independent) load chains side by side: segment bounds, first wire row id, its
// words, the destination row; further entries of a segment (rare) follow in a loop.
template <int VEC>
__global__ __launch_bounds__(kDqWavesPerBlock *kWave) void dequantize_bwd_kernel(
    const uint64_t *__restrict__ wire, int64_t ldw, int d, float *__restrict__ dst, int64_t ld,
    const int64_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_rows,
    int64_t n_dst_rows, const int32_t *__restrict__ dst_ids)
{
    using V = typename VecT<VEC>::type;
    constexpr int D = kDqDstPerWave;
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k0 = (static_cast<int64_t>(blockIdx.x) * kDqWavesPerBlock + wave) * D;
    if (k0 >= n_dst_rows) return;
    const int W = (d + 63) >> 6;
    // every load below is unconditional (indices clamped to something valid) so that the
    // loads of the D chains are issued together; a slot past the end gets an empty segment
    int64_t j0[D], j1[D];
    float *orow[D];
#pragma unroll
    for (int q = 0; q < D; ++q) {
        const bool valid = k0 + q < n_dst_rows;
        const int64_t kk = valid ? k0 + q : k0;
        j0[q] = seg_ptr[kk];
        j1[q] = seg_ptr[kk + 1];
        orow[q] = dst + static_cast<int64_t>(dst_ids[kk]) * ld;
        if (!valid) j1[q] = j0[q];
    }
#pragma unroll
    for (int q = 0; q < D; ++q) {
        j0[q] = uniform(j0[q]);
        j1[q] = uniform(j1[q]);
    }
    for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
        float acc[D][VEC];
        const uint64_t *prow[D];
        uint64_t meta[D], word[D];
#pragma unroll
        for (int q = 0; q < D; ++q) {
            stream_load<VEC>(acc[q], orow[q] + c0);   // read-modify-write rows: touched once
            // an empty segment reads nothing of seg_rows (which may then have no elements at
            // all): its load goes to a location that always exists and wire row 0 stands in
            const bool some = j0[q] < j1[q];
            const int32_t *pid = some ? seg_rows + j0[q] : dst_ids + k0;
            const int32_t id = *pid;
            prow[q] = wire + static_cast<int64_t>(some ? id : 0) * ldw;
        }
#pragma unroll
        for (int q = 0; q < D; ++q) {
            meta[q] = prow[q][W];
            word[q] = prow[q][c0 >> 6];
        }
#pragma unroll
        for (int q = 0; q < D; ++q) {
            if (j0[q] >= j1[q]) continue;
            for (int64_t j = j0[q];;) {
                const float zp = __uint_as_float(static_cast<uint32_t>(meta[q] >> 32));
                const float hi = zp + __uint_as_float(static_cast<uint32_t>(meta[q]));
                const uint32_t bits = static_cast<uint32_t>(word[q] >> (c0 & 63));
#pragma unroll
                for (int t = 0; t < VEC; ++t) acc[q][t] = acc[q][t] + (((bits >> t) & 1u) ? hi : zp);
                if (++j >= j1[q]) break;
                const uint64_t *pr = wire + static_cast<int64_t>(seg_rows[j]) * ldw;
                meta[q] = pr[W];
                word[q] = pr[c0 >> 6];
            }
            stream_store<VEC>(orow[q] + c0, acc[q]);
        }
    }
}

static int pick_vec(int d, int64_t ld, const void *p)
{
    if (d % 4 == 0 && ld % 4 == 0 && aligned(p, 16)) return 4;
    if (d % 2 == 0 && ld % 2 == 0 && aligned(p, 8)) return 2;
    return 1;
}

static int32_t check_wire(const char *name, const uint64_t *wire, int64_t ld_wire, int64_t n_rows,
                          int32_t d, const float *dst, int64_t ld)
{
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_rows %lld out of range", name, (long long)n_rows);
    if (d < 1 || d > 65536) return fail(SYLVIE_ERR_INVALID_ARG, "%s: d %d out of range", name, d);
    if (ld < d) return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_dst %lld < d %d", name, (long long)ld, d);
    if (ld_wire != 0 && ld_wire < (static_cast<int64_t>(d) + 63) / 64 + 1)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_wire %lld shorter than a wire row", name, (long long)ld_wire);
    if (n_rows == 0) return SYLVIE_OK;
    if (!wire || !dst) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(wire, 8) || !aligned(dst, 4))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned pointer", name);
    return SYLVIE_OK;
}

}  // namespace sylvie

extern "C" int32_t sylvie_dequantize_1bit_fwd(const uint64_t *wire, int64_t ld_wire, int64_t n_rows,
                                              int32_t d, float *dst, int64_t ld_dst, int64_t row_offset,
                                              void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_dequantize_1bit_fwd";
    const int32_t rc = check_wire(name, wire, ld_wire, n_rows, d, dst, ld_dst);
    const int64_t ldw = ld_wire ? ld_wire : (static_cast<int64_t>(d) + 63) / 64 + 1;
    if (rc != SYLVIE_OK) return rc;
    if (row_offset < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative row_offset", name);
    if (n_rows == 0) return SYLVIE_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t per_block = kDqWavesPerBlock * kDqRowsPerWave;
    const dim3 grid(static_cast<unsigned>((n_rows + per_block - 1) / per_block));
    const dim3 block(kDqWavesPerBlock * kWave);
    // the vector width must also hold for the first written row
    const int vec = pick_vec(d, ld_dst, dst + row_offset * ld_dst);
#define SYLVIE_DQ_LAUNCH(V, ONE)                                                                  \
    hipLaunchKernelGGL((dequantize_fwd_kernel<V, ONE>), grid, block, 0, st, wire, ldw, n_rows, d, \
                       dst, ld_dst, row_offset)
    if (vec == 4) {
        if (d <= 256) SYLVIE_DQ_LAUNCH(4, true); else SYLVIE_DQ_LAUNCH(4, false);
    } else if (vec == 2) {
        if (d <= 128) SYLVIE_DQ_LAUNCH(2, true); else SYLVIE_DQ_LAUNCH(2, false);
    } else {
        if (d <= 64) SYLVIE_DQ_LAUNCH(1, true); else SYLVIE_DQ_LAUNCH(1, false);
    }
#undef SYLVIE_DQ_LAUNCH
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_dequantize_1bit_bwd(const uint64_t *wire, int64_t ld_wire, int64_t n_rows,
                                              int32_t d, float *dst, int64_t ld_dst,
                                              const int64_t *seg_ptr, const int32_t *seg_rows,
                                              int64_t n_dst_rows, const int32_t *dst_ids, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_dequantize_1bit_bwd";
    const int32_t rc = check_wire(name, wire, ld_wire, n_rows, d, dst, ld_dst);
    const int64_t ldw = ld_wire ? ld_wire : (static_cast<int64_t>(d) + 63) / 64 + 1;
    if (rc != SYLVIE_OK) return rc;
    if (n_dst_rows < 0 || n_dst_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_dst_rows out of range", name);
    if (n_rows == 0 || n_dst_rows == 0) return SYLVIE_OK;
    if (!seg_ptr || !seg_rows || !dst_ids) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(seg_ptr, 8) || !aligned(seg_rows, 4) || !aligned(dst_ids, 4))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned index array", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (validate_enabled()) {
        Validator v(name, st);
        v.segments(seg_ptr, seg_rows, n_dst_rows, n_rows, dst_ids);
        const int32_t rc = v.finish();
        if (rc != SYLVIE_OK) return rc;
    }
    const int64_t per_block = kDqWavesPerBlock * kDqDstPerWave;
    const dim3 grid(static_cast<unsigned>((n_dst_rows + per_block - 1) / per_block));
    const dim3 block(kDqWavesPerBlock * kWave);
    const int vec = pick_vec(d, ld_dst, dst);
    if (vec == 4)
        hipLaunchKernelGGL(dequantize_bwd_kernel<4>, grid, block, 0, st, wire, ldw, d, dst,
                           ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    else if (vec == 2)
        hipLaunchKernelGGL(dequantize_bwd_kernel<2>, grid, block, 0, st, wire, ldw, d, dst,
                           ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    else
        hipLaunchKernelGGL(dequantize_bwd_kernel<1>, grid, block, 0, st, wire, ldw, d, dst,
                           ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}
