// 1-bit stochastic-rounding quantizer with fused row gather, row extrema and bit
// packing (Sec. 3.2 "Quantizer" / "Communicator", Eq. 3-4 with b = 1).
//
// One wavefront owns one wire row at a time.  Lane L holds columns L, L+64,
// L+128, ... of the row in registers, so a single wave-wide compare produces a
// 64-bit lane mask that IS packed word k of the row (bit j = column 64k + j): the
// packing costs no instructions.  Row minimum and maximum are a DPP reduction;
// the per-row hash key lives on the scalar unit.
#include <utility>

#include "common.hpp"
#include "rounding.hpp"
#include "validate.hpp"

namespace sylvie {

constexpr int kWavesPerBlock = 4;

// lo[LANE] = low half, hi[LANE] = high half of a wave-uniform 64-bit value held in
// scalar registers; other lanes keep theirs.  The lane select has to be an inline
// constant (data and select may not both be scalar registers).  The value is
// usually the result of the vector compare just before: a scalar register written
// by the vector unit needs two wait states before the vector unit reads it back,
// and the compiler does not look inside an asm block, hence the s_nop.
template <int LANE>
__device__ __forceinline__ void write_lane64(int &lo, int &hi, uint64_t value)
{
    asm volatile("s_nop 1\n\t"
                 "v_writelane_b32 %0, %2, %4\n\t"
                 "v_writelane_b32 %1, %3, %4"
                 : "+v"(lo), "+v"(hi)
                 : "s"(static_cast<int>(value)), "s"(static_cast<int>(value >> 32)), "n"(LANE));
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): loop indices that
// are constant expressions inside the body
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// rows per wave: as many as fit one 64-lane store of (P + 1)-word wire rows, at most 4
constexpr int rows_per_wave(int P) { return 64 / (P + 1) < 4 ? 64 / (P + 1) : 4; }

// P = number of 64-column chunks held in registers (64 (P-1) < d <= 64 P);
// FULL = (d == 64 P): no ragged last chunk.
//
// A wave owns R consecutive wire rows.  The loads of row r+1 are issued before
// row r is processed.  Columns past d re-read column d-1, which leaves the
// extrema unchanged and needs no predicate; their bits are masked off.  A wire
// row is P bit words followed by one metadata word (scale in the low half, zero
// in the high half); the words of all the wave's rows are collected into lanes
// r*(P+1) + k and leave in one contiguous store.
template <int P, bool FULL>
__global__ __launch_bounds__(kWavesPerBlock *kWave) void quantize_rows_kernel(
    const float *__restrict__ src, int64_t ld, int d, const int32_t *__restrict__ idx,
    int64_t row_offset, int64_t n_rows, CallKey ck, uint64_t *__restrict__ wire, int64_t ldw)
{
    const uint32_t ckey = call_key_of(ck);
    constexpr int R = rows_per_wave(P);
    static_assert(R >= 1 && R * (P + 1) <= 64, "one store must hold all words of a wave");
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave) * R;
    if (first >= n_rows) return;
    const int nrows = static_cast<int>(n_rows - first < R ? n_rows - first : R);
    constexpr int W1 = P + 1;       // words per wire row
    constexpr float kTwoM24 = 1.0f / 16777216.0f;

    int my_src = 0;
    if (idx && lane < nrows) my_src = idx[first + lane];

    int coff[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = p * 64 + lane;
        coff[p] = FULL ? c : (c < d ? c : d - 1);
    }
    const uint64_t tail_mask =
        FULL ? ~uint64_t(0) : (~uint64_t(0) >> (63 - ((d - 1) & 63)));

    auto row_base = [&](int r) -> const float * {
        const int64_t srow = idx ? static_cast<int64_t>(__builtin_amdgcn_readlane(my_src, r))
                                 : row_offset + first + r;
        return src + srow * ld;
    };

    float cur[P], nxt[P];
    {
        const float *row = row_base(0);
#pragma unroll
        for (int p = 0; p < P; ++p) cur[p] = row[coff[p]];
    }
    int my_lo = 0, my_hi = 0;       // this lane's word of the wave's output run
    const uint32_t lane_ctr = static_cast<uint32_t>(lane) * kColStride;

    static_for<R>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        if (r < nrows) {
            if (r + 1 < nrows) {
                const float *row = row_base(r + 1);
#pragma unroll
                for (int p = 0; p < P; ++p) nxt[p] = row[coff[p]];
            }
            float mn = cur[0], mx = cur[0];
#pragma unroll
            for (int p = 1; p < P; ++p) {
                mn = fmin_sel(mn, cur[p]);
                mx = fmax_sel(mx, cur[p]);
            }
            wave_minmax(mn, mx);
            mn = mn + 0.0f;
            mx = mx + 0.0f;
            const float sc = mx - mn;
            const uint32_t rkey = mix32(ckey ^ static_cast<uint32_t>(first + r));
            uint32_t ctr = rkey + lane_ctr;
            // u * scale with u = k * 2^-24: folding the exact power of two into the
            // scale gives the same single rounding unless scale * 2^-24 is subnormal.
            const bool fold = sc >= 0x1p-102f || sc == 0.0f;
            const float sc24 = sc * kTwoM24;
            auto emit = [&](auto pc, bool on) {
                constexpr int p = decltype(pc)::value;
                uint64_t word = __ballot(on);
                if (!FULL && p == P - 1) word &= tail_mask;
                write_lane64<r * W1 + p>(my_lo, my_hi, word);
            };
            if (__builtin_expect(fold, 1)) {
                static_for<P>([&](auto pc) {
                    constexpr int p = decltype(pc)::value;
                    const float k = static_cast<float>(draw24(ctr + static_cast<uint32_t>(p) * 64u * kColStride));
                    emit(pc, k * sc24 < cur[p] - mn);
                });
            } else {
                static_for<P>([&](auto pc) {
                    constexpr int p = decltype(pc)::value;
                    const float k = static_cast<float>(draw24(ctr + static_cast<uint32_t>(p) * 64u * kColStride));
                    emit(pc, (k * kTwoM24) * sc < cur[p] - mn);
                });
            }
            write_lane64<r * W1 + P>(my_lo, my_hi,
                                     (static_cast<uint64_t>(uniform(__float_as_uint(mn))) << 32) |
                                         uniform(__float_as_uint(sc)));
#pragma unroll
            for (int p = 0; p < P; ++p) cur[p] = nxt[p];
        }
    });
    // lane l holds word l % W1 of the wave's row l / W1; rows sit ldw words apart
    if (lane < nrows * W1) {
        const int r = lane / W1;
        wire[(first + r) * ldw + (lane - r * W1)] =
            (static_cast<uint64_t>(static_cast<uint32_t>(my_hi)) << 32) | static_cast<uint32_t>(my_lo);
    }
}

// Any width: the row is read twice (the second read hits the cache).
__global__ __launch_bounds__(kWavesPerBlock *kWave) void quantize_rows_wide_kernel(
    const float *__restrict__ src, int64_t ld, int d, const int32_t *__restrict__ idx,
    int64_t row_offset, int64_t n_rows, CallKey ck, uint64_t *__restrict__ wire, int64_t ldw)
{
    const uint32_t ckey = call_key_of(ck);
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave;
    if (i >= n_rows) return;
    const int W = (d + 63) >> 6;
    constexpr float kTwoM24 = 1.0f / 16777216.0f;
    const int64_t srow = idx ? static_cast<int64_t>(uniform(idx[i])) : row_offset + i;
    const float *row = src + srow * ld;
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int c = lane; c < d; c += 64) {
        const float x = row[c];
        mn = fmin_sel(mn, x);
        mx = fmax_sel(mx, x);
    }
    wave_minmax(mn, mx);
    mn = mn + 0.0f;
    mx = mx + 0.0f;
    const float sc = mx - mn;
    const uint32_t rkey = mix32(ckey ^ static_cast<uint32_t>(i));
    uint32_t ctr = rkey + static_cast<uint32_t>(lane) * kColStride;
    uint64_t *out = wire + i * ldw;
    for (int k = 0; k < W; ++k) {
        const int c = k * 64 + lane;
        const float x = c < d ? row[c] : 0.0f;
        const float u = static_cast<float>(draw24(ctr)) * kTwoM24;
        const bool on = (c < d) && (u * sc < x - mn);
        const uint64_t word = __ballot(on);
        if (lane == 0) out[k] = word;
        ctr += 64u * kColStride;
    }
    if (lane == 0) out[W] = (static_cast<uint64_t>(__float_as_uint(mn)) << 32) | __float_as_uint(sc);
}

template <int P, bool FULL>
static void launch_rows(const float *src, int64_t ld, int d, const int32_t *idx,
                        int64_t row_offset, int64_t n_rows, const CallKey &ckey, uint64_t *wire,
                        int64_t ldw, hipStream_t st)
{
    const int64_t rows_per_block = rows_per_wave(P) * kWavesPerBlock;
    const int64_t blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL((quantize_rows_kernel<P, FULL>), dim3(static_cast<unsigned>(blocks)),
                       dim3(kWavesPerBlock * kWave), 0, st, src, ld, d, idx, row_offset, n_rows,
                       ckey, wire, ldw);
}

static int32_t quantize_common(const char *name, const float *src, int64_t ld, int32_t d,
                               const int32_t *idx, int64_t row_offset, int64_t n_rows,
                               uint64_t seed, uint32_t stream_id, uint64_t *wire, int64_t ld_wire,
                               void *stream)
{
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_rows %lld out of range", name, (long long)n_rows);
    if (d < 1 || d > 65536) return fail(SYLVIE_ERR_INVALID_ARG, "%s: d %d out of range", name, d);
    if (ld < d) return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_src %lld < d %d", name, (long long)ld, d);
    const int64_t ldw = ld_wire ? ld_wire : (static_cast<int64_t>(d) + 63) / 64 + 1;
    if (ldw < (static_cast<int64_t>(d) + 63) / 64 + 1)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_wire %lld shorter than a wire row", name, (long long)ld_wire);
    if (!idx && row_offset < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative row_offset", name);
    if (n_rows == 0) return SYLVIE_OK;
    if (!src || !wire) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(src, 4) || (idx && !aligned(idx, 4)))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: float/int arrays need 4-byte alignment", name);
    if (!aligned(wire, 8))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: wire_out needs 8-byte alignment", name);

    hipStream_t st = static_cast<hipStream_t>(stream);
    if (validate_enabled()) {
        Validator v(name, st);
        v.rows(src, ld, d, idx, row_offset, n_rows);
        const int32_t rc = v.finish();
        if (rc != SYLVIE_OK) return rc;
    }
    const CallKey ckey = make_call_key(seed, stream_id);
    const int P = (d + 63) / 64;
#define SYLVIE_Q_CASE(p)                                                                       \
    case p:                                                                                    \
        if (d == 64 * p)                                                                       \
            launch_rows<p, true>(src, ld, d, idx, row_offset, n_rows, ckey, wire, ldw, st);                \
        else                                                                                   \
            launch_rows<p, false>(src, ld, d, idx, row_offset, n_rows, ckey, wire, ldw, st);              \
        break;
    switch (P) {
        SYLVIE_Q_CASE(1)
        SYLVIE_Q_CASE(2)
        SYLVIE_Q_CASE(3)
        SYLVIE_Q_CASE(4)
        SYLVIE_Q_CASE(5)
        SYLVIE_Q_CASE(6)
        SYLVIE_Q_CASE(7)
        SYLVIE_Q_CASE(8)
        SYLVIE_Q_CASE(9)
        SYLVIE_Q_CASE(10)
        SYLVIE_Q_CASE(11)
        SYLVIE_Q_CASE(12)
        SYLVIE_Q_CASE(13)
        SYLVIE_Q_CASE(14)
        SYLVIE_Q_CASE(15)
        SYLVIE_Q_CASE(16)
    default: {
        const int64_t blocks = (n_rows + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(quantize_rows_wide_kernel, dim3(static_cast<unsigned>(blocks)),
                           dim3(kWavesPerBlock * kWave), 0, st, src, ld, d, idx, row_offset,
                           n_rows, ckey, wire, ldw);
    }
    }
#undef SYLVIE_Q_CASE
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

}  // namespace sylvie

extern "C" int32_t sylvie_quantize_1bit_fwd(const float *src, int64_t ld_src, int32_t d,
                                            const int32_t *idx, int64_t row_offset,
                                            int64_t n_rows, uint64_t seed, uint32_t stream_id,
                                            uint64_t *wire_out, int64_t ld_wire, void *stream)
{
    return sylvie::quantize_common("sylvie_quantize_1bit_fwd", src, ld_src, d, idx, row_offset,
                                   n_rows, seed, stream_id, wire_out, ld_wire, stream);
}

extern "C" int32_t sylvie_quantize_1bit_bwd(const float *src, int64_t ld_src, int32_t d,
                                            const int32_t *idx, int64_t row_offset,
                                            int64_t n_rows, uint64_t seed, uint32_t stream_id,
                                            uint64_t *wire_out, int64_t ld_wire, void *stream)
{
    return sylvie::quantize_common("sylvie_quantize_1bit_bwd", src, ld_src, d, idx, row_offset,
                                   n_rows, seed, stream_id, wire_out, ld_wire, stream);
}
