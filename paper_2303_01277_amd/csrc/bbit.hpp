// Device pieces of the b-bit Low-bit Module (Sec. 3.2, Eq. 3-5 with B = 2^b - 1) shared by the
// stand-alone quantizer / dequantizer kernels and the aggregation's fused forms: the row
// constants, the code of one element, the recovered value of one code, and the one-row
// quantizer for a row that a wavefront holds in LDS.
#pragma once

#include "common.hpp"
#include "rounding.hpp"

namespace sylvie {

template <int VEC>
__device__ __forceinline__ void bb_load(float (&o)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    } else {
        o[0] = *p;
    }
}

// Row constants of Eq. 3 for one wire row (all wave-uniform).
struct BbRow {
    float mn, scale, inv;
    bool tiny;
};
template <int BITS>
__device__ __forceinline__ BbRow bb_row_constants(float mn, float mx)
{
    constexpr float Bf = static_cast<float>((1 << BITS) - 1);
    BbRow r;
    mn = mn + 0.0f;
    mx = mx + 0.0f;
    const float range = mx - mn;
    r.mn = mn;
    r.scale = range / Bf;
    r.tiny = range < 0x1p-60f;
    const float den = r.tiny ? range * 0x1p64f : range;
    r.inv = range > 0.0f ? Bf / den : 0.0f;
    return r;
}

// Code of one element (Eq. 3-4).
template <int BITS, bool TINY>
__device__ __forceinline__ uint32_t bb_code(float x, const BbRow &r, uint32_t ctr)
{
    constexpr float Bf = static_cast<float>((1 << BITS) - 1);
    constexpr float kTwoM24 = 1.0f / 16777216.0f;
    float diff = x - r.mn;
    if constexpr (TINY) diff = diff * 0x1p64f;
    float t = diff * r.inv;
    t = t > Bf ? Bf : t;
    // t >= 0: the conversion truncates to floor(t) and v_fract_f32 is t - floor(t), exact
    const float fr = __builtin_amdgcn_fractf(t);
    const float u = static_cast<float>(draw24(ctr)) * kTwoM24;
    return static_cast<uint32_t>(t) + (u < fr ? 1u : 0u);
}

// The VEC codes of columns c0 .. c0 + VEC - 1 (c0 % VEC == 0): one piece of a dword.
template <int BITS, int VEC>
__device__ __forceinline__ uint32_t bb_piece(const uint64_t *prow, int c0)
{
    const uint32_t bit = static_cast<uint32_t>(c0) * BITS;
    const uint32_t dw = reinterpret_cast<const uint32_t *>(prow)[bit >> 5];
    return dw >> (bit & 31u);
}
template <int BITS>
__device__ __forceinline__ float bb_value(uint32_t piece, int t, float sc, float zp)
{
    const uint32_t q = (piece >> (BITS * t)) & ((1u << BITS) - 1u);
    const float step = sc * static_cast<float>(q);
    return step + zp;
}

// Output rows are written once and read by a later launch: streaming stores.
template <int VEC>
__device__ __forceinline__ void bb_store(float *p, const float (&v)[VEC])
{
    stream_store<VEC>(p, v);
}

// Quantize one row of d floats that this wavefront holds in LDS (row[0..d), d % 4 == 0, 16-byte
// aligned) into wire row `out` (ceil(d BITS / 64) code words + the scale | zero word) with the
// draws of wire row `i`: exactly the arithmetic and the draws of quantize_bbit_kernel.  `img` is
// wave-private LDS of at least d / 4 + 2 dwords that does not overlap `row`.  All 64 lanes call.
template <int BITS>
__device__ __forceinline__ void quantize_row_lds_bbit(const float *row, int d, uint32_t ckey, uint32_t i,
                                                      uint64_t *out, uint32_t *img, int lane)
{
    wave_lds_sync();    // the row was written by other lanes of this wavefront
    const int Wb = (d * BITS + 63) >> 6;
    const int last = d - 4;
    float mn, mx;
    {
        const float4 v = *reinterpret_cast<const float4 *>(row + (lane * 4 < d ? lane * 4 : last));
        mn = fmin_sel(fmin_sel(v.x, v.y), fmin_sel(v.z, v.w));
        mx = fmax_sel(fmax_sel(v.x, v.y), fmax_sel(v.z, v.w));
    }
    for (int c0 = (lane + 64) * 4; c0 < d; c0 += 256) {
        const float4 v = *reinterpret_cast<const float4 *>(row + c0);
        mn = fmin_sel(mn, fmin_sel(fmin_sel(v.x, v.y), fmin_sel(v.z, v.w)));
        mx = fmax_sel(mx, fmax_sel(fmax_sel(v.x, v.y), fmax_sel(v.z, v.w)));
    }
    wave_minmax(mn, mx);
    const BbRow rc = bb_row_constants<BITS>(mn, mx);
    const uint32_t rkey = mix32(ckey ^ i);
    // pieces of 4 codes each; slots past the row (up to the end of its last word) hold zeros
    const int slots = Wb * 64 / (4 * BITS);
    for (int s = lane; s < slots; s += 64) {
        const int c0 = s * 4;
        uint32_t piece = 0;
        if (c0 < d) {
            const float4 v = *reinterpret_cast<const float4 *>(row + c0);
            const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t ctr = rkey + static_cast<uint32_t>(c0 + t) * kColStride;
                const uint32_t q = rc.tiny ? bb_code<BITS, true>(x[t], rc, ctr) : bb_code<BITS, false>(x[t], rc, ctr);
                piece |= q << (BITS * t);
            }
        }
        if constexpr (BITS == 2) reinterpret_cast<uint8_t *>(img)[s] = static_cast<uint8_t>(piece);
        else if constexpr (BITS == 4) reinterpret_cast<uint16_t *>(img)[s] = static_cast<uint16_t>(piece);
        else img[s] = piece;
    }
    wave_lds_sync();
    for (int k = lane; k < Wb; k += 64) out[k] = *reinterpret_cast<const uint64_t *>(img + 2 * k);
    if (lane == (Wb & 63))
        out[Wb] = (static_cast<uint64_t>(__float_as_uint(rc.mn)) << 32) | __float_as_uint(rc.scale);
    wave_lds_sync();
}

// ---- half-precision wire rows (d binary16 values, zero halves up to a multiple of four) --------

template <int VEC>
__device__ __forceinline__ void fp16_load(float (&o)[VEC], const uint16_t *p)
{
    if constexpr (VEC == 4) {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        o[0] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v.x & 0xffffu)));
        o[1] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v.x >> 16)));
        o[2] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v.y & 0xffffu)));
        o[3] = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(v.y >> 16)));
    } else {
        o[0] = static_cast<float>(__builtin_bit_cast(_Float16, *p));
    }
}

// Four floats -> four binary16 values (round to nearest even) as two dwords.
__device__ __forceinline__ uint2 fp16_pack4(const float (&v)[4])
{
    const _Float16 h0 = static_cast<_Float16>(v[0]), h1 = static_cast<_Float16>(v[1]);
    const _Float16 h2 = static_cast<_Float16>(v[2]), h3 = static_cast<_Float16>(v[3]);
    uint2 o;
    o.x = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h0)) |
          (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h1)) << 16);
    o.y = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h2)) |
          (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h3)) << 16);
    return o;
}

// Convert one row of d floats that this wavefront holds in LDS (d % 4 == 0, 16-byte aligned)
// into the half-precision wire row `out`: the arithmetic of convert_fp16_kernel.  All 64 lanes call.
__device__ __forceinline__ void convert_row_lds_fp16(const float *row, int d, uint64_t *out, int lane)
{
    wave_lds_sync();    // the row was written by other lanes of this wavefront
    for (int c0 = lane * 4; c0 < d; c0 += 256) {
        const float4 x = *reinterpret_cast<const float4 *>(row + c0);
        const float v[4] = {x.x, x.y, x.z, x.w};
        *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + c0) = fp16_pack4(v);
    }
    wave_lds_sync();
}

}  // namespace sylvie
