// The rounding draws of the quantizer (Sec. 3.2, Eq. 4) and the one-row quantizer
// that kernels other than the stand-alone quantizer use on a row they hold in LDS.
#pragma once

#include "common.hpp"

namespace sylvie {

// Counter hash behind the rounding draws.  Keys: (seed, stream) -> call key on
// the host; (call key, wire row) -> row key, scalar unit; (row key, column) ->
// 24 uniform bits per element.
constexpr uint32_t kM1 = 0xce6e1acdu;
constexpr uint32_t kM2 = 0x6d3cb3a7u;
constexpr uint32_t kColStride = 0x9e3779b9u;
constexpr uint32_t kDomain = 0x53594c56u;

__host__ __device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= kM1;
    x ^= x >> 15;
    x *= kM2;
    x ^= x >> 16;
    return x;
}

__host__ __device__ __forceinline__ uint32_t call_key(uint64_t seed, uint32_t stream_id)
{
    uint32_t k = mix32(static_cast<uint32_t>(seed) ^ kDomain);
    k = mix32(k ^ static_cast<uint32_t>(seed >> 32));
    return mix32(k ^ stream_id);
}

// The key of one quantizing call as its kernels receive it.  Normally the host has hashed
// (seed, stream) into `key`.  When the caller has named a device-resident seed offset
// (sylvie_seed_offset_source), `offset` points at it and the kernel hashes
// (seed + *offset, stream) itself, on the scalar unit, once per wavefront: a launch recorded in
// a graph then draws the bits of a new seed on every replay.
struct CallKey {
    uint32_t key;
    uint32_t stream_id;
    uint64_t seed;
    const uint64_t *offset;
};
CallKey make_call_key(uint64_t seed, uint32_t stream_id);   // api.hip
__device__ __forceinline__ uint32_t call_key_of(const CallKey &k)
{
    if (!k.offset) return k.key;
    const uint64_t s = k.seed + *k.offset;
    return call_key(s, k.stream_id);
}

// Top 24 bits of the second product: the draw for one element.  Both xor-shifts
// are by 16 so that each is a single VALU op (the shifted operand is a sub-dword
// select of the same register).
__device__ __forceinline__ uint32_t draw24(uint32_t x)
{
    x ^= x >> 16;
    x *= kM1;
    x ^= x >> 16;
    x *= kM2;
    return x >> 8;
}

// Quantize one row of d floats that this wavefront holds in LDS (row[0..d)) into wire
// row `out` (W bit words + the scale|zero word), with the draws of wire row `i`.
// Exactly the arithmetic of the stand-alone quantizer: extrema, + 0.0f, scale =
// max - min, bit = [fl(k * 2^-24 * scale) < fl(x - min)] with the exact fold of the
// power of two unless scale * 2^-24 would be subnormal.  All 64 lanes must call it.
__device__ __forceinline__ void quantize_row_lds(const float *row, int d, uint32_t ckey,
                                                 uint32_t i, uint64_t *out, int lane)
{
    constexpr float kTwoM24 = 1.0f / 16777216.0f;
    const int W = (d + 63) >> 6;
    wave_lds_sync();    // the row was written by other lanes of this wavefront
    // columns past d re-read column d-1: extrema unchanged, no predicate
    float mn = row[lane < d ? lane : d - 1], mx = mn;
    for (int c = lane + 64; c < d; c += 64) {
        const float x = row[c];
        mn = fmin_sel(mn, x);
        mx = fmax_sel(mx, x);
    }
    wave_minmax(mn, mx);
    mn = mn + 0.0f;
    mx = mx + 0.0f;
    const float sc = mx - mn;
    const bool fold = sc >= 0x1p-102f || sc == 0.0f;
    const float sc24 = sc * kTwoM24;
    const uint32_t rkey = mix32(ckey ^ i);
    uint32_t ctr = rkey + static_cast<uint32_t>(lane) * kColStride;
    uint64_t mine = 0;
    for (int k = 0; k < W; ++k) {
        const int c = k * 64 + lane;
        const float x = row[c < d ? c : d - 1];
        const float kf = static_cast<float>(draw24(ctr));
        const float lhs = fold ? kf * sc24 : (kf * kTwoM24) * sc;
        const uint64_t word = __ballot(c < d && lhs < x - mn);
        if (lane == k) mine = word;
        ctr += 64u * kColStride;
    }
    if (lane == W) mine = (static_cast<uint64_t>(__float_as_uint(mn)) << 32) | __float_as_uint(sc);
    // W + 1 <= 64 for every width the callers support (d <= 2048)
    if (lane <= W) out[lane] = mine;
}

}  // namespace sylvie
