// b-bit Low-bit Module (Sec. 3.2, Eq. 3-5 with B = 2^b - 1, b in {2, 4, 8}; the
// bit-width study of Sec. 4.3) and the half-precision wire of the same study.
//
// Quantizer: one wavefront per wire row, as in the 1-bit kernel, but lane L holds VEC
// ADJACENT columns per pass, because the codes of adjacent columns are adjacent in the
// packed row.  A lane's VEC codes form one VEC*b-bit piece that never straddles a
// dword; the pieces are OR-ed into a wave-private LDS image of the packed row, which
// then leaves in one contiguous store together with the scale | zero word.
//
// Per row, single precision, one operation each (no contraction):
//   range = max - min, scale = range / B, g = 2^64 if range < 2^-60 else 1,
//   inv = B / (range g) (0 for a constant row)
// per element
//   t = min(((x - min) g) inv, B), q = floor(t) + [k 2^-24 < t - floor(t)]
// with k the 24-bit draw of (seed, stream, wire row, column).
// Dequantizer (Eq. 5): fl(fl(scale q) + zero).
#include <type_traits>

#include "common.hpp"
#include "rounding.hpp"
#include "bbit.hpp"

namespace sylvie {

constexpr int kBbWavesPerBlock = 4;
constexpr int kBbRowsPerWave = 4;

// P passes of 64 VEC columns cover the row (64 VEC (P-1) < d <= 64 VEC P).  VEC = 4
// needs d % 4 == 0 and 16-byte aligned rows.  A wave takes kBbRowsPerWave consecutive
// rows and issues the loads of the next row before it works on the current one.
template <int BITS, int VEC, int P>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void quantize_bbit_kernel(
    const float *__restrict__ src, int64_t ld, int d, const int32_t *__restrict__ idx,
    int64_t row_offset, int64_t n_rows, CallKey ck, uint64_t *__restrict__ wire)
{
    const uint32_t ckey = call_key_of(ck);
    constexpr int R = kBbRowsPerWave;
    constexpr int kDwords = P * 64 * VEC * BITS / 32;          // packed codes of a full-width row
    __shared__ __align__(8) uint32_t image[kBbWavesPerBlock][kDwords + 2];
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave) * R;
    if (first >= n_rows) return;
    const int nrows = static_cast<int>(n_rows - first < R ? n_rows - first : R);
    const int Wb = (d * BITS + 63) >> 6;                       // code words per wire row
    uint32_t *img = image[wave];

    int my_src = 0;
    if (idx && lane < nrows) my_src = idx[first + lane];
    // columns past d re-read the last vector of the row: extrema unchanged, no predicate
    int coff[P];
    bool valid[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = (p * 64 + lane) * VEC;
        valid[p] = c < d;
        coff[p] = valid[p] ? c : d - VEC;
    }
    auto row_base = [&](int r) -> const float * {
        const int64_t srow = idx ? static_cast<int64_t>(__builtin_amdgcn_readlane(my_src, r))
                                 : row_offset + first + r;
        return src + srow * ld;
    };
    float cur[P][VEC], nxt[P][VEC];
    {
        const float *row = row_base(0);
#pragma unroll
        for (int p = 0; p < P; ++p) bb_load<VEC>(cur[p], row + coff[p]);
    }
#pragma unroll 1
    for (int r = 0; r < nrows; ++r) {
        if (r + 1 < nrows) {
            const float *row = row_base(r + 1);
#pragma unroll
            for (int p = 0; p < P; ++p) bb_load<VEC>(nxt[p], row + coff[p]);
        }
        float mn = cur[0][0], mx = cur[0][0];
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int t = 0; t < VEC; ++t) {
                mn = fmin_sel(mn, cur[p][t]);
                mx = fmax_sel(mx, cur[p][t]);
            }
        wave_minmax(mn, mx);
        const BbRow rc = bb_row_constants<BITS>(mn, mx);
        // A lane's VEC codes are a piece of VEC * BITS bits.  Where that is a whole number of
        // bytes (VEC = 4) every lane stores its piece with one plain sub-dword write - lanes
        // past the row store zeros, which are the padding bits - so the image needs neither
        // clearing nor atomics; otherwise the image is cleared and the pieces are OR-ed in.
        constexpr int kPieceBits = VEC * BITS;
        constexpr bool kPlain = kPieceBits % 8 == 0;
        if constexpr (!kPlain)
            for (int k = lane; k < 2 * Wb; k += 64) img[k] = 0u;
        const uint32_t rkey = mix32(ckey ^ static_cast<uint32_t>(first + r));
        auto encode = [&](auto tiny_c) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const uint32_t c0 = static_cast<uint32_t>((p * 64 + lane) * VEC);
                uint32_t piece = 0;
#pragma unroll
                for (int t = 0; t < VEC; ++t)
                    piece |= bb_code<BITS, decltype(tiny_c)::value>(cur[p][t], rc, rkey + (c0 + t) * kColStride)
                             << (BITS * t);
                if constexpr (kPlain) {
                    const uint32_t v = valid[p] ? piece : 0u;
                    const int slot = p * 64 + lane;                 // piece index inside the row
                    if constexpr (kPieceBits == 8) reinterpret_cast<uint8_t *>(img)[slot] = static_cast<uint8_t>(v);
                    else if constexpr (kPieceBits == 16) reinterpret_cast<uint16_t *>(img)[slot] = static_cast<uint16_t>(v);
                    else img[slot] = v;
                } else if (valid[p]) {
                    const uint32_t bit = c0 * BITS;
                    atomicOr(&img[bit >> 5], piece << (bit & 31u));
                }
            }
        };
        if (__builtin_expect(rc.tiny, 0)) encode(std::true_type{});
        else encode(std::false_type{});
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint64_t *out = wire + (first + r) * (Wb + 1);
        for (int k = lane; k < Wb; k += 64)
            out[k] = *reinterpret_cast<const uint64_t *>(img + 2 * k);
        if (lane == (Wb & 63))
            out[Wb] = (static_cast<uint64_t>(__float_as_uint(rc.mn)) << 32) | __float_as_uint(rc.scale);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int t = 0; t < VEC; ++t) cur[p][t] = nxt[p][t];
    }
}

// Any width and alignment: the row is read twice (the second read hits the cache) and
// the packed row is assembled in global memory word by word through the LDS image of
// 64 columns at a time.
template <int BITS>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void quantize_bbit_wide_kernel(
    const float *__restrict__ src, int64_t ld, int d, const int32_t *__restrict__ idx,
    int64_t row_offset, int64_t n_rows, CallKey ck, uint64_t *__restrict__ wire)
{
    const uint32_t ckey = call_key_of(ck);
    __shared__ __align__(8) uint32_t image[kBbWavesPerBlock][2 * BITS];   // 64 codes
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave;
    if (i >= n_rows) return;
    const int Wb = (d * BITS + 63) >> 6;
    uint32_t *img = image[wave];
    const int64_t srow = idx ? static_cast<int64_t>(uniform(idx[i])) : row_offset + i;
    const float *row = src + srow * ld;
    float mn = row[lane < d ? lane : d - 1], mx = mn;
    for (int c = lane + 64; c < d; c += 64) {
        const float x = row[c];
        mn = fmin_sel(mn, x);
        mx = fmax_sel(mx, x);
    }
    wave_minmax(mn, mx);
    const BbRow rc = bb_row_constants<BITS>(mn, mx);
    const uint32_t rkey = mix32(ckey ^ static_cast<uint32_t>(i));
    uint64_t *out = wire + i * (Wb + 1);
    // 64 columns = BITS 64-bit words of codes per step
    for (int c0 = 0; c0 < d; c0 += 64) {
        if (lane < 2 * BITS) img[lane] = 0u;
        __builtin_amdgcn_wave_barrier();
        const int c = c0 + lane;
        if (c < d) {
            const float x = row[c];
            const uint32_t q = rc.tiny ? bb_code<BITS, true>(x, rc, rkey + static_cast<uint32_t>(c) * kColStride)
                                       : bb_code<BITS, false>(x, rc, rkey + static_cast<uint32_t>(c) * kColStride);
            const uint32_t bit = static_cast<uint32_t>(lane) * BITS;
            atomicOr(&img[bit >> 5], q << (bit & 31u));
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        const int w0 = (c0 / 64) * BITS;                  // first word of this step
        if (lane < BITS && w0 + lane < Wb) out[w0 + lane] = *reinterpret_cast<const uint64_t *>(img + 2 * lane);
        __builtin_amdgcn_wave_barrier();
    }
    if (lane == 0) out[Wb] = (static_cast<uint64_t>(__float_as_uint(rc.mn)) << 32) | __float_as_uint(rc.scale);
}

// ---- dequantizer ------------------------------------------------------------------

// Forward: wire row i overwrites row row_offset + i of dst.  A wave takes
// kBbRowsPerWave rows; for rows of at most 64 VEC columns all their loads are issued
// before the first store.
template <int BITS, int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void dequantize_bbit_fwd_kernel(
    const uint64_t *__restrict__ wire, int64_t n_rows, int d, float *__restrict__ dst, int64_t ld,
    int64_t row_offset)
{
    constexpr int R = kBbRowsPerWave;
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave) * R;
    const int Wb = (d * BITS + 63) >> 6;
    if (d <= 64 * VEC) {
        const int c0 = lane * VEC;
        const int cl = c0 < d ? c0 : 0;
        uint64_t meta[R];
        uint32_t piece[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            meta[r] = 0;
            piece[r] = 0;
            if (first + r < n_rows) {
                const uint64_t *prow = wire + (first + r) * (Wb + 1);
                meta[r] = prow[Wb];
                piece[r] = bb_piece<BITS, VEC>(prow, cl);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (first + r < n_rows && c0 < d) {
                const float zp = __uint_as_float(static_cast<uint32_t>(meta[r] >> 32));
                const float sc = __uint_as_float(static_cast<uint32_t>(meta[r]));
                float v[VEC];
#pragma unroll
                for (int t = 0; t < VEC; ++t) v[t] = bb_value<BITS>(piece[r], t, sc, zp);
                bb_store<VEC>(dst + (row_offset + first + r) * ld + c0, v);
            }
        }
    } else {
#pragma unroll 1
        for (int r = 0; r < R; ++r) {
            const int64_t i = first + r;
            if (i >= n_rows) break;
            const uint64_t *prow = wire + i * (Wb + 1);
            const uint64_t meta = prow[Wb];
            const float zp = __uint_as_float(static_cast<uint32_t>(meta >> 32));
            const float sc = __uint_as_float(static_cast<uint32_t>(meta));
            float *orow = dst + (row_offset + i) * ld;
            for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
                const uint32_t piece = bb_piece<BITS, VEC>(prow, c0);
                float v[VEC];
#pragma unroll
                for (int t = 0; t < VEC; ++t) v[t] = bb_value<BITS>(piece, t, sc, zp);
                bb_store<VEC>(orow + c0, v);
            }
        }
    }
}

// Backward: dst[dst_ids[k]] += the recovered wire rows of segment k in ascending order,
// single precision (Alg. 2, integrate).  One wavefront per destination row.
template <int BITS, int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void dequantize_bbit_bwd_kernel(
    const uint64_t *__restrict__ wire, int d, float *__restrict__ dst, int64_t ld,
    const int64_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_rows,
    int64_t n_dst_rows, const int32_t *__restrict__ dst_ids)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave;
    if (k >= n_dst_rows) return;
    const int Wb = (d * BITS + 63) >> 6;
    const int64_t j0 = uniform(seg_ptr[k]), j1 = uniform(seg_ptr[k + 1]);
    if (j0 >= j1) return;
    float *orow = dst + static_cast<int64_t>(uniform(dst_ids[k])) * ld;
    for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
        float acc[VEC];
        stream_load<VEC>(acc, orow + c0);      // read-modify-write row: touched once
        for (int64_t j = j0; j < j1; ++j) {
            const uint64_t *prow = wire + static_cast<int64_t>(uniform(seg_rows[j])) * (Wb + 1);
            const uint64_t meta = prow[Wb];
            const float zp = __uint_as_float(static_cast<uint32_t>(meta >> 32));
            const float sc = __uint_as_float(static_cast<uint32_t>(meta));
            const uint32_t piece = bb_piece<BITS, VEC>(prow, c0);
#pragma unroll
            for (int t = 0; t < VEC; ++t) acc[t] = acc[t] + bb_value<BITS>(piece, t, sc, zp);
        }
        bb_store<VEC>(orow + c0, acc);
    }
}

// ---- half-precision wire ------------------------------------------------------------

// Wire row: d binary16 values (round to nearest even), zero halves up to a multiple
// of four.  Lane L converts VEC adjacent columns per pass.
template <int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void convert_fp16_kernel(
    const float *__restrict__ src, int64_t ld, int d, const int32_t *__restrict__ idx,
    int64_t row_offset, int64_t n_rows, uint16_t *__restrict__ wire)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave) * kBbRowsPerWave;
    const int dp = ((d + 3) >> 2) << 2;
#pragma unroll 1
    for (int r = 0; r < kBbRowsPerWave; ++r) {
        const int64_t i = first + r;
        if (i >= n_rows) break;
        const int64_t srow = idx ? static_cast<int64_t>(uniform(idx[i])) : row_offset + i;
        const float *row = src + srow * ld;
        uint16_t *out = wire + i * dp;
        for (int c0 = lane * VEC; c0 < dp; c0 += 64 * VEC) {
            if constexpr (VEC == 4) {
                float v[4];
                bb_load<4>(v, row + c0);                 // d % 4 == 0: never ragged
                const _Float16 h0 = static_cast<_Float16>(v[0]), h1 = static_cast<_Float16>(v[1]);
                const _Float16 h2 = static_cast<_Float16>(v[2]), h3 = static_cast<_Float16>(v[3]);
                uint2 o;
                o.x = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h0)) |
                      (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h1)) << 16);
                o.y = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h2)) |
                      (static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h3)) << 16);
                *reinterpret_cast<uint2 *>(out + c0) = o;
            } else {
                const _Float16 h = c0 < d ? static_cast<_Float16>(row[c0]) : static_cast<_Float16>(0.0f);
                out[c0] = c0 < d ? __builtin_bit_cast(uint16_t, h) : static_cast<uint16_t>(0);
            }
        }
    }
}

template <int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void recover_fp16_fwd_kernel(
    const uint16_t *__restrict__ wire, int64_t n_rows, int d, float *__restrict__ dst, int64_t ld,
    int64_t row_offset)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave) * kBbRowsPerWave;
    const int dp = ((d + 3) >> 2) << 2;
#pragma unroll 1
    for (int r = 0; r < kBbRowsPerWave; ++r) {
        const int64_t i = first + r;
        if (i >= n_rows) break;
        for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
            float v[VEC];
            fp16_load<VEC>(v, wire + i * dp + c0);
            bb_store<VEC>(dst + (row_offset + i) * ld + c0, v);
        }
    }
}

template <int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void recover_fp16_bwd_kernel(
    const uint16_t *__restrict__ wire, int d, float *__restrict__ dst, int64_t ld,
    const int64_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_rows,
    int64_t n_dst_rows, const int32_t *__restrict__ dst_ids)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave;
    if (k >= n_dst_rows) return;
    const int dp = ((d + 3) >> 2) << 2;
    const int64_t j0 = uniform(seg_ptr[k]), j1 = uniform(seg_ptr[k + 1]);
    if (j0 >= j1) return;
    float *orow = dst + static_cast<int64_t>(uniform(dst_ids[k])) * ld;
    for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
        float acc[VEC];
        stream_load<VEC>(acc, orow + c0);      // read-modify-write row: touched once
        for (int64_t j = j0; j < j1; ++j) {
            float v[VEC];
            fp16_load<VEC>(v, wire + static_cast<int64_t>(uniform(seg_rows[j])) * dp + c0);
#pragma unroll
            for (int t = 0; t < VEC; ++t) acc[t] = acc[t] + v[t];
        }
        bb_store<VEC>(orow + c0, acc);
    }
}

// ---- full-precision wire (the vanilla exchange the bit-width study compares with) ---------

// Wire row: the d floats of the source row unchanged, one zero float of padding when d is odd
// (rows are whole 64-bit words).  Sending is a row gather, receiving a row copy or, in the
// backward direction, the ordered accumulate of the other wires.
template <int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void copy_rows_out_kernel(
    const float *__restrict__ src, int64_t ld, int d, const int32_t *__restrict__ idx,
    int64_t row_offset, int64_t n_rows, float *__restrict__ wire)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave) * kBbRowsPerWave;
    const int dp = ((d + 1) >> 1) << 1;
#pragma unroll 1
    for (int r = 0; r < kBbRowsPerWave; ++r) {
        const int64_t i = first + r;
        if (i >= n_rows) break;
        const int64_t srow = idx ? static_cast<int64_t>(uniform(idx[i])) : row_offset + i;
        const float *row = src + srow * ld;
        float *out = wire + i * dp;
        for (int c0 = lane * VEC; c0 < dp; c0 += 64 * VEC) {
            if constexpr (VEC == 4) {
                float v[4];
                bb_load<4>(v, row + c0);                 // d % 4 == 0: never ragged
                bb_store<4>(out + c0, v);
            } else {
                out[c0] = c0 < d ? row[c0] : 0.0f;
            }
        }
    }
}

template <int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void copy_rows_in_kernel(
    const float *__restrict__ wire, int64_t n_rows, int d, float *__restrict__ dst, int64_t ld,
    int64_t row_offset)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t first = (static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave) * kBbRowsPerWave;
    const int dp = ((d + 1) >> 1) << 1;
#pragma unroll 1
    for (int r = 0; r < kBbRowsPerWave; ++r) {
        const int64_t i = first + r;
        if (i >= n_rows) break;
        for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
            float v[VEC];
            bb_load<VEC>(v, wire + i * dp + c0);
            bb_store<VEC>(dst + (row_offset + i) * ld + c0, v);
        }
    }
}

template <int VEC>
__global__ __launch_bounds__(kBbWavesPerBlock *kWave) void add_rows_bwd_kernel(
    const float *__restrict__ wire, int d, float *__restrict__ dst, int64_t ld,
    const int64_t *__restrict__ seg_ptr, const int32_t *__restrict__ seg_rows,
    int64_t n_dst_rows, const int32_t *__restrict__ dst_ids)
{
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t k = static_cast<int64_t>(blockIdx.x) * kBbWavesPerBlock + wave;
    if (k >= n_dst_rows) return;
    const int dp = ((d + 1) >> 1) << 1;
    const int64_t j0 = uniform(seg_ptr[k]), j1 = uniform(seg_ptr[k + 1]);
    if (j0 >= j1) return;
    float *orow = dst + static_cast<int64_t>(uniform(dst_ids[k])) * ld;
    for (int c0 = lane * VEC; c0 < d; c0 += 64 * VEC) {
        float acc[VEC];
        stream_load<VEC>(acc, orow + c0);      // read-modify-write row: touched once
        for (int64_t j = j0; j < j1; ++j) {
            float v[VEC];
            bb_load<VEC>(v, wire + static_cast<int64_t>(uniform(seg_rows[j])) * dp + c0);
#pragma unroll
            for (int t = 0; t < VEC; ++t) acc[t] = acc[t] + v[t];
        }
        bb_store<VEC>(orow + c0, acc);
    }
}

// ---- host side ----------------------------------------------------------------------

static bool bits_ok(int32_t bits)
{
    return bits == 1 || bits == 2 || bits == 4 || bits == 8 || bits == 16 || bits == 32;
}

template <int BITS, int VEC>
static void launch_quantize(const float *src, int64_t ld, int d, const int32_t *idx, int64_t row_offset,
                            int64_t n_rows, const CallKey &ckey, uint64_t *wire, hipStream_t st)
{
    const int P = (d + 64 * VEC - 1) / (64 * VEC);
    const int64_t per_block = kBbWavesPerBlock * kBbRowsPerWave;
    const dim3 grid(static_cast<unsigned>((n_rows + per_block - 1) / per_block));
    const dim3 block(kBbWavesPerBlock * kWave);
#define SYLVIE_BB_CASE(p)                                                                          \
    case p:                                                                                        \
        hipLaunchKernelGGL((quantize_bbit_kernel<BITS, VEC, p>), grid, block, 0, st, src, ld, d, idx, \
                           row_offset, n_rows, ckey, wire);                                        \
        return;
    switch (P) {
        SYLVIE_BB_CASE(1)
        SYLVIE_BB_CASE(2)
        SYLVIE_BB_CASE(3)
        SYLVIE_BB_CASE(4)
    default: break;
    }
#undef SYLVIE_BB_CASE
    const dim3 wgrid(static_cast<unsigned>((n_rows + kBbWavesPerBlock - 1) / kBbWavesPerBlock));
    hipLaunchKernelGGL((quantize_bbit_wide_kernel<BITS>), wgrid, block, 0, st, src, ld, d, idx,
                       row_offset, n_rows, ckey, wire);
}

template <int BITS>
static void launch_quantize_bits(const float *src, int64_t ld, int d, const int32_t *idx,
                                 int64_t row_offset, int64_t n_rows, const CallKey &ckey, uint64_t *wire,
                                 hipStream_t st)
{
    const bool v4 = d % 4 == 0 && ld % 4 == 0 && aligned(src, 16);
    if (v4) launch_quantize<BITS, 4>(src, ld, d, idx, row_offset, n_rows, ckey, wire, st);
    else launch_quantize<BITS, 1>(src, ld, d, idx, row_offset, n_rows, ckey, wire, st);
}

static int32_t quantize_bbit_common(const char *name, const float *src, int64_t ld, int32_t d,
                                    const int32_t *idx, int64_t row_offset, int64_t n_rows,
                                    int32_t bits, uint64_t seed, uint32_t stream_id, uint64_t *wire,
                                    void *stream, bool fwd)
{
    if (!bits_ok(bits)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bits must be 1, 2, 4, 8, 16 or 32 (got %d)", name, bits);
    if (bits == 1)
        return fwd ? sylvie_quantize_1bit_fwd(src, ld, d, idx, row_offset, n_rows, seed, stream_id, wire, 0, stream)
                   : sylvie_quantize_1bit_bwd(src, ld, d, idx, row_offset, n_rows, seed, stream_id, wire, 0, stream);
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_rows %lld out of range", name, (long long)n_rows);
    if (d < 1 || d > 65536) return fail(SYLVIE_ERR_INVALID_ARG, "%s: d %d out of range", name, d);
    if (ld < d) return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_src %lld < d %d", name, (long long)ld, d);
    if (!idx && row_offset < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative row_offset", name);
    if (n_rows == 0) return SYLVIE_OK;
    if (!src || !wire) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(src, 4) || (idx && !aligned(idx, 4)))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: float/int arrays need 4-byte alignment", name);
    if (!aligned(wire, 8))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: wire_out needs 8-byte alignment", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (bits == 16) {
        const int64_t per_block = kBbWavesPerBlock * kBbRowsPerWave;
        const dim3 grid(static_cast<unsigned>((n_rows + per_block - 1) / per_block));
        const dim3 block(kBbWavesPerBlock * kWave);
        uint16_t *w16 = reinterpret_cast<uint16_t *>(wire);
        if (d % 4 == 0 && ld % 4 == 0 && aligned(src, 16))
            hipLaunchKernelGGL(convert_fp16_kernel<4>, grid, block, 0, st, src, ld, d, idx, row_offset, n_rows, w16);
        else
            hipLaunchKernelGGL(convert_fp16_kernel<1>, grid, block, 0, st, src, ld, d, idx, row_offset, n_rows, w16);
    } else if (bits == 32) {
        const int64_t per_block = kBbWavesPerBlock * kBbRowsPerWave;
        const dim3 grid(static_cast<unsigned>((n_rows + per_block - 1) / per_block));
        const dim3 block(kBbWavesPerBlock * kWave);
        float *w32 = reinterpret_cast<float *>(wire);
        if (d % 4 == 0 && ld % 4 == 0 && aligned(src, 16) && aligned(wire, 16))
            hipLaunchKernelGGL(copy_rows_out_kernel<4>, grid, block, 0, st, src, ld, d, idx, row_offset, n_rows, w32);
        else
            hipLaunchKernelGGL(copy_rows_out_kernel<1>, grid, block, 0, st, src, ld, d, idx, row_offset, n_rows, w32);
    } else {
        const CallKey ckey = make_call_key(seed, stream_id);
        if (bits == 2) launch_quantize_bits<2>(src, ld, d, idx, row_offset, n_rows, ckey, wire, st);
        else if (bits == 4) launch_quantize_bits<4>(src, ld, d, idx, row_offset, n_rows, ckey, wire, st);
        else launch_quantize_bits<8>(src, ld, d, idx, row_offset, n_rows, ckey, wire, st);
    }
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

static int32_t check_bb_wire(const char *name, const uint64_t *wire, int64_t n_rows, int32_t d,
                             int32_t bits, const float *dst, int64_t ld)
{
    if (!bits_ok(bits)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bits must be 1, 2, 4, 8, 16 or 32 (got %d)", name, bits);
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

extern "C" size_t sylvie_wire_row_words_bits(int32_t d, int32_t bits)
{
    if (d < 1 || !sylvie::bits_ok(bits)) return 0;
    if (bits == 16) return (static_cast<size_t>(d) + 3) / 4;
    if (bits == 32) return (static_cast<size_t>(d) + 1) / 2;
    return (static_cast<size_t>(d) * bits + 63) / 64 + 1;
}

extern "C" int32_t sylvie_quantize_bbit_fwd(const float *src, int64_t ld_src, int32_t d,
                                            const int32_t *idx, int64_t row_offset, int64_t n_rows,
                                            int32_t bits, uint64_t seed, uint32_t stream_id,
                                            uint64_t *wire_out, void *stream)
{
    return sylvie::quantize_bbit_common("sylvie_quantize_bbit_fwd", src, ld_src, d, idx, row_offset,
                                        n_rows, bits, seed, stream_id, wire_out, stream, true);
}

extern "C" int32_t sylvie_quantize_bbit_bwd(const float *src, int64_t ld_src, int32_t d,
                                            const int32_t *idx, int64_t row_offset, int64_t n_rows,
                                            int32_t bits, uint64_t seed, uint32_t stream_id,
                                            uint64_t *wire_out, void *stream)
{
    return sylvie::quantize_bbit_common("sylvie_quantize_bbit_bwd", src, ld_src, d, idx, row_offset,
                                        n_rows, bits, seed, stream_id, wire_out, stream, false);
}

extern "C" int32_t sylvie_dequantize_bbit_fwd(const uint64_t *wire, int64_t n_rows, int32_t d,
                                              int32_t bits, float *dst, int64_t ld_dst,
                                              int64_t row_offset, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_dequantize_bbit_fwd";
    const int32_t rc = check_bb_wire(name, wire, n_rows, d, bits, dst, ld_dst);
    if (rc != SYLVIE_OK) return rc;
    if (bits == 1) return sylvie_dequantize_1bit_fwd(wire, 0, n_rows, d, dst, ld_dst, row_offset, stream);
    if (row_offset < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative row_offset", name);
    if (n_rows == 0) return SYLVIE_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t per_block = kBbWavesPerBlock * kBbRowsPerWave;
    const dim3 grid(static_cast<unsigned>((n_rows + per_block - 1) / per_block));
    const dim3 block(kBbWavesPerBlock * kWave);
    const bool v4 = d % 4 == 0 && ld_dst % 4 == 0 && aligned(dst + row_offset * ld_dst, 16);
#define SYLVIE_BB_DQ(B)                                                                              \
    if (v4) hipLaunchKernelGGL((dequantize_bbit_fwd_kernel<B, 4>), grid, block, 0, st, wire, n_rows, d, dst, ld_dst, row_offset); \
    else hipLaunchKernelGGL((dequantize_bbit_fwd_kernel<B, 1>), grid, block, 0, st, wire, n_rows, d, dst, ld_dst, row_offset)
    if (bits == 2) { SYLVIE_BB_DQ(2); }
    else if (bits == 4) { SYLVIE_BB_DQ(4); }
    else if (bits == 8) { SYLVIE_BB_DQ(8); }
    else if (bits == 32) {
        const float *w32 = reinterpret_cast<const float *>(wire);
        if (v4 && aligned(wire, 16)) hipLaunchKernelGGL(copy_rows_in_kernel<4>, grid, block, 0, st, w32, n_rows, d, dst, ld_dst, row_offset);
        else hipLaunchKernelGGL(copy_rows_in_kernel<1>, grid, block, 0, st, w32, n_rows, d, dst, ld_dst, row_offset);
    } else {
        const uint16_t *w16 = reinterpret_cast<const uint16_t *>(wire);
        if (v4) hipLaunchKernelGGL(recover_fp16_fwd_kernel<4>, grid, block, 0, st, w16, n_rows, d, dst, ld_dst, row_offset);
        else hipLaunchKernelGGL(recover_fp16_fwd_kernel<1>, grid, block, 0, st, w16, n_rows, d, dst, ld_dst, row_offset);
    }
#undef SYLVIE_BB_DQ
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_dequantize_bbit_bwd(const uint64_t *wire, int64_t n_rows, int32_t d,
                                              int32_t bits, float *dst, int64_t ld_dst,
                                              const int64_t *seg_ptr, const int32_t *seg_rows,
                                              int64_t n_dst_rows, const int32_t *dst_ids, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_dequantize_bbit_bwd";
    const int32_t rc = check_bb_wire(name, wire, n_rows, d, bits, dst, ld_dst);
    if (rc != SYLVIE_OK) return rc;
    if (bits == 1)
        return sylvie_dequantize_1bit_bwd(wire, 0, n_rows, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids, stream);
    if (n_dst_rows < 0 || n_dst_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_dst_rows out of range", name);
    if (n_rows == 0 || n_dst_rows == 0) return SYLVIE_OK;
    if (!seg_ptr || !seg_rows || !dst_ids) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(seg_ptr, 8) || !aligned(seg_rows, 4) || !aligned(dst_ids, 4))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned index array", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(static_cast<unsigned>((n_dst_rows + kBbWavesPerBlock - 1) / kBbWavesPerBlock));
    const dim3 block(kBbWavesPerBlock * kWave);
    const bool v4 = d % 4 == 0 && ld_dst % 4 == 0 && aligned(dst, 16);
#define SYLVIE_BB_DQB(B)                                                                             \
    if (v4) hipLaunchKernelGGL((dequantize_bbit_bwd_kernel<B, 4>), grid, block, 0, st, wire, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids); \
    else hipLaunchKernelGGL((dequantize_bbit_bwd_kernel<B, 1>), grid, block, 0, st, wire, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids)
    if (bits == 2) { SYLVIE_BB_DQB(2); }
    else if (bits == 4) { SYLVIE_BB_DQB(4); }
    else if (bits == 8) { SYLVIE_BB_DQB(8); }
    else if (bits == 32) {
        const float *w32 = reinterpret_cast<const float *>(wire);
        if (v4 && aligned(wire, 16)) hipLaunchKernelGGL(add_rows_bwd_kernel<4>, grid, block, 0, st, w32, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
        else hipLaunchKernelGGL(add_rows_bwd_kernel<1>, grid, block, 0, st, w32, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    } else {
        const uint16_t *w16 = reinterpret_cast<const uint16_t *>(wire);
        if (v4) hipLaunchKernelGGL(recover_fp16_bwd_kernel<4>, grid, block, 0, st, w16, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
        else hipLaunchKernelGGL(recover_fp16_bwd_kernel<1>, grid, block, 0, st, w16, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows, dst_ids);
    }
#undef SYLVIE_BB_DQB
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}
