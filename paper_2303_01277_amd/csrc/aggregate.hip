// CSR neighbour aggregation Y = diag(rs) * A * diag(cs) * X (Eq. 1; Alg. 1 the
// product A_n * H~; Alg. 2 its transpose on the transposed CSR).
//
// The work is a gather of whole feature rows: every entry of A pulls one row of
// X (d floats, contiguous) and adds it, weighted, into the output row.  It is
// bound by memory, not arithmetic, so the layout goal is: every load a full
// contiguous row segment, many rows in flight per wavefront, and no pass over
// the data that does not have to happen.
//
//   * One wavefront sums one output row (or one <= `chunk`-entry piece of a long
//     row).  G lanes cover one gathered row with VEC-wide loads and P passes
//     (G*VEC*P >= d); when G < 64 the wave gathers 64/G rows at once and folds
//     the lane groups together at the end.
//   * Column indices and weights are read 64 at a time, one per lane, and handed
//     to the gathering lanes through lane reads (scalar unit for G = 64), not
//     through LDS: the values are needed exactly once.
//   * U gathers are issued back to back before the first is consumed.
//   * Long rows (hubs of a power-law graph) are cut into tasks so no wavefront
//     runs away with the tail of the launch; the tasks share the launch with the
//     ordinary rows and go first.  Partial sums are written to a workspace and
//     added in task order by a second tiny kernel, so results do not depend on
//     scheduling.
//   * What happens to a finished row is a template choice: store it; or, for the
//     halo block of the backward pass, quantize it on the spot (the row goes
//     through LDS once to change from "lane = 4 adjacent columns" to "lane =
//     columns 64 apart", the layout in which a wave-wide compare is a packed word)
//     and write only the wire row; or, for the inner block, add the dequantized
//     wire rows that belong to it (Alg. 2 "integrate") before the one store.
#include <mutex>
#include <type_traits>

#include "common.hpp"
#include "bbit.hpp"
#include "rounding.hpp"
#include "validate.hpp"


namespace sylvie {

// Wavefronts per workgroup.  A workgroup keeps its slots until its last wavefront ends, and row
// lengths vary widely, so small workgroups keep more wavefronts in flight: one per workgroup for
// the wire-reading forward launch, whose rows walk the longest chain of dependent fetches
// (measured on the four large workloads: -8 to -14 %), two for the others (-1 %; one is slower
// for the backward halo launch).
constexpr int kAgWavesPerBlock = 2;
constexpr int kAgWavesPerBlockWire = 1;
template <int WB, int EPI>
constexpr int waves_per_block() { return (EPI == 0 && WB > 0) ? kAgWavesPerBlockWire : kAgWavesPerBlock; }

struct AggArgs {
    const int64_t *rowptr;
    const int32_t *col;
    const float *w;
    const float *row_scale;
    const float *col_scale;
    int64_t n_rows;
    const float *X;
    int64_t ld_x;
    int d;
    float *Y;
    int64_t ld_y;
    const float *addend;
    int64_t ld_addend;
    int64_t addend_rows;
    int chunk;          // 0: never split
    const int32_t *long_rows;
    const int64_t *long_ptr;
    int64_t n_long;
    float *workspace;
    // optional packed tail of X: columns >= n_dense are rows of a 1-bit wire
    int64_t n_dense;
    const uint32_t *wire32;     // wire rows (W bit words + 1 metadata word) seen as dwords
    int64_t ldw;                // 64-bit words from one wire row to the next (>= W + 1)
    // rows handled by this launch are row_begin .. row_begin + n_rows - 1 (absolute
    // indices into rowptr / Y / addend / row_scale)
    int64_t row_begin;
    // optional processing order: wavefront i of the launch takes row row_begin + row_order[i]
    // (a permutation of [0, n_rows)); results do not depend on it, the cache traffic does
    const int32_t *row_order;
    // epilogue "quantize": wire row (v - row_begin) <- quantized row v
    uint64_t *wire_out;
    int64_t ldw_out;            // row stride of wire_out in 64-bit words
    CallKey ck;
    // epilogue "integrate": row v += dequantized wire rows seg_rows[seg_ptr[v - row_begin] ..)
    const int64_t *seg_ptr;
    const int32_t *seg_rows;
};

enum : int { kEpiStore = 0, kEpiQuantize = 1, kEpiIntegrate = 2 };

// o[0..VEC) += the dequantized elements cc .. cc+VEC-1 of the wire rows of segment s,
// in order (single-precision adds, Alg. 2 "integrate feature gradients").  WB = bits per
// element of the wire (1, or 2 / 4 / 8: the recovered value is then fl(fl(scale q) + zero); 16: the
// rows are binary16 values).
template <int VEC, int WB>
__device__ __forceinline__ void integrate_vec(const AggArgs &a, int64_t s, int cc, float (&o)[VEC])
{
    const int64_t j0 = a.seg_ptr[s], j1 = a.seg_ptr[s + 1];
    for (int64_t j = j0; j < j1; ++j) {
        const uint32_t *pr = a.wire32 + static_cast<int64_t>(a.seg_rows[j]) * (2 * a.ldw);
        if constexpr (WB == 16) {       // half-precision rows carry no metadata
            float v[VEC];
            fp16_load<VEC>(v, reinterpret_cast<const uint16_t *>(pr) + cc);
#pragma unroll
            for (int t = 0; t < VEC; ++t) o[t] = o[t] + v[t];
        } else {
            const int W32 = ((a.d * WB + 63) >> 6) * 2;
            const uint2 meta = *reinterpret_cast<const uint2 *>(pr + W32);
            const float zp = __uint_as_float(meta.y);
            if constexpr (WB == 1) {
                const float hi = zp + __uint_as_float(meta.x);
                const uint32_t bits = pr[cc >> 5] >> (cc & 31);
#pragma unroll
                for (int t = 0; t < VEC; ++t) o[t] = o[t] + (((bits >> t) & 1u) ? hi : zp);
            } else {
                const float sc = __uint_as_float(meta.x);
                const uint32_t piece = bb_piece<WB, VEC>(reinterpret_cast<const uint64_t *>(pr), cc);
#pragma unroll
                for (int t = 0; t < VEC; ++t) o[t] = o[t] + bb_value<WB>(piece, t, sc, zp);
            }
        }
    }
}

// N scalar loads of LW dwords each (one wire row's mask words per load) and the wait for all of
// them, as ONE asm statement: the compiler never sees a destination register as defined before
// its data has arrived, so it cannot copy or spill it in between; early-clobber outputs keep a
// destination from sharing registers with an address that a later load still has to read.
typedef const __attribute__((address_space(4))) uint64_t *const_words;
template <int LW>
struct SVec { typedef uint32_t type __attribute__((ext_vector_type(LW))); };
template <int LW, int N>
__device__ __forceinline__ void scalar_rows(typename SVec<LW>::type (&m)[N], const const_words (&p)[N])
{
    static_assert((LW == 8 && (N == 8 || N == 1)) || (LW == 4 && (N == 12 || N == 1)) ||
                  (LW == 2 && (N == 16 || N == 1)), "block sizes the wire loops use");
    if constexpr (N == 1) {
        if constexpr (LW == 8)
            asm volatile("s_load_dwordx8 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=&s"(m[0]) : "s"(p[0]) : "memory");
        else if constexpr (LW == 4)
            asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=&s"(m[0]) : "s"(p[0]) : "memory");
        else
            asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=&s"(m[0]) : "s"(p[0]) : "memory");
    } else if constexpr (LW == 8) {
            asm volatile(
                "s_load_dwordx8 %0, %8, 0x0\n\t"
                "s_load_dwordx8 %1, %9, 0x0\n\t"
                "s_load_dwordx8 %2, %10, 0x0\n\t"
                "s_load_dwordx8 %3, %11, 0x0\n\t"
                "s_load_dwordx8 %4, %12, 0x0\n\t"
                "s_load_dwordx8 %5, %13, 0x0\n\t"
                "s_load_dwordx8 %6, %14, 0x0\n\t"
                "s_load_dwordx8 %7, %15, 0x0\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&s"(m[0]), "=&s"(m[1]), "=&s"(m[2]), "=&s"(m[3]), "=&s"(m[4]), "=&s"(m[5]), "=&s"(m[6]), "=&s"(m[7])
                : "s"(p[0]), "s"(p[1]), "s"(p[2]), "s"(p[3]), "s"(p[4]), "s"(p[5]), "s"(p[6]), "s"(p[7])
                : "memory");
    } else if constexpr (LW == 4) {
            asm volatile(
                "s_load_dwordx4 %0, %12, 0x0\n\t"
                "s_load_dwordx4 %1, %13, 0x0\n\t"
                "s_load_dwordx4 %2, %14, 0x0\n\t"
                "s_load_dwordx4 %3, %15, 0x0\n\t"
                "s_load_dwordx4 %4, %16, 0x0\n\t"
                "s_load_dwordx4 %5, %17, 0x0\n\t"
                "s_load_dwordx4 %6, %18, 0x0\n\t"
                "s_load_dwordx4 %7, %19, 0x0\n\t"
                "s_load_dwordx4 %8, %20, 0x0\n\t"
                "s_load_dwordx4 %9, %21, 0x0\n\t"
                "s_load_dwordx4 %10, %22, 0x0\n\t"
                "s_load_dwordx4 %11, %23, 0x0\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&s"(m[0]), "=&s"(m[1]), "=&s"(m[2]), "=&s"(m[3]), "=&s"(m[4]), "=&s"(m[5]), "=&s"(m[6]), "=&s"(m[7]), "=&s"(m[8]), "=&s"(m[9]), "=&s"(m[10]), "=&s"(m[11])
                : "s"(p[0]), "s"(p[1]), "s"(p[2]), "s"(p[3]), "s"(p[4]), "s"(p[5]), "s"(p[6]), "s"(p[7]), "s"(p[8]), "s"(p[9]), "s"(p[10]), "s"(p[11])
                : "memory");
    } else {
            asm volatile(
                "s_load_dwordx2 %0, %16, 0x0\n\t"
                "s_load_dwordx2 %1, %17, 0x0\n\t"
                "s_load_dwordx2 %2, %18, 0x0\n\t"
                "s_load_dwordx2 %3, %19, 0x0\n\t"
                "s_load_dwordx2 %4, %20, 0x0\n\t"
                "s_load_dwordx2 %5, %21, 0x0\n\t"
                "s_load_dwordx2 %6, %22, 0x0\n\t"
                "s_load_dwordx2 %7, %23, 0x0\n\t"
                "s_load_dwordx2 %8, %24, 0x0\n\t"
                "s_load_dwordx2 %9, %25, 0x0\n\t"
                "s_load_dwordx2 %10, %26, 0x0\n\t"
                "s_load_dwordx2 %11, %27, 0x0\n\t"
                "s_load_dwordx2 %12, %28, 0x0\n\t"
                "s_load_dwordx2 %13, %29, 0x0\n\t"
                "s_load_dwordx2 %14, %30, 0x0\n\t"
                "s_load_dwordx2 %15, %31, 0x0\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&s"(m[0]), "=&s"(m[1]), "=&s"(m[2]), "=&s"(m[3]), "=&s"(m[4]), "=&s"(m[5]), "=&s"(m[6]), "=&s"(m[7]), "=&s"(m[8]), "=&s"(m[9]), "=&s"(m[10]), "=&s"(m[11]), "=&s"(m[12]), "=&s"(m[13]), "=&s"(m[14]), "=&s"(m[15])
                : "s"(p[0]), "s"(p[1]), "s"(p[2]), "s"(p[3]), "s"(p[4]), "s"(p[5]), "s"(p[6]), "s"(p[7]), "s"(p[8]), "s"(p[9]), "s"(p[10]), "s"(p[11]), "s"(p[12]), "s"(p[13]), "s"(p[14]), "s"(p[15])
                : "memory");
    }
}

// acc[p][t] += sum over entries [e0, e1) of w_e * cs[col_e] * X[col_e][column(p, t)]
//
// WIRE: columns >= n_dense are not rows of X but rows of a packed 1-bit wire
// (Eq. 5 applied on the fly: the element is zero or fl(zero + scale) by its bit), so a
// halo row costs 8 W + 8 bytes instead of 4 d.  Inside a row all dense columns
// precede all wire columns (columns ascending), so each 64-entry batch splits
// at one point found with a ballot.
//
// WIRE with a full-width lane group (G == 64): the wire entries are summed in a second
// set of accumulators, accw[k] = column 64 k + lane, because in that layout word k of a
// wire row IS the lane mask of the select between its two levels: the words come in
// through scalar loads, one v_cndmask + one v_fma per word and entry.  The weight and
// the two levels of an entry reach all lanes through a broadcast read of a record that
// the lane owning the entry put into LDS (`bcast`, 64 records of 16 bytes per wave).
// The caller folds accw into acc afterwards (merge_wire_sums); `used_w` says whether
// there is anything to fold.
template <int VEC, int G, int P, int WIRE>
__device__ __forceinline__ void gather_sum(float (&acc)[P][VEC], int64_t e0, int64_t e1,
                                           const AggArgs &a, int lane,
                                           [[maybe_unused]] float (&accw)[P * VEC],
                                           [[maybe_unused]] float *bcast,
                                           [[maybe_unused]] bool &used_w)
{
    constexpr int EP = 64 / G;                 // rows gathered at once
    constexpr int U = (P >= 4) ? 2 : (8 / P);  // gathers in flight per lane group
    const int sub = EP == 1 ? 0 : lane / G;
    const int gl = lane % G;
    // column offsets of this lane; lanes past the row width re-read its last
    // vector (never stored) so that no load needs a predicate
    int coff[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int cc = (p * G + gl) * VEC;
        coff[p] = cc < a.d ? cc : a.d - VEC;
    }
    // code dwords per wire row (WIRE = bits per element); 2 metadata dwords follow
    const int W32 = ((a.d * (WIRE ? WIRE : 1) + 63) >> 6) * 2;
    for (int64_t base = e0; base < e1; base += 64) {
        const int cnt = static_cast<int>(e1 - base < 64 ? e1 - base : 64);
        int my_c = 0;
        float my_w = 0.0f;
        if (lane < cnt) {
            // index and weight streams are read once per launch: past the caches' retention,
            // which is better spent on the gathered rows
            // (ordinary loads: neighbouring rows share the lines of the index and weight streams;
            // the streaming hint was measured here and costs 3 - 12 % on three of four workloads)
            my_c = a.col[base + lane];
            my_w = a.w ? a.w[base + lane] : 1.0f;
            if (a.col_scale) my_w *= a.col_scale[my_c];
        }
        // address of the lane's own gathered row, computed once on the vector unit; an entry's
        // row is then addressed by two lane reads instead of a 64-bit scalar multiply-add
        const uintptr_t my_xrow = reinterpret_cast<uintptr_t>(a.X + static_cast<int64_t>(my_c) * a.ld_x);
        [[maybe_unused]] const int my_xlo = static_cast<int>(static_cast<uint32_t>(my_xrow));
        [[maybe_unused]] const int my_xhi = static_cast<int>(static_cast<uint32_t>(my_xrow >> 32));
        [[maybe_unused]] auto xrow_of_slot = [&](int slot) -> const float * {
            const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(my_xlo, slot));
            const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(my_xhi, slot));
            return reinterpret_cast<const float *>((static_cast<uint64_t>(hi) << 32) | lo);
        };
        int nd = cnt;                          // entries [0, nd) are dense, [nd, cnt) wire
        if constexpr (WIRE)
            nd = __builtin_popcountll(__ballot(lane < cnt && my_c < a.n_dense));
        // wire entries: each lane fetches the metadata word of ITS entry now, so that the
        // fetch is in flight while the dense rows are gathered
        [[maybe_unused]] uint2 meta = make_uint2(0u, 0u);
        // address of the lane's own wire row, computed once on the vector unit: the per-entry
        // loop then needs two lane reads and no scalar arithmetic to address a row
        [[maybe_unused]] uint32_t my_row_lo = 0, my_row_hi = 0;
        if constexpr (WIRE) {
            if (nd < cnt) {
                const bool mine = lane >= nd && lane < cnt;
                const int64_t my_wr = mine ? static_cast<int64_t>(my_c) - a.n_dense : 0;
                const uint32_t *my_row = a.wire32 + my_wr * (2 * a.ldw);
                if constexpr (WIRE != 16) meta = *reinterpret_cast<const uint2 *>(my_row + W32);
                my_row_lo = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(my_row));
                my_row_hi = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(my_row) >> 32);
            }
        }
        int j = 0;
        // full groups: U * EP valid entries, all gathers issued before any is used
        for (; j + EP * U <= nd; j += EP * U) {
            float x[U][P][VEC];
            float wv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int sl = j + u * EP + sub;
                const float *xr;
                if constexpr (EP == 1) {
                    xr = xrow_of_slot(sl);
                    wv[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), sl));
                } else {
                    xr = a.X + static_cast<int64_t>(__shfl(my_c, sl)) * a.ld_x;
                    wv[u] = __shfl(my_w, sl);
                }
#pragma unroll
                for (int p = 0; p < P; ++p) load_vec_at<VEC>(x[u][p], xr, static_cast<uint32_t>(coff[p]) * 4u);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int p = 0; p < P; ++p)
#pragma unroll
                    for (int t = 0; t < VEC; ++t) acc[p][t] = fmaf(wv[u], x[u][p][t], acc[p][t]);
        }
        // remainder: one gather per lane group; groups past the end add w = 0 times
        // row 0 (lanes >= cnt hold column 0, weight 0)
        for (; j < nd; j += EP) {
            const int sl = j + sub;
            const float *xr;
            float wj;
            if constexpr (EP == 1) {
                xr = xrow_of_slot(sl);
                wj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), sl));
            } else {
                int c = __shfl(my_c, sl & 63);
                wj = __shfl(my_w, sl & 63);
                if (sl >= nd) { wj = 0.0f; c = 0; }
                xr = a.X + static_cast<int64_t>(c) * a.ld_x;
            }
            float x[P][VEC];
#pragma unroll
            for (int p = 0; p < P; ++p) load_vec_at<VEC>(x[p], xr, static_cast<uint32_t>(coff[p]) * 4u);
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int t = 0; t < VEC; ++t) acc[p][t] = fmaf(wj, x[p][t], acc[p][t]);
        }
        if constexpr (WIRE) {
            if (nd < cnt) {
                // Wire entries.  Each lane has fetched the two levels of ITS entry (zero and
                // fl(zero + scale), Eq. 5) and publishes them with its weight as a 16-byte
                // record; then, entry by entry, the record is broadcast, the row's mask words
                // arrive by scalar loads and one select + one FMA per word does the rest.
                const bool mine = lane >= nd && lane < cnt;
                const float my_zp = __uint_as_float(meta.y);
                const float my_hi = my_zp + __uint_as_float(meta.x);
                const float my_ww = mine ? my_w : 0.0f;
                static_assert(!WIRE || EP == 1, "rows that read a wire take a whole wavefront");
                if constexpr (WIRE == 1) {
                    constexpr int NW = P * VEC;                     // >= words per wire row
                    const int W = W32 >> 1;
                    wave_lds_sync();    // the previous batch's records have been read
                    reinterpret_cast<float4 *>(bcast)[lane] = make_float4(my_ww, my_zp, my_hi, 0.0f);
                    wave_lds_sync();    // every lane reads every record below
                    used_w = true;
                    auto row_of_slot = [&](int slot) -> const_words {
                        const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(my_row_lo), slot));
                        const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(my_row_hi), slot));
                        return (const_words)((static_cast<uint64_t>(hi) << 32) | lo);
                    };
                    if constexpr (NW == 4) {
                        // Rows of up to 256 columns: 1 to 4 mask words.  One scalar load brings an
                        // entry's words (2, 4 or 8 dwords: a row of 3 words is loaded with its
                        // metadata word, which feeds an accumulator nobody reads), and the narrower
                        // the row, the more entries are in flight before the one wait: the row's
                        // dependent fetches, not bandwidth, bound these launches.
                        auto entries = [&](auto lw_c, auto n_c, int j0) {
                            constexpr int LW = decltype(lw_c)::value;   // dwords per load
                            constexpr int N = decltype(n_c)::value;
                            constexpr int WU = LW / 2;                  // words used per entry
                            typename SVec<LW>::type m[N];
                            const_words prow[N];
                            float4 rec[N];
                            const float4 *recs = reinterpret_cast<const float4 *>(bcast) + j0;
#pragma unroll
                            for (int u = 0; u < N; ++u) {
                                prow[u] = row_of_slot(j0 + u);
                                rec[u] = recs[u];
                            }
                            scalar_rows<LW, N>(m, prow);
#pragma unroll
                            for (int u = 0; u < N; ++u)
#pragma unroll
                                for (int k = 0; k < WU; ++k) {
                                    const uint64_t mk = (static_cast<uint64_t>(m[u][2 * k + 1]) << 32) | m[u][2 * k];
                                    float x;
                                    asm("v_cndmask_b32_e64 %0, %1, %2, %3"
                                        : "=v"(x)
                                        : "v"(rec[u].y), "v"(rec[u].z), "s"(mk));
                                    accw[k] = fmaf(rec[u].x, x, accw[k]);
                                }
                        };
                        auto all_entries = [&](auto lw_c, auto n_c) {
                            constexpr int N = decltype(n_c)::value;
                            int jj = nd;
                            for (; jj + N <= cnt; jj += N) entries(lw_c, n_c, jj);
                            for (; jj < cnt; ++jj) entries(lw_c, std::integral_constant<int, 1>{}, jj);
                        };
                        if (W == 1) all_entries(std::integral_constant<int, 2>{}, std::integral_constant<int, 16>{});
                        else if (W == 2) all_entries(std::integral_constant<int, 4>{}, std::integral_constant<int, 12>{});
                        else all_entries(std::integral_constant<int, 8>{}, std::integral_constant<int, 8>{});
                    } else {
                        // wider rows: word by word.  FULLW: the row has exactly NW words, so the
                        // loads have constant offsets and merge into wide ones; otherwise the
                        // words past the row's last one re-read the metadata word and feed
                        // accumulators nobody reads.
                        constexpr int UW = NW <= 8 ? 2 : 1;
                        auto entries = [&](auto n_c, auto full_c, int j0) {
                            constexpr int N = decltype(n_c)::value;
                            constexpr bool FULLW = decltype(full_c)::value;
                            float4 rec[N];
                            const float4 *recs = reinterpret_cast<const float4 *>(bcast) + j0;
                            uint64_t m[N][NW];
#pragma unroll
                            for (int u = 0; u < N; ++u) {
                                const_words prow = row_of_slot(j0 + u);
#pragma unroll
                                for (int k = 0; k < NW; ++k) m[u][k] = prow[FULLW ? k : (k < W ? k : W)];
                                rec[u] = recs[u];
                            }
#pragma unroll
                            for (int u = 0; u < N; ++u)
#pragma unroll
                                for (int k = 0; k < NW; ++k) {
                                    float x;
                                    asm("v_cndmask_b32_e64 %0, %1, %2, %3"
                                        : "=v"(x)
                                        : "v"(rec[u].y), "v"(rec[u].z), "s"(m[u][k]));
                                    accw[k] = fmaf(rec[u].x, x, accw[k]);
                                }
                        };
                        auto all_entries = [&](auto full_c) {
                            int jj = nd;
                            for (; jj + UW <= cnt; jj += UW) entries(std::integral_constant<int, UW>{}, full_c, jj);
                            for (; jj < cnt; ++jj) entries(std::integral_constant<int, 1>{}, full_c, jj);
                        };
                        if (W == NW) all_entries(std::true_type{});
                        else all_entries(std::false_type{});
                    }
                } else if constexpr (WIRE == 16) {
                    // half-precision wire: a lane's four adjacent columns are eight bytes at the
                    // matching place of the wire row; UB rows in flight, four conversions and the
                    // weight's FMAs per entry.
                    static_assert(VEC == 4, "half-precision wire rows are gathered four columns per lane");
                    typedef const __attribute__((address_space(1))) char *global_bytes;
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    typedef const __attribute__((address_space(1))) u32x2 *global_u2;
                    constexpr int UB = (P >= 4) ? 2 : (8 / P);
                    const int my_wwi = __float_as_int(my_ww);
                    auto hentries = [&](auto n_c, int j0) {
                        constexpr int N = decltype(n_c)::value;
                        u32x2 pc[N][P];
                        float ww[N];
#pragma unroll
                        for (int u = 0; u < N; ++u) {
                            const int sl = j0 + u;
                            const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(my_row_lo), sl));
                            const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(my_row_hi), sl));
                            global_bytes row = (global_bytes)((static_cast<uint64_t>(hi) << 32) | lo);
                            ww[u] = __int_as_float(__builtin_amdgcn_readlane(my_wwi, sl));
#pragma unroll
                            for (int p = 0; p < P; ++p) pc[u][p] = *(global_u2)(row + static_cast<uint32_t>(coff[p]) * 2u);
                        }
#pragma unroll
                        for (int u = 0; u < N; ++u)
#pragma unroll
                            for (int p = 0; p < P; ++p) {
                                const float x0 = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(pc[u][p].x & 0xffffu)));
                                const float x1 = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(pc[u][p].x >> 16)));
                                const float x2 = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(pc[u][p].y & 0xffffu)));
                                const float x3 = static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(pc[u][p].y >> 16)));
                                acc[p][0] = fmaf(ww[u], x0, acc[p][0]);
                                acc[p][1] = fmaf(ww[u], x1, acc[p][1]);
                                acc[p][2] = fmaf(ww[u], x2, acc[p][2]);
                                acc[p][3] = fmaf(ww[u], x3, acc[p][3]);
                            }
                    };
                    int jj = nd;
                    for (; jj + UB <= cnt; jj += UB) hentries(std::integral_constant<int, UB>{}, jj);
                    for (; jj < cnt; ++jj) hentries(std::integral_constant<int, 1>{}, jj);
                } else {
                    // b-bit wire (2, 4, 8 bits): a lane's VEC adjacent columns are one piece of
                    // VEC * WIRE bits at the matching place of the wire row, so wire entries use
                    // the dense rows' accumulators and loop shape: UB rows in flight, then per
                    // element one field extract, one convert, fl(fl(scale q) + zero) (Eq. 5) and
                    // the weight's FMA.  Scale, zero and weight of an entry come from the lane
                    // that owns it by lane reads.
                    static_assert(VEC == 4, "b-bit wire rows are gathered four columns per lane");
                    typedef const __attribute__((address_space(1))) char *global_bytes;
                    constexpr int UB = (P >= 4) ? 2 : (8 / P);
                    constexpr uint32_t kMask = (1u << WIRE) - 1u;
                    const int my_sc = static_cast<int>(meta.x), my_zpi = static_cast<int>(meta.y);
                    const int my_wwi = __float_as_int(my_ww);
                    auto piece_at = [&](global_bytes row, int p) -> uint32_t {
                        const uint32_t off = static_cast<uint32_t>(coff[p]) * WIRE / 8u;
                        if constexpr (WIRE == 8)
                            return *reinterpret_cast<const __attribute__((address_space(1))) uint32_t *>(row + off);
                        else if constexpr (WIRE == 4)
                            return *reinterpret_cast<const __attribute__((address_space(1))) uint16_t *>(row + off);
                        else
                            return *reinterpret_cast<const __attribute__((address_space(1))) uint8_t *>(row + off);
                    };
                    auto bentries = [&](auto n_c, int j0) {
                        constexpr int N = decltype(n_c)::value;
                        uint32_t pc[N][P];
                        float ww[N], sc[N], zp[N];
#pragma unroll
                        for (int u = 0; u < N; ++u) {
                            const int sl = j0 + u;
                            const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(my_row_lo), sl));
                            const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(my_row_hi), sl));
                            global_bytes row = (global_bytes)((static_cast<uint64_t>(hi) << 32) | lo);
                            ww[u] = __int_as_float(__builtin_amdgcn_readlane(my_wwi, sl));
                            sc[u] = __int_as_float(__builtin_amdgcn_readlane(my_sc, sl));
                            zp[u] = __int_as_float(__builtin_amdgcn_readlane(my_zpi, sl));
#pragma unroll
                            for (int p = 0; p < P; ++p) pc[u][p] = piece_at(row, p);
                        }
#pragma unroll
                        for (int u = 0; u < N; ++u)
#pragma unroll
                            for (int p = 0; p < P; ++p)
#pragma unroll
                                for (int t = 0; t < VEC; ++t) {
                                    const float q = static_cast<float>((pc[u][p] >> (WIRE * t)) & kMask);
                                    const float step = sc[u] * q;
                                    const float x = step + zp[u];
                                    acc[p][t] = fmaf(ww[u], x, acc[p][t]);
                                }
                    };
                    int jj = nd;
                    for (; jj + UB <= cnt; jj += UB) bentries(std::integral_constant<int, UB>{}, jj);
                    for (; jj < cnt; ++jj) bentries(std::integral_constant<int, 1>{}, jj);
                }
            }
        }
    }
    // fold the lane groups: afterwards every group holds the full sums
    if constexpr (EP > 1) {
#pragma unroll
        for (int s = G; s < 64; s <<= 1)
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int t = 0; t < VEC; ++t) acc[p][t] += __shfl_xor(acc[p][t], s);
    }
}

// acc += accw, the latter moved from "lane = column 64 k + lane" to the lane's own VEC
// adjacent columns through a wave-private LDS row of 64 P VEC floats.
template <int VEC, int P>
__device__ __forceinline__ void merge_wire_sums(float (&acc)[P][VEC], const float (&accw)[P * VEC],
                                                float *row, int d, int lane)
{
    wave_lds_sync();    // `row` shares its memory with the broadcast records read above
#pragma unroll
    for (int k = 0; k < P * VEC; ++k) row[64 * k + lane] = accw[k];
    wave_lds_sync();    // a lane now reads columns that other lanes wrote
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int cc = (p * 64 + lane) * VEC;
        if (cc < d) {
#pragma unroll
            for (int t = 0; t < VEC; ++t) acc[p][t] += row[cc + t];
        }
    }
}

// One launch covers everything that gathers.  The first workgroups
// take the pieces of the long rows (they start first, so the heaviest rows never
// trail the launch); every later wavefront takes one ordinary row and skips the
// long ones.  Pieces write partial sums to workspace[task][0..d).
template <int VEC, int G, int P, int WB, int EPI>
__global__ __launch_bounds__((waves_per_block<WB, EPI>() * kWave)) void aggregate_gather_kernel(AggArgs a,
                                                                                              int64_t n_tasks)
{
    constexpr int kWPB = waves_per_block<WB, EPI>();
    [[maybe_unused]] const uint32_t ckey = EPI == kEpiQuantize ? call_key_of(a.ck) : 0u;
    // WB = bits per element of the wire this launch reads (EPI store: the halo columns;
    // EPI integrate: the received gradients) or writes (EPI quantize); 0 = no wire
    constexpr int WIRE = EPI == kEpiStore ? WB : 0;            // wire read by the gather itself
    // quantize epilogue: the finished row as floats, for b > 1 followed by the packed image
    constexpr int kRowStage = VEC * G * P;
    constexpr int kStage = EPI == kEpiQuantize ? kRowStage + (WB > 1 && WB < 16 ? kRowStage / 4 + 4 : 0) : 4;
    __shared__ __align__(16) float stage[kWPB][kStage];
    // wire entries of full-width rows: broadcast records, then the fold of their sums
    constexpr bool kWireAcc = WIRE == 1 && G == 64;
    constexpr int kWStage = kWireAcc ? (64 * P * VEC > 256 ? 64 * P * VEC : 256) : 4;
    __shared__ __align__(16) float wstage[kWPB][kWStage];
    float accw[P * VEC];
#pragma unroll
    for (int k = 0; k < P * VEC; ++k) accw[k] = 0.0f;
    bool used_w = false;
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t task_blocks = (n_tasks + kWPB - 1) / kWPB;
    float acc[P][VEC];
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
        for (int t = 0; t < VEC; ++t) acc[p][t] = 0.0f;

    if (static_cast<int64_t>(blockIdx.x) < task_blocks) {
        const int64_t t = static_cast<int64_t>(blockIdx.x) * kWPB + wave;
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
        gather_sum<VEC, G, P, WIRE>(acc, e0, e1, a, lane, accw, wstage[wave], used_w);
        if constexpr (kWireAcc) {
            if (used_w) merge_wire_sums<VEC, P>(acc, accw, wstage[wave], a.d, lane);
        }
        if (lane >= G) return;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int cc = (p * G + lane) * VEC;
            if (cc < a.d) store_vec<VEC>(a.workspace + t * a.d + cc, acc[p]);
        }
        return;
    }

    const int64_t pos = (static_cast<int64_t>(blockIdx.x) - task_blocks) * kWPB + wave;
    if (pos >= a.n_rows) return;
    const int64_t local = a.row_order ? static_cast<int64_t>(uniform(a.row_order[pos])) : pos;
    const int64_t v = a.row_begin + local;
    const int64_t e0 = uniform(a.rowptr[v]);
    const int64_t e1 = uniform(a.rowptr[v + 1]);
    if (a.chunk > 0 && e1 - e0 > a.chunk) return;
    gather_sum<VEC, G, P, WIRE>(acc, e0, e1, a, lane, accw, wstage[wave], used_w);
    if constexpr (kWireAcc) {
        if (used_w) merge_wire_sums<VEC, P>(acc, accw, wstage[wave], a.d, lane);
    }
    const float rs = a.row_scale ? a.row_scale[v] : 1.0f;
    const bool add = a.addend && v < a.addend_rows;
    if (lane < G) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int cc = (p * G + lane) * VEC;
            if (cc < a.d) {
                float o[VEC];
#pragma unroll
                for (int t = 0; t < VEC; ++t) o[t] = rs * acc[p][t];
                if (add) {
                    float ad[VEC];
                    load_vec<VEC>(ad, a.addend + v * a.ld_addend + cc);
#pragma unroll
                    for (int t = 0; t < VEC; ++t) o[t] += ad[t];
                }
                if constexpr (EPI == kEpiIntegrate) integrate_vec<VEC, WB>(a, local, cc, o);
                if constexpr (EPI == kEpiQuantize) {
#pragma unroll
                    for (int t = 0; t < VEC; ++t) stage[wave][cc + t] = o[t];
                } else {
                    stream_store<VEC>(a.Y + v * a.ld_y + cc, o);    // written once, read by a later launch
                }
            }
        }
    }
    if constexpr (EPI == kEpiQuantize) {
        if constexpr (WB == 1)
            quantize_row_lds(stage[wave], a.d, ckey, static_cast<uint32_t>(local),
                             a.wire_out + local * a.ldw_out, lane);
        else if constexpr (WB == 16)
            convert_row_lds_fp16(stage[wave], a.d, a.wire_out + local * a.ldw_out, lane);
        else
            quantize_row_lds_bbit<WB>(stage[wave], a.d, ckey, static_cast<uint32_t>(local),
                                      a.wire_out + local * a.ldw_out,
                                      reinterpret_cast<uint32_t *>(stage[wave] + kRowStage), lane);
    }
}

// One wavefront per long row: add its partial sums in task order, scale, finish.
template <int VEC, int WB, int EPI>
__global__ __launch_bounds__(kAgWavesPerBlock *kWave) void aggregate_reduce_kernel(AggArgs a)
{
    // EPI quantize: per wave d floats (rounded up to 4) and, for b > 1, d / 4 + 4 image dwords
    extern __shared__ __align__(16) float rstage[];
    [[maybe_unused]] const uint32_t ckey = EPI == kEpiQuantize ? call_key_of(a.ck) : 0u;
    const int lane = lane_id();
    const int wave = uniform(static_cast<int>(threadIdx.x) >> 6);
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kAgWavesPerBlock + wave;
    if (i >= a.n_long) return;
    const int64_t v = a.long_rows[i];
    const int64_t local = v - a.row_begin;
    const int64_t t0 = a.long_ptr[i], t1 = a.long_ptr[i + 1];
    const float rs = a.row_scale ? a.row_scale[v] : 1.0f;
    const bool add = a.addend && v < a.addend_rows;
    const int d4 = (a.d + 3) & ~3;
    const int per_wave = d4 + (WB > 1 && WB < 16 ? d4 / 4 + 4 : 0);
    float *srow = rstage + wave * per_wave;
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
#pragma unroll
        for (int q = 0; q < VEC; ++q) acc[q] *= rs;
        if (add) {
            float ad[VEC];
            load_vec<VEC>(ad, a.addend + v * a.ld_addend + cc);
#pragma unroll
            for (int q = 0; q < VEC; ++q) acc[q] += ad[q];
        }
        if constexpr (EPI == kEpiIntegrate) integrate_vec<VEC, WB>(a, local, cc, acc);
        if constexpr (EPI == kEpiQuantize) {
#pragma unroll
            for (int q = 0; q < VEC; ++q) srow[cc + q] = acc[q];
        } else {
            stream_store<VEC>(a.Y + v * a.ld_y + cc, acc);
        }
    }
    if constexpr (EPI == kEpiQuantize) {
        if constexpr (WB == 1)
            quantize_row_lds(srow, a.d, ckey, static_cast<uint32_t>(local),
                             a.wire_out + local * a.ldw_out, lane);
        else if constexpr (WB == 16)
            convert_row_lds_fp16(srow, a.d, a.wire_out + local * a.ldw_out, lane);
        else
            quantize_row_lds_bbit<WB>(srow, a.d, ckey, static_cast<uint32_t>(local),
                                      a.wire_out + local * a.ldw_out,
                                      reinterpret_cast<uint32_t *>(srow + d4), lane);
    }
}

template <int VEC, int G, int P, int WB, int EPI>
static void launch_kernels(const AggArgs &a, int64_t nt, hipStream_t st)
{
    constexpr int kWPB = waves_per_block<WB, EPI>();
    const int64_t blocks = (nt + kWPB - 1) / kWPB + (a.n_rows + kWPB - 1) / kWPB;
    hipLaunchKernelGGL((aggregate_gather_kernel<VEC, G, P, WB, EPI>),
                       dim3(static_cast<unsigned>(blocks)), dim3(kWPB * kWave), 0, st, a, nt);
    if (a.n_long > 0) {
        const dim3 block(kAgWavesPerBlock * kWave);
        const dim3 rg(static_cast<unsigned>((a.n_long + kAgWavesPerBlock - 1) / kAgWavesPerBlock));
        const int d4 = (a.d + 3) & ~3;
        const size_t lds = EPI == kEpiQuantize
                               ? sizeof(float) * kAgWavesPerBlock * (d4 + (WB > 1 && WB < 16 ? d4 / 4 + 4 : 0)) : 0;
        hipLaunchKernelGGL((aggregate_reduce_kernel<VEC, WB, EPI>), rg, block, lds, st, a);
    }
}

template <int VEC, int G, int P>
static void launch_shape(const AggArgs &a, int64_t n_tasks, int epi, int bits, hipStream_t st)
{
    const int64_t nt = a.n_long > 0 ? n_tasks : 0;
    // wires wider than one bit are read and written four columns per lane (the caller has
    // checked the alignment); launch_vec gives every wire-reading launch a whole wavefront per row
    if constexpr (VEC == 4) {
        if (bits > 1) {
#define SYLVIE_AG_BITS(B)                                                                      \
    if (epi == kEpiQuantize) launch_kernels<VEC, G, P, B, kEpiQuantize>(a, nt, st);             \
    else if (epi == kEpiIntegrate) launch_kernels<VEC, G, P, B, kEpiIntegrate>(a, nt, st);      \
    else if constexpr (G == 64) launch_kernels<VEC, G, P, B, kEpiStore>(a, nt, st);
            if (bits == 2) { SYLVIE_AG_BITS(2) }
            else if (bits == 4) { SYLVIE_AG_BITS(4) }
            else if (bits == 8) { SYLVIE_AG_BITS(8) }
            else { SYLVIE_AG_BITS(16) }
#undef SYLVIE_AG_BITS
            return;
        }
    }
    if (epi == kEpiQuantize) launch_kernels<VEC, G, P, 1, kEpiQuantize>(a, nt, st);
    else if (epi == kEpiIntegrate) launch_kernels<VEC, G, P, 1, kEpiIntegrate>(a, nt, st);
    else if (a.wire32) {
        if constexpr (G == 64) launch_kernels<VEC, G, P, 1, kEpiStore>(a, nt, st);
    } else launch_kernels<VEC, G, P, 0, kEpiStore>(a, nt, st);
}

template <int VEC>
static bool launch_vec(const AggArgs &a, int64_t n_tasks, int epi, int bits, hipStream_t st)
{
    const int lanes = (a.d + VEC - 1) / VEC;   // lanes needed for one row, one pass
    // Rows that read a wire take a whole wavefront even when they are narrow: wire entries
    // then go through the scalar path (mask words by scalar loads, one select + FMA per word),
    // which costs half the vector instructions of the shared-wavefront path per entry.
    if (epi == kEpiStore && a.wire32 && lanes <= 64) launch_shape<VEC, 64, 1>(a, n_tasks, epi, bits, st);
    else if (lanes <= 16) launch_shape<VEC, 16, 1>(a, n_tasks, epi, bits, st);
    else if (lanes <= 32) launch_shape<VEC, 32, 1>(a, n_tasks, epi, bits, st);
    else if (lanes <= 64) launch_shape<VEC, 64, 1>(a, n_tasks, epi, bits, st);
    else if (lanes <= 128) launch_shape<VEC, 64, 2>(a, n_tasks, epi, bits, st);
    else if (lanes <= 192) launch_shape<VEC, 64, 3>(a, n_tasks, epi, bits, st);
    else if (lanes <= 256) launch_shape<VEC, 64, 4>(a, n_tasks, epi, bits, st);
    else if (lanes <= 320) launch_shape<VEC, 64, 5>(a, n_tasks, epi, bits, st);
    else if (lanes <= 384) launch_shape<VEC, 64, 6>(a, n_tasks, epi, bits, st);
    else if (lanes <= 512) launch_shape<VEC, 64, 8>(a, n_tasks, epi, bits, st);
    else return false;
    return true;
}

// Everything an aggregation call may carry beyond the plain operands.
struct AggExtra {
    int64_t n_dense = 0;            // forward: columns >= n_dense are wire rows
    const uint64_t *wire = nullptr; // forward: wire to read; integrate: wire to add
    int64_t n_wire = 0;
    int64_t ld_wire = 0;            // row stride of wire / wire_out in words, 0 = W + 1
    int64_t row_begin = 0;
    int epi = kEpiStore;
    uint64_t *wire_out = nullptr;   // quantize epilogue
    CallKey ck = {0u, 0u, 0ull, nullptr};
    const int64_t *seg_ptr = nullptr;
    const int32_t *seg_rows = nullptr;
    const int32_t *row_order = nullptr;
    int bits = 1;                   // bits per element of the wire read / written / added
};

static int32_t aggregate_common(const char *name, const int64_t *rowptr, const int32_t *col,
                                const float *w, const float *row_scale, const float *col_scale,
                                int64_t n_rows, const float *X, int64_t ld_x, int32_t d, float *Y,
                                int64_t ld_y, const float *addend, int64_t ld_addend,
                                int64_t addend_rows, int32_t chunk, const int32_t *long_rows,
                                const int64_t *long_ptr, int64_t n_long, int64_t n_tasks,
                                float *workspace, size_t workspace_bytes, void *stream,
                                const AggExtra &x = AggExtra())
{
    const int64_t n_dense = x.n_dense, n_wire = x.n_wire;
    const uint64_t *wire = x.wire;
    if (n_rows < 0 || n_rows >= (int64_t(1) << 31))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: n_rows %lld out of range", name, (long long)n_rows);
    if (d < 1 || d > 65536) return fail(SYLVIE_ERR_INVALID_ARG, "%s: d %d out of range", name, d);
    if (ld_x < d || ld_y < d) return fail(SYLVIE_ERR_INVALID_ARG, "%s: leading dimension < d", name);
    if (addend && (ld_addend < d || addend_rows < 0))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad addend shape", name);
    if (n_long < 0 || n_tasks < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative count", name);
    if (n_wire < 0 || n_dense < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative count", name);
    if (n_wire > 0 && !wire) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null wire", name);
    if (n_wire > 0 && !aligned(wire, 8))
        return fail(SYLVIE_ERR_BAD_ALIGNMENT, "%s: misaligned wire", name);
    if (x.bits != 1 && x.bits != 2 && x.bits != 4 && x.bits != 8 && x.bits != 16)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bits must be 1, 2, 4, 8 or 16 (got %d)", name, x.bits);
    // half-precision rows (16) have no metadata word
    const int64_t row_words = x.bits == 16 ? (static_cast<int64_t>(d) + 3) / 4
                                           : (static_cast<int64_t>(d) * x.bits + 63) / 64 + 1;
    if (x.ld_wire != 0 && x.ld_wire < row_words)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: ld_wire %lld shorter than a wire row", name, (long long)x.ld_wire);
    if (n_rows == 0) return SYLVIE_OK;
    if (x.row_begin < 0) return fail(SYLVIE_ERR_INVALID_ARG, "%s: negative row_begin", name);
    if (x.epi == kEpiQuantize && (!x.wire_out || !aligned(x.wire_out, 8)))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: wire_out null or misaligned", name);
    if (x.epi == kEpiIntegrate && (!x.seg_ptr || (n_wire > 0 && !x.seg_rows)))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: segment table has null pointers", name);
    if (x.epi == kEpiQuantize && d > 2048)
        return fail(SYLVIE_ERR_UNIMPLEMENTED, "%s: fused quantize supports d <= 2048", name);
    if (!rowptr || !col || !X || (!Y && x.epi != kEpiQuantize))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(rowptr, 8) || !aligned(col, 4) || !aligned(X, 4) || !aligned(Y, 4) ||
        (w && !aligned(w, 4)))
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
    AggArgs a;
    a.rowptr = rowptr; a.col = col; a.w = w; a.row_scale = row_scale; a.col_scale = col_scale;
    a.n_rows = n_rows; a.X = X; a.ld_x = ld_x; a.d = d; a.Y = Y; a.ld_y = ld_y;
    a.addend = addend; a.ld_addend = ld_addend; a.addend_rows = addend_rows;
    a.chunk = n_long > 0 ? chunk : 0;
    a.long_rows = long_rows; a.long_ptr = long_ptr; a.n_long = n_long; a.workspace = workspace;
    a.n_dense = n_dense;
    a.wire32 = n_wire > 0 ? reinterpret_cast<const uint32_t *>(wire) : nullptr;
    a.ldw = a.ldw_out = x.ld_wire ? x.ld_wire : row_words;
    a.row_begin = x.row_begin;
    a.wire_out = x.wire_out;
    a.ck = x.ck;
    a.seg_ptr = x.seg_ptr;
    a.seg_rows = x.seg_rows;
    a.row_order = x.row_order;

    hipStream_t st = static_cast<hipStream_t>(stream);
    if (validate_enabled()) {
        // the number of rows of X is not an argument: columns are checked against it only
        // where the call states it (dense + wire rows of the wire-reading forward)
        Validator v(name, st);
        const bool reads_wire = x.epi == kEpiStore && n_wire > 0;
        v.csr(rowptr, col, x.row_begin, n_rows, reads_wire ? n_dense + n_wire : -1,
              reads_wire ? n_dense : -1);
        if (x.epi == kEpiIntegrate) v.segments(x.seg_ptr, x.seg_rows, n_rows, n_wire, nullptr);
        const int32_t rc = v.finish();
        if (rc != SYLVIE_OK) return rc;
    }
    if (x.epi == kEpiQuantize) { Y = const_cast<float *>(X); ld_y = ld_x; }   // Y is unused
    const bool a16 = aligned(X, 16) && aligned(Y, 16) && ld_x % 4 == 0 && ld_y % 4 == 0 &&
                     d % 4 == 0 && (!addend || (aligned(addend, 16) && ld_addend % 4 == 0));
    const bool a8 = aligned(X, 8) && aligned(Y, 8) && ld_x % 2 == 0 && ld_y % 2 == 0 &&
                    d % 2 == 0 && (!addend || (aligned(addend, 8) && ld_addend % 2 == 0));
    const bool uses_wire = x.epi != kEpiStore || n_wire > 0;
    const int bits = uses_wire ? x.bits : 1;
    if (bits > 1 && !a16)
        return fail(SYLVIE_ERR_UNIMPLEMENTED,
                    "%s: wires of %d bits need d %% 4 == 0 and 16-byte aligned rows "
                    "(dequantize / quantize as separate calls otherwise)", name, bits);
    bool ok;
    if (a16) ok = launch_vec<4>(a, n_tasks, x.epi, bits, st);
    else if (a8) ok = launch_vec<2>(a, n_tasks, x.epi, bits, st);
    else ok = launch_vec<1>(a, n_tasks, x.epi, bits, st);
    if (!ok)
        return fail(SYLVIE_ERR_UNIMPLEMENTED,
                    "%s: d = %d is wider than one launch covers at this alignment "
                    "(2048 / 1024 / 512 columns for 16 / 8 / 4-byte aligned rows); "
                    "split the columns across calls", name, d);
    SYLVIE_HIP_LAUNCH_CHECK(name);
    return SYLVIE_OK;
}

// Scratch of the entry point that may not allocate: the partial sums of the long rows'
// tasks live in this array instead of a caller workspace.  Every GPU the library runs on
// holds its own copy at its own address for the life of the process; the name below is only
// the host-side handle of the symbol, the address kernels can use is looked up per device.
static __device__ __align__(256) unsigned char scratch[SYLVIE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static float *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
static int32_t static_scratch(const char *name, float **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(SYLVIE_ERR_HIP, "%s: hipGetDevice: %s", name, hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(SYLVIE_ERR_UNIMPLEMENTED, "%s: device ordinal %d not supported", name, dev);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(SYLVIE_ERR_HIP, "%s: hipGetSymbolAddress: %s", name, hipGetErrorString(e));
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_scratch_ptr[dev];
    return SYLVIE_OK;
}

}  // namespace sylvie

extern "C" int32_t sylvie_aggregate_csr_fwd_noalloc(const int64_t *rowptr, const int32_t *col,
                                                    const float *w, const float *row_scale,
                                                    const float *col_scale, int64_t n_rows,
                                                    const float *X, int64_t ld_x, int32_t d, float *Y,
                                                    int64_t ld_y, const float *addend,
                                                    int64_t ld_addend, int64_t addend_rows,
                                                    const int32_t *row_order, int32_t chunk, const int32_t *long_rows,
                                                    const int64_t *long_ptr, int64_t n_long,
                                                    int64_t n_tasks, void *stream)
{
    const char *name = "sylvie_aggregate_csr_fwd_noalloc";
    float *ws = nullptr;
    if (n_long > 0) {
        // the size is checked before anything else so that the error names the limit
        if (n_tasks < 0 || d < 1 ||
            static_cast<uint64_t>(n_tasks) > SYLVIE_STATIC_SCRATCH_BYTES / (4ull * static_cast<uint64_t>(d)))
            return sylvie::fail(SYLVIE_ERR_WORKSPACE,
                                "%s: n_tasks * d * 4 = %lld * %d * 4 bytes exceeds the built-in scratch of %llu bytes; "
                                "use sylvie_aggregate_csr_fwd with a workspace of your own",
                                name, (long long)n_tasks, d, (unsigned long long)SYLVIE_STATIC_SCRATCH_BYTES);
        const int32_t rc = sylvie::static_scratch(name, &ws);
        if (rc != SYLVIE_OK) return rc;
    }
    sylvie::AggExtra x;
    x.row_order = row_order;
    return sylvie::aggregate_common(name, rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, Y,
                                    ld_y, addend, ld_addend, addend_rows, chunk, long_rows, long_ptr,
                                    n_long, n_tasks, ws, n_long > 0 ? SYLVIE_STATIC_SCRATCH_BYTES : 0,
                                    stream, x);
}

extern "C" int32_t sylvie_aggregate_csr_fwd(const int64_t *rowptr, const int32_t *col,
                                            const float *w, const float *row_scale,
                                            const float *col_scale, int64_t n_rows,
                                            const float *X, int64_t ld_x, int32_t d, float *Y,
                                            int64_t ld_y, const float *addend, int64_t ld_addend,
                                            int64_t addend_rows, const int32_t *row_order, int32_t chunk,
                                            const int32_t *long_rows, const int64_t *long_ptr,
                                            int64_t n_long, int64_t n_tasks, float *workspace,
                                            size_t workspace_bytes, void *stream)
{
    sylvie::AggExtra x;
    x.row_order = row_order;
    return sylvie::aggregate_common("sylvie_aggregate_csr_fwd", rowptr, col, w, row_scale,
                                    col_scale, n_rows, X, ld_x, d, Y, ld_y, addend, ld_addend,
                                    addend_rows, chunk, long_rows, long_ptr, n_long, n_tasks,
                                    workspace, workspace_bytes, stream, x);
}

extern "C" int32_t sylvie_aggregate_csr_bwd(const int64_t *rowptrT, const int32_t *colT,
                                            const float *wT, const float *row_scale,
                                            const float *col_scale, int64_t n_rowsT,
                                            const float *dY, int64_t ld_dy, int32_t d, float *dX,
                                            int64_t ld_dx, const float *addend, int64_t ld_addend,
                                            int64_t addend_rows, const int32_t *row_order, int32_t chunk,
                                            const int32_t *long_rows, const int64_t *long_ptr,
                                            int64_t n_long, int64_t n_tasks, float *workspace,
                                            size_t workspace_bytes, void *stream)
{
    sylvie::AggExtra x;
    x.row_order = row_order;
    return sylvie::aggregate_common("sylvie_aggregate_csr_bwd", rowptrT, colT, wT, row_scale,
                                    col_scale, n_rowsT, dY, ld_dy, d, dX, ld_dx, addend, ld_addend,
                                    addend_rows, chunk, long_rows, long_ptr, n_long, n_tasks,
                                    workspace, workspace_bytes, stream, x);
}

namespace sylvie {

static int32_t fwd_wire_call(const char *name, int32_t bits, const int64_t *rowptr, const int32_t *col,
                             const float *w, const float *row_scale, const float *col_scale,
                             int64_t n_rows, const float *X, int64_t ld_x, int32_t d, int64_t n_dense,
                             const uint64_t *wire, int64_t ld_wire, int64_t n_wire, float *Y, int64_t ld_y,
                             const int32_t *row_order, int32_t chunk, const int32_t *long_rows,
                             const int64_t *long_ptr, int64_t n_long, int64_t n_tasks, float *workspace,
                             size_t workspace_bytes, void *stream)
{
    AggExtra x;
    x.n_dense = n_dense;
    x.wire = wire;
    x.ld_wire = ld_wire;
    x.n_wire = n_wire;
    x.row_order = row_order;
    x.bits = bits;
    return aggregate_common(name, rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, Y, ld_y,
                            nullptr, 0, 0, chunk, long_rows, long_ptr, n_long, n_tasks, workspace,
                            workspace_bytes, stream, x);
}

static int32_t bwd_quantize_call(const char *name, int32_t bits, const int64_t *rowptrT,
                                 const int32_t *colT, const float *wT, const float *row_scale,
                                 const float *col_scale, int64_t row_begin, int64_t n_rows,
                                 const float *dY, int64_t ld_dy, int32_t d, uint64_t seed,
                                 uint32_t stream_id, uint64_t *wire_out, int64_t ld_wire,
                                 const int32_t *row_order, int32_t chunk, const int32_t *long_rows,
                                 const int64_t *long_ptr, int64_t n_long, int64_t n_tasks,
                                 float *workspace, size_t workspace_bytes, void *stream)
{
    AggExtra x;
    x.row_begin = row_begin;
    x.epi = kEpiQuantize;
    x.wire_out = wire_out;
    x.ld_wire = ld_wire;
    x.ck = make_call_key(seed, stream_id);
    x.row_order = row_order;
    x.bits = bits;
    return aggregate_common(name, rowptrT, colT, wT, row_scale, col_scale, n_rows, dY, ld_dy, d, nullptr,
                            ld_dy, nullptr, 0, 0, chunk, long_rows, long_ptr, n_long, n_tasks, workspace,
                            workspace_bytes, stream, x);
}

static int32_t bwd_integrate_call(const char *name, int32_t bits, const int64_t *rowptrT,
                                  const int32_t *colT, const float *wT, const float *row_scale,
                                  const float *col_scale, int64_t row_begin, int64_t n_rows,
                                  const float *dY, int64_t ld_dy, int32_t d, float *dX, int64_t ld_dx,
                                  const float *addend, int64_t ld_addend, int64_t addend_rows,
                                  const uint64_t *wire, int64_t ld_wire, int64_t n_wire,
                                  const int64_t *seg_ptr, const int32_t *seg_rows, const int32_t *row_order,
                                  int32_t chunk, const int32_t *long_rows, const int64_t *long_ptr,
                                  int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes,
                                  void *stream)
{
    AggExtra x;
    x.row_begin = row_begin;
    x.epi = kEpiIntegrate;
    x.wire = wire;
    x.ld_wire = ld_wire;
    x.n_wire = n_wire;
    x.seg_ptr = seg_ptr;
    x.seg_rows = seg_rows;
    x.row_order = row_order;
    x.bits = bits;
    return aggregate_common(name, rowptrT, colT, wT, row_scale, col_scale, n_rows, dY, ld_dy, d, dX, ld_dx,
                            addend, ld_addend, addend_rows, chunk, long_rows, long_ptr, n_long, n_tasks,
                            workspace, workspace_bytes, stream, x);
}

}  // namespace sylvie

extern "C" int32_t sylvie_aggregate_csr_fwd_wire(
    const int64_t *rowptr, const int32_t *col, const float *w, const float *row_scale,
    const float *col_scale, int64_t n_rows, const float *X, int64_t ld_x, int32_t d,
    int64_t n_dense, const uint64_t *wire, int64_t ld_wire, int64_t n_wire, float *Y, int64_t ld_y,
    const int32_t *row_order, int32_t chunk, const int32_t *long_rows, const int64_t *long_ptr,
    int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes, void *stream)
{
    return sylvie::fwd_wire_call("sylvie_aggregate_csr_fwd_wire", 1, rowptr, col, w, row_scale, col_scale,
                                 n_rows, X, ld_x, d, n_dense, wire, ld_wire, n_wire, Y, ld_y, row_order,
                                 chunk, long_rows, long_ptr, n_long, n_tasks, workspace, workspace_bytes,
                                 stream);
}

extern "C" int32_t sylvie_aggregate_csr_fwd_wire_bbit(
    const int64_t *rowptr, const int32_t *col, const float *w, const float *row_scale,
    const float *col_scale, int64_t n_rows, const float *X, int64_t ld_x, int32_t d, int32_t bits,
    int64_t n_dense, const uint64_t *wire, int64_t ld_wire, int64_t n_wire, float *Y, int64_t ld_y,
    const int32_t *row_order, int32_t chunk, const int32_t *long_rows, const int64_t *long_ptr,
    int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes, void *stream)
{
    return sylvie::fwd_wire_call("sylvie_aggregate_csr_fwd_wire_bbit", bits, rowptr, col, w, row_scale,
                                 col_scale, n_rows, X, ld_x, d, n_dense, wire, ld_wire, n_wire, Y, ld_y,
                                 row_order, chunk, long_rows, long_ptr, n_long, n_tasks, workspace,
                                 workspace_bytes, stream);
}

extern "C" int32_t sylvie_aggregate_csr_bwd_quantize(
    const int64_t *rowptrT, const int32_t *colT, const float *wT, const float *row_scale,
    const float *col_scale, int64_t row_begin, int64_t n_rows, const float *dY, int64_t ld_dy,
    int32_t d, uint64_t seed, uint32_t stream_id, uint64_t *wire_out, int64_t ld_wire,
    const int32_t *row_order, int32_t chunk, const int32_t *long_rows, const int64_t *long_ptr,
    int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes, void *stream)
{
    return sylvie::bwd_quantize_call("sylvie_aggregate_csr_bwd_quantize", 1, rowptrT, colT, wT, row_scale,
                                     col_scale, row_begin, n_rows, dY, ld_dy, d, seed, stream_id, wire_out,
                                     ld_wire, row_order, chunk, long_rows, long_ptr, n_long, n_tasks,
                                     workspace, workspace_bytes, stream);
}

extern "C" int32_t sylvie_aggregate_csr_bwd_quantize_bbit(
    const int64_t *rowptrT, const int32_t *colT, const float *wT, const float *row_scale,
    const float *col_scale, int64_t row_begin, int64_t n_rows, const float *dY, int64_t ld_dy,
    int32_t d, int32_t bits, uint64_t seed, uint32_t stream_id, uint64_t *wire_out, int64_t ld_wire,
    const int32_t *row_order, int32_t chunk, const int32_t *long_rows, const int64_t *long_ptr,
    int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes, void *stream)
{
    return sylvie::bwd_quantize_call("sylvie_aggregate_csr_bwd_quantize_bbit", bits, rowptrT, colT, wT,
                                     row_scale, col_scale, row_begin, n_rows, dY, ld_dy, d, seed, stream_id,
                                     wire_out, ld_wire, row_order, chunk, long_rows, long_ptr, n_long,
                                     n_tasks, workspace, workspace_bytes, stream);
}

extern "C" int32_t sylvie_aggregate_csr_bwd_integrate(
    const int64_t *rowptrT, const int32_t *colT, const float *wT, const float *row_scale,
    const float *col_scale, int64_t row_begin, int64_t n_rows, const float *dY, int64_t ld_dy,
    int32_t d, float *dX, int64_t ld_dx, const float *addend, int64_t ld_addend,
    int64_t addend_rows, const uint64_t *wire, int64_t ld_wire, int64_t n_wire, const int64_t *seg_ptr,
    const int32_t *seg_rows, const int32_t *row_order, int32_t chunk, const int32_t *long_rows,
    const int64_t *long_ptr, int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes,
    void *stream)
{
    return sylvie::bwd_integrate_call("sylvie_aggregate_csr_bwd_integrate", 1, rowptrT, colT, wT, row_scale,
                                      col_scale, row_begin, n_rows, dY, ld_dy, d, dX, ld_dx, addend,
                                      ld_addend, addend_rows, wire, ld_wire, n_wire, seg_ptr, seg_rows,
                                      row_order, chunk, long_rows, long_ptr, n_long, n_tasks, workspace,
                                      workspace_bytes, stream);
}

extern "C" int32_t sylvie_aggregate_csr_bwd_integrate_bbit(
    const int64_t *rowptrT, const int32_t *colT, const float *wT, const float *row_scale,
    const float *col_scale, int64_t row_begin, int64_t n_rows, const float *dY, int64_t ld_dy,
    int32_t d, int32_t bits, float *dX, int64_t ld_dx, const float *addend, int64_t ld_addend,
    int64_t addend_rows, const uint64_t *wire, int64_t ld_wire, int64_t n_wire, const int64_t *seg_ptr,
    const int32_t *seg_rows, const int32_t *row_order, int32_t chunk, const int32_t *long_rows,
    const int64_t *long_ptr, int64_t n_long, int64_t n_tasks, float *workspace, size_t workspace_bytes,
    void *stream)
{
    return sylvie::bwd_integrate_call("sylvie_aggregate_csr_bwd_integrate_bbit", bits, rowptrT, colT, wT,
                                      row_scale, col_scale, row_begin, n_rows, dY, ld_dy, d, dX, ld_dx,
                                      addend, ld_addend, addend_rows, wire, ld_wire, n_wire, seg_ptr,
                                      seg_rows, row_order, chunk, long_rows, long_ptr, n_long, n_tasks,
                                      workspace, workspace_bytes, stream);
}
