// Graph Engine set-up on the device (Sec. 3.2; Alg. 1, the lines before the epoch loop):
// HALO node set and local numbering, receive / send sets, the transposed operator and the
// scatter segments of the backward accumulate.  Integer work only; every result is unique, so
// nothing here depends on the order in which waves run.
//
// Building blocks: an exclusive prefix sum (tile sums, recursive scan of the sums, tile
// rescan) and a stable least-significant-digit radix sort of (key, value) pairs with 8-bit
// digits.  One wave owns a tile of 2048 consecutive items, so the stable order inside a
// digit is (tile, round, lane): a wave counts its digits, the counts are scanned digit-major
// over all tiles, and in the scatter pass a lane's slot is the tile's offset for its digit
// plus the number of earlier items of the tile with that digit (running count in LDS plus the
// rank among the lanes of the round that hold the same digit, found with eight ballots).
#include "common.hpp"

namespace sylvie {
namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kSortTile = 2048;                    // items per wave
constexpr int kSortRounds = kSortTile / kWave;
constexpr int kScanItems = 8;                      // per thread
constexpr int kScanTile = kBlock * kScanItems;

// ---- exclusive prefix sum -------------------------------------------------------------

template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v)
{
    const int lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const T o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan of one value per thread over the block; *total receives the block sum.
template <typename T>
__device__ __forceinline__ T block_exclusive_scan(T v, T *lds /*[kWavesPerBlock]*/, T *total)
{
    const int wave = static_cast<int>(threadIdx.x) / kWave;
    const T inc = wave_inclusive_scan(v);
    if (lane_id() == kWave - 1) lds[wave] = inc;
    __syncthreads();
    T before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        const T s = lds[w];
        if (w < wave) before += s;
        all += s;
    }
    __syncthreads();
    *total = all;
    return before + inc - v;
}

template <typename T>
__global__ __launch_bounds__(kBlock) void scan_tile_sums_kernel(const T *in, int64_t n, T *sums)
{
    __shared__ T lds[kWavesPerBlock];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kScanTile + static_cast<int64_t>(threadIdx.x) * kScanItems;
    T s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k)
        if (base + k < n) s += in[base + k];
    T total;
    block_exclusive_scan(s, lds, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// out[i] = offset of the tile + sum of in[tile start .. i).  offsets == nullptr: single tile.
template <typename T>
__global__ __launch_bounds__(kBlock) void scan_tiles_kernel(const T *in, T *out, int64_t n, const T *offsets)
{
    __shared__ T lds[kWavesPerBlock];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kScanTile + static_cast<int64_t>(threadIdx.x) * kScanItems;
    T v[kScanItems];
    T s = 0;
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        v[k] = base + k < n ? in[base + k] : T(0);
        s += v[k];
    }
    T total;
    T run = block_exclusive_scan(s, lds, &total) + (offsets ? offsets[blockIdx.x] : T(0));
#pragma unroll
    for (int k = 0; k < kScanItems; ++k) {
        if (base + k < n) out[base + k] = run;
        run += v[k];
    }
}

inline int64_t scan_tiles_of(int64_t n) { return (n + kScanTile - 1) / kScanTile; }
inline size_t align256(size_t b) { return (b + 255) & ~size_t(255); }

// Elements of scratch (type T) an exclusive scan of n elements needs.
inline int64_t scan_scratch_elems(int64_t n)
{
    int64_t total = 0;
    while (n > kScanTile) {
        n = scan_tiles_of(n);
        total += n + 32;           // keeps every level 256-byte aligned for 8-byte T
        total &= ~int64_t(31);
    }
    return total;
}

template <typename T>
void exclusive_scan(const T *in, T *out, int64_t n, T *scratch, hipStream_t st)
{
    if (n <= 0) return;
    const int64_t tiles = scan_tiles_of(n);
    if (tiles == 1) {
        hipLaunchKernelGGL(scan_tiles_kernel<T>, dim3(1), dim3(kBlock), 0, st, in, out, n, static_cast<const T *>(nullptr));
        return;
    }
    T *sums = scratch;
    T *next = scratch + ((tiles + 32) & ~int64_t(31));
    hipLaunchKernelGGL(scan_tile_sums_kernel<T>, dim3(static_cast<unsigned>(tiles)), dim3(kBlock), 0, st, in, n, sums);
    exclusive_scan<T>(sums, sums, tiles, next, st);
    hipLaunchKernelGGL(scan_tiles_kernel<T>, dim3(static_cast<unsigned>(tiles)), dim3(kBlock), 0, st, in, out, n,
                       static_cast<const T *>(sums));
}

// ---- stable radix sort of pairs ---------------------------------------------------------

__global__ __launch_bounds__(kBlock) void radix_count_kernel(const uint32_t *keys, int64_t n, int shift,
                                                            uint32_t *hist, int64_t tiles)
{
    __shared__ uint32_t cnt[kWavesPerBlock][256];
    const int wave = static_cast<int>(threadIdx.x) / kWave, lane = lane_id();
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + wave;
    for (int d = lane; d < 256; d += kWave) cnt[wave][d] = 0;
    __syncthreads();
    if (tile < tiles) {
        const int64_t base = tile * kSortTile;
        for (int r = 0; r < kSortRounds; ++r) {
            const int64_t i = base + r * kWave + lane;
            if (i < n) atomicAdd(&cnt[wave][(keys[i] >> shift) & 255u], 1u);
        }
    }
    __syncthreads();
    if (tile < tiles)
        for (int d = lane; d < 256; d += kWave) hist[static_cast<int64_t>(d) * tiles + tile] = cnt[wave][d];
}

// Scatter pass.  A wavefront first sorts its tile by the digit inside LDS (positions from the tile's
// own digit counts, which are the differences of consecutive scanned offsets), then writes the
// tile out in that order: the items of one digit are adjacent lanes writing adjacent addresses,
// runs of eight items on average instead of 64 separate 4-byte writes per instruction.
constexpr int kScatterWaves = 2;        // 2 x (16 KB of staged pairs + 3 KB of tables) of LDS per workgroup

__global__ __launch_bounds__(kScatterWaves *kWave) void radix_scatter_kernel(
    const uint32_t *keys_in, const uint32_t *vals_in, uint32_t *keys_out, uint32_t *vals_out, int64_t n, int shift,
    const uint32_t *offs, int64_t tiles)
{
    __shared__ uint32_t goff[kScatterWaves][256];      // where the tile's items of a digit go
    __shared__ uint32_t lstart[kScatterWaves][256];    // where they start inside the sorted tile
    __shared__ uint32_t lrun[kScatterWaves][256];      // next free place inside the sorted tile
    __shared__ uint32_t skey[kScatterWaves][kSortTile];
    __shared__ uint32_t sval[kScatterWaves][kSortTile];
    const int wave = static_cast<int>(threadIdx.x) / kWave, lane = lane_id();
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kScatterWaves + wave;
    if (tile >= tiles) return;
    const int64_t base = tile * kSortTile;
    const int count = static_cast<int>(n - base < kSortTile ? n - base : kSortTile);
    // lane l owns digits 4 l .. 4 l + 3: global offsets, counts, local starts
    {
        uint32_t c[4], total = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int d = 4 * lane + q;
            const int64_t at = static_cast<int64_t>(d) * tiles + tile;        // digit-major scan order
            const uint32_t here = offs[at];
            const uint32_t next = at + 1 < 256 * tiles ? offs[at + 1] : static_cast<uint32_t>(n);
            goff[wave][d] = here;
            c[q] = next - here;
            total += c[q];
        }
        uint32_t start = wave_inclusive_scan(total) - total;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            lstart[wave][4 * lane + q] = start;
            lrun[wave][4 * lane + q] = start;
            start += c[q];
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const uint64_t below = (uint64_t(1) << lane) - 1;
    for (int r = 0; r < kSortRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        const bool valid = i < n;
        const uint32_t key = valid ? keys_in[i] : 0u;
        const uint32_t val = valid ? vals_in[i] : 0u;
        const uint32_t digit = (key >> shift) & 255u;
        uint64_t same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const bool bit = (digit >> b) & 1u;
            const uint64_t m = __ballot(valid && bit);
            same &= bit ? m : ~m;
        }
        if (valid) {
            const uint32_t first = lrun[wave][digit];
            const uint32_t rank = static_cast<uint32_t>(__popcll(same & below));
            __builtin_amdgcn_wave_barrier();
            if (rank == 0) lrun[wave][digit] = first + static_cast<uint32_t>(__popcll(same));
            const uint32_t pos = first + rank;
            if (pos < static_cast<uint32_t>(kSortTile)) {       // always true for a histogram of these keys
                skey[wave][pos] = key;
                sval[wave][pos] = val;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    for (int j = lane; j < count; j += kWave) {
        const uint32_t key = skey[wave][j];
        const uint32_t digit = (key >> shift) & 255u;
        const uint32_t pos = goff[wave][digit] + (static_cast<uint32_t>(j) - lstart[wave][digit]);
        if (pos < n) {                         // always true for a histogram of these keys
            keys_out[pos] = key;
            vals_out[pos] = sval[wave][j];
        }
    }
}

inline int64_t sort_tiles_of(int64_t n) { return (n + kSortTile - 1) / kSortTile; }

struct SortBuffers {
    uint32_t *keys[2];
    uint32_t *vals[2];
    uint32_t *hist;
    uint32_t *scan_scratch;
};

// Sorts keys[0] / vals[0] (n items, keys < 2^key_bits) by key, stable; returns the index (0 or 1)
// of the buffer pair that holds the result.
int radix_sort_pairs(const SortBuffers &b, int64_t n, int key_bits, hipStream_t st)
{
    int cur = 0;
    if (n <= 0) return cur;
    const int64_t tiles = sort_tiles_of(n);
    const unsigned blocks = static_cast<unsigned>((tiles + kWavesPerBlock - 1) / kWavesPerBlock);
    for (int shift = 0; shift < key_bits; shift += 8) {
        hipLaunchKernelGGL(radix_count_kernel, dim3(blocks), dim3(kBlock), 0, st, b.keys[cur], n, shift, b.hist, tiles);
        exclusive_scan<uint32_t>(b.hist, b.hist, 256 * tiles, b.scan_scratch, st);
        const unsigned sblocks = static_cast<unsigned>((tiles + kScatterWaves - 1) / kScatterWaves);
        hipLaunchKernelGGL(radix_scatter_kernel, dim3(sblocks), dim3(kScatterWaves * kWave), 0, st, b.keys[cur],
                           b.vals[cur], b.keys[cur ^ 1], b.vals[cur ^ 1], n, shift, b.hist, tiles);
        cur ^= 1;
    }
    return cur;
}

inline int bits_for(int64_t n_keys)
{
    int bits = 1;
    while ((int64_t(1) << bits) < n_keys) ++bits;
    return bits;
}

// ---- workspace ------------------------------------------------------------------------------

struct Arena {
    char *base;
    size_t used, cap;
    template <typename T>
    T *take(int64_t elems)
    {
        T *p = reinterpret_cast<T *>(base + used);
        used += align256(sizeof(T) * static_cast<size_t>(elems > 0 ? elems : 1));
        return p;
    }
};

size_t sort_bytes(int64_t n)
{
    const int64_t tiles = sort_tiles_of(n > 0 ? n : 1);
    return 4 * align256(4 * static_cast<size_t>(n > 0 ? n : 1)) + align256(4 * 256 * static_cast<size_t>(tiles)) +
           align256(4 * static_cast<size_t>(scan_scratch_elems(256 * tiles) + 64));
}

SortBuffers take_sort(Arena &a, int64_t n)
{
    SortBuffers b;
    const int64_t tiles = sort_tiles_of(n > 0 ? n : 1);
    b.keys[0] = a.take<uint32_t>(n);
    b.keys[1] = a.take<uint32_t>(n);
    b.vals[0] = a.take<uint32_t>(n);
    b.vals[1] = a.take<uint32_t>(n);
    b.hist = a.take<uint32_t>(256 * tiles);
    b.scan_scratch = a.take<uint32_t>(scan_scratch_elems(256 * tiles) + 64);
    return b;
}

// ---- kernels of the set-up steps ----------------------------------------------------------------

__global__ void clear_status_kernel(int32_t *status) { status[0] = 0; }

// ptr[c] = number of sorted keys below c, for c = 0 .. n_keys (a CSR row pointer).
__global__ __launch_bounds__(kBlock) void boundaries_kernel(const uint32_t *keys, int64_t n, int64_t n_keys, int64_t *ptr)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i > n) return;
    const int64_t prev = i == 0 ? -1 : static_cast<int64_t>(keys[i - 1]);
    int64_t cur = i == n ? n_keys : static_cast<int64_t>(keys[i]);
    if (cur > n_keys) cur = n_keys;
    for (int64_t c = prev + 1; c <= cur; ++c) ptr[c] = i;
}

// Keys from an int32 array with a range check (out of range: status, key 0); values = index.
__global__ __launch_bounds__(kBlock) void keys_from_i32_kernel(const int32_t *src, int64_t n, int64_t n_keys,
                                                              uint32_t *keys, uint32_t *vals, int32_t *status)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n) return;
    int64_t k = src[i];
    if (k < 0 || k >= n_keys) {
        status[0] = 1;
        k = 0;
    }
    keys[i] = static_cast<uint32_t>(k);
    vals[i] = static_cast<uint32_t>(i);
}

// Row of every entry (the r with rowptr[r] <= e < rowptr[r + 1]) and the entry's weight side by
// side, so that the transposition's last step gathers one 8-byte record per entry, not two words
// from two arrays.
__global__ __launch_bounds__(kBlock) void expand_rows_kernel(const int64_t *rowptr, int64_t n_rows, int64_t nnz,
                                                            const float *w, uint2 *row_w, int32_t *status)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (e == 0 && (rowptr[0] != 0 || rowptr[n_rows] != nnz)) status[0] = 2;
    if (e >= nnz) return;
    int64_t lo = 0, hi = n_rows;                   // answer in [lo, hi)
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (rowptr[mid] <= e) lo = mid; else hi = mid;
    }
    if (!(rowptr[lo] <= e && e < rowptr[lo + 1])) status[0] = 2;      // row pointer not ascending
    row_w[e] = make_uint2(static_cast<uint32_t>(lo), w ? __float_as_uint(w[e]) : 0u);
}

__global__ __launch_bounds__(kBlock) void transpose_gather_kernel(const uint32_t *order, int64_t n, const uint2 *row_w,
                                                                 int32_t *colT, float *wT, int64_t *perm)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n) return;
    const uint32_t e = order[i];
    const uint2 rw = row_w[e];
    colT[i] = static_cast<int32_t>(rw.x);
    if (wT) wT[i] = __uint_as_float(rw.y);
    if (perm) perm[i] = static_cast<int64_t>(e);
}

// flags[g] = 1 for an owned node (low half), later 1 << 32 for a named node that is not owned.
__global__ __launch_bounds__(kBlock) void mark_owned_kernel(const int32_t *owner, int64_t n_nodes, int32_t part, uint64_t *flags)
{
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (g > n_nodes) return;
    flags[g] = (g < n_nodes && owner[g] == part) ? 1u : 0u;             // flags[n_nodes] = 0: the scan's total
}

__global__ __launch_bounds__(kBlock) void mark_named_kernel(const int32_t *gcol, int64_t nnz, const int32_t *owner,
                                                           int64_t n_nodes, int32_t part, uint64_t *flags, int32_t *status)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (e >= nnz) return;
    const int64_t g = gcol[e];
    if (g < 0 || g >= n_nodes) {
        status[0] = 1;
        return;
    }
    if (owner[g] != part) flags[g] = uint64_t(1) << 32;                  // every writer stores the same value
}

__global__ __launch_bounds__(kBlock) void assign_pos_kernel(const uint64_t *flags, const uint64_t *ranks, int64_t n_nodes,
                                                           int32_t *pos, int32_t *halo_gid, int64_t cap)
{
    const int64_t g = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (g >= n_nodes) return;
    const uint64_t f = flags[g], r = ranks[g];
    const int64_t n_inner = static_cast<int64_t>(ranks[n_nodes] & 0xffffffffu);
    int64_t p = -1;
    if (f == 1u) p = static_cast<int64_t>(r & 0xffffffffu);
    else if (f != 0) {
        const int64_t j = static_cast<int64_t>(r >> 32);
        p = n_inner + j;
        if (j < cap) halo_gid[j] = static_cast<int32_t>(g);
    }
    pos[g] = static_cast<int32_t>(p);
}

__global__ __launch_bounds__(kBlock) void relabel_kernel(const int32_t *gcol, int64_t nnz, const int32_t *pos, int64_t n_nodes,
                                                        int32_t *col, int32_t *status)
{
    const int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (e >= nnz) return;
    const int64_t g = gcol[e];
    int32_t p = -1;
    if (g >= 0 && g < n_nodes) p = pos[g];
    if (p < 0) status[0] = 1;
    col[e] = p;
}

// row_of[node] = place of the node among the nodes of its owner, from the nodes sorted by owner.
__global__ __launch_bounds__(kBlock) void rank_in_group_kernel(const uint32_t *keys, const uint32_t *vals, int64_t n,
                                                              const int64_t *group_ptr, int32_t *row_of)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n) return;
    row_of[vals[i]] = static_cast<int32_t>(i - group_ptr[keys[i]]);
}

__global__ __launch_bounds__(kBlock) void halo_owner_keys_kernel(const int32_t *halo_gid, int64_t n_halo, const int32_t *owner,
                                                                int64_t n_nodes, int32_t n_parts, uint32_t *keys,
                                                                uint32_t *vals, int32_t *status)
{
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (j >= n_halo) return;
    const int64_t g = halo_gid[j];
    int32_t k = 0;
    if (g < 0 || g >= n_nodes) status[0] = 1;
    else {
        k = owner[g];
        if (k < 0 || k >= n_parts) {
            status[0] = 1;
            k = 0;
        }
    }
    keys[j] = static_cast<uint32_t>(k);
    vals[j] = static_cast<uint32_t>(j);
}

__global__ __launch_bounds__(kBlock) void recv_rows_kernel(const uint32_t *order, int64_t n_halo, const int32_t *halo_gid,
                                                          const int32_t *row_of, int64_t n_nodes, int32_t *R_halo, int32_t *R_row)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n_halo) return;
    const uint32_t j = order[i];
    R_halo[i] = static_cast<int32_t>(j);
    const int64_t g = halo_gid[j];
    R_row[i] = (g >= 0 && g < n_nodes) ? row_of[g] : -1;
}

__global__ __launch_bounds__(kBlock) void copy_u32_to_i32_kernel(const uint32_t *src, int64_t n, int32_t *dst)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n) dst[i] = static_cast<int32_t>(src[i]);
}


// ---- operator weights and launch plans ------------------------------------------------------

// One wavefront per inner row r of the adjacency (no self loops, columns ascending): writes row r
// of D^-1/2 (A + I) D^-1/2 with the self loop merged in column order.  The weight of entry
// (r, c) is 1 / sqrt((deg_r + 1)(deg_c + 1)) evaluated in double (multiplication, square root
// and division are each correctly rounded) and rounded once to float.
__global__ __launch_bounds__(kBlock) void gcn_operator_kernel(const int64_t *rowptr, const int32_t *col,
                                                             const int32_t *deg, int64_t n_in, int64_t n_cols,
                                                             int64_t *rowptr_out, int32_t *col_out, float *w_out,
                                                             int32_t *status)
{
    const int lane = lane_id();
    const int64_t r = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + static_cast<int>(threadIdx.x) / kWave;
    if (r > n_in) return;
    const int64_t e0 = rowptr[r < n_in ? r : n_in];
    if (lane == 0) rowptr_out[r] = e0 + r;
    if (r == n_in) return;
    const int64_t e1 = rowptr[r + 1];
    if (e1 < e0) {
        if (lane == 0) status[0] = 2;
        return;
    }
    const double dr = static_cast<double>(deg[r]) + 1.0;
    const int64_t o0 = e0 + r;
    int64_t below = 0;                                   // columns < r seen so far
    for (int64_t base = e0; base < e1; base += kWave) {
        const int64_t e = base + lane;
        const bool have = e < e1;
        int64_t c = have ? static_cast<int64_t>(col[e]) : n_cols;
        if (have && (c < 0 || c >= n_cols || c == r)) {
            status[0] = 1;
            c = 0;                                       // keeps every access below in range
        }
        const bool lt = have && c < r;
        const uint64_t m = __ballot(lt);
        if (have) {
            const int64_t k = e - e0;                    // position inside the input row
            const int64_t o = o0 + k + (lt ? 0 : 1);     // the self loop sits after the columns < r
            col_out[o] = static_cast<int32_t>(c);
            w_out[o] = static_cast<float>(1.0 / sqrt(dr * (static_cast<double>(deg[c]) + 1.0)));
        }
        below += __popcll(m);
    }
    if (lane == 0) {
        col_out[o0 + below] = static_cast<int32_t>(r);
        w_out[o0 + below] = static_cast<float>(1.0 / sqrt(dr * dr));
    }
}

// Mean aggregator: every entry of row r weighs 1 / len(r), evaluated in double, rounded once.
__global__ __launch_bounds__(kBlock) void mean_weights_kernel(const int64_t *rowptr, int64_t n_rows, float *w,
                                                             int32_t *status)
{
    const int lane = lane_id();
    const int64_t r = static_cast<int64_t>(blockIdx.x) * kWavesPerBlock + static_cast<int>(threadIdx.x) / kWave;
    if (r >= n_rows) return;
    const int64_t e0 = rowptr[r], e1 = rowptr[r + 1];
    if (e1 < e0) {
        if (lane == 0) status[0] = 2;
        return;
    }
    const float v = static_cast<float>(1.0 / static_cast<double>(e1 - e0));
    for (int64_t e = e0 + lane; e < e1; e += kWave) w[e] = v;
}

// item i = row row_begin + i: low half 1 if the row is longer than chunk, high half its number of
// chunk-sized tasks (0 for a row that is not long).  One more item (zeros) closes the scan.
__global__ __launch_bounds__(kBlock) void long_row_items_kernel(const int64_t *rowptr, int64_t row_begin, int64_t n,
                                                               int64_t chunk, uint64_t *items, int32_t *status)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i > n) return;
    uint64_t v = 0;
    if (i < n) {
        const int64_t len = rowptr[row_begin + i + 1] - rowptr[row_begin + i];
        if (len < 0) status[0] = 2;
        if (len > chunk) v = 1ull | (static_cast<uint64_t>((len + chunk - 1) / chunk) << 32);
    }
    items[i] = v;
}

__global__ __launch_bounds__(kBlock) void long_row_fill_kernel(const uint64_t *items, const uint64_t *ranks, int64_t n,
                                                              int64_t row_begin, int32_t *long_rows, int64_t *long_ptr,
                                                              int64_t capacity)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i > n) return;
    const uint64_t rk = ranks[i];
    const int64_t slot = static_cast<int64_t>(rk & 0xffffffffu);
    const bool is_long = i < n && (items[i] & 1ull);
    if ((is_long || i == n) && slot <= capacity) {
        if (is_long && slot < capacity) long_rows[slot] = static_cast<int32_t>(row_begin + i);
        long_ptr[slot] = static_cast<int64_t>(rk >> 32);     // tasks before this row; the total at i == n
    }
}

// pieces of every row: per[i] = ceil(len_i / chunk)
__global__ __launch_bounds__(kBlock) void piece_counts_kernel(const int64_t *rowptr, int64_t n_rows, int64_t chunk,
                                                             uint64_t *per, int32_t *status)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i > n_rows) return;
    uint64_t v = 0;
    if (i < n_rows) {
        const int64_t len = rowptr[i + 1] - rowptr[i];
        if (len < 0) status[0] = 2;
        else v = static_cast<uint64_t>((len + chunk - 1) / chunk);
    }
    per[i] = v;
}

__global__ __launch_bounds__(kBlock) void piece_fill_kernel(const int64_t *rowptr, const uint64_t *first, int64_t n_rows,
                                                           int64_t chunk, int64_t *row_piece, int64_t *piece_ptr,
                                                           int32_t *piece_row, int64_t capacity)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i > n_rows) return;
    const int64_t k0 = static_cast<int64_t>(first[i]);
    row_piece[i] = k0;
    if (i == n_rows) {
        if (k0 <= capacity) piece_ptr[k0] = rowptr[n_rows];
        return;
    }
    const int64_t e0 = rowptr[i], e1 = rowptr[i + 1];
    int64_t k = k0;
    for (int64_t e = e0; e < e1 && k < capacity; e += chunk, ++k) {
        piece_ptr[k] = e;
        piece_row[k] = static_cast<int32_t>(i);
    }
}

// keys that sort rows longest first: 2^32 - 1 - min(len, 2^32 - 1); value = row index in the range
__global__ __launch_bounds__(kBlock) void length_keys_kernel(const int64_t *rowptr, int64_t row_begin, int64_t n,
                                                            uint32_t *keys, uint32_t *vals, int32_t *status)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i >= n) return;
    int64_t len = rowptr[row_begin + i + 1] - rowptr[row_begin + i];
    if (len < 0) {
        status[0] = 2;
        len = 0;
    }
    if (len > 0xffffffffll) len = 0xffffffffll;
    keys[i] = 0xffffffffu - static_cast<uint32_t>(len);
    vals[i] = static_cast<uint32_t>(i);
}

inline unsigned blocks_for(int64_t n) { return static_cast<unsigned>((n + kBlock - 1) / kBlock); }
inline unsigned wave_blocks_for(int64_t n) { return static_cast<unsigned>((n + kWavesPerBlock - 1) / kWavesPerBlock); }

// Waits for the stream and reports what the kernels' range checks found.
int32_t finish(const char *name, int32_t *status, hipStream_t st, const char *what1, const char *what2)
{
    SYLVIE_HIP_LAUNCH_CHECK(name);
    int32_t host = 0;
    hipError_t e = hipMemcpyAsync(&host, status, sizeof(host), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(SYLVIE_ERR_HIP, "%s: %s", name, hipGetErrorString(e));
    if (host == 1) return fail(SYLVIE_ERR_INVALID_ARG, "%s: %s", name, what1);
    if (host == 2) return fail(SYLVIE_ERR_INVALID_ARG, "%s: %s", name, what2);
    return SYLVIE_OK;
}

constexpr int64_t kMaxItems = (int64_t(1) << 31) - 4096;

}  // namespace
}  // namespace sylvie

extern "C" size_t sylvie_graph_workspace_bytes(int64_t n)
{
    using namespace sylvie;
    if (n < 1) n = 1;
    // status word, the sort's buffers, one int32 array and two 8-byte arrays of n + 1, scan scratch
    return 256 + sort_bytes(n) + align256(4 * static_cast<size_t>(n + 1)) + 2 * align256(8 * static_cast<size_t>(n + 1)) +
           align256(8 * static_cast<size_t>(scan_scratch_elems(n + 1) + 64)) + 1024;
}

extern "C" int32_t sylvie_graph_local_index(const int32_t *gcol, int64_t nnz, int64_t n_in, const int32_t *owner, int64_t n_nodes, int32_t part, int32_t *pos,
                                            int32_t *halo_gid, int64_t halo_capacity, int64_t *counts_host,
                                            void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_local_index";
    if (n_in < 0 || nnz < 0 || n_nodes < 1 || n_nodes > kMaxItems || nnz > kMaxItems || halo_capacity < 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!owner || !pos || !counts_host || (nnz > 0 && !gcol) || (halo_capacity > 0 && !halo_gid))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(n_nodes))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    uint64_t *flags = a.take<uint64_t>(n_nodes + 1);
    uint64_t *ranks = a.take<uint64_t>(n_nodes + 1);
    uint64_t *scratch = a.take<uint64_t>(scan_scratch_elems(n_nodes + 1) + 64);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    hipLaunchKernelGGL(mark_owned_kernel, dim3(blocks_for(n_nodes + 1)), dim3(kBlock), 0, st, owner, n_nodes, part, flags);
    if (nnz > 0)
        hipLaunchKernelGGL(mark_named_kernel, dim3(blocks_for(nnz)), dim3(kBlock), 0, st, gcol, nnz, owner, n_nodes, part,
                           flags, status);
    exclusive_scan<uint64_t>(flags, ranks, n_nodes + 1, scratch, st);
    hipLaunchKernelGGL(assign_pos_kernel, dim3(blocks_for(n_nodes)), dim3(kBlock), 0, st, flags, ranks, n_nodes, pos,
                       halo_gid, halo_capacity);
    const int32_t rc = finish(name, status, st, "neighbour id outside [0, n_nodes)", "");
    if (rc != SYLVIE_OK) return rc;
    uint64_t totals = 0;                                   // read back on the caller's stream
    hipError_t e = hipMemcpyAsync(&totals, ranks + n_nodes, sizeof(totals), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(SYLVIE_ERR_HIP, "%s: %s", name, hipGetErrorString(e));
    counts_host[0] = static_cast<int64_t>(totals & 0xffffffffu);
    counts_host[1] = static_cast<int64_t>(totals >> 32);
    if (counts_host[0] != n_in)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: the partition owns %lld nodes, n_in says %lld", name,
                    static_cast<long long>(counts_host[0]), static_cast<long long>(n_in));
    if (counts_host[1] > halo_capacity)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: %lld halo nodes, room for %lld", name,
                    static_cast<long long>(counts_host[1]), static_cast<long long>(halo_capacity));
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_graph_relabel_columns(const int32_t *gcol, int64_t nnz, const int32_t *pos, int64_t n_nodes,
                                                int32_t *col, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_relabel_columns";
    if (nnz < 0 || n_nodes < 1) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (nnz == 0) return SYLVIE_OK;
    if (!gcol || !pos || !col) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < 256) return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t *status = static_cast<int32_t *>(workspace);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    hipLaunchKernelGGL(relabel_kernel, dim3(blocks_for(nnz)), dim3(kBlock), 0, st, gcol, nnz, pos, n_nodes, col, status);
    return finish(name, status, st, "a neighbour is neither an inner nor a halo node of this partition", "");
}

extern "C" int32_t sylvie_graph_rows_in_owner(const int32_t *owner, int64_t n_nodes, int32_t n_parts, int32_t *row_of,
                                              int64_t *part_ptr, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_rows_in_owner";
    if (n_nodes < 1 || n_nodes > kMaxItems || n_parts < 1 || n_parts > (1 << 20))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!owner || !row_of || !part_ptr) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(n_nodes))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    SortBuffers b = take_sort(a, n_nodes);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    hipLaunchKernelGGL(keys_from_i32_kernel, dim3(blocks_for(n_nodes)), dim3(kBlock), 0, st, owner, n_nodes,
                       static_cast<int64_t>(n_parts), b.keys[0], b.vals[0], status);
    const int cur = radix_sort_pairs(b, n_nodes, bits_for(n_parts), st);
    hipLaunchKernelGGL(boundaries_kernel, dim3(blocks_for(n_nodes + 1)), dim3(kBlock), 0, st, b.keys[cur], n_nodes,
                       static_cast<int64_t>(n_parts), part_ptr);
    hipLaunchKernelGGL(rank_in_group_kernel, dim3(blocks_for(n_nodes)), dim3(kBlock), 0, st, b.keys[cur], b.vals[cur],
                       n_nodes, part_ptr, row_of);
    return finish(name, status, st, "owner outside [0, n_parts)", "");
}

extern "C" int32_t sylvie_graph_recv_sets(const int32_t *halo_gid, int64_t n_halo, const int32_t *owner,
                                          const int32_t *row_of, int64_t n_nodes, int32_t n_parts, int64_t *R_ptr,
                                          int32_t *R_halo, int32_t *R_row, void *workspace, size_t workspace_bytes,
                                          void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_recv_sets";
    if (n_halo < 0 || n_halo > kMaxItems || n_nodes < 1 || n_parts < 1 || n_parts > (1 << 20))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!owner || !row_of || !R_ptr || (n_halo > 0 && (!halo_gid || !R_halo || !R_row)))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(n_halo))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    SortBuffers b = take_sort(a, n_halo);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    if (n_halo > 0)
        hipLaunchKernelGGL(halo_owner_keys_kernel, dim3(blocks_for(n_halo)), dim3(kBlock), 0, st, halo_gid, n_halo, owner,
                           n_nodes, n_parts, b.keys[0], b.vals[0], status);
    const int cur = radix_sort_pairs(b, n_halo, bits_for(n_parts), st);
    hipLaunchKernelGGL(boundaries_kernel, dim3(blocks_for(n_halo + 1)), dim3(kBlock), 0, st, b.keys[cur], n_halo,
                       static_cast<int64_t>(n_parts), R_ptr);
    if (n_halo > 0)
        hipLaunchKernelGGL(recv_rows_kernel, dim3(blocks_for(n_halo)), dim3(kBlock), 0, st, b.vals[cur], n_halo, halo_gid,
                           row_of, n_nodes, R_halo, R_row);
    return finish(name, status, st, "halo id outside [0, n_nodes) or owner outside [0, n_parts)", "");
}

extern "C" int32_t sylvie_graph_transpose_csr(const int64_t *rowptr, const int32_t *col, const float *w, int64_t n_rows,
                                              int64_t n_cols, int64_t nnz, int64_t *rowptrT, int32_t *colT, float *wT,
                                              int64_t *perm, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_transpose_csr";
    if (n_rows < 1 || n_cols < 1 || nnz < 0 || nnz > kMaxItems || n_rows > kMaxItems || n_cols > kMaxItems)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!rowptr || !rowptrT || (nnz > 0 && (!col || !colT)) || ((w == nullptr) != (wT == nullptr)))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer (w and wT go together)", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(nnz))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    SortBuffers b = take_sort(a, nnz);
    uint2 *row_w = a.take<uint2>(nnz + 1);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    hipLaunchKernelGGL(expand_rows_kernel, dim3(blocks_for(nnz > 0 ? nnz : 1)), dim3(kBlock), 0, st, rowptr, n_rows, nnz,
                       wT ? w : nullptr, row_w, status);
    if (nnz > 0)
        hipLaunchKernelGGL(keys_from_i32_kernel, dim3(blocks_for(nnz)), dim3(kBlock), 0, st, col, nnz, n_cols, b.keys[0],
                           b.vals[0], status);
    const int cur = radix_sort_pairs(b, nnz, bits_for(n_cols), st);
    hipLaunchKernelGGL(boundaries_kernel, dim3(blocks_for(nnz + 1)), dim3(kBlock), 0, st, b.keys[cur], nnz, n_cols, rowptrT);
    if (nnz > 0)
        hipLaunchKernelGGL(transpose_gather_kernel, dim3(blocks_for(nnz)), dim3(kBlock), 0, st, b.vals[cur], nnz, row_w,
                           colT, wT, perm);
    return finish(name, status, st, "column outside [0, n_cols)", "row pointer does not ascend from 0 to nnz");
}

extern "C" int32_t sylvie_graph_scatter_segments(const int32_t *dst_row, int64_t n, int64_t n_dst, int64_t *seg_ptr,
                                                 int32_t *seg_rows, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_scatter_segments";
    if (n < 0 || n > kMaxItems || n_dst < 1 || n_dst > kMaxItems) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!seg_ptr || (n > 0 && (!dst_row || !seg_rows))) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(n))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    SortBuffers b = take_sort(a, n);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    if (n > 0)
        hipLaunchKernelGGL(keys_from_i32_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, st, dst_row, n, n_dst, b.keys[0],
                           b.vals[0], status);
    const int cur = radix_sort_pairs(b, n, bits_for(n_dst), st);
    hipLaunchKernelGGL(boundaries_kernel, dim3(blocks_for(n + 1)), dim3(kBlock), 0, st, b.keys[cur], n, n_dst, seg_ptr);
    if (n > 0)
        hipLaunchKernelGGL(copy_u32_to_i32_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, st, b.vals[cur], n, seg_rows);
    return finish(name, status, st, "destination row outside [0, n_dst)", "");
}

extern "C" int32_t sylvie_graph_gcn_operator(const int64_t *rowptr, const int32_t *col, const int32_t *deg, int64_t n_in,
                                             int64_t n_cols, int64_t nnz, int64_t *rowptr_out, int32_t *col_out,
                                             float *w_out, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_gcn_operator";
    if (n_in < 0 || n_in > kMaxItems || n_cols < n_in || n_cols > kMaxItems || nnz < 0 || nnz + n_in > kMaxItems)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!rowptr || !rowptr_out || (n_cols > 0 && !deg) || (nnz > 0 && !col) || (nnz + n_in > 0 && (!col_out || !w_out)))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < 256) return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t *status = static_cast<int32_t *>(workspace);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    hipLaunchKernelGGL(gcn_operator_kernel, dim3(wave_blocks_for(n_in + 1)), dim3(kBlock), 0, st, rowptr, col, deg, n_in,
                       n_cols, rowptr_out, col_out, w_out, status);
    return finish(name, status, st, "column outside [0, n_cols) or a self loop in the adjacency",
                  "row pointer does not ascend");
}

extern "C" int32_t sylvie_graph_mean_weights(const int64_t *rowptr, int64_t n_rows, int64_t nnz, float *w_out,
                                             void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_mean_weights";
    if (n_rows < 0 || n_rows > kMaxItems || nnz < 0 || nnz > kMaxItems) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!rowptr || (nnz > 0 && !w_out)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < 256) return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t *status = static_cast<int32_t *>(workspace);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    if (n_rows > 0)
        hipLaunchKernelGGL(mean_weights_kernel, dim3(wave_blocks_for(n_rows)), dim3(kBlock), 0, st, rowptr, n_rows, w_out,
                           status);
    return finish(name, status, st, "", "row pointer does not ascend");
}

extern "C" int32_t sylvie_graph_long_row_plan(const int64_t *rowptr, int64_t row_begin, int64_t n_rows, int32_t chunk,
                                              int32_t *long_rows, int64_t *long_ptr, int64_t capacity,
                                              int64_t *counts_host, void *workspace, size_t workspace_bytes,
                                              void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_long_row_plan";
    if (row_begin < 0 || n_rows < 0 || n_rows > kMaxItems || capacity < 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (chunk <= 0 || chunk % 64 != 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: chunk must be a positive multiple of 64", name);
    if (!rowptr || !long_ptr || !counts_host || (capacity > 0 && !long_rows))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(n_rows))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    uint64_t *items = a.take<uint64_t>(n_rows + 1);
    uint64_t *ranks = a.take<uint64_t>(n_rows + 1);
    uint64_t *scratch = a.take<uint64_t>(scan_scratch_elems(n_rows + 1) + 64);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    hipLaunchKernelGGL(long_row_items_kernel, dim3(blocks_for(n_rows + 1)), dim3(kBlock), 0, st, rowptr, row_begin, n_rows,
                       static_cast<int64_t>(chunk), items, status);
    exclusive_scan<uint64_t>(items, ranks, n_rows + 1, scratch, st);
    hipLaunchKernelGGL(long_row_fill_kernel, dim3(blocks_for(n_rows + 1)), dim3(kBlock), 0, st, items, ranks, n_rows,
                       row_begin, long_rows, long_ptr, capacity);
    const int32_t rc = finish(name, status, st, "", "row pointer does not ascend");
    if (rc != SYLVIE_OK) return rc;
    uint64_t totals = 0;
    hipError_t e = hipMemcpyAsync(&totals, ranks + n_rows, sizeof(totals), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(SYLVIE_ERR_HIP, "%s: %s", name, hipGetErrorString(e));
    counts_host[0] = static_cast<int64_t>(totals & 0xffffffffu);
    counts_host[1] = static_cast<int64_t>(totals >> 32);
    if (counts_host[0] > capacity)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: %lld long rows, room for %lld", name,
                    static_cast<long long>(counts_host[0]), static_cast<long long>(capacity));
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_graph_piece_table(const int64_t *rowptr, int64_t n_rows, int32_t chunk, int64_t *row_piece,
                                            int64_t *piece_ptr, int32_t *piece_row, int64_t capacity,
                                            int64_t *n_pieces_host, void *workspace, size_t workspace_bytes,
                                            void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_piece_table";
    if (n_rows < 0 || n_rows > kMaxItems || capacity < 0 || chunk <= 0)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!rowptr || !row_piece || !piece_ptr || !n_pieces_host || (capacity > 0 && !piece_row))
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(n_rows))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    uint64_t *per = a.take<uint64_t>(n_rows + 1);
    uint64_t *first = a.take<uint64_t>(n_rows + 1);
    uint64_t *scratch = a.take<uint64_t>(scan_scratch_elems(n_rows + 1) + 64);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    hipLaunchKernelGGL(piece_counts_kernel, dim3(blocks_for(n_rows + 1)), dim3(kBlock), 0, st, rowptr, n_rows,
                       static_cast<int64_t>(chunk), per, status);
    exclusive_scan<uint64_t>(per, first, n_rows + 1, scratch, st);
    hipLaunchKernelGGL(piece_fill_kernel, dim3(blocks_for(n_rows + 1)), dim3(kBlock), 0, st, rowptr, first, n_rows,
                       static_cast<int64_t>(chunk), row_piece, piece_ptr, piece_row, capacity);
    const int32_t rc = finish(name, status, st, "", "row pointer does not ascend");
    if (rc != SYLVIE_OK) return rc;
    uint64_t total = 0;
    hipError_t e = hipMemcpyAsync(&total, first + n_rows, sizeof(total), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(SYLVIE_ERR_HIP, "%s: %s", name, hipGetErrorString(e));
    n_pieces_host[0] = static_cast<int64_t>(total);
    if (n_pieces_host[0] > capacity)
        return fail(SYLVIE_ERR_INVALID_ARG, "%s: %lld pieces, room for %lld", name,
                    static_cast<long long>(n_pieces_host[0]), static_cast<long long>(capacity));
    return SYLVIE_OK;
}

extern "C" int32_t sylvie_graph_rows_by_length(const int64_t *rowptr, int64_t row_begin, int64_t n_rows,
                                               int32_t *order, void *workspace, size_t workspace_bytes, void *stream)
{
    using namespace sylvie;
    const char *name = "sylvie_graph_rows_by_length";
    if (row_begin < 0 || n_rows < 0 || n_rows > kMaxItems) return fail(SYLVIE_ERR_INVALID_ARG, "%s: bad sizes", name);
    if (!rowptr || (n_rows > 0 && !order)) return fail(SYLVIE_ERR_INVALID_ARG, "%s: null pointer", name);
    if (!workspace || workspace_bytes < sylvie_graph_workspace_bytes(n_rows))
        return fail(SYLVIE_ERR_WORKSPACE, "%s: workspace too small", name);
    hipStream_t st = static_cast<hipStream_t>(stream);
    Arena a{static_cast<char *>(workspace), 0, workspace_bytes};
    int32_t *status = a.take<int32_t>(1);
    SortBuffers b = take_sort(a, n_rows);
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
    if (n_rows > 0)
        hipLaunchKernelGGL(length_keys_kernel, dim3(blocks_for(n_rows)), dim3(kBlock), 0, st, rowptr, row_begin, n_rows,
                           b.keys[0], b.vals[0], status);
    const int cur = radix_sort_pairs(b, n_rows, 32, st);
    if (n_rows > 0)
        hipLaunchKernelGGL(copy_u32_to_i32_kernel, dim3(blocks_for(n_rows)), dim3(kBlock), 0, st, b.vals[cur], n_rows, order);
    return finish(name, status, st, "", "row pointer does not ascend");
}
