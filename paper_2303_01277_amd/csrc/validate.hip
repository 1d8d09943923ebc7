// Precondition checks of the debug mode SYLVIE_VALIDATE=1.
//
// The hot entry points trust their inputs (finite values below 2^126, indices in range,
// dense columns before wire columns inside a CSR row) and never synchronise.  With the
// environment variable SYLVIE_VALIDATE set to 1 they first run the checks below on the
// caller's stream, wait for them, and return SYLVIE_ERR_INVALID_ARG with the first kind of
// violation found instead of enqueueing the real work.  The checks only read the caller's
// arrays; their one status record lives in the library's device image.
#include <stdlib.h>
#include <string.h>

#include "common.hpp"
#include "validate.hpp"

namespace sylvie {

// [0] = bit mask of violations, [1] = an offending position (any one)
static __device__ __align__(16) unsigned long long g_check[2];

constexpr int kBlock = 256;

__global__ void check_clear_kernel(unsigned long long *rec)
{
    rec[0] = 0ull;
    rec[1] = 0ull;
}

__device__ __forceinline__ void flag(unsigned long long *rec, unsigned bit, unsigned long long where)
{
    atomicOr(&rec[0], 1ull << bit);
    rec[1] = where;
}

// rows idx[i] (or row_offset + i) of src: every element finite with |x| < 2^126; idx >= 0
__global__ __launch_bounds__(kBlock) void check_rows_kernel(const float *src, int64_t ld, int d,
                                                            const int32_t *idx, int64_t row_offset,
                                                            int64_t n_rows, unsigned long long *rec)
{
    const int64_t total = n_rows * d;
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; e < total;
         e += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int64_t i = e / d;
        const int c = static_cast<int>(e - i * d);
        int64_t r = row_offset + i;
        if (idx) {
            r = idx[i];
            if (r < 0) {
                if (c == 0) flag(rec, kBadIndex, static_cast<unsigned long long>(i));
                continue;
            }
        }
        const float x = src[r * ld + c];
        if (!(fabsf(x) < 0x1p126f)) flag(rec, kBadValue, static_cast<unsigned long long>(e));
    }
}

// rows [row_begin, row_begin + n_rows) of a CSR: row pointer ascending, columns in
// [0, n_cols) when n_cols >= 0, and (n_dense >= 0) no column < n_dense after one >= n_dense
__global__ __launch_bounds__(kBlock) void check_csr_kernel(const int64_t *rowptr, const int32_t *col,
                                                           int64_t row_begin, int64_t n_rows,
                                                           int64_t n_cols, int64_t n_dense,
                                                           unsigned long long *rec)
{
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; i < n_rows;
         i += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int64_t v = row_begin + i;
        const int64_t e0 = rowptr[v], e1 = rowptr[v + 1];
        if (e0 < 0 || e1 < e0) {
            flag(rec, kBadRowPtr, static_cast<unsigned long long>(v));
            continue;
        }
        bool wire_seen = false;
        for (int64_t e = e0; e < e1; ++e) {
            const int64_t c = col[e];
            if (c < 0 || (n_cols >= 0 && c >= n_cols)) flag(rec, kBadIndex, static_cast<unsigned long long>(e));
            if (n_dense >= 0) {
                if (c >= n_dense) wire_seen = true;
                else if (wire_seen) flag(rec, kBadOrder, static_cast<unsigned long long>(e));
            }
        }
    }
}

// seg_ptr[0 .. n_seg] ascending from 0; seg_rows[j] in [0, n_wire) for j < seg_ptr[n_seg];
// ids[k] >= 0 (ids may be null)
__global__ __launch_bounds__(kBlock) void check_segments_kernel(const int64_t *seg_ptr,
                                                                const int32_t *seg_rows, int64_t n_seg,
                                                                int64_t n_wire, const int32_t *ids,
                                                                unsigned long long *rec)
{
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x; k < n_seg;
         k += static_cast<int64_t>(gridDim.x) * kBlock) {
        const int64_t j0 = seg_ptr[k], j1 = seg_ptr[k + 1];
        if ((k == 0 && j0 != 0) || j1 < j0 || j1 > n_wire) {
            flag(rec, kBadRowPtr, static_cast<unsigned long long>(k));
            continue;
        }
        if (ids && ids[k] < 0) flag(rec, kBadIndex, static_cast<unsigned long long>(k));
        for (int64_t j = j0; j < j1; ++j) {
            const int32_t r = seg_rows[j];
            if (r < 0 || r >= n_wire) flag(rec, kBadIndex, static_cast<unsigned long long>(j));
            if (j > j0 && seg_rows[j - 1] >= r) flag(rec, kBadOrder, static_cast<unsigned long long>(j));
        }
    }
}

bool validate_enabled()
{
    const char *v = getenv("SYLVIE_VALIDATE");
    return v && strcmp(v, "1") == 0;
}

static int32_t record_address(const char *name, unsigned long long **rec)
{
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_check));
    if (e != hipSuccess || !p) return fail(SYLVIE_ERR_HIP, "%s: validate: %s", name, hipGetErrorString(e));
    *rec = static_cast<unsigned long long *>(p);
    return SYLVIE_OK;
}

static unsigned grid_for(int64_t n)
{
    const int64_t b = (n + kBlock - 1) / kBlock;
    return static_cast<unsigned>(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

Validator::Validator(const char *name, hipStream_t st) : name_(name), st_(st)
{
    rc_ = record_address(name, &rec_);
    if (rc_ == SYLVIE_OK) hipLaunchKernelGGL(check_clear_kernel, dim3(1), dim3(1), 0, st_, rec_);
}

void Validator::rows(const float *src, int64_t ld, int d, const int32_t *idx, int64_t row_offset,
                     int64_t n_rows)
{
    if (rc_ != SYLVIE_OK || n_rows <= 0 || !src) return;
    hipLaunchKernelGGL(check_rows_kernel, dim3(grid_for(n_rows * d)), dim3(kBlock), 0, st_, src, ld, d, idx,
                       row_offset, n_rows, rec_);
}

void Validator::csr(const int64_t *rowptr, const int32_t *col, int64_t row_begin, int64_t n_rows,
                    int64_t n_cols, int64_t n_dense)
{
    if (rc_ != SYLVIE_OK || n_rows <= 0 || !rowptr || !col) return;
    hipLaunchKernelGGL(check_csr_kernel, dim3(grid_for(n_rows)), dim3(kBlock), 0, st_, rowptr, col, row_begin,
                       n_rows, n_cols, n_dense, rec_);
}

void Validator::segments(const int64_t *seg_ptr, const int32_t *seg_rows, int64_t n_seg, int64_t n_wire,
                         const int32_t *ids)
{
    if (rc_ != SYLVIE_OK || n_seg <= 0 || !seg_ptr) return;
    hipLaunchKernelGGL(check_segments_kernel, dim3(grid_for(n_seg)), dim3(kBlock), 0, st_, seg_ptr, seg_rows,
                       n_seg, n_wire, ids, rec_);
}

int32_t Validator::finish()
{
    if (rc_ != SYLVIE_OK) return rc_;
    unsigned long long host[2] = {0, 0};
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(host, rec_, sizeof(host), hipMemcpyDeviceToHost, st_);
    if (e == hipSuccess) e = hipStreamSynchronize(st_);
    if (e != hipSuccess) return fail(SYLVIE_ERR_HIP, "%s: validate: %s", name_, hipGetErrorString(e));
    if (host[0] == 0) return SYLVIE_OK;
    const char *what = (host[0] & (1ull << kBadValue)) ? "a value that is not finite or not below 2^126"
                     : (host[0] & (1ull << kBadIndex)) ? "an index out of range"
                     : (host[0] & (1ull << kBadRowPtr)) ? "a row / segment pointer that does not ascend within bounds"
                     : "entries out of order (dense columns must precede wire columns; segment rows must ascend)";
    return fail(SYLVIE_ERR_INVALID_ARG, "%s: SYLVIE_VALIDATE found %s (near position %llu; violation mask 0x%llx)",
                name_, what, host[1], host[0]);
}

}  // namespace sylvie
