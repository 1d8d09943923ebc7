// Debug-mode precondition checks (SYLVIE_VALIDATE=1): see validate.hip.
#pragma once

#include "common.hpp"

namespace sylvie {

enum : unsigned { kBadValue = 0, kBadIndex = 1, kBadRowPtr = 2, kBadOrder = 3 };

// True when the environment asks for the checks (read at every call: a test may switch it).
bool validate_enabled();

// Enqueues checks on the caller's stream, then finish() waits for them and turns the first
// kind of violation into SYLVIE_ERR_INVALID_ARG.  One status record per device image: calls
// that validate concurrently on one GPU would share it (it is a debug mode).
class Validator {
public:
    Validator(const char *name, hipStream_t st);
    // source rows idx[i] | row_offset + i: finite, |x| < 2^126, idx[i] >= 0
    void rows(const float *src, int64_t ld, int d, const int32_t *idx, int64_t row_offset, int64_t n_rows);
    // CSR rows [row_begin, row_begin + n_rows): pointers ascend; 0 <= col (< n_cols if n_cols >= 0);
    // with n_dense >= 0, columns < n_dense come before columns >= n_dense inside a row
    void csr(const int64_t *rowptr, const int32_t *col, int64_t row_begin, int64_t n_rows, int64_t n_cols,
             int64_t n_dense);
    // segment table: seg_ptr ascends from 0 to <= n_wire, seg_rows in [0, n_wire) ascending inside
    // a segment, ids[k] >= 0 when given
    void segments(const int64_t *seg_ptr, const int32_t *seg_rows, int64_t n_seg, int64_t n_wire,
                  const int32_t *ids);
    int32_t finish();

private:
    const char *name_;
    hipStream_t st_;
    unsigned long long *rec_ = nullptr;
    int32_t rc_ = SYLVIE_OK;
};

}  // namespace sylvie
