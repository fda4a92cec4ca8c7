// CPU oracle for y <- alpha*A*x + beta*y with A in coordinate (COO), compressed-sparse-column
// (CSC) and ELL storage.  TEST INFRASTRUCTURE ONLY; shares no code with the GPU library.
//
// The benchmark's tasks 8, 10 and 14 (App. C): the same product as the CSR task with A held as
//   COO  values[nnz], row_indices[nnz], col_indices[nnz]            (any order, repeats add up)
//   CSC  values[nnz], row_indices[nnz], col_offsets[cols+1]
//   ELL  values[rows*width], col_ids[rows*width], row-major, padding marked by col_id = -1
// Each y_i is accumulated in IEEE double in the order the entries are stored; S_i = sum |a x|.
// dtype 0: values and x are binary32; dtype 1: bf16 bit patterns (upper half of a binary32).
//
// Pins (tests/test_oracle_formats.py): scipy's own format conversions of a CSR matrix fed to
// these functions must reproduce the pinned CSR oracle; hand-worked fixtures; padding and
// empty rows/columns; repeated coordinates.

#include <cmath>
#include <cstdint>
#include <cstring>

namespace {

inline double widen_at(const void* p, int64_t i, int dtype) {
    if (dtype == 0) return static_cast<double>(static_cast<const float*>(p)[i]);
    const uint32_t u = static_cast<uint32_t>(static_cast<const uint16_t*>(p)[i]) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

void finish(int64_t m, const double* acc, const float* y0, float alpha, float beta, double* y_ref) {
    for (int64_t i = 0; i < m; ++i) {
        double r = static_cast<double>(alpha) * acc[i];
        if (beta != 0.0f) r += static_cast<double>(beta) * static_cast<double>(y0[i]);
        y_ref[i] = r;
    }
}

}  // namespace

extern "C" {

// y_ref doubles as the accumulator (it is overwritten at the end).  Returns 1 for an index out of range.
int oracle_spmv_coo(int64_t m, int64_t n, int64_t nnz, const int32_t* row, const int32_t* col, const void* vals,
                    int dtype, const void* x, const float* y0, float alpha, float beta, double* y_ref, double* S_ref) {
    for (int64_t i = 0; i < m; ++i) y_ref[i] = S_ref[i] = 0.0;
    for (int64_t e = 0; e < nnz; ++e) {
        if (row[e] < 0 || row[e] >= m || col[e] < 0 || col[e] >= n) return 1;
        const double p = widen_at(vals, e, dtype) * widen_at(x, col[e], dtype);
        y_ref[row[e]] += p;
        S_ref[row[e]] += std::fabs(p);
    }
    finish(m, y_ref, y0, alpha, beta, y_ref);
    return 0;
}

int oracle_spmv_csc(int64_t m, int64_t n, const int32_t* col_offsets, const int32_t* row, const void* vals, int dtype,
                    const void* x, const float* y0, float alpha, float beta, double* y_ref, double* S_ref) {
    for (int64_t i = 0; i < m; ++i) y_ref[i] = S_ref[i] = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        if (col_offsets[j + 1] < col_offsets[j]) return 1;
        for (int64_t e = col_offsets[j]; e < col_offsets[j + 1]; ++e) {
            if (row[e] < 0 || row[e] >= m) return 1;
            const double p = widen_at(vals, e, dtype) * widen_at(x, j, dtype);
            y_ref[row[e]] += p;
            S_ref[row[e]] += std::fabs(p);
        }
    }
    finish(m, y_ref, y0, alpha, beta, y_ref);
    return 0;
}

// A slot is padding exactly when its col_id is -1 (its value is then ignored, whatever it is).
int oracle_spmv_ell(int64_t m, int64_t n, int64_t width, const int32_t* col_ids, const void* vals, int dtype,
                    const void* x, const float* y0, float alpha, float beta, double* y_ref, double* S_ref) {
    for (int64_t i = 0; i < m; ++i) {
        double acc = 0.0, S = 0.0;
        for (int64_t s = 0; s < width; ++s) {
            const int32_t j = col_ids[i * width + s];
            if (j == -1) continue;
            if (j < 0 || j >= n) return 1;
            const double p = widen_at(vals, i * width + s, dtype) * widen_at(x, j, dtype);
            acc += p;
            S += std::fabs(p);
        }
        y_ref[i] = acc;
        S_ref[i] = S;
    }
    finish(m, y_ref, y0, alpha, beta, y_ref);
    return 0;
}

}  // extern "C"
