// CPU oracle for the CSR sparse-times-dense matrix product.  TEST INFRASTRUCTURE ONLY.
//
// The benchmark's "SpMM CSR" task (App. C, task 13): C = A B with A sparse in CSR (values /
// col_indices / row_offsets, shape rows x cols) and B dense (cols x K), C dense (rows x K).
// Computed here in the BLAS form  C <- alpha * A * B + beta * C  with B and C row-major with
// leading dimensions ldb, ldc.  Every element of C is one sum over the stored entries of its
// row, in storage order, in IEEE double precision: three nested loops, nothing blocked.
// Shares no code with the GPU library and is never called by it.
//
// Pins (tests/test_oracle_spmm.py): a dense matrix product on small matrices (numpy), K = 1
// against the pinned SpMV oracle, identity A (C = B), a hand-worked fixture, linearity in B.
//
// Also the order in which the GPU kernel is handed the rows (its own scheduling aid, not part of
// the paper's task): the definition written out as a stable sort.  Pins: a hand-worked fixture,
// and the defining properties checked with numpy on random lengths.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>

extern "C" {

// C_ref[i*K + k] = alpha * sum_e vals[e] * B[colidx[e]*ldb + k] + beta * C0[i*ldc + k]   (double, dense m x K)
// S_ref[i*K + k] = sum_e |vals[e] * B[colidx[e]*ldb + k]|
// beta == 0: C0 is not read (may be NULL).  Returns 0, or 1 for a malformed structure.
int oracle_spmm_csr_f32(int64_t m, int64_t n, int64_t K, const int32_t* rowptr, const int32_t* colidx,
                        const float* vals, const float* B, int64_t ldb, const float* C0, int64_t ldc, float alpha,
                        float beta, double* C_ref, double* S_ref) {
    for (int64_t i = 0; i < m; ++i) {
        if (rowptr[i + 1] < rowptr[i]) return 1;
        for (int64_t k = 0; k < K; ++k) {
            double acc = 0.0, S = 0.0;
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const int32_t j = colidx[e];
                if (j < 0 || j >= n) return 1;
                const double p = static_cast<double>(vals[e]) * static_cast<double>(B[j * ldb + k]);
                acc += p;
                S += std::fabs(p);
            }
            double r = static_cast<double>(alpha) * acc;
            if (beta != 0.0f) r += static_cast<double>(beta) * static_cast<double>(C0[i * ldc + k]);
            C_ref[i * K + k] = r;
            S_ref[i * K + k] = S;
        }
    }
    return 0;
}

// The rows are cut into windows of `window` consecutive rows (the last one may be shorter).
// rows[0..m) lists, window after window, the window's row ids sorted by decreasing
// key(i) = min(ceil(len_i / 4), 64), len_i = rowptr[i+1] - rowptr[i]; rows of equal key keep
// their ascending order.
void oracle_spmm_row_order(int64_t m, const int32_t* rowptr, int64_t window, int32_t* rows) {
    auto key = [&](int32_t i) {
        const int64_t len = static_cast<int64_t>(rowptr[i + 1]) - rowptr[i];
        return std::min<int64_t>((len + 3) / 4, 64);
    };
    std::iota(rows, rows + m, 0);
    for (int64_t w0 = 0; w0 < m; w0 += window)
        std::stable_sort(rows + w0, rows + std::min(w0 + window, m), [&](int32_t a, int32_t b) { return key(a) > key(b); });
}

}  // extern "C"
