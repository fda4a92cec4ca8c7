// CPU oracle for the CSR sparse matrix-vector product.  TEST INFRASTRUCTURE ONLY.
//
// This file is the reference that the HIP kernels are judged against.  It is plain,
// single-threaded, deliberately slow, shares no code with the GPU library and is
// never called by it.  Only tests, the smoke check and the benchmark's CPU-baseline
// leg may use it.
//
// What it computes: the operation of the benchmark's "SpMV CSR" task (App. C, task 12:
// y = A x with A given by values / col_indices / row_offsets), extended with the BLAS
// scalars:  y <- alpha * A * x + beta * y.  The sum of every row is taken in the order
// the entries are stored, in IEEE double precision.  Nothing is blocked, reordered or
// vectorised by hand.
//
// Pins (tests/test_oracle_*.py): dense matvec on tiny matrices, identity and diagonal
// matrices, A*1 = row sums (closed form 0/1/2 for the 5-point Laplacian), integer-valued
// matrices whose result is exact, an independent library CSR product, linearity and
// row-permutation invariants, and small hand-worked fixtures under tests/golden/.

#include <cmath>
#include <cstdint>
#include <cstring>

namespace {

// bf16 is the upper half of an IEEE binary32: widening is exact.
inline float bf16_bits_to_float(uint16_t b) {
    uint32_t u = static_cast<uint32_t>(b) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
}

}  // namespace

extern "C" {

// FP32 storage.  y_ref[i] = alpha * sum_k vals[k]*x[colidx[k]] + beta*y0[i]   (double)
//                S_ref[i] = sum_k |vals[k]*x[colidx[k]]|                        (double)
// beta == 0 means y0 is not read at all (it may be NULL or hold NaN).
// Returns 0, or 1 if a column index is outside [0, n) or rowptr is not a valid offset array.
int oracle_spmv_csr_f32(int64_t m, int64_t n, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                        const float* x, const float* y0, float alpha, float beta, double* y_ref, double* S_ref) {
    for (int64_t i = 0; i < m; ++i) {
        if (rowptr[i + 1] < rowptr[i]) return 1;
        double acc = 0.0;
        double S = 0.0;
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
            const int32_t j = colidx[k];
            if (j < 0 || j >= n) return 1;
            const double p = static_cast<double>(vals[k]) * static_cast<double>(x[j]);
            acc += p;
            S += std::fabs(p);
        }
        double r = static_cast<double>(alpha) * acc;
        if (beta != 0.0f) r += static_cast<double>(beta) * static_cast<double>(y0[i]);
        y_ref[i] = r;
        S_ref[i] = S;
    }
    return 0;
}

// BF16 storage of vals and x (bit patterns), same arithmetic in double on the widened values.
int oracle_spmv_csr_bf16(int64_t m, int64_t n, const int32_t* rowptr, const int32_t* colidx, const uint16_t* vals,
                         const uint16_t* x, const float* y0, float alpha, float beta, double* y_ref, double* S_ref) {
    for (int64_t i = 0; i < m; ++i) {
        if (rowptr[i + 1] < rowptr[i]) return 1;
        double acc = 0.0;
        double S = 0.0;
        for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
            const int32_t j = colidx[k];
            if (j < 0 || j >= n) return 1;
            const double p = static_cast<double>(bf16_bits_to_float(vals[k])) * static_cast<double>(bf16_bits_to_float(x[j]));
            acc += p;
            S += std::fabs(p);
        }
        double r = static_cast<double>(alpha) * acc;
        if (beta != 0.0f) r += static_cast<double>(beta) * static_cast<double>(y0[i]);
        y_ref[i] = r;
        S_ref[i] = S;
    }
    return 0;
}

}  // extern "C"
