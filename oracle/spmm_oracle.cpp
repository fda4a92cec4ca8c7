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
// and the defining properties checked with numpy on random lengths.  And the packed copy of A in
// that order, slot by slot from its definition.  Pins: a hand-worked fixture; every entry found
// exactly once, everything else padding; rows with equally many columns of every residue (a closed form).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <numeric>
#include <utility>
#include <vector>

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

// The same product with A's values and B stored as bf16 (the upper half of an IEEE binary32, here as uint16 bit
// patterns; App. C task 13 in the benchmark's BF16 variant, section 3.1).  Every stored number is widened exactly
// (bits << 16 read as a binary32); products and sums in double as above; C0, alpha, beta stay binary32.
static double bf16_to_double(uint16_t b) {
    const uint32_t u = static_cast<uint32_t>(b) << 16;
    float f;
    static_assert(sizeof f == sizeof u, "binary32");
    __builtin_memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

int oracle_spmm_csr_bf16(int64_t m, int64_t n, int64_t K, const int32_t* rowptr, const int32_t* colidx,
                         const uint16_t* vals, const uint16_t* B, int64_t ldb, const float* C0, int64_t ldc, float alpha,
                         float beta, double* C_ref, double* S_ref) {
    for (int64_t i = 0; i < m; ++i) {
        if (rowptr[i + 1] < rowptr[i]) return 1;
        for (int64_t k = 0; k < K; ++k) {
            double acc = 0.0, S = 0.0;
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
                const int32_t j = colidx[e];
                if (j < 0 || j >= n) return 1;
                const double p = bf16_to_double(vals[e]) * bf16_to_double(B[j * ldb + k]);
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

// Packed copy, layout.  Group g = the rows at positions 16g .. 16g+15 of rows[] (positions from m
// on count as empty rows); L_g = its longest row.  desc[2g] = sum over earlier groups of
// ceil(L / 16), desc[2g+1] = ceil(L_g / 4); closing pair (total blocks, 0).  Returns the total.
int64_t oracle_spmm_packed_layout(int64_t m, const int32_t* rowptr, const int32_t* rows, int32_t* desc) {
    const int64_t groups = (m + 15) / 16;
    int64_t blocks = 0;
    for (int64_t g = 0; g < groups; ++g) {
        int64_t L = 0;
        for (int64_t i = 0; i < 16; ++i) {
            const int64_t p = 16 * g + i;
            if (p < m) L = std::max<int64_t>(L, static_cast<int64_t>(rowptr[rows[p] + 1]) - rowptr[rows[p]]);
        }
        desc[2 * g] = static_cast<int32_t>(blocks);
        desc[2 * g + 1] = static_cast<int32_t>((L + 3) / 4);
        blocks += (L + 15) / 16;
    }
    desc[2 * groups] = static_cast<int32_t>(blocks);
    desc[2 * groups + 1] = 0;
    return blocks;
}

// Packed copy, the order of a row's entries.  The row at position p of rows[] takes its entries by increasing
// key(e) = 4 * (earlier entries of the row whose column is congruent to e's modulo 4) + (column of e - p) mod 4
// (the keys of a row are distinct).  The kernel keeps B's rows 64 bytes apart in LDS, four to a cycle of the banks, and
// reads entry number t of 16 rows at once: this way neighbouring rows ask for different quarters of the banks as long
// as each has entries of every residue left.
static std::vector<int64_t> packed_entry_order(const int32_t* colidx, int64_t first, int64_t len, int64_t p) {
    std::vector<std::pair<int64_t, int64_t>> keyed(static_cast<size_t>(len));
    int64_t seen[4] = {0, 0, 0, 0};
    for (int64_t t = 0; t < len; ++t) {
        const int64_t c = colidx[first + t];
        keyed[static_cast<size_t>(t)] = {4 * seen[c % 4]++ + ((c - p) % 4 + 4) % 4, t};
    }
    std::sort(keyed.begin(), keyed.end());
    std::vector<int64_t> order(static_cast<size_t>(len));
    for (int64_t t = 0; t < len; ++t) order[static_cast<size_t>(t)] = keyed[static_cast<size_t>(t)].second;
    return order;
}

// Packed copy, contents: slot ((desc[2g] + b) * 64 + 4 i + q) * 4 + e holds the entry of rank 16 b + 4 q + e (in the
// order above) of the i-th row of group g, or padding (column -1, value 0) where the row has no such entry.
void oracle_spmm_pack(int64_t m, const int32_t* rowptr, const int32_t* colidx, const float* vals, const int32_t* rows,
                      const int32_t* desc, int32_t* pcol, float* pval) {
    const int64_t groups = (m + 15) / 16;
    for (int64_t g = 0; g < groups; ++g)
        for (int64_t i = 0; i < 16; ++i) {
            const int64_t p = 16 * g + i;
            const int64_t first = p < m ? rowptr[rows[p]] : 0, len = p < m ? rowptr[rows[p] + 1] - first : 0;
            const std::vector<int64_t> order = packed_entry_order(colidx, first, len, p);
            for (int64_t b = 0; b < desc[2 * g + 2] - desc[2 * g]; ++b)
                for (int64_t q = 0; q < 4; ++q)
                    for (int64_t e = 0; e < 4; ++e) {
                        const int64_t slot = ((desc[2 * g] + b) * 64 + 4 * i + q) * 4 + e;
                        const int64_t t = 16 * b + 4 * q + e;
                        pcol[slot] = -1;
                        pval[slot] = 0.0f;
                        if (t < len) {
                            pcol[slot] = colidx[first + order[static_cast<size_t>(t)]];
                            pval[slot] = vals[first + order[static_cast<size_t>(t)]];
                        }
                    }
        }
}

// The packed copy is built when it has at most 2 * nnz slots (256 per block) and 2^22 blocks.
int oracle_spmm_packed_choice(int64_t nnz, int64_t blocks) {
    return nnz > 0 && 256 * blocks <= 2 * nnz && blocks <= (int64_t{1} << 22);
}

}  // extern "C"
