// Host-side analysis of the CSR row structure: statistics, length bins, row blocks,
// merge-path splits, plan.  Integer work only; O(m) plus O(P log m).
#pragma once
#include <cstdint>
#include <vector>

#include "spmv_mi355.h"

namespace spmv {

// 2040 + (vector width - 1) stays inside 2048 slots: a default tile is at most two 128-bit
// vectors per lane of a 256-lane workgroup in FP32 and one in bf16.
constexpr int kDefaultBlockNnz = 2040;
constexpr int kDefaultRowsMax = 256;
constexpr int kDefaultItemsPerChunk = 2040;
constexpr int kMaxBlockNnz = 8192;
constexpr int kMaxRowsMax = 1024;
constexpr int kMaxItemsPerChunk = 8192;

struct Analysis {
    spmv_analysis_info_t info{};
    int32_t bin_count[SPMV_NUM_BINS]{};
    int32_t bin_offset[SPMV_NUM_BINS + 1]{};
    std::vector<int32_t> bin_rows;    // [m]
    std::vector<int32_t> row_blocks;  // [nb+1]
    std::vector<int32_t> mp_row;      // [P+1]
    std::vector<int32_t> mp_nz;       // [P+1]
};

// Fills in defaults and range-checks the parameters.  Returns SPMV_OK or SPMV_ERR_INVALID_ARG.
spmv_status_t resolve_params(const spmv_analyze_params_t* in, spmv_analyze_params_t* out);

// rowptr is a HOST array of m+1 entries.  Returns SPMV_OK, SPMV_ERR_BAD_STRUCTURE or SPMV_ERR_ALLOC.
spmv_status_t analyze_rowptr(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr,
                             const spmv_analyze_params_t& params, Analysis* out);

}  // namespace spmv
