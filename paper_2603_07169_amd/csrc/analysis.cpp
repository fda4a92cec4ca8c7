// Host-side analysis of the CSR row structure (row_offsets as laid out in App. C task 12).
#include "analysis.h"

#include <algorithm>
#include <climits>
#include <new>

namespace spmv {

namespace {

inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// bin index of a row length: 0 for an empty row, otherwise 1 + ceil(log2(len)).
inline int length_bin(uint32_t len) {
    if (len <= 1) return static_cast<int>(len);
    return 33 - __builtin_clz(len - 1);
}

// Merge-path split on diagonal d: the number of finished rows i at the point where the path
// has made d steps.  rowptr[i+1] + i is strictly increasing, so the first i with
// rowptr[i+1] + i > d - 1 can be found by bisection inside the feasible window.
inline int64_t split_rows_on_diagonal(int64_t d, int64_t m, int64_t nnz, const int32_t* rowptr) {
    int64_t lo = std::max<int64_t>(0, d - nnz);
    int64_t hi = std::min<int64_t>(d, m);
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (static_cast<int64_t>(rowptr[mid + 1]) + mid > d - 1)
            hi = mid;
        else
            lo = mid + 1;
    }
    return lo;
}

}  // namespace

spmv_status_t resolve_params(const spmv_analyze_params_t* in, spmv_analyze_params_t* out) {
    spmv_analyze_params_t p{};
    if (in) p = *in;
    if (p.reserved != 0 || (p.prepare_spmm != 0 && p.prepare_spmm != 1)) return SPMV_ERR_INVALID_ARG;
    if (p.plan < SPMV_PLAN_AUTO || p.plan > SPMV_PLAN_COLBLOCK) return SPMV_ERR_INVALID_ARG;
    if (p.items_per_chunk == 0) p.items_per_chunk = kDefaultItemsPerChunk;
    if (p.block_nnz < 0 || p.block_nnz > kMaxBlockNnz) return SPMV_ERR_INVALID_ARG;
    if (p.rows_max < 0 || p.rows_max > kMaxRowsMax) return SPMV_ERR_INVALID_ARG;
    if (p.items_per_chunk < 1 || p.items_per_chunk > kMaxItemsPerChunk) return SPMV_ERR_INVALID_ARG;
    if (p.vector_lanes != 0 && (!is_pow2(p.vector_lanes) || p.vector_lanes < 2 || p.vector_lanes > 64))
        return SPMV_ERR_INVALID_ARG;
    *out = p;
    return SPMV_OK;
}

// The tile kernel gives a row to a team of G lanes, G = the largest power of two with
// 16*G <= mean row length + 15, and runs 256 lanes: a block of 256/G rows keeps every lane busy.
// The entry limit is set so that the row limit is the one that binds on a regular matrix.
// Small matrices get small blocks so that there are enough of them to spread over the chip.
void default_tile_shape(int64_t m, int64_t nnz, int32_t* block_nnz, int32_t* rows_max) {
    if (m <= 0 || nnz <= (int64_t{1} << 20)) {
        *block_nnz = 1024;
        *rows_max = 64;
        return;
    }
    const int64_t mean_up = (nnz + m - 1) / m;
    int lanes = 1;
    while (lanes < 64 && 16 * static_cast<int64_t>(lanes) < mean_up) lanes <<= 1;
    const int rows = 256 / lanes;
    int64_t entries = (rows * mean_up + 7) & ~int64_t{7};
    entries = std::max<int64_t>(2048, std::min<int64_t>(entries, kMaxBlockNnz));
    *block_nnz = static_cast<int32_t>(entries);
    *rows_max = rows;
}

spmv_status_t analyze_rowptr(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr,
                             const spmv_analyze_params_t& params_in, Analysis* out) try {
    Analysis& a = *out;
    a = Analysis{};
    spmv_analyze_params_t params = params_in;
    {
        int32_t bn = 0, rm = 0;
        default_tile_shape(m, nnz, &bn, &rm);
        if (params.block_nnz == 0) params.block_nnz = bn;
        if (params.rows_max == 0) params.rows_max = rm;
    }

    // ---- structure check + statistics + bin histogram, one sweep
    if (rowptr[0] != 0 || rowptr[m] != nnz) return SPMV_ERR_BAD_STRUCTURE;
    int64_t min_len = m > 0 ? INT64_MAX : 0, max_len = 0, n_empty = 0;
    for (int64_t i = 0; i < m; ++i) {
        const int64_t len = static_cast<int64_t>(rowptr[i + 1]) - rowptr[i];
        if (len < 0) return SPMV_ERR_BAD_STRUCTURE;
        min_len = std::min(min_len, len);
        max_len = std::max(max_len, len);
        n_empty += (len == 0);
        a.bin_count[length_bin(static_cast<uint32_t>(len))] += 1;
    }

    // ---- stable counting sort of the row ids by bin
    for (int b = 0; b < SPMV_NUM_BINS; ++b) a.bin_offset[b + 1] = a.bin_offset[b] + a.bin_count[b];
    a.bin_rows.resize(static_cast<size_t>(m));
    {
        int32_t cursor[SPMV_NUM_BINS];
        std::copy(a.bin_offset, a.bin_offset + SPMV_NUM_BINS, cursor);
        for (int64_t i = 0; i < m; ++i) {
            const uint32_t len = static_cast<uint32_t>(rowptr[i + 1] - rowptr[i]);
            a.bin_rows[static_cast<size_t>(cursor[length_bin(len)]++)] = static_cast<int32_t>(i);
        }
    }

    // ---- greedy row blocks: close the open block when the next row would overflow it
    a.row_blocks.clear();
    a.row_blocks.push_back(0);
    {
        int64_t open_first = 0;  // first row of the open block
        for (int64_t i = 0; i < m; ++i) {
            const int64_t with_row = static_cast<int64_t>(rowptr[i + 1]) - rowptr[open_first];
            const bool fits = (i - open_first) < params.rows_max && with_row <= params.block_nnz;
            if (!fits && i > open_first) {
                a.row_blocks.push_back(static_cast<int32_t>(i));
                open_first = i;
            }
            // A row that alone exceeds block_nnz opens a block at i and is cut off by the next row:
            // with_row for row i+1 is then > block_nnz as well, so the block closes at i+1.
        }
        if (m > 0) a.row_blocks.push_back(static_cast<int32_t>(m));
    }

    // ---- merge-path splits by bisection on each chunk's diagonal
    const int64_t T = m + nnz;
    const int64_t ipc = params.items_per_chunk;
    const int64_t P = (T + ipc - 1) / ipc;
    a.mp_row.resize(static_cast<size_t>(P + 1));
    a.mp_nz.resize(static_cast<size_t>(P + 1));
    for (int64_t p = 0; p <= P; ++p) {
        const int64_t d = std::min(p * ipc, T);
        const int64_t i = split_rows_on_diagonal(d, m, nnz, rowptr);
        a.mp_row[static_cast<size_t>(p)] = static_cast<int32_t>(i);
        a.mp_nz[static_cast<size_t>(p)] = static_cast<int32_t>(d - i);
    }

    // ---- plan
    int32_t plan = params.plan;
    if (plan == SPMV_PLAN_AUTO) {
        if (m == 0 || nnz == 0)
            plan = SPMV_PLAN_SCALAR;
        else if (max_len > params.block_nnz)
            plan = SPMV_PLAN_MERGE;
        else
            plan = SPMV_PLAN_ADAPTIVE;
    }
    int32_t lanes = params.vector_lanes;
    if (lanes == 0) {
        lanes = 2;
        if (m > 0) {
            const int64_t mean_up = (nnz + m - 1) / m;
            while (lanes < 64 && 8 * static_cast<int64_t>(lanes) < mean_up) lanes <<= 1;
        }
    }

    a.info.m = m;
    a.info.n = n;
    a.info.nnz = nnz;
    a.info.min_len = min_len;
    a.info.max_len = max_len;
    a.info.n_empty = n_empty;
    a.info.num_row_blocks = static_cast<int64_t>(a.row_blocks.size()) - 1;
    a.info.num_chunks = P;
    a.info.plan = plan;
    a.info.vector_lanes = lanes;
    a.info.block_nnz = params.block_nnz;
    a.info.rows_max = params.rows_max;
    a.info.items_per_chunk = params.items_per_chunk;
    return SPMV_OK;
} catch (const std::bad_alloc&) {
    return SPMV_ERR_ALLOC;
}

}  // namespace spmv

namespace spmv {

int64_t column_block_width(spmv_dtype_t dtype) { return (int64_t{4} << 20) / (dtype == SPMV_F32 ? 4 : 2); }

bool column_block_choice(int64_t n, int64_t nnz, spmv_dtype_t dtype, int32_t plan) {
    const int64_t width = column_block_width(dtype);
    const int64_t blocks = (n + width - 1) / width;
    return (plan == SPMV_PLAN_ADAPTIVE || plan == SPMV_PLAN_MERGE) && n > 2 * width && blocks <= 16 && nnz >= (int64_t{1} << 22);
}

bool window_choice(const int32_t* nv, int64_t nb, int64_t nnz, int64_t* total, int32_t* largest) {
    int64_t sum = 0;
    int32_t mx = 0;
    for (int64_t b = 0; b < nb; ++b) {
        sum += nv[b];
        if (nv[b] > mx) mx = nv[b];
    }
    *total = sum;
    *largest = mx;
    return nnz > 0 && mx <= SPMV_MAX_X_VECTORS && 4 * nb * static_cast<int64_t>(mx) <= nnz;
}

void spmm_row_order(int64_t m, const int32_t* rowptr, std::vector<int32_t>* rows) {
    // window after window, a counting sort: one pass to size the classes, one to place the rows
    // (ascending inside a class)
    auto key_of = [&](int64_t i) {
        const int64_t steps = (static_cast<int64_t>(rowptr[i + 1]) - rowptr[i] + 3) / 4;
        return static_cast<int>(steps < kSpmmMaxKey ? steps : kSpmmMaxKey);
    };
    rows->resize(static_cast<size_t>(m));
    for (int64_t w0 = 0; w0 < m; w0 += SPMV_SPMM_WINDOW) {
        const int64_t w1 = w0 + SPMV_SPMM_WINDOW < m ? w0 + SPMV_SPMM_WINDOW : m;
        int64_t count[kSpmmMaxKey + 1] = {};
        for (int64_t i = w0; i < w1; ++i) count[key_of(i)] += 1;
        int64_t cursor[kSpmmMaxKey + 1];
        int64_t run = w0;
        for (int k = kSpmmMaxKey; k >= 0; --k) {  // the largest key comes first
            cursor[k] = run;
            run += count[k];
        }
        for (int64_t i = w0; i < w1; ++i) (*rows)[static_cast<size_t>(cursor[key_of(i)]++)] = static_cast<int32_t>(i);
    }
}

bool spmm_packed_layout(int64_t m, int64_t nnz, const int32_t* rowptr, const int32_t* rows, std::vector<int32_t>* desc,
                        int64_t* num_blocks) {
    const int64_t groups = (m + 15) / 16;
    desc->assign(static_cast<size_t>(2 * groups + 2), 0);
    int64_t blocks = 0;
    for (int64_t g = 0; g < groups; ++g) {
        int64_t longest = 0;
        for (int64_t p = 16 * g; p < 16 * g + 16 && p < m; ++p) {
            const int64_t r = rows[p];
            longest = std::max<int64_t>(longest, static_cast<int64_t>(rowptr[r + 1]) - rowptr[r]);
        }
        // (when the count leaves the int32 range the layout is not used: see the return value)
        (*desc)[static_cast<size_t>(2 * g)] = static_cast<int32_t>(std::min<int64_t>(blocks, INT32_MAX));
        (*desc)[static_cast<size_t>(2 * g + 1)] = static_cast<int32_t>((longest + 3) / 4);
        blocks += (longest + 15) / 16;
    }
    (*desc)[static_cast<size_t>(2 * groups)] = static_cast<int32_t>(std::min<int64_t>(blocks, INT32_MAX));
    *num_blocks = blocks;
    return nnz > 0 && blocks * 256 <= 2 * nnz && blocks <= kSpmmMaxBlocks;
}

}  // namespace spmv
