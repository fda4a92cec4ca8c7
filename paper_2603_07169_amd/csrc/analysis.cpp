// Host-side analysis of the CSR row structure (row_offsets as laid out in App. C task 12).
#include "analysis.h"

#include <algorithm>
#include <climits>
#include <system_error>
#include <thread>
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

// Runs fn(t, begin, end) over [0, count) cut into contiguous, ascending pieces, one per thread.  Small
// inputs run on the calling thread; the passes below are memory-bound, so a handful of threads is enough.
constexpr int kMaxHostThreads = 8;
constexpr int64_t kRowsPerThread = int64_t{1} << 17;

inline int host_threads(int64_t count) {
    const int64_t by_size = count / kRowsPerThread;
    const int64_t hw = static_cast<int64_t>(std::thread::hardware_concurrency());
    const int64_t t = std::min<int64_t>({by_size, hw > 0 ? hw : 1, kMaxHostThreads});
    return static_cast<int>(t < 1 ? 1 : t);
}

template <typename F>
void parallel_pieces(int64_t count, int threads, F fn) {
    if (threads <= 1) {
        fn(0, int64_t{0}, count);
        return;
    }
    std::vector<std::thread> pool;
    pool.reserve(static_cast<size_t>(threads));
    int started = 0;
    try {
        for (; started < threads; ++started)
            pool.emplace_back([=]() { fn(started, count * started / threads, count * (started + 1) / threads); });
    } catch (const std::system_error&) {
        // no more threads to be had: the pieces not handed out yet are done here, in order
    }
    for (int t = started; t < threads; ++t) fn(t, count * t / threads, count * (t + 1) / threads);
    for (std::thread& th : pool) th.join();
}

}  // namespace

spmv_status_t resolve_params(const spmv_analyze_params_t* in, spmv_analyze_params_t* out) {
    spmv_analyze_params_t p{};
    if (in) p = *in;
    if (p.reserved != 0 || (p.prepare_spmm != 0 && p.prepare_spmm != 1)) return SPMV_ERR_INVALID_ARG;
    if (p.plan < SPMV_PLAN_AUTO || p.plan > SPMV_PLAN_SELL) return SPMV_ERR_INVALID_ARG;
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

void merge_path_splits(int64_t m, int64_t nnz, const int32_t* rowptr, int64_t ipc, std::vector<int32_t>* rows,
                       std::vector<int32_t>* entries) {
    const int64_t T = m + nnz;
    const int64_t P = (T + ipc - 1) / ipc;
    rows->resize(static_cast<size_t>(P + 1));
    entries->resize(static_cast<size_t>(P + 1));
    int32_t* mp_row = rows->data();
    int32_t* mp_nz = entries->data();
    parallel_pieces(P + 1, host_threads((P + 1) * 16), [=](int, int64_t lo, int64_t hi) {
        // The split on diagonal d + ipc lies at most ipc rows past the one on diagonal d (every row passed costs a step),
        // so after a piece's first split each bisection runs over a window of ipc rows: a few steps in memory just touched.
        int64_t prev = -1;
        for (int64_t p = lo; p < hi; ++p) {
            const int64_t d = std::min(p * ipc, T);
            int64_t i;
            if (prev < 0) {
                i = split_rows_on_diagonal(d, m, nnz, rowptr);
            } else {
                int64_t a = std::max<int64_t>(prev, d - nnz), b = std::min<int64_t>({d, m, prev + ipc});
                while (a < b) {
                    const int64_t mid = a + (b - a) / 2;
                    if (static_cast<int64_t>(rowptr[mid + 1]) + mid > d - 1)
                        b = mid;
                    else
                        a = mid + 1;
                }
                i = a;
            }
            prev = i;
            mp_row[p] = static_cast<int32_t>(i);
            mp_nz[p] = static_cast<int32_t>(d - i);
        }
    });
}

bool merge_path_splits_snapped(int64_t m, int64_t nnz, const int32_t* rowptr, int64_t ipc, int64_t snap, std::vector<int32_t>* rows,
                               std::vector<int32_t>* entries) {
    const int64_t T = m + nnz;
    rows->clear();
    entries->clear();
    rows->push_back(0);
    entries->push_back(0);
    bool cuts = false;
    int64_t i = 0, j = 0;
    while (i + j < T) {
        // the point ipc steps on: the rows finished there lie within ipc rows of the split before (a bisection as in
        // merge_path_splits)
        const int64_t d = std::min(i + j + ipc, T);
        int64_t a = std::max<int64_t>(i, d - nnz), b = std::min<int64_t>({d, m, i + ipc});
        while (a < b) {
            const int64_t mid = a + (b - a) / 2;
            if (static_cast<int64_t>(rowptr[mid + 1]) + mid > d - 1)
                b = mid;
            else
                a = mid + 1;
        }
        i = a;
        j = d - i;
        if (i < m && rowptr[i] < j) {  // entries of row i taken, row i not finished
            if (static_cast<int64_t>(rowptr[i + 1]) - rowptr[i] <= snap)
                j = rowptr[i];
            else
                cuts = true;
        }
        rows->push_back(static_cast<int32_t>(i));
        entries->push_back(static_cast<int32_t>(j));
    }
    return cuts;
}

void bin_rows_of(int64_t m, const int32_t* rowptr, std::vector<int32_t>* rows) {
    // a stable counting sort, in one thread: the lengths are counted per bin, then every row goes behind the rows
    // before it in its bin
    int64_t cursor[SPMV_NUM_BINS + 1] = {};
    for (int64_t i = 0; i < m; ++i) cursor[length_bin(static_cast<uint32_t>(rowptr[i + 1] - rowptr[i])) + 1] += 1;
    for (int b = 0; b < SPMV_NUM_BINS; ++b) cursor[b + 1] += cursor[b];
    rows->resize(static_cast<size_t>(m));
    for (int64_t i = 0; i < m; ++i)
        (*rows)[static_cast<size_t>(cursor[length_bin(static_cast<uint32_t>(rowptr[i + 1] - rowptr[i]))]++)] = static_cast<int32_t>(i);
}

spmv_status_t analyze_rowptr(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr,
                             const spmv_analyze_params_t& params_in, Analysis* out, bool want_bin_rows) try {
    Analysis& a = *out;
    a = Analysis{};
    spmv_analyze_params_t params = params_in;
    {
        int32_t bn = 0, rm = 0;
        default_tile_shape(m, nnz, &bn, &rm);
        if (params.block_nnz == 0) params.block_nnz = bn;
        if (params.rows_max == 0) params.rows_max = rm;
    }

    // ---- structure check + statistics + bin histogram, one sweep (per thread: its own rows and counts)
    if (rowptr[0] != 0 || rowptr[m] != nnz) return SPMV_ERR_BAD_STRUCTURE;
    const int threads = host_threads(m);
    struct Part {
        int64_t min_len = INT64_MAX, max_len = 0, n_empty = 0;
        bool bad = false;
        int32_t hist[SPMV_NUM_BINS] = {};
    };
    std::vector<Part> parts(static_cast<size_t>(threads));
    parallel_pieces(m, threads, [&](int t, int64_t lo, int64_t hi) {
        Part& q = parts[static_cast<size_t>(t)];
        for (int64_t i = lo; i < hi; ++i) {
            const int64_t len = static_cast<int64_t>(rowptr[i + 1]) - rowptr[i];
            if (len < 0) {
                q.bad = true;
                return;
            }
            q.min_len = std::min(q.min_len, len);
            q.max_len = std::max(q.max_len, len);
            q.n_empty += (len == 0);
            q.hist[length_bin(static_cast<uint32_t>(len))] += 1;
        }
    });
    int64_t min_len = m > 0 ? INT64_MAX : 0, max_len = 0, n_empty = 0;
    for (const Part& q : parts) {
        if (q.bad) return SPMV_ERR_BAD_STRUCTURE;
        min_len = std::min(min_len, q.min_len);
        max_len = std::max(max_len, q.max_len);
        n_empty += q.n_empty;
        for (int b = 0; b < SPMV_NUM_BINS; ++b) a.bin_count[b] += q.hist[b];
    }

    // ---- stable counting sort of the row ids by bin: thread t writes behind the rows of the threads before it.
    // Only the BINNED plan's kernels read the list, so it is built when that plan is asked for (want_bin_rows); for any
    // other plan bin_rows_of() builds it when the caller reads the analysis back.
    for (int b = 0; b < SPMV_NUM_BINS; ++b) a.bin_offset[b + 1] = a.bin_offset[b] + a.bin_count[b];
    if (want_bin_rows) {
        a.bin_rows.resize(static_cast<size_t>(m));
        std::vector<int32_t> first(static_cast<size_t>(threads) * SPMV_NUM_BINS);
        for (int b = 0; b < SPMV_NUM_BINS; ++b) {
            int32_t at = a.bin_offset[b];
            for (int t = 0; t < threads; ++t) {
                first[static_cast<size_t>(t) * SPMV_NUM_BINS + b] = at;
                at += parts[static_cast<size_t>(t)].hist[b];
            }
        }
        int32_t* bin_rows = a.bin_rows.data();
        parallel_pieces(m, threads, [&, bin_rows](int t, int64_t lo, int64_t hi) {
            int32_t cursor[SPMV_NUM_BINS];
            std::copy(first.begin() + static_cast<size_t>(t) * SPMV_NUM_BINS,
                      first.begin() + static_cast<size_t>(t + 1) * SPMV_NUM_BINS, cursor);
            for (int64_t i = lo; i < hi; ++i) {
                const uint32_t len = static_cast<uint32_t>(rowptr[i + 1] - rowptr[i]);
                bin_rows[cursor[length_bin(len)]++] = static_cast<int32_t>(i);
            }
        });
    }

    // ---- greedy row blocks.  The block opened at row s takes rows while it has fewer than rows_max of
    // them and stays within block_nnz entries, i.e. it ends at the last r with r - s <= rows_max and
    // rowptr[r] - rowptr[s] <= block_nnz (found by bisection: rowptr does not decrease), and a row that
    // alone exceeds block_nnz stands alone.
    a.row_blocks.clear();
    a.row_blocks.push_back(0);
    for (int64_t s = 0; s < m;) {
        const int64_t limit = static_cast<int64_t>(rowptr[s]) + params.block_nnz;
        const int64_t cap = std::min<int64_t>(m, s + params.rows_max);
        // first index in (s, cap] whose offset exceeds the limit, or cap + 1
        const int32_t* past = std::upper_bound(rowptr + s + 1, rowptr + cap + 1, limit,
                                               [](int64_t v, int32_t off) { return v < static_cast<int64_t>(off); });
        int64_t end = (past - rowptr) - 1;
        if (end == s) end = s + 1;
        a.row_blocks.push_back(static_cast<int32_t>(end));
        s = end;
    }

    // ---- merge-path splits by bisection on each chunk's diagonal
    merge_path_splits(m, nnz, rowptr, params.items_per_chunk, &a.mp_row, &a.mp_nz);
    const int64_t P = static_cast<int64_t>(a.mp_row.size()) - 1;

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

bool columns_scattered(int64_t x_vectors_counted, int64_t entries_counted) {
    return x_vectors_counted >= 0 && 4 * x_vectors_counted >= 3 * entries_counted;
}

bool column_block_sizes_ok(int64_t n, int64_t nnz, spmv_dtype_t dtype) {
    const int64_t width = column_block_width(dtype);
    const int64_t blocks = (n + width - 1) / width;
    return n > 2 * width && blocks <= 16 && nnz >= (int64_t{1} << 22);
}

bool column_block_choice(int64_t n, int64_t nnz, spmv_dtype_t dtype, int32_t plan, int64_t x_vectors_counted, int64_t entries_counted) {
    // clustered columns keep the row-wise gathers cheap, whatever the size of x: only scattered ones are regrouped
    return (plan == SPMV_PLAN_ADAPTIVE || plan == SPMV_PLAN_MERGE) && column_block_sizes_ok(n, nnz, dtype) &&
           columns_scattered(x_vectors_counted, entries_counted);
}

int two_phase_shift(int64_t n) {
    (void)n;
    return 14;
}

bool two_phase_sizes_ok(int64_t m, int64_t n, int64_t nnz, spmv_dtype_t dtype) {
    // 1.5 * 2^22 entries or more: below that the row-wise kernels' gathers (one address-unit slot each, wherever x
    // lies) cost less than writing the products out and reading them back over three launches; x of 256 KiB or more
    // (measured down to there: 80 against 64 us on 16.8 M entries)
    if (16 * n < column_block_width(dtype) || nnz < 3 * (int64_t{1} << 21)) return false;
    const int64_t C = (n + (int64_t{1} << two_phase_shift(n)) - 1) >> two_phase_shift(n);
    const int64_t P = (m + nnz + kTwoPhaseItems - 1) / kTwoPhaseItems;
    // tiles of at least eight entries on average: the padding to whole groups of four then stays below a fifth
    return C <= 65535 && C * P <= kTwoPhaseMaxTiles && 8 * C * P <= nnz;
}

bool two_phase_choice(int64_t m, int64_t n, int64_t nnz, spmv_dtype_t dtype, int32_t plan, int64_t x_vectors_counted,
                      int64_t entries_counted) {
    if (!(plan == SPMV_PLAN_ADAPTIVE || plan == SPMV_PLAN_MERGE)) return false;
    // columns that cluster (a band, a stencil too wide for the x windows) keep the row-wise gathers cheap:
    // neighbouring lanes share cache lines.  Only scattered columns go through the two passes.
    return columns_scattered(x_vectors_counted, entries_counted) && two_phase_sizes_ok(m, n, nnz, dtype);
}

int two_phase_group_shift(spmv_dtype_t dtype) { return dtype == SPMV_BF16 ? 12 : 11; }

bool grouped_two_phase_choice(int64_t m, int64_t n, int64_t nnz, spmv_dtype_t dtype, int32_t plan, bool group_aligned,
                              int64_t x_vectors_counted, int64_t entries_counted) {
    if (!(plan == SPMV_PLAN_ADAPTIVE || plan == SPMV_PLAN_MERGE) || !group_aligned) return false;
    const int64_t elem_bytes = dtype == SPMV_F32 ? 4 : 2, vec_elems = 16 / elem_bytes;
    if (x_vectors_counted < 0 || 4 * vec_elems * x_vectors_counted < 3 * entries_counted) return false;
    const int shift = two_phase_group_shift(dtype);
    const int64_t groups = nnz / kTpGroup, cols = (n + kTpGroup - 1) / kTpGroup;
    const int64_t C = (cols + (int64_t{1} << shift) - 1) >> shift;
    const int64_t P = (m + groups + kTwoPhaseItems - 1) / kTwoPhaseItems;
    return n * elem_bytes >= (int64_t{1} << 20) && groups >= 3 * (int64_t{1} << 21) && C <= 65535 && C * P <= kTwoPhaseMaxTiles &&
           8 * C * P <= groups;
}

int32_t two_phase_piece_groups(int64_t C, const int32_t* block_first, int32_t resident, int32_t waves) {
    const int64_t total = block_first[C] / 4;
    auto pieces_at = [&](int64_t cap) {
        int64_t q = 0;
        for (int64_t c = 0; c < C; ++c) q += (block_first[c + 1] / 4 - block_first[c] / 4 + cap - 1) / cap;
        return q;
    };
    if (resident < 1) resident = 1;
    int64_t k = total >= static_cast<int64_t>(waves) * resident * kTwoPhasePieceFloor ? waves : 1;
    while (pieces_at(kTwoPhasePieceGroups) > k * resident) ++k;
    // pieces_at falls as the cap grows: the smallest cap that keeps within k rounds
    int64_t lo = 1, hi = kTwoPhasePieceGroups;
    while (lo < hi) {
        const int64_t mid = (lo + hi) / 2;
        if (pieces_at(mid) <= k * resident)
            hi = mid;
        else
            lo = mid + 1;
    }
    return static_cast<int32_t>(lo < kTwoPhasePieceFloor ? kTwoPhasePieceFloor : lo);
}

void two_phase_pieces(int64_t C, const int32_t* block_first, int32_t piece_groups, std::vector<int32_t>* piece_c,
                      std::vector<int32_t>* piece_g) {
    piece_c->clear();
    piece_g->clear();
    for (int64_t c = 0; c < C; ++c) {
        // the block's groups in the fewest pieces the cap allows, all of one size (the last may be shorter)
        const int64_t first_group = block_first[c] / 4, groups = block_first[c + 1] / 4 - first_group;
        const int64_t pieces = (groups + piece_groups - 1) / piece_groups;
        const int64_t size = pieces > 0 ? (groups + pieces - 1) / pieces : 1;
        for (int64_t g = first_group; g < first_group + groups; g += size) {
            piece_c->push_back(static_cast<int32_t>(c));
            piece_g->push_back(static_cast<int32_t>(g));
        }
    }
    piece_g->push_back(block_first[C] / 4);
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
