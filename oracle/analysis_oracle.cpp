// CPU oracle for the integer outputs of the analysis step.  TEST INFRASTRUCTURE ONLY.
//
// The GPU library's spmv_csr_analyze() derives, from the CSR row offsets alone, the row
// statistics, a length-binned row list, a row-block partition and a merge-path split.
// The definitions are restated here in their most literal form (counting loops, a
// sequential greedy scan, a step-by-step merge walk) so that each can be checked by eye.
// Nothing here is shared with, or called by, the library; results must match bit for bit.
//
// The paper fixes only the CSR layout (App. C task 12: row_offsets holds "the starting
// index of each row", length rows+1).  The partitions themselves are this project's
// definitions; they are spelled out in the function comments below.

#include <algorithm>
#include <cstdint>
#include <vector>

extern "C" {

// ---- row statistics ---------------------------------------------------------------
// out[0] = min row length, out[1] = max row length, out[2] = number of empty rows.
// m == 0 gives 0, 0, 0.
void oracle_row_stats(int64_t m, const int32_t* rowptr, int64_t* out) {
    int64_t mn = 0, mx = 0, empty = 0;
    for (int64_t i = 0; i < m; ++i) {
        const int64_t len = static_cast<int64_t>(rowptr[i + 1]) - rowptr[i];
        if (i == 0 || len < mn) mn = len;
        if (i == 0 || len > mx) mx = len;
        if (len == 0) ++empty;
    }
    out[0] = mn;
    out[1] = mx;
    out[2] = empty;
}

// ---- length bins ------------------------------------------------------------------
// bin(0) = 0; for len >= 1, bin(len) = the smallest b >= 1 with 2^(b-1) >= len
// (1->1, 2->2, 3..4->3, 5..8->4, 9..16->5, ...).  33 bins cover every int32 length.
static int bin_of(int64_t len) {
    if (len == 0) return 0;
    int b = 1;
    int64_t cap = 1;
    while (cap < len) {
        cap *= 2;
        ++b;
    }
    return b;
}

// bin_count[33], bin_offset[34] = exclusive prefix sums of bin_count,
// bin_rows[m] = row ids grouped by bin, ascending row id inside every bin.
void oracle_row_bins(int64_t m, const int32_t* rowptr, int32_t* bin_count, int32_t* bin_offset, int32_t* bin_rows) {
    for (int b = 0; b < 33; ++b) bin_count[b] = 0;
    for (int64_t i = 0; i < m; ++i) bin_count[bin_of(static_cast<int64_t>(rowptr[i + 1]) - rowptr[i])] += 1;
    bin_offset[0] = 0;
    for (int b = 0; b < 33; ++b) bin_offset[b + 1] = bin_offset[b] + bin_count[b];
    // one pass per bin, rows visited in ascending order: trivially stable
    int64_t w = 0;
    for (int b = 0; b < 33; ++b)
        for (int64_t i = 0; i < m; ++i)
            if (bin_of(static_cast<int64_t>(rowptr[i + 1]) - rowptr[i]) == b) bin_rows[w++] = static_cast<int32_t>(i);
}

// ---- row blocks -------------------------------------------------------------------
// Greedy left-to-right partition of the rows into contiguous blocks.  A block takes the
// next row while it has fewer than rows_max rows and the row still fits under block_nnz
// stored entries; a row longer than block_nnz forms a block of its own.
// Writes block boundaries (first row of each block, then m) to out; returns the number
// of blocks nb (out holds nb+1 entries; m == 0 gives nb = 0 and out = [0]).
// `out` must have room for m+1 entries.
int64_t oracle_row_blocks(int64_t m, const int32_t* rowptr, int32_t block_nnz, int32_t rows_max, int32_t* out) {
    int64_t nb = 0;
    out[0] = 0;
    int64_t r = 0;
    while (r < m) {
        const int64_t first = r;
        int64_t held = 0;
        while (r < m) {
            const int64_t len = static_cast<int64_t>(rowptr[r + 1]) - rowptr[r];
            if (r - first >= rows_max) break;
            if (held + len > block_nnz) break;
            held += len;
            ++r;
        }
        if (r == first) ++r;  // a single row that is longer than block_nnz
        ++nb;
        out[nb] = static_cast<int32_t>(r);
    }
    return nb;
}

// ---- merge path -------------------------------------------------------------------
// The merge path interleaves two sorted lists: the m row ends (row i ends at rowptr[i+1])
// and the nnz entry positions 0..nnz-1.  Standing at (i rows finished, j entries taken),
// the next step takes entry j if it belongs to row i (i < m, j < nnz, rowptr[i+1] > j),
// otherwise it finishes row i.  The path has T = m + nnz steps.  Split p (p = 0..P,
// P = ceil(T / ipc)) is the point reached after min(p*ipc, T) steps.
// Writes mp_row[P+1], mp_nz[P+1]; returns P.
int64_t oracle_merge_path(int64_t m, int64_t nnz, const int32_t* rowptr, int32_t ipc, int32_t* mp_row, int32_t* mp_nz) {
    const int64_t T = m + nnz;
    const int64_t P = (T + ipc - 1) / ipc;
    int64_t i = 0, j = 0, p = 0;
    for (int64_t step = 0;; ++step) {
        if (step == p * ipc || step == T) {
            mp_row[p] = static_cast<int32_t>(i);
            mp_nz[p] = static_cast<int32_t>(j);
            ++p;
        }
        if (step == T) break;
        if (i < m && j < nnz && rowptr[i + 1] > j)
            ++j;
        else
            ++i;
    }
    return P;
}

// The chunks of the two-pass plan: the same walk, cut every ipc steps, except that a cut which falls inside a row of at
// most `snap` entries - some of its entries taken, the row not finished - is moved back to that row's first entry: the
// chunk ends there, and the next ipc steps are counted from there.  A chunk then cuts only rows longer than snap
// (snap = 0: the plain merge path; snap < ipc, so every chunk moves forward).  Writes the splits to row[], nz[] (room for
// (m + nnz) / (ipc - snap) + 2 entries); returns P, the number of chunks.
int64_t oracle_merge_path_snapped(int64_t m, int64_t nnz, const int32_t* rowptr, int32_t ipc, int32_t snap, int32_t* row,
                                  int32_t* nz) {
    const int64_t T = m + nnz;
    int64_t i = 0, j = 0, p = 0, in_chunk = 0;
    row[0] = 0;
    nz[0] = 0;
    while (i + j < T) {
        if (i < m && j < nnz && rowptr[i + 1] > j)
            ++j;
        else
            ++i;
        ++in_chunk;
        if (in_chunk == ipc || i + j == T) {
            // inside row i: back to its first entry (the next chunk walks those steps again)
            if (i < m && rowptr[i] < j && j <= rowptr[i + 1] && rowptr[i + 1] - rowptr[i] <= snap) j = rowptr[i];
            ++p;
            row[p] = static_cast<int32_t>(i);
            nz[p] = static_cast<int32_t>(j);
            in_chunk = 0;
        }
    }
    return p;
}

// ---- default row-block shape ---------------------------------------------------------
// Used when the caller leaves block_nnz / rows_max at 0.  Matrices of at most 2^20 entries
// (or no rows): 1024 entries, 64 rows.  Otherwise, with mean = ceil(nnz / m) and G the
// largest power of two <= 64 such that 16*G <= mean + 15 (G doubles while 16*G < mean):
// rows_max = 256 / G, block_nnz = rows_max * mean rounded up to a multiple of 8, then
// clamped to [2048, 8192].
void oracle_tile_shape(int64_t m, int64_t nnz, int32_t* block_nnz, int32_t* rows_max) {
    if (m <= 0 || nnz <= 1048576) {
        *block_nnz = 1024;
        *rows_max = 64;
        return;
    }
    const int64_t mean = (nnz + m - 1) / m;
    int64_t G = 1;
    while (G < 64 && 16 * G < mean) G *= 2;
    const int64_t rows = 256 / G;
    int64_t entries = rows * mean;
    while (entries % 8 != 0) ++entries;
    if (entries < 2048) entries = 2048;
    if (entries > 8192) entries = 8192;
    *block_nnz = static_cast<int32_t>(entries);
    *rows_max = static_cast<int32_t>(rows);
}

// ---- plan -------------------------------------------------------------------------
// Plans: 1 scalar (one lane per row), 2 vector (a group of lanes per row), 3 binned
// (scalar/vector per length bin), 4 adaptive (row blocks through LDS), 5 merge (merge-path
// chunks + carry fix-up).  The automatic choice is a pure integer function:
//   no rows or no entries                    -> 1
//   some row is longer than one row block    -> 5
//   otherwise                                -> 4
int32_t oracle_plan(int64_t m, int64_t nnz, int64_t max_len, int32_t block_nnz) {
    if (m == 0 || nnz == 0) return 1;
    if (max_len > block_nnz) return 5;
    return 4;
}

// Lanes per row of the vector plan: the smallest power of two G in [2, 64] with
// 8*G >= ceil(nnz / m)  (every lane then takes about eight entries, one 128-bit load of bf16
// values); 64 when none is.
int32_t oracle_vector_lanes(int64_t m, int64_t nnz) {
    if (m == 0) return 2;
    const int64_t mean_up = (nnz + m - 1) / m;
    int32_t G = 2;
    while (G < 64 && 8 * static_cast<int64_t>(G) < mean_up) G *= 2;
    return G;
}

// ---- x windows of row blocks --------------------------------------------------------
// A row block touches x only at its entries' columns.  Cut x into aligned vectors of
// `vec_elems` elements (16 bytes: 4 binary32 or 8 bf16 values).  For block b,
//   keys_b      = the distinct values of colidx[k] / vec_elems over the block's entries,
//                 in ascending order;
//   nv[b]       = how many there are;
//   xv_start    = all blocks' key lists one after the other, each key times vec_elems
//                 (the index of the vector's first element);
//   lidx[k]     = rank(colidx[k] / vec_elems in keys_b) * vec_elems + colidx[k] % vec_elems,
//                 the position of x[colidx[k]] once the block's vectors are laid out back to
//                 back in that order.
// A block with more than block_nnz entries (a single long row) takes no vectors and its
// lidx entries are 0.  xv_start and lidx may be null (count only).  Returns sum of nv.
int64_t oracle_x_windows(int64_t nb, const int32_t* row_blocks, const int32_t* rowptr, const int32_t* colidx,
                         int32_t block_nnz, int32_t vec_elems, int32_t* nv, int32_t* xv_start, uint16_t* lidx) {
    int64_t total = 0;
    for (int64_t b = 0; b < nb; ++b) {
        const int64_t k0 = rowptr[row_blocks[b]], k1 = rowptr[row_blocks[b + 1]];
        if (k1 - k0 > block_nnz) {
            nv[b] = 0;
            if (lidx)
                for (int64_t k = k0; k < k1; ++k) lidx[k] = 0;
            continue;
        }
        std::vector<int32_t> keys;
        for (int64_t k = k0; k < k1; ++k) keys.push_back(colidx[k] / vec_elems);
        std::sort(keys.begin(), keys.end());
        keys.erase(std::unique(keys.begin(), keys.end()), keys.end());
        nv[b] = static_cast<int32_t>(keys.size());
        if (xv_start)
            for (size_t j = 0; j < keys.size(); ++j) xv_start[total + static_cast<int64_t>(j)] = keys[j] * vec_elems;
        if (lidx)
            for (int64_t k = k0; k < k1; ++k) {
                const int32_t key = colidx[k] / vec_elems;
                const int64_t rank = std::find(keys.begin(), keys.end(), key) - keys.begin();
                lidx[k] = static_cast<uint16_t>(rank * vec_elems + colidx[k] % vec_elems);
            }
        total += static_cast<int64_t>(keys.size());
    }
    return total;
}

// Whether the automatic plan serves x from those windows.  The kernel reads every block's list
// at a fixed stride of V = the largest nv, so the lists cost nb * V words: V must fit the
// kernel's buffer (at most max_vectors) and 4 * nb * V must not exceed the entry count.
int32_t oracle_window_choice(int64_t nb, const int32_t* nv, int64_t nnz, int32_t max_vectors) {
    if (nnz == 0) return 0;
    int64_t V = 0;
    for (int64_t b = 0; b < nb; ++b)
        if (nv[b] > V) V = nv[b];
    if (V > max_vectors) return 0;
    return 4 * nb * V <= nnz ? 1 : 0;
}

// ---- column blocks ----------------------------------------------------------------------
// Columns are cut into blocks of `width` consecutive columns (block b = columns b*width ..
// (b+1)*width - 1).  The entries are regrouped block after block; inside a block they keep the
// order they have in the row-major arrays (row after row, and inside a row the stored order).
//   cb_ptr[b]  = number of entries in blocks before b  (C + 1 values, C = ceil(n / width))
//   cb_row[k]  = row of the k-th regrouped entry
//   cb_col[k]  = its column minus the first column of its block
//   cb_src[k]  = its position in the original arrays (so its value is vals[cb_src[k]])
// Returns C.
int64_t oracle_column_blocks(int64_t m, int64_t n, const int32_t* rowptr, const int32_t* colidx, int64_t width,
                             int32_t* cb_ptr, int32_t* cb_row, int32_t* cb_col, int32_t* cb_src) {
    const int64_t C = (n + width - 1) / width;
    int64_t k = 0;
    for (int64_t b = 0; b < C; ++b) {
        cb_ptr[b] = static_cast<int32_t>(k);
        for (int64_t i = 0; i < m; ++i)
            for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e)
                if (colidx[e] / width == b) {
                    cb_row[k] = static_cast<int32_t>(i);
                    cb_col[k] = static_cast<int32_t>(colidx[e] - b * width);
                    cb_src[k] = static_cast<int32_t>(e);
                    ++k;
                }
    }
    cb_ptr[C] = static_cast<int32_t>(k);
    return C;
}

// Block width and the automatic choice.  A block of x is 4 MiB (2^20 binary32 or 2^21 bf16
// columns: what one die's L2 holds).  The column-blocked plan is taken when the matrix would
// otherwise run on row blocks or merge-path chunks with x gathered from memory (plan 4 or 5),
// x is larger than two blocks, there are at most 16 blocks and at least 2^22 entries, and the columns
// are scattered (oracle_scatter_counts: three distinct x vectors per four counted entries, or more).
int64_t oracle_column_block_width(int32_t elem_bytes) { return (int64_t{4} << 20) / elem_bytes; }

int32_t oracle_column_block_choice(int64_t n, int64_t nnz, int32_t elem_bytes, int32_t plan, int64_t vectors, int64_t entries) {
    const int64_t width = oracle_column_block_width(elem_bytes);
    const int64_t C = (n + width - 1) / width;
    if (vectors < 0 || 4 * vectors < 3 * entries) return 0;  // clustered columns (or none counted): the row-wise plan stays
    return ((plan == 4 || plan == 5) && n > 2 * width && C <= 16 && nnz >= (int64_t{1} << 22)) ? 1 : 0;
}

// The window positions are grouped when every row block starts at a multiple of eight entries and every
// whole aligned group of eight entries 8g .. 8g+7 sits at eight consecutive positions (rows made of aligned
// runs of columns).  Entries past the last whole group do not matter.
int32_t oracle_lidx_grouped(int64_t nnz, const uint16_t* lidx, int64_t nb, const int32_t* row_blocks, const int32_t* rowptr) {
    if (nnz < 8) return 0;
    for (int64_t b = 0; b < nb; ++b)
        if (rowptr[row_blocks[b]] % 8 != 0) return 0;
    for (int64_t g = 0; g < nnz / 8; ++g)
        for (int64_t i = 1; i < 8; ++i)
            if (lidx[8 * g + i] != lidx[8 * g] + i) return 0;
    return 1;
}

// ---- row patterns of the window positions -----------------------------------------------
// Inside a row block of a stencil the window positions of one row are those of the row before, moved on by a
// constant.  Row i of a block (entries k_i .. k_i + len_i - 1) has
//   base_i = lidx[k_i]  (0 for an empty row),   rel_i[j] = lidx[k_i + j] - base_i   (j = 0 .. len_i - 1).
// A run is a stretch of consecutive rows of the block, found greedily from the block's first row on: the run that
// holds row i - 1 also takes row i when len_i = len_{i-1}, rel_i = rel_{i-1} and, if the run already has two rows
// or more, base_i - base_{i-1} equals the step between those (the run's stride; a run of one row has stride 0).
// The block is patterned when it is staged (at most block_nnz entries), no row is longer than max_len, no rel is
// negative (a row's first entry sits lowest in the window) and it has at most max_runs runs.  Then, for its runs
// r = 0 .. n_runs[b] - 1, slot q = b * max_runs + r holds run_rows[q] (rows in the run), run_len[q] (entries per row),
// run_base[q] (base of its first row) and run_stride[q]; the block's pattern list is rel of the first row of run 0,
// then of run 1, ..., pat_ptr[b] .. pat_ptr[b+1] - 1 in pat (which may be null: sizes only).  A block that is not
// patterned has n_runs 0, zeros in its slots and no pattern entries.  Returns the entries held by patterned blocks.
int64_t oracle_row_patterns(int64_t nb, const int32_t* row_blocks, const int32_t* rowptr, const uint16_t* lidx, int32_t block_nnz,
                            int32_t max_runs, int32_t max_len, int32_t* n_runs, int32_t* run_rows, int32_t* run_len,
                            int32_t* run_base, int32_t* run_stride, int32_t* pat_ptr, uint16_t* pat) {
    int64_t covered = 0;
    pat_ptr[0] = 0;
    for (int64_t b = 0; b < nb; ++b) {
        const int64_t first = row_blocks[b], last = row_blocks[b + 1];
        for (int r = 0; r < max_runs; ++r) run_rows[b * max_runs + r] = run_len[b * max_runs + r] = run_base[b * max_runs + r] = run_stride[b * max_runs + r] = 0;
        n_runs[b] = 0;
        pat_ptr[b + 1] = pat_ptr[b];
        const int64_t entries = static_cast<int64_t>(rowptr[last]) - rowptr[first];
        bool ok = entries <= block_nnz;
        // the rows one by one: base and rel of each
        std::vector<int64_t> base;
        std::vector<std::vector<int64_t>> rel;
        for (int64_t i = first; i < last && ok; ++i) {
            const int64_t k = rowptr[i], len = static_cast<int64_t>(rowptr[i + 1]) - k;
            if (len > max_len) ok = false;
            base.push_back(len > 0 ? lidx[k] : 0);
            rel.emplace_back();
            for (int64_t j = 0; j < len && ok; ++j) {
                const int64_t d = static_cast<int64_t>(lidx[k + j]) - base.back();
                if (d < 0) ok = false;
                rel.back().push_back(d);
            }
        }
        if (!ok) continue;
        // greedy runs
        std::vector<int64_t> start;  // first row (within the block) of every run
        std::vector<int64_t> stride;
        for (int64_t i = 0; i < last - first; ++i) {
            bool joins = false;
            if (!start.empty() && rel[i] == rel[i - 1]) {
                const int64_t rows_so_far = i - start.back();
                const int64_t step = base[i] - base[i - 1];
                if (rows_so_far == 1) {
                    joins = true;
                    stride.back() = step;
                } else if (step == stride.back()) {
                    joins = true;
                }
            }
            if (!joins) {
                start.push_back(i);
                stride.push_back(0);
            }
        }
        if (static_cast<int64_t>(start.size()) > max_runs) continue;
        n_runs[b] = static_cast<int32_t>(start.size());
        for (size_t r = 0; r < start.size(); ++r) {
            const int64_t end = r + 1 < start.size() ? start[r + 1] : last - first;
            const int64_t q = b * max_runs + static_cast<int64_t>(r);
            run_rows[q] = static_cast<int32_t>(end - start[r]);
            run_len[q] = static_cast<int32_t>(rel[start[r]].size());
            run_base[q] = static_cast<int32_t>(base[start[r]]);
            run_stride[q] = static_cast<int32_t>(stride[r]);
            for (int64_t d : rel[start[r]]) {
                if (pat) pat[pat_ptr[b + 1]] = static_cast<uint16_t>(d);
                pat_ptr[b + 1] += 1;
            }
        }
        covered += entries;
    }
    return covered;
}

// The kernel that works from the patterns is taken when the patterned blocks hold at least half of the entries.
int32_t oracle_pattern_choice(int64_t nnz, int64_t covered) { return (nnz > 0 && 2 * covered >= nnz) ? 1 : 0; }

// ---- the two-pass layout ---------------------------------------------------------------
// Column blocks of 2^shift columns (C of them); chunks = the stretches of the CSR entry list
// between consecutive splits of oracle_merge_path_snapped (every `items` steps, rows of at most `snap` entries kept whole; P of them).  Tile (c, p) =
// the entries of column block c in chunk p, in CSR order, padded to a multiple of four slots.
// Multiply order: tiles by (c, p); reduce order: tiles by (p, c).  Sizes first: S = padded slots,
// Q = pieces (every column block's groups of four slots cut evenly into the fewest runs of at most piece_groups).
void oracle_two_phase_sizes(int64_t m, int64_t n, const int32_t* rowptr, const int32_t* colidx, int32_t shift, int32_t items,
                            int32_t snap, int32_t piece_groups, int64_t* S, int64_t* Q, int64_t* P_out, int64_t* C_out) {
    const int64_t nnz = rowptr[m];
    const int64_t C = (n + (int64_t{1} << shift) - 1) >> shift;
    const size_t room = static_cast<size_t>((m + nnz) / (items - snap) + 2);
    std::vector<int32_t> sr(room), sz(room);
    const int64_t P = oracle_merge_path_snapped(m, nnz, rowptr, items, snap, sr.data(), sz.data());
    std::vector<int64_t> cnt(static_cast<size_t>(C * P), 0);
    int64_t p = 0;
    for (int64_t k = 0; k < nnz; ++k) {
        while (sz[static_cast<size_t>(p + 1)] <= k) ++p;  // the chunk whose stretch holds entry k
        ++cnt[static_cast<size_t>((colidx[k] >> shift) * P + p)];
    }
    int64_t slots = 0, pieces = 0;
    for (int64_t c = 0; c < C; ++c) {
        int64_t groups = 0;
        for (int64_t q = 0; q < P; ++q) groups += (cnt[static_cast<size_t>(c * P + q)] + 3) / 4;
        slots += 4 * groups;
        pieces += (groups + piece_groups - 1) / piece_groups;
    }
    *S = slots;
    *Q = pieces;
    *P_out = P;
    *C_out = C;
}

// Fills tp_row[P+1], tp_nz[P+1] (room for (m + nnz) / (items - snap) + 2), piece_c[Q], piece_g[Q+1], chunk_g[P+1], col[S],
// src[S], from[S/4], pos[S].
// from[g] = the group of the multiply order whose four slots are group g of the reduce order (the products stay where
// the multiply pass made them; the reduce pass fetches them).
void oracle_two_phase_layout(int64_t m, int64_t n, const int32_t* rowptr, const int32_t* colidx, int32_t shift, int32_t items,
                             int32_t snap, int32_t piece_groups, int32_t* tp_row, int32_t* tp_nz, int32_t* piece_c, int32_t* piece_g,
                             int32_t* chunk_g, uint16_t* col, int32_t* src, int32_t* from, uint16_t* pos) {
    const int64_t nnz = rowptr[m];
    const int64_t C = (n + (int64_t{1} << shift) - 1) >> shift;
    const int64_t P = oracle_merge_path_snapped(m, nnz, rowptr, items, snap, tp_row, tp_nz);
    std::vector<int64_t> cnt(static_cast<size_t>(C * P), 0), start1(static_cast<size_t>(C * P)), start2(static_cast<size_t>(C * P));
    std::vector<int64_t> chunk_of(static_cast<size_t>(nnz));
    int64_t p = 0;
    for (int64_t k = 0; k < nnz; ++k) {
        while (tp_nz[p + 1] <= k) ++p;
        chunk_of[static_cast<size_t>(k)] = p;
        ++cnt[static_cast<size_t>((colidx[k] >> shift) * P + p)];
    }
    // where every tile starts in the two orders, and the pieces
    int64_t slot = 0, q = 0;
    for (int64_t c = 0; c < C; ++c) {
        const int64_t block_first_group = slot / 4;
        for (int64_t pp = 0; pp < P; ++pp) {
            start1[static_cast<size_t>(c * P + pp)] = slot;
            slot += (cnt[static_cast<size_t>(c * P + pp)] + 3) / 4 * 4;
        }
        // the block's groups go into the fewest pieces that hold at most piece_groups each, cut evenly:
        // piece i starts i * ceil(groups / pieces) groups into the block
        const int64_t groups = slot / 4 - block_first_group;
        const int64_t pieces = (groups + piece_groups - 1) / piece_groups;
        for (int64_t i = 0; i < pieces; ++i) {
            piece_c[q] = static_cast<int32_t>(c);
            piece_g[q] = static_cast<int32_t>(block_first_group + i * ((groups + pieces - 1) / pieces));
            ++q;
        }
    }
    const int64_t S = slot;
    piece_g[q] = static_cast<int32_t>(S / 4);
    slot = 0;
    for (int64_t pp = 0; pp < P; ++pp) {
        chunk_g[pp] = static_cast<int32_t>(slot / 4);
        for (int64_t c = 0; c < C; ++c) {
            start2[static_cast<size_t>(c * P + pp)] = slot;
            slot += (cnt[static_cast<size_t>(c * P + pp)] + 3) / 4 * 4;
        }
    }
    chunk_g[P] = static_cast<int32_t>(slot / 4);
    // padding everywhere, then the entries in CSR order, each to the next free slot of its tile
    for (int64_t s = 0; s < S; ++s) {
        col[s] = static_cast<uint16_t>(1u << shift);
        src[s] = -1;
        pos[s] = 0xFFFF;
    }
    std::vector<int64_t> used(static_cast<size_t>(C * P), 0);
    for (int64_t k = 0; k < nnz; ++k) {
        const int64_t c = colidx[k] >> shift;
        const int64_t pp = chunk_of[static_cast<size_t>(k)];
        const size_t t = static_cast<size_t>(c * P + pp);
        const int64_t o = used[t]++;
        const int64_t s1 = start1[t] + o, s2 = start2[t] + o;
        col[s1] = static_cast<uint16_t>(colidx[k] - (c << shift));
        src[s1] = static_cast<int32_t>(k);
        pos[s2] = static_cast<uint16_t>(k - tp_nz[pp]);
        if (o % 4 == 0) from[s2 / 4] = static_cast<int32_t>(s1 / 4);
    }
}

// The cap on a piece's groups that the library chooses for a device holding `resident` workgroups of the multiply pass
// at once (groups[c] = groups of four slots of column block c).  pieces(t) = sum_c ceil(groups[c] / t).  The pass is cut
// for k rounds of resident workgroups: k = waves when the matrix has waves * resident * floor groups or more, else 1, and
// raised until pieces(cap) <= k * resident; the answer is the smallest t <= cap with pieces(t) <= k * resident, but never
// below floor.
int32_t oracle_two_phase_piece_groups(int64_t C, const int64_t* groups, int32_t resident, int32_t waves, int32_t cap, int32_t floor) {
    int64_t total = 0;
    for (int64_t c = 0; c < C; ++c) total += groups[c];
    int64_t k = total >= static_cast<int64_t>(waves) * resident * floor ? waves : 1;
    for (;; ++k)
        for (int64_t t = 1; t <= cap; ++t) {
            int64_t pieces = 0;
            for (int64_t c = 0; c < C; ++c) pieces += (groups[c] + t - 1) / t;
            if (pieces <= k * resident) return static_cast<int32_t>(t < floor ? floor : t);
        }
}

// When AUTO takes the two-pass plan on groups of eight.  Candidates are group-aligned matrices that the row-length rule
// sent to the adaptive or the merge plan.  Taken when x holds at least 1 MiB, the matrix of groups meets the two-pass
// plan's own size conditions (3 * 2^21 entries, at most 65535 column blocks of 2^shift columns and 2^24 tiles, eight
// entries or more per tile on average) and the groups are scattered: the counted row blocks touch at least three
// distinct x vectors per four vectors their entries would fill (vec_elems entries each; vectors < 0: not counted, no).
int32_t oracle_grouped_two_phase_choice(int64_t m, int64_t n, int64_t nnz, int32_t elem_bytes, int32_t vec_elems, int32_t plan,
                                        int32_t group_aligned, int32_t shift, int32_t items, int64_t vectors, int64_t entries) {
    if (!(plan == 4 || plan == 5) || !group_aligned) return 0;
    if (vectors < 0 || 4 * vec_elems * vectors < 3 * entries) return 0;
    const int64_t ng = nnz / 8, ncol = (n + 7) / 8;
    const int64_t C = (ncol + (int64_t{1} << shift) - 1) >> shift;
    const int64_t P = (m + ng + items - 1) / items;
    return (n * elem_bytes >= (int64_t{1} << 20) && ng >= 3 * (int64_t{1} << 21) && C <= 65535 && C * P <= (int64_t{1} << 24) &&
            8 * C * P <= ng)
               ? 1
               : 0;
}

// How scattered the columns are: the distinct x vectors of the row blocks (nv from oracle_x_windows), summed,
// against the entries of the blocks that were counted (every block but a single row longer than block_nnz).
void oracle_scatter_counts(int64_t nb, const int32_t* row_blocks, const int32_t* rowptr, int32_t block_nnz, const int32_t* nv,
                           int64_t* vectors, int64_t* entries) {
    *vectors = 0;
    *entries = 0;
    for (int64_t b = 0; b < nb; ++b) {
        const int64_t in_block = static_cast<int64_t>(rowptr[row_blocks[b + 1]]) - rowptr[row_blocks[b]];
        *vectors += nv[b];
        if (in_block <= block_nnz) *entries += in_block;
    }
}

// AUTO takes the two-pass plan (ahead of the column-blocked one) when x holds at least a sixteenth of a column
// block of the column-blocked plan's width (256 KiB), there are at least 3 * 2^21 entries, at most 65535
// column blocks and 2^24 tiles, the tiles hold eight entries or more on average, and the columns are
// scattered: at least three distinct x vectors per four counted entries (vectors < 0: not counted, no).
int32_t oracle_two_phase_choice(int64_t m, int64_t n, int64_t nnz, int32_t elem_bytes, int32_t plan, int32_t shift, int32_t items,
                                int64_t vectors, int64_t entries) {
    const int64_t width = oracle_column_block_width(elem_bytes);
    const int64_t C = (n + (int64_t{1} << shift) - 1) >> shift;
    const int64_t P = (m + nnz + items - 1) / items;
    if (vectors < 0 || 4 * vectors < 3 * entries) return 0;
    return ((plan == 4 || plan == 5) && 16 * n >= width && nnz >= 3 * (int64_t{1} << 21) && C <= 65535 && C * P <= (int64_t{1} << 24) &&
            8 * C * P <= nnz)
               ? 1
               : 0;
}

// Sliced ELL re-layout (the ELL storage of App. C task 14 - fixed width, col_id -1 marks padding - applied to slices
// of `height` consecutive rows, each slice with a width of its own): slice s holds rows s*height .. s*height+height-1
// (rows from m on count as empty), its width is its longest row, and it takes width * height slots stored column by
// column: slot slice_ptr[s] + j * height + i belongs to entry j of the slice's i-th row.
// slice_ptr[s] = slots of the slices before s (ns + 1 numbers, ns = ceil(m / height)); returns the total.
int64_t oracle_sell_slices(int64_t m, const int32_t* rowptr, int64_t height, int64_t* slice_ptr) {
    const int64_t ns = (m + height - 1) / height;
    int64_t slots = 0;
    for (int64_t s = 0; s < ns; ++s) {
        int64_t width = 0;
        for (int64_t i = 0; i < height; ++i) {
            const int64_t r = s * height + i;
            if (r < m) width = std::max<int64_t>(width, rowptr[r + 1] - rowptr[r]);
        }
        slice_ptr[s] = slots;
        slots += width * height;
    }
    slice_ptr[ns] = slots;
    return slots;
}

// sell_col[slot] = the entry's column, sell_src[slot] = its position in colidx / vals; a slot without an entry
// (a row shorter than its slice is wide, a row from m on) holds -1 in both.
void oracle_sell_fill(int64_t m, const int32_t* rowptr, const int32_t* colidx, int64_t height, const int64_t* slice_ptr,
                      int32_t* sell_col, int32_t* sell_src) {
    const int64_t ns = (m + height - 1) / height;
    for (int64_t s = 0; s < ns; ++s) {
        const int64_t width = (slice_ptr[s + 1] - slice_ptr[s]) / height;
        for (int64_t j = 0; j < width; ++j)
            for (int64_t i = 0; i < height; ++i) {
                const int64_t slot = slice_ptr[s] + j * height + i;
                const int64_t r = s * height + i;
                sell_col[slot] = -1;
                sell_src[slot] = -1;
                if (r < m && j < rowptr[r + 1] - rowptr[r]) {
                    sell_col[slot] = colidx[rowptr[r] + j];
                    sell_src[slot] = static_cast<int32_t>(rowptr[r] + j);
                }
            }
    }
}

// Group-aligned CSR: every row starts at a multiple of `width` entries (so it holds whole groups of `width`), and
// every group k = width*g .. width*g + width - 1 has the columns c, c+1, .., c+width-1 with c a multiple of width: the
// x values a group multiplies are one aligned run.  On such a matrix the two-pass plan works on groups instead of
// entries.  Returns 1 or 0 (0 also when there is no entry).
int32_t oracle_csr_groups(int64_t m, int64_t nnz, const int32_t* rowptr, const int32_t* colidx, int32_t width) {
    if (nnz == 0) return 0;
    for (int64_t i = 0; i <= m; ++i)
        if (rowptr[i] % width != 0) return 0;
    for (int64_t g = 0; g < nnz / width; ++g) {
        const int64_t c = colidx[width * g];
        if (c % width != 0) return 0;
        for (int64_t i = 1; i < width; ++i)
            if (colidx[width * g + i] != c + i) return 0;
    }
    return 1;
}

// The matrix of groups of a group-aligned matrix: m rows, ceil(n / width) columns, nnz / width entries;
// rowptr_g[i] = rowptr[i] / width, col_g[g] = colidx[width * g] / width.
void oracle_group_matrix(int64_t m, int64_t nnz, const int32_t* rowptr, const int32_t* colidx, int32_t width, int32_t* rowptr_g,
                         int32_t* col_g) {
    for (int64_t i = 0; i <= m; ++i) rowptr_g[i] = rowptr[i] / width;
    for (int64_t g = 0; g < nnz / width; ++g) col_g[g] = colidx[width * g] / width;
}

}  // extern "C"
