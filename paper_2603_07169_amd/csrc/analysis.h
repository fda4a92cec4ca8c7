// Host-side analysis of the CSR row structure: statistics, length bins, row blocks,
// merge-path splits, plan.  Integer work only; O(m) plus O(P log m).
#pragma once
#include <cstdint>
#include <vector>

#include "spmv_mi355.h"

namespace spmv {

constexpr int kDefaultItemsPerChunk = 2048;
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
    // How scattered the columns are, from the count pass of the x windows (-1: not counted): the distinct
    // 16-byte x vectors of the row blocks, summed, and the entries of the blocks that were counted
    // (all but single rows longer than block_nnz).
    int64_t x_vectors_counted = -1;
    int64_t entries_counted = 0;
    // AUTO found the matrix group-aligned and takes the two-pass plan on its groups: the groups' columns (device memory,
    // nnz / 8 numbers, released once the plan is built)
    bool two_phase_on_groups = false;
    int32_t* d_group_cols = nullptr;
};

// Range-checks the parameters and fills in the defaults that do not depend on the matrix
// (block_nnz / rows_max left at 0 are resolved by analyze_rowptr from the mean row length).
// Returns SPMV_OK or SPMV_ERR_INVALID_ARG.
spmv_status_t resolve_params(const spmv_analyze_params_t* in, spmv_analyze_params_t* out);

// Row-block shape for a matrix of m rows and nnz entries when the caller gives none.
void default_tile_shape(int64_t m, int64_t nnz, int32_t* block_nnz, int32_t* rows_max);

// rowptr is a HOST array of m+1 entries.  Returns SPMV_OK, SPMV_ERR_BAD_STRUCTURE or SPMV_ERR_ALLOC.
// want_bin_rows: also build out->bin_rows (the one output only the BINNED plan's kernels read: 4 bytes a row that
// every other plan can do without until somebody reads the analysis back; bin_count / bin_offset are always filled).
spmv_status_t analyze_rowptr(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr,
                             const spmv_analyze_params_t& params, Analysis* out, bool want_bin_rows);
// The same list on its own (rowptr: HOST array of m+1 checked entries).  May throw std::bad_alloc.
void bin_rows_of(int64_t m, const int32_t* rowptr, std::vector<int32_t>* rows);

// Columns per block of the column-blocked plan (4 MiB of x), and whether the automatic plan
// takes it: only in place of ADAPTIVE / MERGE, with x beyond two blocks, at most 16 blocks and
// at least 2^22 entries.
int64_t column_block_width(spmv_dtype_t dtype);
// scattered: at least three distinct x vectors per four counted entries (x_vectors_counted < 0, nothing counted: no).
bool columns_scattered(int64_t x_vectors_counted, int64_t entries_counted);
bool column_block_sizes_ok(int64_t n, int64_t nnz, spmv_dtype_t dtype);
bool column_block_choice(int64_t n, int64_t nnz, spmv_dtype_t dtype, int32_t plan, int64_t x_vectors_counted, int64_t entries_counted);

// Merge-path splits every ipc steps: rows finished and entries taken at each split (P+1 of each).
void merge_path_splits(int64_t m, int64_t nnz, const int32_t* rowptr, int64_t ipc, std::vector<int32_t>* rows,
                       std::vector<int32_t>* entries);

// The two-pass plan.
constexpr int kTwoPhaseItems = 8192;               // merge-path steps per chunk of the reduce pass
constexpr int kTwoPhaseSnap = SPMV_TP_SNAP;         // rows of at most this many entries are never cut by a chunk
constexpr int kTwoPhasePieceGroups = 16384;        // most groups of four slots a workgroup of the multiply pass takes
constexpr int kTwoPhasePieceFloor = 2048;          // pieces are not made smaller than this to fill the device
constexpr int kTwoPhaseWaves = 2;                  // rounds of resident workgroups the multiply pass is cut for, where the matrix is large enough
constexpr int64_t kTwoPhaseMaxTiles = 1 << 24;     // most (column block, chunk) pairs
int two_phase_shift(int64_t n);                    // log2 of the columns per block
// Sizes alone: x of 256 KiB or more, 3 * 2^21 entries or more, tiles few and dense enough.
bool two_phase_sizes_ok(int64_t m, int64_t n, int64_t nnz, spmv_dtype_t dtype);
// The whole rule: the sizes, a row-wise plan to replace, and scattered columns (at least three distinct x vectors
// per four counted entries; x_vectors_counted < 0, nothing counted, says no).
bool two_phase_choice(int64_t m, int64_t n, int64_t nnz, spmv_dtype_t dtype, int32_t plan, int64_t x_vectors_counted,
                      int64_t entries_counted);
// The pieces of the multiply pass from where the column blocks start in the multiply order (block_first[C+1], in slots,
// the last entry = all slots): every block's groups cut evenly into the fewest pieces of at most piece_groups.
// The two-pass plan on groups of eight entries (a group-aligned matrix: every row starts at a multiple of eight entries and
// every group of eight is an aligned run of eight consecutive columns).  The matrix of groups has m rows, ceil(n / 8)
// columns and nnz / 8 entries; its column blocks hold 2^two_phase_group_shift columns (64 KB of x either way).
constexpr int kTpGroup = 8;
int two_phase_group_shift(spmv_dtype_t dtype);
// The chunks of the two-pass plan: the merge path cut every ipc steps, a cut that falls inside a row of at most snap
// entries (some of its entries taken, the row not finished) moved back to that row's first entry, the next ipc steps
// counted from there (snap < ipc).  Returns whether any chunk still cuts a row: without one there are no carries.
bool merge_path_splits_snapped(int64_t m, int64_t nnz, const int32_t* rowptr, int64_t ipc, int64_t snap, std::vector<int32_t>* rows,
                               std::vector<int32_t>* entries);
void two_phase_pieces(int64_t C, const int32_t* block_first, int32_t piece_groups, std::vector<int32_t>* piece_c,
                      std::vector<int32_t>* piece_g);
// AUTO's rule for the two-pass plan on groups of eight (a group-aligned matrix; plan = what the row-length rule chose):
// x of 1 MiB or more, the matrix of groups within the two-pass plan's size conditions, scattered groups (three distinct
// x vectors or more per four that the counted entries would fill).
bool grouped_two_phase_choice(int64_t m, int64_t n, int64_t nnz, spmv_dtype_t dtype, int32_t plan, bool group_aligned,
                              int64_t x_vectors_counted, int64_t entries_counted);
// The cap on a piece's groups for a device that keeps `resident` workgroups of the multiply pass at once.  A launch of a
// few more pieces than that leaves the device nearly idle while the last ones run (519 pieces on 512 places: 92 us
// instead of 71 on the 1 M-row block-clustered matrix), so the cap is the smallest one with which the column blocks make
// at most k * resident pieces, k the fewest rounds that kTwoPhasePieceGroups allows - at least `waves` rounds where
// pieces of kTwoPhasePieceFloor groups or more remain; never below kTwoPhasePieceFloor.
int32_t two_phase_piece_groups(int64_t C, const int32_t* block_first, int32_t resident, int32_t waves);

// Sums and maximises the blocks' x vector counts; true when the automatic plan should serve x
// from the windows: every block within SPMV_MAX_X_VECTORS, and the fixed-stride address lists
// (one slot per block and possible vector) no longer than a quarter of the entries.
bool window_choice(const int32_t* nv, int64_t nb, int64_t nnz, int64_t* total, int32_t* largest);

// Row order of the sparse-times-dense kernel: inside every window of SPMV_SPMM_WINDOW consecutive
// rows, the row ids by decreasing min(ceil(len / 4), 64), rows of equal key ascending.  rowptr is
// a HOST array of m+1 checked entries.  May throw std::bad_alloc.
constexpr int kSpmmMaxKey = 64;
void spmm_row_order(int64_t m, const int32_t* rowptr, std::vector<int32_t>* rows);

// Packed layout of the sparse-times-dense kernel.  Group g holds the rows at positions 16g .. 16g+15
// of `rows` and is stored as ceil(longest row / 16) blocks of 16 rows x 16 entries.
// desc[2g] = blocks of the groups before g, desc[2g+1] = ceil(longest row of g / 4); one closing
// pair (all blocks, 0).  Returns whether the packed copy is to be built: at most twice as many
// slots (256 per block) as the matrix has entries, and at most kSpmmMaxBlocks blocks.  May throw
// std::bad_alloc.
constexpr int64_t kSpmmMaxBlocks = int64_t{1} << 22;
bool spmm_packed_layout(int64_t m, int64_t nnz, const int32_t* rowptr, const int32_t* rows, std::vector<int32_t>* desc,
                        int64_t* num_blocks);

}  // namespace spmv
