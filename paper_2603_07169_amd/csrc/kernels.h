// Launch interface between the C ABI (host) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstdint>

namespace spmv {

struct MatrixView {
    int32_t m, n, nnz;
    const int32_t* rowptr;  // device [m+1]
    const int32_t* colidx;  // device [nnz]
    const void* vals;       // device [nnz] float or bf16 bits
    bool bf16;
    bool vec_ok;            // colidx and vals are 16-byte aligned: 128-bit loads allowed
};

constexpr int kMaxColBlocks = 16;  // most column blocks of the column-blocked plan
constexpr int kCbTile = 2048;      // entries a wavefront regroups at a time
constexpr int kMaxXVectors = 1024;     // most 16-byte x vectors a row block may keep in LDS
constexpr int kMaxTileEntries = 8192;  // most entries of a row block
constexpr int kMaxRowsPerBlock = 1024; // most rows of a row block
constexpr int kMaxPatternRuns = 4;     // most runs of rows in a patterned block
constexpr int kMaxPatternLen = 64;     // longest row of a patterned block

// x windows of the row blocks (device arrays owned by the handle).
struct XWindows {
    const int32_t* xv_ptr;    // [nb+1]
    const int32_t* xv_start;  // [xv_ptr[nb]]
    const int32_t* xv_pad;    // [nb * max_vectors] xv_start at a fixed stride per block, -1 padded: what the kernel reads
    const uint16_t* lidx8;    // [nnz / 8] lidx[8g] where the positions are grouped (see launch_lidx_groups), else null
    const uint16_t* lidx;     // [nnz rounded up to a multiple of 8]
    int32_t max_vectors;      // largest xv_ptr[b+1] - xv_ptr[b]
    const int32_t* run_desc;  // [8 * nb] packed runs of the row patterns (see launch_pattern_build), or null: no patterns
    const uint16_t* pat_pad;  // [nb * pt_cap] the blocks' pattern lists
    int32_t pt_cap;           // a multiple of 8, at most kMaxPatternRuns * kMaxPatternLen
};

struct Scalars {
    float alpha, beta;
};

// Records a failing HIP call for spmv_last_hip_error() and clears the runtime's sticky error; true when e is an error.
bool note_hip_error(hipError_t e);

// rows == nullptr: rows 0..count-1; otherwise the `count` row ids listed in rows[].
hipError_t launch_scalar(const MatrixView& A, const int32_t* rows, int32_t count, const void* x, float* y, Scalars s,
                         hipStream_t st);
// lanes: power of two in [2, 64].
hipError_t launch_vector(const MatrixView& A, int lanes, const int32_t* rows, int32_t count, const void* x, float* y,
                         Scalars s, hipStream_t st);
// block_desc: device [2*(nb+1)], pairs (row_blocks[b], rowptr[row_blocks[b]]).
// block_nnz, rows_max: the limits the partition was built with.
hipError_t launch_adaptive(const MatrixView& A, const int32_t* block_desc, int32_t nb,
                           int32_t block_nnz, int32_t rows_max, const void* x, float* y, Scalars s, hipStream_t st);
// The adaptive plan with x served from per-block windows in LDS.  staged_max: the most entries
// of any block that is staged (i.e. not a single over-long row); <= block_nnz.
hipError_t launch_windowed(const MatrixView& A, const int32_t* block_desc, int32_t nb,
                           int32_t block_nnz, int32_t staged_max, int32_t rows_max, const XWindows& w, const void* x,
                           float* y, Scalars s, hipStream_t st);
// Analysis-time construction of the x windows.  fill == false: nv[b] = distinct x vectors of
// block b.  fill == true: writes xv_start, xv_pad (stride x_cap >= every nv[b]) and lidx given
// xv_ptr = exclusive prefix sums of nv.
hipError_t launch_window_build(const MatrixView& A, const int32_t* block_nz, int32_t nb, int32_t block_nnz, bool fill,
                               int32_t* nv, const int32_t* xv_ptr, int32_t* xv_start, int32_t* xv_pad, int32_t x_cap,
                               uint16_t* lidx, hipStream_t st);
// chunk_desc: device [2*(P+1)], pairs (mp_row[p], mp_nz[p]); carry_row/carry_val: device [P] scratch owned by the handle.
hipError_t launch_merge(const MatrixView& A, const int32_t* chunk_desc, int32_t P,
                        int32_t items_per_chunk, int32_t* carry_row, float* carry_val, const void* x, float* y,
                        Scalars s, hipStream_t st);
// C <- alpha*A*B + beta*C; A CSR, B device [n x ldb] in A's storage type, C device float[m x ldc], row-major, K columns used.
// rows: device int32[m], the order in which the rows are handed to the wavefronts (a permutation
// of 0..m-1), or NULL for the natural order.
hipError_t launch_spmm(const MatrixView& A, const int32_t* rows, const void* B, int64_t ldb, float* C, int64_t ldc,
                       int32_t K, Scalars s, hipStream_t st);
// The packed copy of A the sparse-times-dense product can run from (device pointers).
constexpr int kSpmmCol16MaxN = 32768;  // up to this many columns the packed column numbers take 16 bits
struct PackedRows {
    const int32_t* rows;  // [m] row order
    const int32_t* desc;  // [2 * (num_groups + 1)] pairs (first block, steps of 4 entries)
    const void* pcol;     // [(blocks + 1) * 256] uint16 (col16) or int32
    const float* pval;    // [(blocks + 1) * 256]
    int32_t num_groups;
    bool col16;
};
// Fills pcol / pval of all blocks of all groups from the CSR arrays (the extra closing block is not written).
hipError_t launch_spmm_pack(const MatrixView& A, const int32_t* rows, const int32_t* desc, int32_t num_groups, bool col16,
                            void* pcol, float* pval, hipStream_t st);
hipError_t launch_spmm_packed(const MatrixView& A, const PackedRows& P, const void* B, int64_t ldb, float* C, int64_t ldc,
                              int32_t K, Scalars s, hipStream_t st);
const char* spmm_packed_kernel_name();
// Whole aligned groups of eight entries (groups = nnz / 8): lidx8[g] = lidx[8g]; *flag (device int32, 0 on entry) is set to 1
// if some group's eight positions are not consecutive numbers.
hipError_t launch_lidx_groups(const uint16_t* lidx, int32_t groups, uint16_t* lidx8, int32_t* flag, hipStream_t st);
// Row patterns of the window positions (analysis).  block_desc as for launch_adaptive.  fill == false: run_desc[8b..8b+7] =
// the runs of block b, packed: words 0-1 rows per run, 3-4 base of the run's first row, 5-6 stride (two's complement), 16 bits
// each in run order; word 2 entries per row, 8 bits each; word 7 the number of runs (0: the block has no pattern, all words 0);
// *max_table (device int32, 0 on entry) = longest pattern list of any block; *covered (device uint64, 0 on entry) = entries
// of the patterned blocks.  fill == true: pat_pad[b * pt_cap ..] = block b's list (rel of the first row of every run), then zeros.
hipError_t launch_pattern_build(const int32_t* block_desc, int32_t nb, const int32_t* rowptr, const uint16_t* lidx, int32_t block_nnz,
                                bool fill, int32_t* run_desc, int32_t* max_table, unsigned long long* covered, uint16_t* pat_pad,
                                int32_t pt_cap, hipStream_t st);
// flag: device int32, must be 0 on entry; set to 1 if any colidx is outside [0, n).
hipError_t launch_validate_columns(const MatrixView& A, int32_t* flag, hipStream_t st);

// y <- alpha*A*x + beta*y for A in COO / CSC / ELL storage (stateless; indices are not checked).
// COO and CSC first scale y by beta, then add every entry's contribution with float atomics.
hipError_t launch_coo(bool bf16, int32_t m, int32_t nnz, const int32_t* row, const int32_t* col, const void* vals,
                      const void* x, float* y, Scalars s, hipStream_t st);
hipError_t launch_csc(bool bf16, int32_t m, int32_t n, int32_t nnz, const int32_t* col_offsets, const int32_t* row,
                      const void* vals, const void* x, float* y, Scalars s, hipStream_t st);
hipError_t launch_ell(bool bf16, int32_t m, int32_t width, const int32_t* col_ids, const void* vals, const void* x,
                      float* y, Scalars s, hipStream_t st);

// Pieces of the COO product for callers that run several of them into one y.
hipError_t launch_scale_y(float* y, int32_t m, float beta, hipStream_t st);  // y <- beta*y (0 when beta == 0)
hipError_t launch_coo_accumulate(bool bf16, int32_t nnz, const int32_t* row, const int32_t* col, const void* vals,
                                 const void* x, float* y, float alpha, hipStream_t st);  // y += alpha*A*x, atomics

// Column-blocked regrouping (analysis).  Block of column c = c >> shift; C blocks.  ntiles =
// column_block_tiles(nnz).  count: tile_counts[b*ntiles + t].  scatter: tile_base = exclusive
// prefix sums of tile_counts in that order; writes row, column within block, source position
// and value of every regrouped entry.
int32_t column_block_tiles(int32_t nnz);
hipError_t launch_column_block_count(const MatrixView& A, int shift, int C, int32_t* tile_counts, hipStream_t st);
hipError_t launch_column_block_scatter(const MatrixView& A, int shift, int C, const int32_t* tile_base, int32_t* cb_row,
                                       int32_t* cb_col, int32_t* cb_src, void* cb_vals, hipStream_t st);
// cb_vals[k] = vals[cb_src[k]] for the nnz regrouped entries (the caller's values may have changed).
hipError_t launch_column_block_values(const MatrixView& A, const int32_t* cb_src, void* cb_vals, hipStream_t st);

// The carry fix-up of the merge-path kernels: y[carry_row[p]] += alpha * carry_val[p], runs of equal rows summed in chunk order.
hipError_t launch_merge_fixup(const int32_t* carry_row, const float* carry_val, int32_t P, float* y, float alpha,
                              hipStream_t st);

// The two-pass plan (device arrays owned by the handle).
struct TwoPhase {
    int32_t shift;              // column blocks of 2^shift columns (of 2^shift groups' columns when group == 8)
    int32_t group;              // 1, or 8: a slot stands for a group of eight entries (group-aligned matrix)
    int32_t num_pieces;         // multiply pass: workgroups
    int32_t num_chunks;         // reduce pass: merge-path chunks
    bool carries;               // some chunk cuts a row: the fix-up kernel has to run
    size_t reduce_lds;          // two_phase_reduce_lds() of the largest chunk
    const int32_t* piece_c;     // [num_pieces]   column block of each piece
    const int32_t* piece_g;     // [num_pieces+1] first group of each piece (pieces are contiguous)
    const uint16_t* tp_col;     // [slots] column within the block; padding: 2^shift
    const void* tp_val;         // [slots] values in the handle's dtype; padding: 0
    const int32_t* tp_from;     // [slots/4] group of the multiply order that each group of the reduce order is fed by
    const uint16_t* tp_pos;     // [slots] reduce order: CSR position within the chunk; padding: 0xFFFF
    const int32_t* chunk_desc;  // [2*(num_chunks+1)] pairs (rows finished, entries taken)
    const int32_t* chunk_g;     // [num_chunks+1] first group of each chunk in the reduce order
    float* prod;                // [slots] scratch: the products between the two passes, in the multiply order
    int32_t* carry_row;         // [num_chunks] scratch
    float* carry_val;           // [num_chunks] scratch
};
constexpr int kTpMaxShift = 15;  // column blocks of at most 32768 columns (16-bit columns, one more value for padding)
size_t two_phase_reduce_lds(int32_t entries, int32_t rows);
hipError_t launch_two_phase(const TwoPhase& t, const MatrixView& A, const void* x, float* y, Scalars s, hipStream_t st);
// Analysis time.  Scratch of the regrouping (device, T = C*P tiles): all of it is temporary.
struct TwoPhaseTables {
    int32_t* padded;       // [T]    slots of tile t = c*P + p (entries rounded up to whole groups of four)
    int32_t* base1;        // [T]    slots before it in the multiply order
    int32_t* within;       // [T]    slots of its chunk in the column blocks before its own
    int32_t* in_chunk;     // [P+1]  slots of every chunk, then 0
    int32_t* chunk_first;  // [P+1]  slots before every chunk in the reduce order, then all slots
    int32_t* block_first;  // [C+1]  slots before every column block in the multiply order, then all slots
    int32_t* scan_sums;    // [two_phase_scan_blocks(T)] scratch of the prefix sums
};
int64_t two_phase_scan_blocks(int64_t count);
// Counts every chunk's entries per column block and derives every table above, and chunk_g[P+1] (first group of
// every chunk in the reduce order).  Integer arithmetic only: the result does not depend on scheduling.
hipError_t launch_two_phase_tables(const MatrixView& A, int shift, int32_t C, int32_t P, const int32_t* chunk_desc,
                                   const TwoPhaseTables& w, int32_t* chunk_g, hipStream_t st);
// Fills the padding and places every entry (CSR order kept inside a tile).
// group == 8: A is the matrix of groups (its colidx the groups' columns) and no value is placed.
hipError_t launch_two_phase_place(const MatrixView& A, int shift, int32_t C, int32_t P, const TwoPhaseTables& w,
                                  const int32_t* chunk_desc, int64_t slots, int group, uint16_t* tp_col, void* tp_val,
                                  int32_t* tp_src, int32_t* tp_from, uint16_t* tp_pos, hipStream_t st);
// tp_val[s] = vals[tp_src[s]] wherever tp_src[s] >= 0; group == 8: A is the caller's matrix, a slot holds the eight values of
// group tp_src[s].
hipError_t launch_two_phase_values(const MatrixView& A, const int32_t* tp_src, void* tp_val, int64_t slots, int group,
                                   hipStream_t st);
// gcol[g] = colidx[8g] / 8; *flag (cleared by the caller) is set when some group of eight entries is not an aligned run
// of eight consecutive columns.
hipError_t launch_two_phase_groups(const int32_t* colidx, int32_t ngroups, int32_t* gcol, int32_t* flag, hipStream_t st);

// The sliced ELL plan.  slice_ptr[ns+1]: slots before each slice of kSellHeight rows (a slice takes width * kSellHeight
// slots, stored column by column).  fill: column, source position and value of every slot (-1, -1, 0 for padding).
constexpr int kSellHeight = 64;
hipError_t launch_sell_fill(const MatrixView& A, const int32_t* slice_ptr, int32_t ns, int32_t* sell_col, int32_t* sell_src,
                            void* sell_val, hipStream_t st);
// sell_val[s] = vals[sell_src[s]] wherever sell_src[s] >= 0.
hipError_t launch_sell_values(const MatrixView& A, const int32_t* sell_src, void* sell_val, int64_t slots, hipStream_t st);
hipError_t launch_sell(const MatrixView& A, const int32_t* slice_ptr, int32_t ns, const int32_t* sell_col, const void* sell_val,
                       const void* x, float* y, Scalars s, hipStream_t st);

// Cross-lane reduction self-check on one wavefront.  in: device float[64], lane l contributes in[l].
// out: device float[14*64]; out[gi*64 + l] = sum over lane l's aligned group of G = 2^gi lanes,
// gi = 0..6 from the compile-time variant, then the same seven again from the run-time variant.
hipError_t launch_reduce_selftest(const float* in, float* out, hipStream_t st);

const char* scalar_kernel_name();
const char* vector_kernel_name();
const char* tile_kernel_name();  // kernel of the adaptive and merge plans
const char* window_kernel_name();
const char* pattern_kernel_name();
const char* spmm_kernel_name();
const char* sell_kernel_name();

}  // namespace spmv
