/* spmv_mi355.h -- C ABI of the gfx950 CSR sparse matrix-vector product library.
 *
 * Operation.  The benchmark's "SpMV CSR" task (paper App. C, task 12) multiplies a sparse
 * matrix A, held as three arrays
 *     values[nnz], col_indices[nnz], row_offsets[rows+1]  (row_offsets[i] = index of the first
 *     stored entry of row i),
 * with a dense vector x of length cols and writes y of length rows.  This library computes
 * the BLAS form of it,
 *     y <- alpha * A * x + beta * y,
 * with A and x stored either as IEEE binary32 or as bf16 (upper half of a binary32), products
 * and sums always taken in binary32, y always binary32.  The paper classes this operation
 * as bound by memory bandwidth (App. A, bottleneck distribution), so every kernel behind
 * this interface is organised around streaming values/col_indices once with wide loads.
 *
 * Conventions.
 *   - Indices are 0-based int32.  m, n, nnz (and K, width) are passed as int64 and must not
 *     exceed SPMV_MAX_SIZE = 2^31 - 2^22: index arithmetic in the kernels is 32-bit, and the
 *     margin keeps an index plus one grid stride inside int32.
 *   - Every array argument of create/run is a DEVICE pointer, BORROWED: the caller owns the
 *     memory and must keep rowptr/colidx/vals alive and unchanged until spmv_destroy()
 *     (vals may be changed in place if spmv_csr_refresh_values() is called before the next run).
 *     The library owns only the metadata it allocates in spmv_csr_analyze().
 *   - Column indices inside a row may be in any order and may repeat (repeats add up).
 *   - Every function returns a status; nothing throws, aborts or prints.
 *   - spmv_csr_run() only enqueues kernels on the given stream: no synchronisation, no
 *     allocation, no host<->device copy.  Runs of one handle on one stream follow each other; runs
 *     on several streams may overlap under every plan except MERGE and TWOPHASE, whose kernels pass
 *     carries / products through scratch kept in the handle: there a run on another stream while
 *     the last one is still in flight is refused with SPMV_ERR_BUSY and enqueues nothing (order the
 *     streams with an event, or give each stream a handle of its own; the check is an event query
 *     and is left out on a stream that is being captured into a graph).
 *   - Read-back functions copy to caller-owned HOST buffers and synchronise the device.
 */
#ifndef SPMV_MI355_H
#define SPMV_MI355_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spmv_csr_s* spmv_handle_t;

/* Largest m, n, nnz, K or ELL width any entry point accepts. */
#define SPMV_MAX_SIZE ((int64_t)2147483647 - 4194303)

/* Storage type of vals AND x.  y, alpha, beta are always float. */
typedef enum { SPMV_F32 = 0, SPMV_BF16 = 1 } spmv_dtype_t;

typedef enum {
    SPMV_OK = 0,
    SPMV_ERR_INVALID_ARG = 1,   /* null pointer, negative size, unknown enum, parameter out of range */
    SPMV_ERR_BAD_STRUCTURE = 2, /* rowptr[0] != 0, rowptr decreasing, rowptr[m] != nnz, column outside [0,n) */
    SPMV_ERR_UNSUPPORTED = 3,   /* a size > SPMV_MAX_SIZE, or pointers not aligned to the element size */
    SPMV_ERR_NOT_ANALYZED = 4,  /* run or read-back before a successful analyze */
    SPMV_ERR_ALLOC = 5,         /* host or device allocation failed */
    SPMV_ERR_HIP = 6,           /* a HIP runtime call failed; see spmv_last_hip_error() */
    SPMV_ERR_BUSY = 7           /* spmv_csr_run: the plan's scratch is still in use by a run on another stream */
} spmv_status_t;

/* Execution plans.  AUTO lets analyze choose (rule documented at spmv_csr_analyze). */
typedef enum {
    SPMV_PLAN_AUTO = 0,
    SPMV_PLAN_SCALAR = 1,   /* one lane per row                                                  */
    SPMV_PLAN_VECTOR = 2,   /* a power-of-two group of lanes (2..64) per row, cross-lane reduce */
    SPMV_PLAN_BINNED = 3,   /* rows grouped by length bin; scalar or vector kernel per bin      */
    SPMV_PLAN_ADAPTIVE = 4, /* contiguous row blocks streamed through LDS (CSR-Adaptive)        */
    SPMV_PLAN_MERGE = 5,    /* equal-work merge-path chunks + carry fix-up                      */
    SPMV_PLAN_WINDOWED = 6, /* ADAPTIVE row blocks whose x values are served from a per-block
                               window in LDS, entries addressed by 16-bit window positions      */
    SPMV_PLAN_COLBLOCK = 7, /* entries regrouped by blocks of columns (one 4 MiB stretch of x per
                               block), each block multiplied in coordinate form with atomics    */
    SPMV_PLAN_TWOPHASE = 8, /* two passes, neither gathering from memory: products by column block
                               with the block of x in LDS, then row sums by merge-path chunk with
                               the products dropped into LDS at their CSR positions             */
    SPMV_PLAN_SELL = 9      /* a sliced ELL copy built at analysis time (the ELL storage of paper
                               App. C task 14, col_id -1 = padding, slice by slice): one wavefront
                               per slice of 64 rows, one lane per row, no row offsets read       */
} spmv_plan_t;

#define SPMV_SELL_HEIGHT 64 /* rows per slice of the SELL plan */
/* Rows of at most this many entries (groups, on a group-aligned matrix) are never cut by a chunk of the two-pass plan. */
#define SPMV_TP_SNAP 512

#define SPMV_MAX_X_VECTORS 1024 /* most 16-byte x vectors in one row block's window */

#define SPMV_NUM_BINS 33

#define SPMV_SPMM_WINDOW 4096 /* rows per window of the spmm_rows order */

/* Analysis parameters.  Zero in any field selects that field's default. */
typedef struct {
    int32_t plan;             /* spmv_plan_t; default AUTO */
    int32_t block_nnz;        /* row blocks: most stored entries per block, 1..8192; default: see analyze */
    int32_t rows_max;         /* row blocks: most rows per block, 1..1024;           default: see analyze */
    int32_t items_per_chunk;  /* merge path: steps (row ends + entries) per chunk; default 2048, 1..8192 */
    int32_t vector_lanes;     /* VECTOR plan: lanes per row, power of two 2..64; default: chosen from nnz/m */
    int32_t skip_validation;  /* nonzero: do not scan colidx for out-of-range columns in analyze */
    int32_t prepare_spmm;     /* 1: also build spmm_rows, the row order spmm_csr_run() then works in
                                 (and, where it pays, a packed copy of A); 0: spmm_csr_run() takes the rows as they come */
    int32_t reserved;         /* must be zero */
} spmv_analyze_params_t;

typedef struct {
    int64_t m, n, nnz;
    int64_t min_len, max_len, n_empty; /* row length statistics (all 0 when m == 0) */
    int64_t num_row_blocks;            /* nb: row_blocks holds nb+1 entries */
    int64_t num_chunks;                /* P:  mp_row / mp_nz hold P+1 entries */
    int64_t num_x_vectors;             /* WINDOWED plan: length of xv_start; 0 otherwise */
    int32_t plan;                      /* the plan run() will use (never AUTO) */
    int32_t vector_lanes;              /* lanes per row the VECTOR plan uses */
    int32_t block_nnz, rows_max, items_per_chunk; /* parameters in effect */
    int32_t max_x_vectors;             /* most x vectors of any row block (0 when the windows were not counted) */
    int32_t num_col_blocks;            /* COLBLOCK plan: C, the number of column blocks; 0 otherwise */
    int32_t col_block_width;           /* COLBLOCK plan: columns per block (a power of two); 0 otherwise */
    int32_t spmm_prepared;             /* prepare_spmm: 0 not asked for, 1 spmm_rows built, 2 the packed copy as well */
    int32_t spmm_col_bytes;            /* packed copy: bytes per column number (2 while n <= 32768, else 4); 0 without it */
    int64_t spmm_num_blocks;           /* packed copy: blocks of 16 rows x 16 entries; 0 without it */
    /* TWOPHASE plan (all 0 otherwise): */
    int64_t tp_slots;                  /* S: padded entries (a multiple of 4)                        */
    int32_t tp_col_shift;              /* column blocks of 2^tp_col_shift columns                    */
    int32_t tp_items;                  /* merge-path steps per chunk of the reduce pass              */
    int32_t tp_num_col_blocks;         /* C2                                                          */
    int32_t tp_num_chunks;             /* P2: tp_row / tp_nz hold P2+1 entries                        */
    int32_t tp_num_pieces;             /* Q: workgroups of the multiply pass                          */
    int32_t lidx_grouped;              /* WINDOWED plan: 1 when the window positions are grouped (see analyze)  */
    int32_t lidx_patterned;            /* WINDOWED plan: 1 when run() works from row patterns (see analyze)      */
    int32_t pat_cap;                   /* ... then: entries per block in pat_pad (a multiple of 8); 0 otherwise  */
    int64_t pat_entries;               /* ... then: stored entries held by the patterned blocks; 0 otherwise     */
    /* SELL plan (all 0 otherwise): */
    int64_t sell_slots;                /* slots of the sliced copy, padding included (a multiple of 64)          */
    int32_t sell_num_slices;           /* ns = ceil(m / 64): sell_ptr holds ns+1 entries                          */
    int32_t tp_group;                  /* TWOPHASE plan: entries a slot stands for, 1 or 8 (see analyze); 0 otherwise */
    int32_t tp_piece_groups;           /* TWOPHASE plan: most groups of four slots in a piece of the multiply pass     */
    int32_t tp_resident;               /* ... and the workgroups of that pass the device holds at once, for which it was chosen */
} spmv_analysis_info_t;

/* Caller-allocated HOST buffers for spmv_csr_get_analysis(); a NULL member is skipped. */
typedef struct {
    int32_t* bin_count;  /* [SPMV_NUM_BINS]                                   */
    int32_t* bin_offset; /* [SPMV_NUM_BINS + 1] exclusive prefix of bin_count */
    int32_t* bin_rows;   /* [m]    row ids grouped by bin, ascending in each bin */
    int32_t* row_blocks; /* [nb+1] first row of each block, then m            */
    int32_t* mp_row;     /* [P+1]  rows finished at each merge-path split     */
    int32_t* mp_nz;      /* [P+1]  entries taken at each merge-path split     */
    /* WINDOWED plan only (skipped otherwise): */
    int32_t* xv_ptr;     /* [nb+1] exclusive prefix of the blocks' x vector counts   */
    int32_t* xv_start;   /* [num_x_vectors] first x element of each vector           */
    int32_t* xv_pad;     /* [nb * max(1, max_x_vectors)] block b's part of xv_start at
                            xv_pad[b*max_x_vectors ...], then -1 up to the next block:
                            the fixed-stride copy the kernel reads                    */
    uint16_t* lidx;      /* [nnz]  window position of every entry's x value          */
    /* ... with lidx_patterned only (skipped otherwise): */
    int32_t* run_desc;   /* [8 nb] the runs of every block, packed (see analyze)      */
    uint16_t* pat_pad;   /* [nb * pat_cap] the blocks' pattern lists, zero padded     */
    /* COLBLOCK plan only (skipped otherwise): */
    int32_t* cb_ptr;     /* [C+1]  entries in the blocks before block b              */
    int32_t* cb_row;     /* [nnz]  row of every regrouped entry                      */
    int32_t* cb_col;     /* [nnz]  its column minus the block's first column         */
    int32_t* cb_src;     /* [nnz]  its position in the caller's colidx / vals        */
    /* TWOPHASE plan only (skipped otherwise): */
    int32_t* tp_row;     /* [P2+1] rows finished at each split of the reduce pass     */
    int32_t* tp_nz;      /* [P2+1] entries taken at each split                        */
    int32_t* tp_piece_c; /* [Q]    column block of each piece of the multiply pass    */
    int32_t* tp_piece_g; /* [Q+1]  first group of four slots of each piece            */
    int32_t* tp_chunk_g; /* [P2+1] first group of each chunk in the reduce order      */
    uint16_t* tp_col;    /* [S]    multiply order: column within the block            */
    int32_t* tp_src;     /* [S]    multiply order: position in colidx / vals, -1 pad  */
    int32_t* tp_from;    /* [S/4]  reduce order: the multiply-order group that is this group */
    uint16_t* tp_pos;    /* [S]    reduce order: CSR position within the chunk        */
    /* With prepare_spmm only (skipped otherwise): */
    int32_t* spmm_rows;  /* [m]    inside each window of SPMV_SPMM_WINDOW consecutive rows:
                            row ids by decreasing min(ceil(len / 4), 64), ties ascending */
    /* With the packed copy only (spmm_prepared == 2; G = ceil(m / 16) groups): */
    int32_t* spmm_desc;  /* [2G+2] pairs (blocks of the groups before g, ceil(longest row of g / 4)),
                            then (spmm_num_blocks, 0)                                  */
    void* spmm_col;      /* [spmm_num_blocks * 256] uint16 or int32 (spmm_col_bytes)   */
    float* spmm_val;     /* [spmm_num_blocks * 256]                                    */
    /* SELL plan only (skipped otherwise): */
    int32_t* sell_ptr;   /* [ns+1] slots of the slices before slice s                  */
    int32_t* sell_col;   /* [sell_slots] column of every slot, -1 = padding            */
    int32_t* sell_src;   /* [sell_slots] its position in colidx / vals, -1 = padding   */
} spmv_analysis_host_t;

/* Records the matrix (paper App. C task 12: values / col_indices / row_offsets).
 *   out      receives the handle; set to NULL on any error.
 *   m, n     rows, columns (>= 0);  nnz  stored entries (>= 0).
 *   rowptr   device int32[m+1];  colidx  device int32[nnz];
 *   vals     device float[nnz] (SPMV_F32) or uint16 bf16 bit patterns [nnz] (SPMV_BF16).
 *            colidx and vals may be NULL only when nnz == 0.
 * Touches no device memory.  Errors: INVALID_ARG, UNSUPPORTED, ALLOC. */
spmv_status_t spmv_csr_create(spmv_handle_t* out, int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr,
                              const int32_t* colidx, const void* vals, spmv_dtype_t dtype);

/* One-time inspection of the row structure.  Copies rowptr to the host, checks it
 * (rowptr[0] == 0, non-decreasing, rowptr[m] == nnz), optionally checks 0 <= colidx < n on the
 * device, then derives and uploads:
 *   - row statistics; bin(len) = 0 for len 0, else the smallest b >= 1 with 2^(b-1) >= len;
 *     bin_rows = stable grouping of row ids by bin (kept on the device for the BINNED plan, whose kernels read it;
 *     under any other plan it is built when spmv_csr_get_analysis() is asked for it, from rowptr as it then is);
 *   - row blocks: greedy left-to-right, a block takes the next row while it has < rows_max
 *     rows and the row keeps it at <= block_nnz entries; a longer row stands alone.
 *     Defaults (a field left 0): with mean = ceil(nnz/m) and G the largest power of two <= 64
 *     with 16*G <= mean + 15, rows_max = 256/G and block_nnz = rows_max*mean rounded up to a
 *     multiple of 8 and clamped to [2048, 8192]; matrices of at most 2^20 entries get
 *     rows_max = 64, block_nnz = 1024;
 *   - merge-path splits: the path over (row ends, entry positions) cut every items_per_chunk
 *     steps;
 *   - the plan: params->plan if not AUTO, else SCALAR when m == 0 or nnz == 0, MERGE when
 *     some row is longer than block_nnz, else ADAPTIVE, upgraded to WINDOWED by the x windows:
 *   - x windows (plan AUTO that arrived at ADAPTIVE, or plan WINDOWED; built on the device from
 *     colidx).  x is cut into aligned 16-byte vectors (4 floats / 8 bf16).  For row block b,
 *     keys_b = the distinct colidx/VE of its entries in ascending order (VE = elements per
 *     vector); xv_start lists keys_b*VE block after block, xv_ptr its block boundaries;
 *     lidx[k] = rank(colidx[k]/VE in keys_b)*VE + colidx[k]%VE.  A block that is one row longer
 *     than block_nnz has no vectors and lidx 0.  With V = the largest vector count of any
 *     block, AUTO picks WINDOWED when V <= SPMV_MAX_X_VECTORS and 4 * nb * V <= nnz (the kernel
 *     reads the lists at a fixed stride of V per block); a forced WINDOWED plan fails with
 *     UNSUPPORTED when V is larger.  The library then holds 2 bytes per
 *     stored entry of its own (lidx) and run() no longer reads colidx.  The positions are
 *     grouped (lidx_grouped = 1) when every row block starts at a multiple of eight entries and
 *     every aligned group of eight entries 8g .. 8g+7 (8g+8 <= nnz) has lidx[8g+i] = lidx[8g] + i:
 *     rows made of aligned runs of columns.  run() then reads one position per group (a copy of
 *     lidx[8g], 2 bytes per eight entries) and counts the other seven up from it.
 *     Row patterns (looked for when the positions are not grouped).  Row i of a block has base_i = lidx of its first
 *     entry (0 for an empty row) and rel_i[j] = lidx of its j-th entry minus base_i.  The rows of a block are cut
 *     greedily into runs: the run of row i-1 also takes row i when rel_i = rel_{i-1} (same length, same numbers) and,
 *     if the run already has two rows or more, base_i - base_{i-1} equals the step between those (the run's stride; a
 *     run of one row has stride 0).  A block is patterned when it is staged (at most block_nnz entries), no row is longer
 *     than 64 entries, no rel is negative and it has at most 4 runs.  When the patterned blocks hold at least half of
 *     the stored entries (lidx_patterned = 1) the library keeps, per block b, run_desc[8b .. 8b+7] - words 0-1: rows of
 *     runs 0..3, words 3-4: base of each run's first row, words 5-6: stride (two's complement), 16 bits each, low half
 *     first; word 2: entries per row of runs 0..3, 8 bits each, low byte first; word 7: number of runs, 0 for a block
 *     without a pattern (then all eight words are 0) - and pat_pad[b * pat_cap ..]: rel of the first row of run 0, of
 *     run 1, .., then zeros (pat_cap = the longest such list rounded up to a multiple of 8).  run() then reads neither the
 *     positions nor the row offsets of a patterned block: the position of entry j of the q-th row of a run is
 *     base + q * stride + rel[j].  Blocks without a pattern are served from lidx as before.
 *   - column blocks (plan AUTO that arrived at ADAPTIVE or MERGE, or plan COLBLOCK; built on the
 *     device).  Columns are cut into blocks of W = 4 MiB / element size columns; the entries are
 *     regrouped block after block, keeping their row-major order inside a block, each with its
 *     row (cb_row), its column within the block (cb_col) and its source position (cb_src); the
 *     library keeps a copy of the values in that order.  AUTO picks COLBLOCK when n > 2 W, there
 *     are at most 16 blocks, nnz >= 2^22, the columns are scattered (the condition on nv_b given
 *     with the two-pass layout below) and that layout was not taken: x then no longer fits the
 *     L2s and the row-wise kernels would fetch a cache line per entry.  run() multiplies block after block with
 *     float atomics into y: results are reproducible to rounding, not bit for bit.  The copy is
 *     taken at analyze time (spmv_csr_refresh_values() renews it).  A forced COLBLOCK
 *     plan fails with UNSUPPORTED when there would be more than 16 blocks.
 *   - the two-pass layout (plan TWOPHASE, or plan AUTO where the rule below holds; built on the
 *     device).  Columns are cut into C2 blocks of 2^tp_col_shift (= 16384) columns; the CSR entry
 *     list is cut into P2 chunks (tp_row / tp_nz: rows finished and entries taken at every cut) by
 *     walking the merge path as for mp_row / mp_nz and cutting every tp_items (= 8192) steps, except
 *     that a cut which falls inside a row of at most SPMV_TP_SNAP entries - some of its entries
 *     taken, the row not finished - is moved back to that row's first entry, and the next tp_items
 *     steps are counted from there: a chunk cuts only rows longer than SPMV_TP_SNAP, and where no
 *     row is cut at all, run() launches no fix-up kernel.  Tile (c, p) = the entries of column block c in chunk
 *     p, in CSR order, padded to a multiple of four slots.  The multiply order lists the tiles by
 *     (c, p), the reduce order by (p, c); S slots each.  Per slot of the multiply order: tp_col
 *     (column - c * 2^tp_col_shift; padding: 2^tp_col_shift), tp_src (position k in colidx / vals;
 *     padding: -1) and a copy of the value (padding: 0).  Per slot of the reduce order: tp_pos =
 *     k - tp_nz[p] (padding: 0xFFFF); per group of four slots of the reduce order tp_from, the
 *     number of the same group in the multiply order.  Column block c's groups are cut evenly into
 *     the fewest pieces of at most t = tp_piece_groups groups: q = ceil(groups / t) pieces of
 *     ceil(groups / q), the last one shorter.  t is chosen for the device: with R = tp_resident
 *     workgroups of the multiply pass held at once (two per compute unit), t is the smallest cap
 *     with which the pieces number at most k R, k the fewest rounds that a cap of 16384 allows, at
 *     least 2 when the matrix has 2 * 2048 * R groups or more; t is never below 2048.  (A launch of
 *     slightly more than a whole number of rounds leaves the device idle while the last pieces run.)
 *     (tp_piece_c, tp_piece_g; pieces are contiguous, tp_piece_g[Q] = S/4); tp_chunk_g[p] = first
 *     group of chunk p in the reduce order.  run() multiplies piece by piece with the block of x
 *     in LDS and writes the products, in the multiply order, to a scratch array of S floats owned
 *     by the handle (runs of one handle with this plan must therefore not overlap), then sums
 *     chunk by chunk, fetching every group of the chunk through tp_from; sums are
 *     taken in a fixed order, so results are reproducible bit for bit.  AUTO picks TWOPHASE ahead
 *     of COLBLOCK when 16 n >= W (W as above: x of 256 KiB or more), nnz >= 3 * 2^21, C2 * P' <= 2^24,
 *     8 * C2 * P' <= nnz (tiles of eight entries or more on average; the rule takes P' = ceil((m +
 *     nnz) / tp_items), the chunk count before any cut is moved) and the columns are scattered:
 *     4 * sum_b nv_b >= 3 * E, with nv_b the distinct x vectors of row block b (the count pass of
 *     the x windows, which AUTO then also runs on a matrix headed for MERGE) and E the entries of
 *     the blocks counted (all but single rows longer than block_nnz).  Clustered columns - a band,
 *     a stencil too wide for the x windows - stay with the row-wise plans, whose gathers then
 *     share cache lines.  A forced TWOPHASE plan fails with UNSUPPORTED
 *     when C2 > 65535, C2 * P2 > 2^24 or nnz + 3 * C2 * P2 > SPMV_MAX_SIZE (a bound on S); with m == 0 or nnz == 0 it runs as
 *     SCALAR.  The library holds 13 + (4 or 2) bytes per slot of its own
 *     (13 + 8 * (4 or 2) per slot on groups, where a slot stands for eight entries).
 *     On groups (tp_group = 8).  A matrix is group-aligned when every row starts at a multiple of eight entries and every
 *     group of entries 8g .. 8g+7 has the columns c, c+1, .., c+7 with c a multiple of eight.  The two-pass plan is then
 *     laid out over the matrix of groups - m rows, ceil(n / 8) columns, nnz / 8 entries with rowptr / 8 and
 *     colidx[8g] / 8 - by the rules above, with column blocks of 2^12 (bf16) or 2^11 (binary32) groups' columns
 *     (64 KB of x either way): tp_src holds group numbers, tp_pos group positions within the chunk, a slot's value copy
 *     the group's eight values, and the product written for a slot is the dot product of those eight with their run of
 *     x.  An eighth of the slots; every size limit above then applies to the matrix of groups.  AUTO takes this
 *     form - ahead of the x windows, which are then not built - for a group-aligned matrix that the row lengths sent to
 *     ADAPTIVE or MERGE when x holds 1 MiB or more, the matrix of groups has 3 * 2^21 entries or more, C2 <= 65535,
 *     C2 * P' <= 2^24, 8 * C2 * P' <= nnz / 8 (P' = ceil((m + nnz / 8) / tp_items)), and the groups are scattered: 4 * VE * sum_b nv_b >= 3 * E (VE = x values per
 *     16-byte vector, nv_b and E as above).
 *   - the sliced ELL copy (plan SELL only; AUTO never picks it: on every matrix it measured the windowed or the
 *     tile kernel did better).  The ELL storage of paper App. C task 14 - rows of one width, col_id -1 marking
 *     padding - applied to slices of SPMV_SELL_HEIGHT = 64 consecutive rows (rows from m on count as
 *     empty): slice s is as wide as its longest row and takes width_s * 64 slots stored column by
 *     column, slot sell_ptr[s] + j * 64 + i belonging to entry j of the slice's i-th row; sell_col /
 *     sell_src hold the entry's column / its position in colidx and vals, -1 in both where the row
 *     has no such entry, and the library keeps a copy of the values in the same order (padding 0).
 *     run() gives a wavefront to every slice and a lane to every row: aligned contiguous loads,
 *     no row offsets, no cross-lane sums, x gathered from memory.  Fails with UNSUPPORTED when the copy would
 *     exceed SPMV_MAX_SIZE slots; with m == 0 or nnz == 0 it runs as SCALAR.  8 + (4 or 2) bytes per slot.
 *   - with prepare_spmm = 1: spmm_rows.  The rows
 *     are cut into windows of SPMV_SPMM_WINDOW consecutive rows; inside a window the row ids are
 *     sorted by decreasing key(len) = min(ceil(len / 4), 64), rows of equal key in ascending
 *     order.  spmm_csr_run() advances through a row four entries at a time, so rows of equal
 *     key keep a wavefront busy for the same number of steps; the windows keep the rows of C
 *     that are written at about the same time close together.
 *     On top of it, a packed copy of A in that order: group g = the rows at positions 16g ..
 *     16g+15 of spmm_rows (positions from m on: empty rows), stored as ceil(L_g / 16) blocks, L_g
 *     the longest row of the group.  Slot ((first_g + b) * 64 + 4 i + q) * 4 + e of spmm_col /
 *     spmm_val holds the entry of rank 16 b + 4 q + e of the group's i-th row (i = 0..15, q = 0..3,
 *     e = 0..3), or padding past the row's end: value 0 and column 2048 when n <= 2048, else all
 *     ones.  The ranks inside the row at position p of spmm_rows go by increasing
 *     4 * (earlier entries of the row whose column is congruent to the entry's modulo 4) +
 *     (column - p) mod 4: the entries are dealt out by column residue, turned by the row's position, so that the 16 rows
 *     a wavefront reads at once ask for different quarters of the LDS banks.  It is built when it has at most 2 * nnz slots and 2^22 blocks (spmm_prepared = 2);
 *     otherwise only spmm_rows is (spmm_prepared = 1) and spmm_csr_run() reads CSR.  The copy
 *     holds the values as they were at analyze time, as binary32 (bf16 values widened).
 * params == NULL means all defaults.  May be called again to re-plan (old metadata is freed).
 * Synchronises the device.  Errors: INVALID_ARG, BAD_STRUCTURE, ALLOC, HIP. */
spmv_status_t spmv_csr_analyze(spmv_handle_t h, const spmv_analyze_params_t* params);

/* Enqueues y <- alpha*A*x + beta*y on `stream` (a hipStream_t passed as void*; NULL = the
 * default stream).
 *   x  device, n elements of the handle's dtype;   y  device float[m], read only if beta != 0.
 *   x and y must not overlap.  beta == 0 never reads y (NaN/Inf there do not propagate).
 * m == 0 is a no-op; nnz == 0 gives y <- beta*y.
 * Errors: INVALID_ARG (null x or y with m, n > 0), NOT_ANALYZED, BUSY (see the conventions), HIP (launch failure). */
spmv_status_t spmv_csr_run(spmv_handle_t h, const void* x, float* y, float alpha, float beta, void* stream);

/* Sparse times dense (paper App. C task 13: C = A B, A in CSR, B of shape cols x K), in the BLAS
 * form  C <- alpha * A * B + beta * C,  enqueued on `stream`.
 *   h    an analyzed handle of either storage type (the benchmark gives every task an FP32 and a BF16
 *        variant, paper section 3.1): with SPMV_BF16 the values of A and B are bf16, products and
 *        sums binary32, C binary32.  The analysis validates the structure; the
 *        product itself uses rowptr / colidx / vals as they are.  A wavefront works on 16 rows
 *        at a time, for as long as the longest of them lasts: analysed with prepare_spmm = 1
 *        it takes them from spmm_rows, where rows of like length are neighbours (and from the
 *        packed copy where that was built: then vals as they were at analyze time);
 *        otherwise in their natural order.  The result is the same to rounding either way.
 *   B    device, elements of the handle's storage type (float, or uint16 bf16 bit patterns), n rows
 *        of K used columns, row-major, leading dimension ldb >= K (in elements).
 *   C    device float, m rows of K used columns, row-major, leading dimension ldc >= K; read only
 *        if beta != 0 (or when n exceeds 2048, where B is taken in several passes that accumulate
 *        into C).  B and C must not overlap.
 * Wide accesses are used when C is 16-byte aligned, B 16-byte (float) or 8-byte (bf16) aligned and
 * ldb, ldc are multiples of 4; any other layout works element by element.  m == 0 or K == 0 is a no-op.
 * Errors: INVALID_ARG (null B or C, K < 0, ldb or ldc < K), UNSUPPORTED (K > SPMV_MAX_SIZE,
 * pointers not aligned to their element size), NOT_ANALYZED, HIP. */
spmv_status_t spmm_csr_run(spmv_handle_t h, const void* B, int64_t ldb, float* C, int64_t ldc, int64_t K, float alpha,
                           float beta, void* stream);

/* The same product y <- alpha*A*x + beta*y with A in the benchmark's other storage layouts
 * (paper App. C tasks 8, 10, 14).  Stateless: every call takes the arrays (all DEVICE pointers,
 * borrowed for the duration of the enqueued work) and enqueues its kernels on `stream`.
 * dtype is the storage type of vals and x as for CSR.  Indices are NOT checked: rows must lie in
 * [0, m) and columns in [0, n), except for ELL padding slots.
 *   COO  vals[nnz], row_indices[nnz], col_indices[nnz] in any order; repeated coordinates add up.
 *   CSC  vals[nnz], row_indices[nnz], col_offsets[n+1] (col_offsets[j] = first entry of column j).
 *   ELL  vals[m*width], col_ids[m*width], row-major; a slot with col_id -1 is padding (its value
 *        is ignored).  width >= 0; m*width may exceed SPMV_MAX_SIZE (slots are addressed with
 *        64-bit offsets).
 * COO and CSC add the entries' contributions to y with float atomics (after y <- beta*y), so
 * their results are reproducible to rounding but not bit for bit; ELL is bit-reproducible.
 * beta == 0 never reads y.  Errors: INVALID_ARG (null pointer with a non-empty array, negative
 * size, unknown dtype), UNSUPPORTED (a size > SPMV_MAX_SIZE, misaligned pointer), HIP. */
spmv_status_t spmv_coo_run(int64_t m, int64_t n, int64_t nnz, const int32_t* row_indices, const int32_t* col_indices,
                           const void* vals, spmv_dtype_t dtype, const void* x, float* y, float alpha, float beta,
                           void* stream);
spmv_status_t spmv_csc_run(int64_t m, int64_t n, int64_t nnz, const int32_t* col_offsets, const int32_t* row_indices,
                           const void* vals, spmv_dtype_t dtype, const void* x, float* y, float alpha, float beta,
                           void* stream);
spmv_status_t spmv_ell_run(int64_t m, int64_t n, int64_t width, const int32_t* col_ids, const void* vals,
                           spmv_dtype_t dtype, const void* x, float* y, float alpha, float beta, void* stream);

/* Brings the library's own copies of the matrix values up to date after the caller has changed vals
 * in place (same structure, new numbers: the case of a nonlinear or time-stepping solver).  Four
 * things hold such copies: the COLBLOCK, TWOPHASE and SELL plans (values regrouped by column blocks / by
 * tiles / by slices) and the packed copy of the sparse-times-dense product; with none of them, this does nothing.  Enqueues on `stream`: no
 * allocation, no copy to the host, no synchronisation.  rowptr and colidx must be unchanged.
 * Errors: INVALID_ARG (null handle), NOT_ANALYZED, HIP. */
spmv_status_t spmv_csr_refresh_values(spmv_handle_t h, void* stream);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The product y <- alpha*A*x + beta*y of spmv_csr_run() under the MERGE plan (items_per_chunk 2048),
 * without a handle and without an analysis step: the merge-path splits are found by a small kernel, then the same
 * kernels run, so the result equals that of spmv_csr_run() on a handle analyzed with plan MERGE bit for bit.  Calls
 * no hipMalloc / hipFree and nothing else that allocates: the splits and the carries of cut rows (16 bytes per chunk of
 * 2048 steps) go to a fixed 2 MiB array in device memory that every GPU the library runs on holds until the process
 * ends, which limits the size to  m + nnz <= SPMV_STATIC_MAX_ITEMS  (larger: UNSUPPORTED, nothing is enqueued).
 * All calls on one GPU share that array: calls that overlap on one GPU (two streams, two threads) race; calls on one
 * stream, or ordered by events, are safe.  Nothing in the array has to be cleared between calls.
 *   rowptr / colidx / vals / x / y  DEVICE pointers as for spmv_csr_create() and spmv_csr_run(), borrowed until the
 *   enqueued work has finished.  The structure is NOT checked: rowptr must be non-decreasing from 0 to nnz and every
 *   column must lie in [0, n).  m == 0 is a no-op; nnz == 0 gives y <- beta*y.  Enqueues on `stream`, no synchronisation.
 * Errors: INVALID_ARG (null pointer with a non-empty array, negative size, unknown dtype), UNSUPPORTED (too large,
 * misaligned pointer), HIP. */
#define SPMV_STATIC_MAX_ITEMS (((int64_t)1 << 28) - 2048)
spmv_status_t spmv_csr_run_static(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr, const int32_t* colidx,
                                  const void* vals, spmv_dtype_t dtype, const void* x, float* y, float alpha, float beta,
                                  void* stream);

/* Frees the handle and the library-owned device metadata.  spmv_destroy(NULL) is OK. */
spmv_status_t spmv_destroy(spmv_handle_t h);

/* Sizes and scalars of the analysis, so the caller can size read-back buffers. */
spmv_status_t spmv_csr_get_analysis_info(spmv_handle_t h, spmv_analysis_info_t* out);

/* Copies the integer analysis outputs to the host buffers in `out`: from the device what the kernels read (x windows, row
 * patterns, column blocks, the two-pass layout, the sparse-times-dense order and packed copy), from the handle's own host
 * memory what was derived from rowptr on the host and is read by the kernels only through the interleaved descriptors
 * (bin_rows unless the plan is BINNED, row_blocks, mp_row, mp_nz). */
spmv_status_t spmv_csr_get_analysis(spmv_handle_t h, const spmv_analysis_host_t* out);

/* The analysis of spmv_csr_analyze() on a HOST copy of rowptr, with HOST outputs and no device
 * involved (same definitions, same code path; the column check is skipped, and with no colidx
 * there are no x windows and no column blocks: AUTO never yields WINDOWED or COLBLOCK here, and
 * asking for them is INVALID_ARG).  `info` is
 * required; `out` may be NULL or have NULL members.  bin_rows needs m entries, row_blocks
 * up to m+1, mp_row/mp_nz ceil((m+nnz)/items_per_chunk)+1.
 * Errors: INVALID_ARG, UNSUPPORTED, BAD_STRUCTURE, ALLOC. */
spmv_status_t spmv_analyze_host(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr_host,
                                const spmv_analyze_params_t* params, spmv_analysis_info_t* info,
                                const spmv_analysis_host_t* out);

/* Self-check of the cross-lane reductions the kernels use (DPP quad/mirror steps, ds_swizzle,
 * v_permlane32_swap).  in_dev: device float[64], one value per lane of a wavefront.
 * out_dev: device float[14*64]: out[gi*64 + l] = sum over the aligned group of 2^gi lanes that
 * contains lane l, gi = 0..6 (compile-time group size), then the same seven rows again from
 * the run-time-group-size variant.  Enqueues one wavefront on `stream`. */
spmv_status_t spmv_selftest_reduce(const float* in_dev, float* out_dev, void* stream);

/* Name of the kernel that carries the nnz stream for the handle's current plan ("" before
 * analyze); lets a profiler summary be matched to the plan. */
const char* spmv_csr_main_kernel_name(spmv_handle_t h);

const char* spmv_status_string(spmv_status_t s);

/* hipError_t (as int) of the most recent failing HIP call made by this library on the calling
 * thread; 0 if none. */
int spmv_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SPMV_MI355_H */
