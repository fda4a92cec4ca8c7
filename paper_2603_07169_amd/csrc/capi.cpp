// C ABI of the library: handle life cycle, analysis upload, plan dispatch.
// See include/spmv_mi355.h for the contract of every entry point.
#include <hip/hip_runtime_api.h>

#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "analysis.h"
#include "kernels.h"
#include "spmv_mi355.h"

namespace {

thread_local int g_last_hip_error = 0;

inline bool hip_failed(hipError_t e) {
    if (e == hipSuccess) return false;
    g_last_hip_error = static_cast<int>(e);
    (void)hipGetLastError();  // clear the sticky per-thread error so later calls start clean
    return true;
}

constexpr int64_t kMaxCount = SPMV_MAX_SIZE;  // an index plus a grid stride (at most 2^21) stays inside int32

}  // namespace

namespace spmv {
bool note_hip_error(hipError_t e) { return hip_failed(e); }
}  // namespace spmv

struct spmv_csr_s {
    int64_t m = 0, n = 0, nnz = 0;
    const int32_t* rowptr = nullptr;
    const int32_t* colidx = nullptr;
    const void* vals = nullptr;
    spmv_dtype_t dtype = SPMV_F32;
    bool vec_ok = false;

    bool analyzed = false;
    spmv_analysis_info_t info{};
    int32_t bin_count[SPMV_NUM_BINS]{};
    int32_t bin_offset[SPMV_NUM_BINS + 1]{};
    // device metadata, owned
    int32_t* d_bin_rows = nullptr;  // uploaded for the BINNED plan only (the one plan whose kernels read it)
    // analysis outputs that no kernel reads in this form stay on the host, for the read-back
    std::vector<int32_t> bin_rows, row_blocks, mp_row, mp_nz;
    int32_t* d_block_nz = nullptr;  // rowptr[row_blocks[b]]: spares the kernels a dependent load
    int32_t* d_block_desc = nullptr;  // pairs (row_blocks[b], block_nz[b]): one scalar load per workgroup
    int32_t* d_chunk_desc = nullptr;  // pairs (mp_row[p], mp_nz[p])
    int32_t* d_cb_row = nullptr;   // column blocks (COLBLOCK plan)
    int32_t* d_cb_col = nullptr;
    int32_t* d_cb_src = nullptr;
    void* d_cb_vals = nullptr;
    std::vector<int32_t> cb_ptr;   // host: [C+1]
    int32_t max_block_entries = 0;  // most entries of any row block that is not a single over-long row
    int32_t* d_carry_row = nullptr;
    float* d_carry_val = nullptr;
    int32_t* d_xv_ptr = nullptr;  // x windows (WINDOWED plan)
    int32_t* d_xv_start = nullptr;
    int32_t* d_xv_pad = nullptr;
    uint16_t* d_lidx = nullptr;
    uint16_t* d_lidx8 = nullptr;  // lidx[8g], kept when the window positions are grouped (info.lidx_grouped)
    int32_t* d_run_desc = nullptr;  // row patterns of the window positions, kept when info.lidx_patterned
    uint16_t* d_pat_pad = nullptr;
    // the two-pass plan (TWOPHASE)
    int32_t* d_tp_desc = nullptr;     // pairs (tp_row[p], tp_nz[p])
    int32_t* d_tp_piece_c = nullptr;
    int32_t* d_tp_piece_g = nullptr;
    int32_t* d_tp_chunk_g = nullptr;
    uint16_t* d_tp_col = nullptr;
    void* d_tp_val = nullptr;
    int32_t* d_tp_src = nullptr;
    int32_t* d_tp_from = nullptr;
    uint16_t* d_tp_pos = nullptr;
    float* d_tp_prod = nullptr;
    int32_t* d_tp_carry_row = nullptr;
    float* d_tp_carry_val = nullptr;
    size_t tp_reduce_lds = 0;
    std::vector<int32_t> tp_row, tp_nz;  // host copies for the read-back
    bool tp_carries = true;              // some chunk of the two-pass plan cuts a row
    // The MERGE and TWOPHASE plans keep scratch in the handle (carries, products): a run on another stream while one is
    // still in flight would share it.  An event recorded behind every such run tells.
    hipEvent_t scratch_free = nullptr;
    hipStream_t scratch_stream = nullptr;
    bool scratch_used = false;
    int32_t* d_sell_ptr = nullptr;  // the sliced ELL copy (SELL plan)
    int32_t* d_sell_col = nullptr;
    int32_t* d_sell_src = nullptr;
    void* d_sell_val = nullptr;
    std::vector<int32_t> sell_ptr;  // host copy for the read-back
    int32_t* d_spmm_rows = nullptr;  // row order of spmm_csr_run (prepare_spmm)
    int32_t* d_spmm_desc = nullptr;  // packed copy of A in that order (spmm_prepared == 2)
    void* d_spmm_col = nullptr;
    float* d_spmm_val = nullptr;
};

namespace {

void free_metadata(spmv_csr_s* h) {
    void* ptrs[] = {h->d_bin_rows, h->d_block_nz,
                    h->d_carry_row, h->d_carry_val, h->d_xv_ptr,   h->d_xv_start, h->d_lidx,
                    h->d_xv_pad,    h->d_block_desc, h->d_chunk_desc, h->d_cb_row, h->d_cb_col,
                    h->d_cb_src,    h->d_cb_vals,   h->d_spmm_rows, h->d_spmm_desc, h->d_spmm_col,
                    h->d_spmm_val,  h->d_tp_desc,   h->d_tp_piece_c, h->d_tp_piece_g, h->d_tp_chunk_g,
                    h->d_tp_col,    h->d_tp_val,    h->d_tp_src,    h->d_tp_from,    h->d_tp_pos,
                    h->d_tp_prod,   h->d_tp_carry_row, h->d_tp_carry_val, h->d_lidx8, h->d_run_desc, h->d_pat_pad,
                    h->d_sell_ptr,  h->d_sell_col,  h->d_sell_src,  h->d_sell_val};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    h->d_tp_desc = h->d_tp_piece_c = h->d_tp_piece_g = h->d_tp_chunk_g = h->d_tp_src = h->d_tp_from = nullptr;
    h->d_tp_carry_row = nullptr;
    h->d_tp_col = h->d_tp_pos = nullptr;
    h->d_tp_val = nullptr;
    h->d_tp_prod = h->d_tp_carry_val = nullptr;
    h->tp_row.clear();
    h->tp_nz.clear();
    h->d_bin_rows = h->d_block_nz = h->d_carry_row = nullptr;
    h->bin_rows.clear();
    h->row_blocks.clear();
    h->mp_row.clear();
    h->mp_nz.clear();
    h->d_carry_val = nullptr;
    h->d_xv_ptr = h->d_xv_start = h->d_xv_pad = h->d_block_desc = h->d_chunk_desc = nullptr;
    h->d_cb_row = h->d_cb_col = h->d_cb_src = nullptr;
    h->d_cb_vals = nullptr;
    h->cb_ptr.clear();
    h->d_lidx = h->d_lidx8 = h->d_pat_pad = nullptr;
    h->d_run_desc = nullptr;
    h->d_sell_ptr = h->d_sell_col = h->d_sell_src = nullptr;
    h->d_sell_val = nullptr;
    h->sell_ptr.clear();
    h->d_spmm_rows = h->d_spmm_desc = nullptr;
    h->d_spmm_col = nullptr;
    h->d_spmm_val = nullptr;
    if (h->scratch_free) (void)hipEventDestroy(h->scratch_free);
    h->scratch_free = nullptr;
    h->scratch_used = false;
    h->analyzed = false;
}

// Plans whose kernels write scratch owned by the handle.
inline bool plan_has_scratch(int32_t plan) { return plan == SPMV_PLAN_MERGE || plan == SPMV_PLAN_TWOPHASE; }

// Before a run that uses the handle's scratch: SPMV_ERR_BUSY when an earlier run on another stream has not finished.
// Nothing is asked of a stream under capture (the queries are not allowed there): *tracked says whether to record.
spmv_status_t scratch_acquire(spmv_csr_s* h, hipStream_t st, bool* tracked) {
    *tracked = false;
    if (!h->scratch_free) return SPMV_OK;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (st != nullptr && (hip_failed(hipStreamIsCapturing(st, &cs)) || cs != hipStreamCaptureStatusNone)) return SPMV_OK;
    *tracked = true;
    if (h->scratch_used && st != h->scratch_stream) {
        const hipError_t e = hipEventQuery(h->scratch_free);
        if (e == hipErrorNotReady) {
            (void)hipGetLastError();
            return SPMV_ERR_BUSY;
        }
        if (hip_failed(e)) return SPMV_ERR_HIP;
    }
    return SPMV_OK;
}

template <typename T>
spmv_status_t upload(const std::vector<T>& src, T** dst) {
    const size_t bytes = sizeof(T) * (src.empty() ? 1 : src.size());
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(dst), bytes))) return SPMV_ERR_ALLOC;
    if (!src.empty() && hip_failed(hipMemcpy(*dst, src.data(), sizeof(T) * src.size(), hipMemcpyHostToDevice)))
        return SPMV_ERR_HIP;
    return SPMV_OK;
}

spmv::MatrixView view_of(const spmv_csr_s* h) {
    spmv::MatrixView A{};
    A.m = static_cast<int32_t>(h->m);
    A.n = static_cast<int32_t>(h->n);
    A.nnz = static_cast<int32_t>(h->nnz);
    A.rowptr = h->rowptr;
    A.colidx = h->colidx;
    A.vals = h->vals;
    A.bf16 = h->dtype == SPMV_BF16;
    A.vec_ok = h->vec_ok;
    return A;
}

// Counts the x vectors of every row block on the device, settles the plan (AUTO: ADAPTIVE or
// WINDOWED) and, for WINDOWED, builds xv_ptr / xv_start / lidx.  Needs d_block_nz.
// count_only: stop after the count (it also says how scattered the columns are).
// The host copy of rowptr that the analysis works on.  The copy lands in pinned memory (a pageable destination makes the
// runtime stage it piece by piece: 1.3 ms for 16 MB against 0.4 ms), in one process-wide buffer that grows as needed and is
// handed to one analysis at a time; an analysis that finds it taken uses pageable memory of its own.
class HostRowptr {
   public:
    HostRowptr() = default;
    HostRowptr(const HostRowptr&) = delete;
    HostRowptr& operator=(const HostRowptr&) = delete;
    ~HostRowptr() {
        if (pinned_) pool().busy.unlock();
    }
    // Copies count numbers from device memory; false on failure (allocation or copy).
    bool download(const int32_t* device, size_t count) {
        count_ = count;
        Pool& pl = pool();
        if (pl.busy.try_lock()) {
            pinned_ = true;
            if (pl.capacity < count) {
                if (pl.data) (void)hipHostFree(pl.data);
                pl.data = nullptr;
                pl.capacity = 0;
                void* fresh = nullptr;
                if (hipHostMalloc(&fresh, sizeof(int32_t) * count, hipHostMallocDefault) == hipSuccess) {
                    pl.data = static_cast<int32_t*>(fresh);
                    pl.capacity = count;
                } else {
                    (void)hipGetLastError();
                }
            }
            if (pl.data) {
                data_ = pl.data;
                return hipMemcpy(pl.data, device, sizeof(int32_t) * count, hipMemcpyDeviceToHost) == hipSuccess;
            }
            pinned_ = false;
            pl.busy.unlock();
        }
        own_.reset(new (std::nothrow) int32_t[count]);
        if (!own_) return false;
        data_ = own_.get();
        return hipMemcpy(own_.get(), device, sizeof(int32_t) * count, hipMemcpyDeviceToHost) == hipSuccess;
    }
    const int32_t* data() const { return data_; }
    size_t size() const { return count_; }
    int32_t operator[](size_t i) const { return data_[i]; }
    const int32_t* begin() const { return data_; }
    const int32_t* end() const { return data_ + count_; }

   private:
    struct Pool {
        std::mutex busy;
        int32_t* data = nullptr;  // never freed: it outlives every handle, and the runtime may be gone at exit
        size_t capacity = 0;
    };
    static Pool& pool() {
        static Pool* p = new Pool;
        return *p;
    }
    const int32_t* data_ = nullptr;
    size_t count_ = 0;
    bool pinned_ = false;
    std::unique_ptr<int32_t[]> own_;
};

spmv_status_t check_groups(spmv_csr_s* h, const HostRowptr& rowptr_host, bool* aligned, int32_t** d_gcol);

spmv_status_t build_x_windows(spmv_csr_s* h, bool forced, bool count_only, const HostRowptr& rowptr_host,
                              spmv::Analysis* a) {
    const int64_t nb = a->info.num_row_blocks;
    const spmv::MatrixView A = view_of(h);
    std::vector<int32_t> nv, xv_ptr;
    try {
        nv.assign(static_cast<size_t>(nb > 0 ? nb : 1), 0);
        xv_ptr.assign(static_cast<size_t>(nb) + 1, 0);
    } catch (const std::bad_alloc&) {
        return SPMV_ERR_ALLOC;
    }
    int32_t* d_nv = nullptr;
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(&d_nv), sizeof(int32_t) * nv.size()))) return SPMV_ERR_ALLOC;
    bool bad = hip_failed(spmv::launch_window_build(A, h->d_block_nz, static_cast<int32_t>(nb), a->info.block_nnz, false,
                                                    d_nv, nullptr, nullptr, nullptr, 0, nullptr, nullptr));
    bad = bad || (nb > 0 && hip_failed(hipMemcpy(nv.data(), d_nv, sizeof(int32_t) * static_cast<size_t>(nb),
                                                 hipMemcpyDeviceToHost)));
    (void)hipFree(d_nv);
    if (bad) return SPMV_ERR_HIP;

    int64_t total = 0;
    int32_t largest = 0;
    const bool pays = spmv::window_choice(nv.data(), nb, h->nnz, &total, &largest);
    a->info.max_x_vectors = largest;
    a->x_vectors_counted = total;
    a->entries_counted = 0;
    for (int64_t b = 0; b < nb; ++b) {
        const int64_t entries = static_cast<int64_t>(rowptr_host[static_cast<size_t>(a->row_blocks[static_cast<size_t>(b) + 1])]) -
                                rowptr_host[static_cast<size_t>(a->row_blocks[static_cast<size_t>(b)])];
        if (entries <= a->info.block_nnz) a->entries_counted += entries;
    }
    // AUTO: a group-aligned matrix with scattered groups goes through the two passes on its groups instead (the windows
    // are then not built); the sizes are looked at first, the columns only when they allow it
    if (!forced && spmv::grouped_two_phase_choice(h->m, h->n, h->nnz, h->dtype, a->info.plan, true, total, a->entries_counted)) {
        bool aligned = false;
        const spmv_status_t gs = check_groups(h, rowptr_host, &aligned, &a->d_group_cols);
        if (gs != SPMV_OK) return gs;
        if (aligned) {
            a->two_phase_on_groups = true;
            return SPMV_OK;
        }
    }
    if (count_only) return SPMV_OK;
    if (forced && largest > SPMV_MAX_X_VECTORS) return SPMV_ERR_UNSUPPORTED;
    if (!forced && !pays) return SPMV_OK;  // stays ADAPTIVE
    const int32_t x_cap = largest > 0 ? largest : 1;
    const int64_t padded = nb * static_cast<int64_t>(x_cap);
    if (padded > kMaxCount) return SPMV_ERR_UNSUPPORTED;

    for (int64_t b = 0; b < nb; ++b) xv_ptr[static_cast<size_t>(b) + 1] = xv_ptr[static_cast<size_t>(b)] + nv[static_cast<size_t>(b)];
    spmv_status_t st = upload(xv_ptr, &h->d_xv_ptr);
    if (st != SPMV_OK) return st;
    const size_t lidx_slots = (static_cast<size_t>(h->nnz) + 7) / 8 * 8 + 8;
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_xv_start), sizeof(int32_t) * static_cast<size_t>(total > 0 ? total : 1))) ||
        hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_xv_pad), sizeof(int32_t) * static_cast<size_t>(padded > 0 ? padded : 1))) ||
        hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_lidx), sizeof(uint16_t) * lidx_slots)))
        return SPMV_ERR_ALLOC;
    if (hip_failed(hipMemset(h->d_lidx, 0, sizeof(uint16_t) * lidx_slots))) return SPMV_ERR_HIP;
    if (hip_failed(spmv::launch_window_build(A, h->d_block_nz, static_cast<int32_t>(nb), a->info.block_nnz, true, nullptr,
                                             h->d_xv_ptr, h->d_xv_start, h->d_xv_pad, x_cap, h->d_lidx, nullptr)))
        return SPMV_ERR_HIP;
    // Grouped positions: every aligned group of eight entries inside one row block (all blocks start at a multiple
    // of eight) and at eight consecutive window positions.  The kernel then reads one position per group.
    bool aligned_blocks = h->nnz >= 8;
    for (int64_t b = 0; b < nb && aligned_blocks; ++b)
        aligned_blocks = rowptr_host[static_cast<size_t>(a->row_blocks[static_cast<size_t>(b)])] % 8 == 0;
    if (aligned_blocks) {
        const int32_t groups = static_cast<int32_t>(h->nnz / 8);
        int32_t* d_flag = nullptr;
        int32_t flag = 0;
        if (hip_failed(hipMalloc(reinterpret_cast<void**>(&d_flag), sizeof(int32_t))) ||
            hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_lidx8), sizeof(uint16_t) * static_cast<size_t>(groups)))) {
            (void)hipFree(d_flag);
            return SPMV_ERR_ALLOC;
        }
        bool failed = hip_failed(hipMemcpy(d_flag, &flag, sizeof flag, hipMemcpyHostToDevice));
        failed = failed || hip_failed(spmv::launch_lidx_groups(h->d_lidx, groups, h->d_lidx8, d_flag, nullptr));
        failed = failed || hip_failed(hipMemcpy(&flag, d_flag, sizeof flag, hipMemcpyDeviceToHost));
        (void)hipFree(d_flag);
        if (failed) return SPMV_ERR_HIP;
        if (flag != 0) {
            (void)hipFree(h->d_lidx8);
            h->d_lidx8 = nullptr;
        }
        a->info.lidx_grouped = flag == 0 ? 1 : 0;
    }
    // Row patterns (stencils): where the positions are not grouped, look for runs of rows whose positions repeat with a
    // constant step; when the patterned blocks hold half of the entries or more, run() works from the patterns.
    if (!a->info.lidx_grouped && nb > 0) {
        struct Counts {
            unsigned long long covered;
            int32_t max_table, pad;
        } counts{0, 0, 0};
        Counts* d_counts = nullptr;
        if (hip_failed(hipMalloc(reinterpret_cast<void**>(&d_counts), sizeof(Counts))) ||
            hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_run_desc), 32 * static_cast<size_t>(nb)))) {
            (void)hipFree(d_counts);
            return SPMV_ERR_ALLOC;
        }
        bool failed = hip_failed(hipMemcpy(d_counts, &counts, sizeof counts, hipMemcpyHostToDevice));
        failed = failed || hip_failed(spmv::launch_pattern_build(h->d_block_desc, static_cast<int32_t>(nb), h->rowptr, h->d_lidx,
                                                                 a->info.block_nnz, false, h->d_run_desc, &d_counts->max_table,
                                                                 &d_counts->covered, nullptr, 0, nullptr));
        failed = failed || hip_failed(hipMemcpy(&counts, d_counts, sizeof counts, hipMemcpyDeviceToHost));
        (void)hipFree(d_counts);
        if (failed) return SPMV_ERR_HIP;
        const int64_t covered = static_cast<int64_t>(counts.covered);
        const int32_t pt_cap = counts.max_table > 0 ? (counts.max_table + 7) / 8 * 8 : 8;
        if (h->nnz > 0 && 2 * covered >= h->nnz && nb * static_cast<int64_t>(pt_cap) <= kMaxCount) {
            if (hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_pat_pad), 2 * static_cast<size_t>(nb) * static_cast<size_t>(pt_cap))))
                return SPMV_ERR_ALLOC;
            if (hip_failed(spmv::launch_pattern_build(h->d_block_desc, static_cast<int32_t>(nb), h->rowptr, h->d_lidx, a->info.block_nnz,
                                                      true, h->d_run_desc, nullptr, nullptr, h->d_pat_pad, pt_cap, nullptr)))
                return SPMV_ERR_HIP;
            a->info.lidx_patterned = 1;
            a->info.pat_cap = pt_cap;
            a->info.pat_entries = covered;
        } else {
            (void)hipFree(h->d_run_desc);
            h->d_run_desc = nullptr;
        }
    }
    a->info.plan = SPMV_PLAN_WINDOWED;
    a->info.num_x_vectors = total;
    return SPMV_OK;
}

// Regroups the entries by blocks of columns on the device (two kernel passes with a prefix sum on
// the host in between) and switches the plan to COLBLOCK.
spmv_status_t build_column_blocks(spmv_csr_s* h, spmv::Analysis* a) {
    const int64_t width = spmv::column_block_width(h->dtype);
    const int64_t C64 = h->n > 0 ? (h->n + width - 1) / width : 1;
    if (C64 > spmv::kMaxColBlocks) return SPMV_ERR_UNSUPPORTED;
    const int C = static_cast<int>(C64);
    int shift = 0;
    while ((int64_t{1} << shift) < width) ++shift;
    const spmv::MatrixView A = view_of(h);
    const int32_t ntiles = spmv::column_block_tiles(A.nnz);
    std::vector<int32_t> counts;
    try {
        counts.assign(static_cast<size_t>(C) * static_cast<size_t>(ntiles > 0 ? ntiles : 1), 0);
        h->cb_ptr.assign(static_cast<size_t>(C) + 1, 0);
    } catch (const std::bad_alloc&) {
        return SPMV_ERR_ALLOC;
    }
    int32_t* d_counts = nullptr;
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(&d_counts), sizeof(int32_t) * counts.size()))) return SPMV_ERR_ALLOC;
    spmv_status_t st = SPMV_OK;
    if (hip_failed(spmv::launch_column_block_count(A, shift, C, d_counts, nullptr)) ||
        hip_failed(hipMemcpy(counts.data(), d_counts, sizeof(int32_t) * counts.size(), hipMemcpyDeviceToHost)))
        st = SPMV_ERR_HIP;
    if (st == SPMV_OK) {
        int64_t run = 0;  // exclusive prefix in (block, tile) order; cb_ptr picks up the block starts
        for (int b = 0; b < C; ++b) {
            h->cb_ptr[static_cast<size_t>(b)] = static_cast<int32_t>(run);
            for (int32_t t = 0; t < ntiles; ++t) {
                int32_t& c = counts[static_cast<size_t>(b) * static_cast<size_t>(ntiles) + static_cast<size_t>(t)];
                const int32_t n_here = c;
                c = static_cast<int32_t>(run);
                run += n_here;
            }
        }
        h->cb_ptr[static_cast<size_t>(C)] = static_cast<int32_t>(run);
        const size_t slots = static_cast<size_t>(h->nnz > 0 ? h->nnz : 1);
        if (hip_failed(hipMemcpy(d_counts, counts.data(), sizeof(int32_t) * counts.size(), hipMemcpyHostToDevice)))
            st = SPMV_ERR_HIP;
        else if (hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_cb_row), sizeof(int32_t) * slots)) ||
                 hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_cb_col), sizeof(int32_t) * slots)) ||
                 hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_cb_src), sizeof(int32_t) * slots)) ||
                 hip_failed(hipMalloc(&h->d_cb_vals, (h->dtype == SPMV_F32 ? 4 : 2) * slots)))
            st = SPMV_ERR_ALLOC;
        else if (hip_failed(hipMemset(h->d_cb_src, 0xFF, sizeof(int32_t) * slots)))  // -1: a slot no entry was placed in
            st = SPMV_ERR_HIP;
        else if (hip_failed(spmv::launch_column_block_scatter(A, shift, C, d_counts, h->d_cb_row, h->d_cb_col, h->d_cb_src,
                                                              h->d_cb_vals, nullptr)) ||
                 hip_failed(hipDeviceSynchronize()))
            st = SPMV_ERR_HIP;
    }
    (void)hipFree(d_counts);
    if (st != SPMV_OK) return st;
    a->info.plan = SPMV_PLAN_COLBLOCK;
    a->info.num_col_blocks = C;
    a->info.col_block_width = static_cast<int32_t>(width);
    return SPMV_OK;
}

// Is the matrix group-aligned (every row a whole number of groups of eight entries, every group an aligned run of eight
// consecutive columns)?  The rows are checked on the host; the columns on the device, which also leaves the groups'
// columns in *d_gcol (allocated here, the caller frees it) when the answer is yes.
spmv_status_t check_groups(spmv_csr_s* h, const HostRowptr& rowptr_host, bool* aligned, int32_t** d_gcol) {
    *aligned = false;
    *d_gcol = nullptr;
    if (h->nnz == 0 || h->nnz % spmv::kTpGroup != 0) return SPMV_OK;
    for (int32_t r : rowptr_host)
        if (r % spmv::kTpGroup != 0) return SPMV_OK;
    const int32_t ngroups = static_cast<int32_t>(h->nnz / spmv::kTpGroup);
    int32_t* d_flag = nullptr;
    int32_t flag = 0;
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(d_gcol), sizeof(int32_t) * static_cast<size_t>(ngroups))) ||
        hip_failed(hipMalloc(reinterpret_cast<void**>(&d_flag), sizeof(int32_t)))) {
        (void)hipFree(*d_gcol);
        *d_gcol = nullptr;
        return SPMV_ERR_ALLOC;
    }
    bool failed = hip_failed(hipMemcpy(d_flag, &flag, sizeof flag, hipMemcpyHostToDevice));
    failed = failed || hip_failed(spmv::launch_two_phase_groups(h->colidx, ngroups, *d_gcol, d_flag, nullptr));
    failed = failed || hip_failed(hipMemcpy(&flag, d_flag, sizeof flag, hipMemcpyDeviceToHost));
    (void)hipFree(d_flag);
    if (failed || flag != 0) {
        (void)hipFree(*d_gcol);
        *d_gcol = nullptr;
        return failed ? SPMV_ERR_HIP : SPMV_OK;
    }
    *aligned = true;
    return SPMV_OK;
}

// Regroups the entries for the two-pass plan on the device (a count per chunk and column block, prefix
// sums in both orders, a placement pass that keeps the CSR order inside a tile) and switches the plan to TWOPHASE.
// d_gcol != nullptr: the matrix is group-aligned and the plan is laid out over its matrix of groups (m rows,
// ceil(n / 8) columns, nnz / 8 entries whose columns are d_gcol): a slot then stands for eight entries.
spmv_status_t build_two_phase(spmv_csr_s* h, const HostRowptr& rowptr_host, spmv::Analysis* a, const int32_t* d_gcol) try {
    if (h->m == 0 || h->nnz == 0) {
        a->info.plan = SPMV_PLAN_SCALAR;
        return SPMV_OK;
    }
    const int group = d_gcol ? spmv::kTpGroup : 1;
    const int shift = d_gcol ? spmv::two_phase_group_shift(h->dtype) : spmv::two_phase_shift(h->n);
    const int64_t ncols = d_gcol ? (h->n + group - 1) / group : h->n, nent = h->nnz / group;
    const int64_t C = (ncols + (int64_t{1} << shift) - 1) >> shift;
    std::vector<int32_t> rowptr_groups;
    if (d_gcol) {
        rowptr_groups.resize(rowptr_host.size());
        for (size_t i = 0; i < rowptr_host.size(); ++i) rowptr_groups[i] = rowptr_host[i] / group;
    }
    const int32_t* const rowptr_used = d_gcol ? rowptr_groups.data() : rowptr_host.data();
    h->tp_carries = spmv::merge_path_splits_snapped(h->m, nent, rowptr_used, spmv::kTwoPhaseItems, spmv::kTwoPhaseSnap, &h->tp_row, &h->tp_nz);
    const int64_t P = static_cast<int64_t>(h->tp_row.size()) - 1;
    if (C > 65535 || C * P > spmv::kTwoPhaseMaxTiles) return SPMV_ERR_UNSUPPORTED;
    spmv::MatrixView A = view_of(h);
    if (d_gcol) {  // the matrix of groups, as far as the regrouping kernels look at it
        A.n = static_cast<int32_t>(ncols);
        A.nnz = static_cast<int32_t>(nent);
        A.colidx = d_gcol;
        A.vals = nullptr;
    }
    const size_t T = static_cast<size_t>(C * P);

    std::vector<int32_t> desc(2 * h->tp_row.size());
    size_t lds = 0;
    for (size_t q = 0; q < h->tp_row.size(); ++q) {
        desc[2 * q] = h->tp_row[q];
        desc[2 * q + 1] = h->tp_nz[q];
        if (q > 0) lds = std::max(lds, spmv::two_phase_reduce_lds(h->tp_nz[q] - h->tp_nz[q - 1], h->tp_row[q] - h->tp_row[q - 1]));
    }
    h->tp_reduce_lds = lds;
    spmv_status_t st = upload(desc, &h->d_tp_desc);
    if (st != SPMV_OK) return st;

    // 32-bit prefix sums on the device: every tile adds at most three slots of padding
    if (nent + 3 * C * P > kMaxCount) return SPMV_ERR_UNSUPPORTED;
    // temporaries of the regrouping: one allocation, cut into 256-byte aligned stretches
    const size_t P1 = static_cast<size_t>(P) + 1, C1 = static_cast<size_t>(C) + 1;
    const size_t stretch[] = {4 * T, 4 * T, 4 * T, 4 * P1, 4 * P1, 4 * C1,
                              4 * static_cast<size_t>(spmv::two_phase_scan_blocks(static_cast<int64_t>(T) + 1))};
    constexpr int kStretches = sizeof(stretch) / sizeof(stretch[0]);
    size_t offset[kStretches + 1] = {0};
    for (int i = 0; i < kStretches; ++i) offset[i + 1] = offset[i] + (stretch[i] + 255) / 256 * 256;
    char* pool = nullptr;
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(&pool), offset[kStretches]))) return SPMV_ERR_ALLOC;
    auto at = [&](int i) { return reinterpret_cast<int32_t*>(pool + offset[i]); };
    spmv::TwoPhaseTables w{};
    w.padded = at(0);
    w.base1 = at(1);
    w.within = at(2);
    w.in_chunk = at(3);
    w.chunk_first = at(4);
    w.block_first = at(5);
    w.scan_sums = at(6);
    auto release = [&] { (void)hipFree(pool); };

    // counts per (column block, chunk) -> prefix sums in both orders, all on the device; the host only needs where the
    // column blocks start (to cut them into pieces) and the total
    std::vector<int32_t> block_first(C1), piece_c, piece_g;
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_chunk_g), 4 * P1))) {
        release();
        return SPMV_ERR_ALLOC;
    }
    if (hip_failed(spmv::launch_two_phase_tables(A, shift, static_cast<int32_t>(C), static_cast<int32_t>(P), h->d_tp_desc, w,
                                                 h->d_tp_chunk_g, nullptr)) ||
        hip_failed(hipMemcpy(block_first.data(), w.block_first, 4 * C1, hipMemcpyDeviceToHost))) {
        release();
        return SPMV_ERR_HIP;
    }
    const int64_t slots = block_first[static_cast<size_t>(C)];
    // the multiply pass keeps two workgroups of 1024 lanes (64 KB of LDS each) on a compute unit
    int dev = 0, cus = 0;
    if (hip_failed(hipGetDevice(&dev)) || hip_failed(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev))) {
        release();
        return SPMV_ERR_HIP;
    }
    const int32_t piece_groups = spmv::two_phase_piece_groups(C, block_first.data(), 2 * cus, spmv::kTwoPhaseWaves);
    spmv::two_phase_pieces(C, block_first.data(), piece_groups, &piece_c, &piece_g);
    const size_t S = static_cast<size_t>(slots);
    st = upload(piece_c, &h->d_tp_piece_c);
    if (st == SPMV_OK) st = upload(piece_g, &h->d_tp_piece_g);
    if (st == SPMV_OK &&
        (hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_col), 2 * S)) ||
         hip_failed(hipMalloc(&h->d_tp_val, static_cast<size_t>(group) * (h->dtype == SPMV_F32 ? 4 : 2) * S)) ||
         hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_src), 4 * S)) ||
         hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_from), S)) ||
         hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_pos), 2 * S)) ||
         hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_prod), 4 * S)) ||
         hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_carry_row), 4 * static_cast<size_t>(P))) ||
         hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_tp_carry_val), 4 * static_cast<size_t>(P)))))
        st = SPMV_ERR_ALLOC;
    if (st == SPMV_OK &&
        (hip_failed(spmv::launch_two_phase_place(A, shift, static_cast<int32_t>(C), static_cast<int32_t>(P), w, h->d_tp_desc,
                                                 slots, group, h->d_tp_col, h->d_tp_val, h->d_tp_src, h->d_tp_from, h->d_tp_pos,
                                                 nullptr)) ||
         (group > 1 && hip_failed(spmv::launch_two_phase_values(view_of(h), h->d_tp_src, h->d_tp_val, slots, group, nullptr))) ||
         hip_failed(hipDeviceSynchronize())))
        st = SPMV_ERR_HIP;
    release();
    if (st != SPMV_OK) return st;
    a->info.plan = SPMV_PLAN_TWOPHASE;
    a->info.tp_slots = slots;
    a->info.tp_col_shift = shift;
    a->info.tp_items = spmv::kTwoPhaseItems;
    a->info.tp_piece_groups = piece_groups;
    a->info.tp_resident = 2 * cus;
    a->info.tp_num_col_blocks = static_cast<int32_t>(C);
    a->info.tp_num_chunks = static_cast<int32_t>(P);
    a->info.tp_num_pieces = static_cast<int32_t>(piece_c.size());
    a->info.tp_group = group;
    return SPMV_OK;
} catch (const std::bad_alloc&) {
    return SPMV_ERR_ALLOC;
}

// Builds the sliced ELL copy (slice widths on the host from rowptr, the slots on the device) and switches the plan to SELL.
spmv_status_t build_sell(spmv_csr_s* h, const HostRowptr& rowptr_host, spmv::Analysis* a) try {
    if (h->m == 0 || h->nnz == 0) {
        a->info.plan = SPMV_PLAN_SCALAR;
        return SPMV_OK;
    }
    constexpr int64_t H = spmv::kSellHeight;
    const int64_t ns = (h->m + H - 1) / H;
    h->sell_ptr.assign(static_cast<size_t>(ns) + 1, 0);
    int64_t slots = 0;
    for (int64_t s = 0; s < ns; ++s) {
        int64_t width = 0;
        const int64_t r1 = std::min<int64_t>(h->m, (s + 1) * H);
        for (int64_t r = s * H; r < r1; ++r)
            width = std::max<int64_t>(width, static_cast<int64_t>(rowptr_host[static_cast<size_t>(r) + 1]) - rowptr_host[static_cast<size_t>(r)]);
        h->sell_ptr[static_cast<size_t>(s)] = static_cast<int32_t>(slots);
        slots += width * H;
        if (slots > kMaxCount) return SPMV_ERR_UNSUPPORTED;
    }
    h->sell_ptr[static_cast<size_t>(ns)] = static_cast<int32_t>(slots);
    spmv_status_t st = upload(h->sell_ptr, &h->d_sell_ptr);
    if (st != SPMV_OK) return st;
    const size_t S = static_cast<size_t>(slots > 0 ? slots : 1);
    if (hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_sell_col), 4 * S)) ||
        hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_sell_src), 4 * S)) ||
        hip_failed(hipMalloc(&h->d_sell_val, (h->dtype == SPMV_F32 ? 4 : 2) * S)))
        return SPMV_ERR_ALLOC;
    if (hip_failed(spmv::launch_sell_fill(view_of(h), h->d_sell_ptr, static_cast<int32_t>(ns), h->d_sell_col, h->d_sell_src,
                                          h->d_sell_val, nullptr)) ||
        hip_failed(hipDeviceSynchronize()))
        return SPMV_ERR_HIP;
    a->info.plan = SPMV_PLAN_SELL;
    a->info.sell_slots = slots;
    a->info.sell_num_slices = static_cast<int32_t>(ns);
    return SPMV_OK;
} catch (const std::bad_alloc&) {
    return SPMV_ERR_ALLOC;
}

spmv::TwoPhase two_phase_of(const spmv_csr_s* h) {
    spmv::TwoPhase t{};
    t.shift = h->info.tp_col_shift;
    t.group = h->info.tp_group > 1 ? h->info.tp_group : 1;
    t.num_pieces = h->info.tp_num_pieces;
    t.num_chunks = h->info.tp_num_chunks;
    t.carries = h->tp_carries;
    t.reduce_lds = h->tp_reduce_lds;
    t.piece_c = h->d_tp_piece_c;
    t.piece_g = h->d_tp_piece_g;
    t.tp_col = h->d_tp_col;
    t.tp_val = h->d_tp_val;
    t.tp_from = h->d_tp_from;
    t.tp_pos = h->d_tp_pos;
    t.chunk_desc = h->d_tp_desc;
    t.chunk_g = h->d_tp_chunk_g;
    t.prod = h->d_tp_prod;
    t.carry_row = h->d_tp_carry_row;
    t.carry_val = h->d_tp_carry_val;
    return t;
}

// Row order of the sparse-times-dense product and, where it pays, the packed copy of A in that order.
spmv_status_t build_spmm_order(spmv_csr_s* h, const HostRowptr& rowptr_host, spmv::Analysis* a) try {
    std::vector<int32_t> order, desc;
    spmv::spmm_row_order(h->m, rowptr_host.data(), &order);
    spmv_status_t st = upload(order, &h->d_spmm_rows);
    if (st != SPMV_OK) return st;
    a->info.spmm_prepared = 1;
    int64_t blocks = 0;
    if (!spmv::spmm_packed_layout(h->m, h->nnz, rowptr_host.data(), order.data(), &desc, &blocks)) return SPMV_OK;
    const bool col16 = h->n <= spmv::kSpmmCol16MaxN;
    const size_t slots = (static_cast<size_t>(blocks) + 1) * 256;  // one closing block that is only ever prefetched
    const size_t col_bytes = col16 ? 2 : 4;
    st = upload(desc, &h->d_spmm_desc);
    if (st != SPMV_OK) return st;
    if (hip_failed(hipMalloc(&h->d_spmm_col, col_bytes * slots)) ||
        hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_spmm_val), sizeof(float) * slots)))
        return SPMV_ERR_ALLOC;
    if (hip_failed(hipMemset(static_cast<char*>(h->d_spmm_col) + col_bytes * (slots - 256), 0, col_bytes * 256)) ||
        hip_failed(hipMemset(h->d_spmm_val + (slots - 256), 0, sizeof(float) * 256)) ||
        hip_failed(spmv::launch_spmm_pack(view_of(h), h->d_spmm_rows, h->d_spmm_desc, static_cast<int32_t>((h->m + 15) / 16),
                                          col16, h->d_spmm_col, h->d_spmm_val, nullptr)))
        return SPMV_ERR_HIP;
    a->info.spmm_prepared = 2;
    a->info.spmm_col_bytes = static_cast<int32_t>(col_bytes);
    a->info.spmm_num_blocks = blocks;
    return SPMV_OK;
} catch (const std::bad_alloc&) {
    return SPMV_ERR_ALLOC;
}

// Lanes per row the binned plan gives to length bin b (b >= 4: rows of 2^(b-2)+1 .. 2^(b-1) entries).
inline int lanes_for_bin(int b) {
    const int g = 1 << (b - 3);
    return g > 64 ? 64 : g;
}

}  // namespace

extern "C" {

spmv_status_t spmv_csr_create(spmv_handle_t* out, int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr,
                              const int32_t* colidx, const void* vals, spmv_dtype_t dtype) {
    if (!out) return SPMV_ERR_INVALID_ARG;
    *out = nullptr;
    if (m < 0 || n < 0 || nnz < 0) return SPMV_ERR_INVALID_ARG;
    if (dtype != SPMV_F32 && dtype != SPMV_BF16) return SPMV_ERR_INVALID_ARG;
    if (!rowptr) return SPMV_ERR_INVALID_ARG;
    if (nnz > 0 && (!colidx || !vals)) return SPMV_ERR_INVALID_ARG;
    if (nnz > 0 && n == 0) return SPMV_ERR_INVALID_ARG;
    if (m > kMaxCount || n > kMaxCount || nnz > kMaxCount) return SPMV_ERR_UNSUPPORTED;
    const uintptr_t esz = dtype == SPMV_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(rowptr) % 4 || reinterpret_cast<uintptr_t>(colidx) % 4 ||
        reinterpret_cast<uintptr_t>(vals) % esz)
        return SPMV_ERR_UNSUPPORTED;
    spmv_csr_s* h = new (std::nothrow) spmv_csr_s;
    if (!h) return SPMV_ERR_ALLOC;
    h->m = m;
    h->n = n;
    h->nnz = nnz;
    h->rowptr = rowptr;
    h->colidx = colidx;
    h->vals = vals;
    h->dtype = dtype;
    h->vec_ok = reinterpret_cast<uintptr_t>(colidx) % 16 == 0 && reinterpret_cast<uintptr_t>(vals) % 16 == 0;
    *out = h;
    return SPMV_OK;
}

spmv_status_t spmv_csr_analyze(spmv_handle_t h, const spmv_analyze_params_t* params) {
    if (!h) return SPMV_ERR_INVALID_ARG;
    spmv_analyze_params_t p{};
    spmv_status_t st = spmv::resolve_params(params, &p);
    if (st != SPMV_OK) return st;
    free_metadata(h);

    HostRowptr rowptr_host;
    if (!rowptr_host.download(h->rowptr, static_cast<size_t>(h->m) + 1)) return hip_failed(hipGetLastError()) ? SPMV_ERR_HIP : SPMV_ERR_ALLOC;

    spmv::Analysis a;
    st = spmv::analyze_rowptr(h->m, h->n, h->nnz, rowptr_host.data(), p, &a, p.plan == SPMV_PLAN_BINNED);
    if (st != SPMV_OK) return st;

    if (!p.skip_validation && h->nnz > 0) {
        int32_t* d_flag = nullptr;
        int32_t flag = 0;
        if (hip_failed(hipMalloc(reinterpret_cast<void**>(&d_flag), sizeof(int32_t)))) return SPMV_ERR_ALLOC;
        bool bad = hip_failed(hipMemcpy(d_flag, &flag, sizeof flag, hipMemcpyHostToDevice));
        bad = bad || hip_failed(spmv::launch_validate_columns(view_of(h), d_flag, nullptr));
        bad = bad || hip_failed(hipMemcpy(&flag, d_flag, sizeof flag, hipMemcpyDeviceToHost));
        (void)hipFree(d_flag);
        if (bad) return SPMV_ERR_HIP;
        if (flag != 0) return SPMV_ERR_BAD_STRUCTURE;
    }

    if (p.plan == SPMV_PLAN_BINNED) st = upload(a.bin_rows, &h->d_bin_rows);
    if (st == SPMV_OK) {
        try {
            std::vector<int32_t> block_nz(a.row_blocks.size());
            for (size_t b = 0; b < block_nz.size(); ++b) block_nz[b] = rowptr_host[static_cast<size_t>(a.row_blocks[b])];
            h->max_block_entries = 0;
            for (size_t b = 0; b + 1 < block_nz.size(); ++b) {
                const int32_t entries = block_nz[b + 1] - block_nz[b];
                if (entries <= a.info.block_nnz && entries > h->max_block_entries) h->max_block_entries = entries;
            }
            st = upload(block_nz, &h->d_block_nz);
            std::vector<int32_t> desc(2 * block_nz.size());
            for (size_t b = 0; b < block_nz.size(); ++b) {
                desc[2 * b] = a.row_blocks[b];
                desc[2 * b + 1] = block_nz[b];
            }
            if (st == SPMV_OK) st = upload(desc, &h->d_block_desc);
            desc.resize(2 * a.mp_row.size());
            for (size_t q = 0; q < a.mp_row.size(); ++q) {
                desc[2 * q] = a.mp_row[q];
                desc[2 * q + 1] = a.mp_nz[q];
            }
            if (st == SPMV_OK) st = upload(desc, &h->d_chunk_desc);
        } catch (const std::bad_alloc&) {
            st = SPMV_ERR_ALLOC;
        }
    }
    if (st == SPMV_OK) {
        const bool forced = p.plan == SPMV_PLAN_WINDOWED;
        // a matrix headed for the merge plan is counted too where a regrouping plan could take it: is it scattered?
        const bool count_only = p.plan == SPMV_PLAN_AUTO && a.info.plan == SPMV_PLAN_MERGE &&
                                (spmv::two_phase_sizes_ok(h->m, h->n, h->nnz, h->dtype) ||
                                 spmv::column_block_sizes_ok(h->n, h->nnz, h->dtype) ||
                                 spmv::grouped_two_phase_choice(h->m, h->n, h->nnz, h->dtype, a.info.plan, true, 1, 0));
        if (forced || count_only || (p.plan == SPMV_PLAN_AUTO && a.info.plan == SPMV_PLAN_ADAPTIVE))
            st = build_x_windows(h, forced, count_only, rowptr_host, &a);
    }
    if (st == SPMV_OK) {
        const bool automatic = p.plan == SPMV_PLAN_AUTO &&
                               (a.two_phase_on_groups || spmv::two_phase_choice(h->m, h->n, h->nnz, h->dtype, a.info.plan,
                                                                                a.x_vectors_counted, a.entries_counted));
        if (p.plan == SPMV_PLAN_TWOPHASE || automatic) {
            // a group-aligned matrix is laid out over its groups of eight entries: an eighth of the slots
            bool aligned = false;
            if (!a.d_group_cols) st = check_groups(h, rowptr_host, &aligned, &a.d_group_cols);
            if (st == SPMV_OK) st = build_two_phase(h, rowptr_host, &a, a.d_group_cols);
            if (automatic && st == SPMV_ERR_UNSUPPORTED) st = SPMV_OK;  // too many padded slots: the plan stays what it was
        }
    }
    if (a.d_group_cols) {
        (void)hipFree(a.d_group_cols);
        a.d_group_cols = nullptr;
    }
    if (st == SPMV_OK) {
        const bool automatic = p.plan == SPMV_PLAN_AUTO && spmv::column_block_choice(h->n, h->nnz, h->dtype, a.info.plan,
                                                                                     a.x_vectors_counted, a.entries_counted);
        if (p.plan == SPMV_PLAN_COLBLOCK || automatic) st = build_column_blocks(h, &a);
    }
    if (st == SPMV_OK && p.plan == SPMV_PLAN_SELL) st = build_sell(h, rowptr_host, &a);
    if (st == SPMV_OK && p.prepare_spmm) st = build_spmm_order(h, rowptr_host, &a);
    if (st == SPMV_OK) {
        const size_t P = static_cast<size_t>(a.info.num_chunks > 0 ? a.info.num_chunks : 1);
        if (hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_carry_row), sizeof(int32_t) * P)) ||
            hip_failed(hipMalloc(reinterpret_cast<void**>(&h->d_carry_val), sizeof(float) * P)))
            st = SPMV_ERR_ALLOC;
    }
    if (st == SPMV_OK && plan_has_scratch(a.info.plan) &&
        hip_failed(hipEventCreateWithFlags(&h->scratch_free, hipEventDisableTiming)))
        st = SPMV_ERR_HIP;
    if (st == SPMV_OK && hip_failed(hipDeviceSynchronize())) st = SPMV_ERR_HIP;
    if (st != SPMV_OK) {
        free_metadata(h);
        return st;
    }
    h->info = a.info;
    h->bin_rows = std::move(a.bin_rows);
    h->row_blocks = std::move(a.row_blocks);
    h->mp_row = std::move(a.mp_row);
    h->mp_nz = std::move(a.mp_nz);
    std::memcpy(h->bin_count, a.bin_count, sizeof h->bin_count);
    std::memcpy(h->bin_offset, a.bin_offset, sizeof h->bin_offset);
    h->analyzed = true;
    return SPMV_OK;
}

spmv_status_t spmv_csr_run(spmv_handle_t h, const void* x, float* y, float alpha, float beta, void* stream) {
    if (!h) return SPMV_ERR_INVALID_ARG;
    if (!h->analyzed) return SPMV_ERR_NOT_ANALYZED;
    if (h->m == 0) return SPMV_OK;
    if (!y) return SPMV_ERR_INVALID_ARG;
    if (h->nnz > 0 && !x) return SPMV_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(y) % 4 || reinterpret_cast<uintptr_t>(x) % (h->dtype == SPMV_F32 ? 4 : 2))
        return SPMV_ERR_UNSUPPORTED;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const spmv::MatrixView A = view_of(h);
    const spmv::Scalars s{alpha, beta};
    const int32_t m = A.m;
    hipError_t e = hipSuccess;
    bool tracked = false;
    if (plan_has_scratch(h->info.plan)) {
        const spmv_status_t busy = scratch_acquire(h, st, &tracked);
        if (busy != SPMV_OK) return busy;
    }
    switch (h->info.plan) {
        case SPMV_PLAN_SCALAR:
            e = spmv::launch_scalar(A, nullptr, m, x, y, s, st);
            break;
        case SPMV_PLAN_VECTOR:
            e = spmv::launch_vector(A, h->info.vector_lanes, nullptr, m, x, y, s, st);
            break;
        case SPMV_PLAN_BINNED: {
            // bins 0..3 (at most 4 entries a row): one lane per row; every higher bin: a team per row
            const int32_t short_rows = h->bin_offset[4];
            e = spmv::launch_scalar(A, h->d_bin_rows, short_rows, x, y, s, st);
            for (int b = 4; b < SPMV_NUM_BINS && e == hipSuccess; ++b) {
                // bins whose team is the full wavefront are launched together
                int last = b;
                if (lanes_for_bin(b) == 64) last = SPMV_NUM_BINS - 1;
                const int32_t first_row = h->bin_offset[b];
                const int32_t count = h->bin_offset[last + 1] - first_row;
                if (count > 0)
                    e = spmv::launch_vector(A, lanes_for_bin(b), h->d_bin_rows + first_row, count, x, y, s, st);
                b = last;
            }
            break;
        }
        case SPMV_PLAN_ADAPTIVE:
            e = spmv::launch_adaptive(A, h->d_block_desc, static_cast<int32_t>(h->info.num_row_blocks),
                                      h->info.block_nnz, h->info.rows_max, x, y, s, st);
            break;
        case SPMV_PLAN_WINDOWED: {
            const spmv::XWindows w{h->d_xv_ptr, h->d_xv_start, h->d_xv_pad, h->d_lidx8, h->d_lidx, h->info.max_x_vectors,
                                   h->d_run_desc, h->d_pat_pad, h->info.pat_cap};
            e = spmv::launch_windowed(A, h->d_block_desc, static_cast<int32_t>(h->info.num_row_blocks),
                                      h->info.block_nnz, h->max_block_entries, h->info.rows_max, w, x, y, s, st);
            break;
        }
        case SPMV_PLAN_COLBLOCK: {
            // y <- beta*y once, then every block adds its part; block b reads x from its first column on
            e = spmv::launch_scale_y(y, m, beta, st);
            const size_t esz = A.bf16 ? 2 : 4;
            for (int b = 0; b < h->info.num_col_blocks && e == hipSuccess; ++b) {
                const int32_t k0 = h->cb_ptr[static_cast<size_t>(b)], k1 = h->cb_ptr[static_cast<size_t>(b) + 1];
                e = spmv::launch_coo_accumulate(A.bf16, k1 - k0, h->d_cb_row + k0, h->d_cb_col + k0,
                                                static_cast<const char*>(h->d_cb_vals) + esz * static_cast<size_t>(k0),
                                                static_cast<const char*>(x) + esz * static_cast<size_t>(b) * h->info.col_block_width,
                                                y, alpha, st);
            }
            break;
        }
        case SPMV_PLAN_TWOPHASE:
            e = spmv::launch_two_phase(two_phase_of(h), A, x, y, s, st);
            break;
        case SPMV_PLAN_SELL:
            e = spmv::launch_sell(A, h->d_sell_ptr, h->info.sell_num_slices, h->d_sell_col, h->d_sell_val, x, y, s, st);
            break;
        case SPMV_PLAN_MERGE:
            e = spmv::launch_merge(A, h->d_chunk_desc, static_cast<int32_t>(h->info.num_chunks),
                                   h->info.items_per_chunk, h->d_carry_row, h->d_carry_val, x, y, s, st);
            break;
        default:
            return SPMV_ERR_INVALID_ARG;
    }
    if (tracked && e == hipSuccess) {
        e = hipEventRecord(h->scratch_free, st);
        h->scratch_stream = st;
        h->scratch_used = true;
    }
    return hip_failed(e) ? SPMV_ERR_HIP : SPMV_OK;
}

spmv_status_t spmm_csr_run(spmv_handle_t h, const void* B, int64_t ldb, float* C, int64_t ldc, int64_t K, float alpha,
                           float beta, void* stream) {
    if (!h) return SPMV_ERR_INVALID_ARG;
    if (!h->analyzed) return SPMV_ERR_NOT_ANALYZED;
    if (K < 0) return SPMV_ERR_INVALID_ARG;
    if (K > kMaxCount) return SPMV_ERR_UNSUPPORTED;
    if (h->m == 0 || K == 0) return SPMV_OK;
    if (!C || ldc < K) return SPMV_ERR_INVALID_ARG;
    if (h->n > 0 && (!B || ldb < K)) return SPMV_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(B) % (h->dtype == SPMV_F32 ? 4 : 2) || reinterpret_cast<uintptr_t>(C) % 4) return SPMV_ERR_UNSUPPORTED;
    hipError_t e;
    if (h->info.spmm_prepared == 2) {
        const spmv::PackedRows P{h->d_spmm_rows, h->d_spmm_desc, h->d_spmm_col, h->d_spmm_val,
                                 static_cast<int32_t>((h->m + 15) / 16), h->info.spmm_col_bytes == 2};
        e = spmv::launch_spmm_packed(view_of(h), P, B, ldb, C, ldc, static_cast<int32_t>(K), spmv::Scalars{alpha, beta},
                                     static_cast<hipStream_t>(stream));
    } else {
        e = spmv::launch_spmm(view_of(h), h->d_spmm_rows, B, ldb, C, ldc, static_cast<int32_t>(K), spmv::Scalars{alpha, beta},
                              static_cast<hipStream_t>(stream));
    }
    return hip_failed(e) ? SPMV_ERR_HIP : SPMV_OK;
}

namespace {

// Common argument checks of the stateless layouts: sizes, dtype, pointer alignment.
spmv_status_t check_stateless(int64_t m, int64_t n, int64_t count, spmv_dtype_t dtype, const void* idx_a,
                              const void* idx_b, const void* vals, const void* x, const float* y) {
    if (m < 0 || n < 0 || count < 0) return SPMV_ERR_INVALID_ARG;
    if (dtype != SPMV_F32 && dtype != SPMV_BF16) return SPMV_ERR_INVALID_ARG;
    if (m > kMaxCount || n > kMaxCount || count > kMaxCount) return SPMV_ERR_UNSUPPORTED;
    if (m > 0 && !y) return SPMV_ERR_INVALID_ARG;
    if (count > 0 && (!idx_a || !idx_b || !vals || !x)) return SPMV_ERR_INVALID_ARG;
    const uintptr_t esz = dtype == SPMV_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(idx_a) % 4 || reinterpret_cast<uintptr_t>(idx_b) % 4 ||
        reinterpret_cast<uintptr_t>(vals) % esz || reinterpret_cast<uintptr_t>(x) % esz ||
        reinterpret_cast<uintptr_t>(y) % 4)
        return SPMV_ERR_UNSUPPORTED;
    return SPMV_OK;
}

}  // namespace

spmv_status_t spmv_coo_run(int64_t m, int64_t n, int64_t nnz, const int32_t* row_indices, const int32_t* col_indices,
                           const void* vals, spmv_dtype_t dtype, const void* x, float* y, float alpha, float beta,
                           void* stream) {
    const spmv_status_t st = check_stateless(m, n, nnz, dtype, row_indices, col_indices, vals, x, y);
    if (st != SPMV_OK) return st;
    const hipError_t e = spmv::launch_coo(dtype == SPMV_BF16, static_cast<int32_t>(m), static_cast<int32_t>(nnz),
                                          row_indices, col_indices, vals, x, y, spmv::Scalars{alpha, beta},
                                          static_cast<hipStream_t>(stream));
    return hip_failed(e) ? SPMV_ERR_HIP : SPMV_OK;
}

spmv_status_t spmv_csc_run(int64_t m, int64_t n, int64_t nnz, const int32_t* col_offsets, const int32_t* row_indices,
                           const void* vals, spmv_dtype_t dtype, const void* x, float* y, float alpha, float beta,
                           void* stream) {
    const spmv_status_t st = check_stateless(m, n, nnz, dtype, row_indices, row_indices, vals, x, y);
    if (st != SPMV_OK) return st;
    if (!col_offsets || reinterpret_cast<uintptr_t>(col_offsets) % 4) return SPMV_ERR_INVALID_ARG;
    if (n > 0 && !x) return SPMV_ERR_INVALID_ARG;
    const hipError_t e = spmv::launch_csc(dtype == SPMV_BF16, static_cast<int32_t>(m), static_cast<int32_t>(n),
                                          static_cast<int32_t>(nnz), col_offsets, row_indices, vals, x, y,
                                          spmv::Scalars{alpha, beta}, static_cast<hipStream_t>(stream));
    return hip_failed(e) ? SPMV_ERR_HIP : SPMV_OK;
}

spmv_status_t spmv_ell_run(int64_t m, int64_t n, int64_t width, const int32_t* col_ids, const void* vals,
                           spmv_dtype_t dtype, const void* x, float* y, float alpha, float beta, void* stream) {
    if (width < 0) return SPMV_ERR_INVALID_ARG;
    if (width > kMaxCount) return SPMV_ERR_UNSUPPORTED;
    // m * width itself may exceed the limit: slots are addressed with 64-bit offsets
    // without columns x may point at nothing: only the slot arrays are then checked for alignment
    const spmv_status_t st = check_stateless(m, n, m > 0 && n > 0 ? width : 0, dtype, col_ids, col_ids, vals, n > 0 ? x : nullptr, y);
    if (st != SPMV_OK) return st;
    // without columns every slot is padding: y <- beta*y, and x (which may point at nothing) is never read
    const hipError_t e =
        n == 0 ? spmv::launch_scale_y(y, static_cast<int32_t>(m), beta, static_cast<hipStream_t>(stream))
               : spmv::launch_ell(dtype == SPMV_BF16, static_cast<int32_t>(m), static_cast<int32_t>(width), col_ids, vals, x, y,
                                  spmv::Scalars{alpha, beta}, static_cast<hipStream_t>(stream));
    return hip_failed(e) ? SPMV_ERR_HIP : SPMV_OK;
}

spmv_status_t spmv_csr_refresh_values(spmv_handle_t h, void* stream) {
    if (!h) return SPMV_ERR_INVALID_ARG;
    if (!h->analyzed) return SPMV_ERR_NOT_ANALYZED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const spmv::MatrixView A = view_of(h);
    hipError_t e = hipSuccess;
    if (h->info.plan == SPMV_PLAN_COLBLOCK) e = spmv::launch_column_block_values(A, h->d_cb_src, h->d_cb_vals, st);
    if (h->info.plan == SPMV_PLAN_TWOPHASE)
        e = spmv::launch_two_phase_values(A, h->d_tp_src, h->d_tp_val, h->info.tp_slots, h->info.tp_group > 1 ? h->info.tp_group : 1, st);
    if (h->info.plan == SPMV_PLAN_SELL) e = spmv::launch_sell_values(A, h->d_sell_src, h->d_sell_val, h->info.sell_slots, st);
    if (e == hipSuccess && h->info.spmm_prepared == 2)
        e = spmv::launch_spmm_pack(A, h->d_spmm_rows, h->d_spmm_desc, static_cast<int32_t>((h->m + 15) / 16),
                                   h->info.spmm_col_bytes == 2, h->d_spmm_col, h->d_spmm_val, st);
    return hip_failed(e) ? SPMV_ERR_HIP : SPMV_OK;
}

spmv_status_t spmv_destroy(spmv_handle_t h) {
    if (!h) return SPMV_OK;
    free_metadata(h);
    delete h;
    return SPMV_OK;
}

spmv_status_t spmv_csr_get_analysis_info(spmv_handle_t h, spmv_analysis_info_t* out) {
    if (!h || !out) return SPMV_ERR_INVALID_ARG;
    if (!h->analyzed) return SPMV_ERR_NOT_ANALYZED;
    *out = h->info;
    return SPMV_OK;
}

spmv_status_t spmv_csr_get_analysis(spmv_handle_t h, const spmv_analysis_host_t* out) {
    if (!h || !out) return SPMV_ERR_INVALID_ARG;
    if (!h->analyzed) return SPMV_ERR_NOT_ANALYZED;
    if (out->bin_count) std::memcpy(out->bin_count, h->bin_count, sizeof h->bin_count);
    if (out->bin_offset) std::memcpy(out->bin_offset, h->bin_offset, sizeof h->bin_offset);
    struct Copy {
        int32_t* dst;
        const int32_t* src;
        int64_t count;
    };
    // derived on the host from rowptr and kept there (kernels read the interleaved descriptors instead)
    const struct {
        int32_t* dst;
        const std::vector<int32_t>* src;
    } host_copies[] = {{out->bin_rows, &h->bin_rows}, {out->row_blocks, &h->row_blocks}, {out->mp_row, &h->mp_row}, {out->mp_nz, &h->mp_nz}};
    if (out->bin_rows && h->bin_rows.empty() && h->m > 0) {
        // not built at analyze time (no kernel of this plan reads it): built now, from the caller's rowptr
        try {
            std::vector<int32_t> rowptr_host(static_cast<size_t>(h->m) + 1);
            if (hip_failed(hipMemcpy(rowptr_host.data(), h->rowptr, sizeof(int32_t) * rowptr_host.size(), hipMemcpyDeviceToHost)))
                return SPMV_ERR_HIP;
            spmv::bin_rows_of(h->m, rowptr_host.data(), &h->bin_rows);
        } catch (const std::bad_alloc&) {
            return SPMV_ERR_ALLOC;
        }
    }
    for (const auto& c : host_copies)
        if (c.dst && !c.src->empty()) std::memcpy(c.dst, c.src->data(), sizeof(int32_t) * c.src->size());
    if (h->info.spmm_prepared && out->spmm_rows && h->info.m > 0 &&
        hip_failed(hipMemcpy(out->spmm_rows, h->d_spmm_rows, sizeof(int32_t) * static_cast<size_t>(h->info.m), hipMemcpyDeviceToHost)))
        return SPMV_ERR_HIP;
    if (h->info.spmm_prepared == 2) {
        const size_t groups = static_cast<size_t>((h->info.m + 15) / 16), slots = static_cast<size_t>(h->info.spmm_num_blocks) * 256;
        if (out->spmm_desc &&
            hip_failed(hipMemcpy(out->spmm_desc, h->d_spmm_desc, sizeof(int32_t) * (2 * groups + 2), hipMemcpyDeviceToHost)))
            return SPMV_ERR_HIP;
        if (out->spmm_col && slots > 0 &&
            hip_failed(hipMemcpy(out->spmm_col, h->d_spmm_col, static_cast<size_t>(h->info.spmm_col_bytes) * slots, hipMemcpyDeviceToHost)))
            return SPMV_ERR_HIP;
        if (out->spmm_val && slots > 0 &&
            hip_failed(hipMemcpy(out->spmm_val, h->d_spmm_val, sizeof(float) * slots, hipMemcpyDeviceToHost)))
            return SPMV_ERR_HIP;
    }
    if (h->info.plan == SPMV_PLAN_COLBLOCK) {
        if (out->cb_ptr) std::memcpy(out->cb_ptr, h->cb_ptr.data(), sizeof(int32_t) * h->cb_ptr.size());
        const Copy ccopies[] = {{out->cb_row, h->d_cb_row, h->info.nnz}, {out->cb_col, h->d_cb_col, h->info.nnz},
                                {out->cb_src, h->d_cb_src, h->info.nnz}};
        for (const Copy& c : ccopies)
            if (c.dst && c.count > 0 &&
                hip_failed(hipMemcpy(c.dst, c.src, sizeof(int32_t) * static_cast<size_t>(c.count), hipMemcpyDeviceToHost)))
                return SPMV_ERR_HIP;
    }
    if (h->info.plan == SPMV_PLAN_TWOPHASE) {
        const size_t P1 = static_cast<size_t>(h->info.tp_num_chunks) + 1, S = static_cast<size_t>(h->info.tp_slots);
        if (out->tp_row) std::memcpy(out->tp_row, h->tp_row.data(), sizeof(int32_t) * P1);
        if (out->tp_nz) std::memcpy(out->tp_nz, h->tp_nz.data(), sizeof(int32_t) * P1);
        const Copy tcopies[] = {{out->tp_piece_c, h->d_tp_piece_c, h->info.tp_num_pieces},
                                {out->tp_piece_g, h->d_tp_piece_g, h->info.tp_num_pieces + 1},
                                {out->tp_chunk_g, h->d_tp_chunk_g, h->info.tp_num_chunks + 1},
                                {out->tp_src, h->d_tp_src, h->info.tp_slots},
                                {out->tp_from, h->d_tp_from, h->info.tp_slots / 4}};
        for (const Copy& c : tcopies)
            if (c.dst && c.count > 0 &&
                hip_failed(hipMemcpy(c.dst, c.src, sizeof(int32_t) * static_cast<size_t>(c.count), hipMemcpyDeviceToHost)))
                return SPMV_ERR_HIP;
        if (out->tp_col && S > 0 && hip_failed(hipMemcpy(out->tp_col, h->d_tp_col, sizeof(uint16_t) * S, hipMemcpyDeviceToHost)))
            return SPMV_ERR_HIP;
        if (out->tp_pos && S > 0 && hip_failed(hipMemcpy(out->tp_pos, h->d_tp_pos, sizeof(uint16_t) * S, hipMemcpyDeviceToHost)))
            return SPMV_ERR_HIP;
    }
    if (h->info.plan == SPMV_PLAN_SELL) {
        if (out->sell_ptr) std::memcpy(out->sell_ptr, h->sell_ptr.data(), sizeof(int32_t) * h->sell_ptr.size());
        const Copy scopies[] = {{out->sell_col, h->d_sell_col, h->info.sell_slots}, {out->sell_src, h->d_sell_src, h->info.sell_slots}};
        for (const Copy& c : scopies)
            if (c.dst && c.count > 0 &&
                hip_failed(hipMemcpy(c.dst, c.src, sizeof(int32_t) * static_cast<size_t>(c.count), hipMemcpyDeviceToHost)))
                return SPMV_ERR_HIP;
    }
    if (h->info.plan == SPMV_PLAN_WINDOWED) {
        const Copy wcopies[] = {{out->xv_ptr, h->d_xv_ptr, h->info.num_row_blocks + 1},
                                {out->xv_start, h->d_xv_start, h->info.num_x_vectors},
                                {out->xv_pad, h->d_xv_pad,
                                 h->info.num_row_blocks * (h->info.max_x_vectors > 0 ? h->info.max_x_vectors : 1)}};
        for (const Copy& c : wcopies)
            if (c.dst && c.count > 0 &&
                hip_failed(hipMemcpy(c.dst, c.src, sizeof(int32_t) * static_cast<size_t>(c.count), hipMemcpyDeviceToHost)))
                return SPMV_ERR_HIP;
        if (out->lidx && h->nnz > 0 &&
            hip_failed(hipMemcpy(out->lidx, h->d_lidx, sizeof(uint16_t) * static_cast<size_t>(h->nnz), hipMemcpyDeviceToHost)))
            return SPMV_ERR_HIP;
        if (h->info.lidx_patterned) {
            const size_t nb = static_cast<size_t>(h->info.num_row_blocks);
            if (out->run_desc && hip_failed(hipMemcpy(out->run_desc, h->d_run_desc, 32 * nb, hipMemcpyDeviceToHost))) return SPMV_ERR_HIP;
            if (out->pat_pad &&
                hip_failed(hipMemcpy(out->pat_pad, h->d_pat_pad, 2 * nb * static_cast<size_t>(h->info.pat_cap), hipMemcpyDeviceToHost)))
                return SPMV_ERR_HIP;
        }
    }
    return SPMV_OK;
}

spmv_status_t spmv_analyze_host(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr_host,
                                const spmv_analyze_params_t* params, spmv_analysis_info_t* info,
                                const spmv_analysis_host_t* out) {
    if (!rowptr_host || !info || m < 0 || n < 0 || nnz < 0) return SPMV_ERR_INVALID_ARG;
    if (m > kMaxCount || n > kMaxCount || nnz > kMaxCount) return SPMV_ERR_UNSUPPORTED;
    spmv_analyze_params_t p{};
    spmv_status_t st = spmv::resolve_params(params, &p);
    if (st != SPMV_OK) return st;
    if (p.plan == SPMV_PLAN_WINDOWED || p.plan == SPMV_PLAN_COLBLOCK || p.plan == SPMV_PLAN_TWOPHASE || p.plan == SPMV_PLAN_SELL)
        return SPMV_ERR_INVALID_ARG;  // they need colidx: device only
    spmv::Analysis a;
    st = spmv::analyze_rowptr(m, n, nnz, rowptr_host, p, &a, out && out->bin_rows);
    if (st != SPMV_OK) return st;
    std::vector<int32_t> order, desc;
    if (p.prepare_spmm) {
        try {
            spmv::spmm_row_order(m, rowptr_host, &order);
            a.info.spmm_prepared = 1;
            int64_t blocks = 0;
            if (spmv::spmm_packed_layout(m, nnz, rowptr_host, order.data(), &desc, &blocks)) {
                a.info.spmm_prepared = 2;  // the layout only: packing needs colidx and vals, which live on the device
                a.info.spmm_col_bytes = n <= spmv::kSpmmCol16MaxN ? 2 : 4;
                a.info.spmm_num_blocks = blocks;
            }
        } catch (const std::bad_alloc&) {
            return SPMV_ERR_ALLOC;
        }
    }
    *info = a.info;
    if (out) {
        if (out->spmm_rows && !order.empty()) std::memcpy(out->spmm_rows, order.data(), sizeof(int32_t) * order.size());
        if (out->spmm_desc && a.info.spmm_prepared == 2) std::memcpy(out->spmm_desc, desc.data(), sizeof(int32_t) * desc.size());
        if (out->bin_count) std::memcpy(out->bin_count, a.bin_count, sizeof a.bin_count);
        if (out->bin_offset) std::memcpy(out->bin_offset, a.bin_offset, sizeof a.bin_offset);
        if (out->bin_rows && !a.bin_rows.empty())
            std::memcpy(out->bin_rows, a.bin_rows.data(), sizeof(int32_t) * a.bin_rows.size());
        if (out->row_blocks) std::memcpy(out->row_blocks, a.row_blocks.data(), sizeof(int32_t) * a.row_blocks.size());
        if (out->mp_row) std::memcpy(out->mp_row, a.mp_row.data(), sizeof(int32_t) * a.mp_row.size());
        if (out->mp_nz) std::memcpy(out->mp_nz, a.mp_nz.data(), sizeof(int32_t) * a.mp_nz.size());
    }
    return SPMV_OK;
}

spmv_status_t spmv_selftest_reduce(const float* in_dev, float* out_dev, void* stream) {
    if (!in_dev || !out_dev) return SPMV_ERR_INVALID_ARG;
    return hip_failed(spmv::launch_reduce_selftest(in_dev, out_dev, static_cast<hipStream_t>(stream))) ? SPMV_ERR_HIP
                                                                                                       : SPMV_OK;
}

const char* spmv_csr_main_kernel_name(spmv_handle_t h) {
    if (!h || !h->analyzed) return "";
    switch (h->info.plan) {
        case SPMV_PLAN_SCALAR: return spmv::scalar_kernel_name();
        case SPMV_PLAN_VECTOR:
        case SPMV_PLAN_BINNED: return spmv::vector_kernel_name();
        case SPMV_PLAN_ADAPTIVE:
        case SPMV_PLAN_MERGE: return spmv::tile_kernel_name();
        case SPMV_PLAN_WINDOWED: return h->info.lidx_patterned ? spmv::pattern_kernel_name() : spmv::window_kernel_name();
        case SPMV_PLAN_COLBLOCK: return "spmv_coo_kernel";
        case SPMV_PLAN_TWOPHASE: return h->info.tp_group > 1 ? "tp_multiply_group_kernel" : "tp_multiply_kernel";
        case SPMV_PLAN_SELL: return spmv::sell_kernel_name();
        default: return "";
    }
}

const char* spmv_status_string(spmv_status_t s) {
    switch (s) {
        case SPMV_OK: return "ok";
        case SPMV_ERR_INVALID_ARG: return "invalid argument";
        case SPMV_ERR_BAD_STRUCTURE: return "malformed CSR structure";
        case SPMV_ERR_UNSUPPORTED: return "unsupported size or alignment";
        case SPMV_ERR_NOT_ANALYZED: return "handle not analyzed";
        case SPMV_ERR_ALLOC: return "allocation failed";
        case SPMV_ERR_HIP: return "HIP runtime error";
        case SPMV_ERR_BUSY: return "the handle's scratch is in use by a run on another stream";
        default: return "unknown status";
    }
}

int spmv_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
