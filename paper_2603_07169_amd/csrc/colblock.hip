// Analysis-time regrouping of a CSR matrix by blocks of columns (gfx950).
//
// With columns spread over more of x than an L2 holds, almost every x gather of the row-wise
// kernels misses and drags a whole cache line across the fabric.  Regrouped block after block,
// the entries of one block only touch one 4 MiB stretch of x, which stays in the L2s while
// that block is multiplied.  Inside a block the entries keep their row-major order, each with
// its row number, so a block is multiplied by the coordinate-format kernel.
//
// Two passes of one kernel, one wavefront per tile of kCbTile consecutive entries:
//   count    tile_counts[b * ntiles + t] = entries of tile t that fall into block b
//   scatter  entry e of tile t, the r-th of the tile's entries in block b, goes to position
//            tile_base[b * ntiles + t] + r, where tile_base is the exclusive prefix sum of
//            tile_counts in (b, t) order (taken on the host between the passes)
// Positions inside a tile come from ballots, so the order of the entries is kept exactly.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"

namespace spmv {
namespace {

template <bool SCATTER>
__global__ __launch_bounds__(64) void cb_tile_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                     const void* __restrict__ vals, int elem_bytes, int m, int nnz, int shift,
                                                     int C, int ntiles, int32_t* __restrict__ tile_counts,
                                                     const int32_t* __restrict__ tile_base, int32_t* __restrict__ cb_row,
                                                     int32_t* __restrict__ cb_col, int32_t* __restrict__ cb_src,
                                                     void* __restrict__ cb_vals) {
    // Entries of this tile seen so far, per block.  Ballots are uniform over the wavefront, so every
    // lane keeps the same counts in its own registers (the loops over blocks are fully unrolled).
    int running[kMaxColBlocks];
#pragma unroll
    for (int b = 0; b < kMaxColBlocks; ++b) running[b] = 0;
    const int lane = threadIdx.x;
    const int tile = blockIdx.x;
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int step = 0; step < kCbTile / 64; ++step) {
        const int e = tile * kCbTile + step * 64 + lane;
        const bool live = e < nnz;
        const int c = live ? colidx[e] : 0;
        int blk = live ? c >> shift : -1;
        if (blk >= C) blk = -1;  // a column beyond n (only possible when the caller skipped validation): dropped
        int rank = 0;
#pragma unroll
        for (int b = 0; b < kMaxColBlocks; ++b) {
            if (b < C) {
                const unsigned long long mask = __builtin_amdgcn_ballot_w64(blk == b);
                if (blk == b) rank = running[b] + __popcll(mask & below);
                running[b] += __popcll(mask);
            }
        }
        if constexpr (SCATTER) {
            if (blk >= 0) {
                const int dest = tile_base[blk * ntiles + tile] + rank;
                int lo = 0, hi = m;  // the row of entry e: the last i with rowptr[i] <= e
                while (lo < hi) {
                    const int mid = lo + ((hi - lo + 1) >> 1);
                    if (rowptr[mid] <= e) lo = mid;
                    else hi = mid - 1;
                }
                cb_row[dest] = lo;
                cb_col[dest] = c - (blk << shift);
                cb_src[dest] = e;
                if (elem_bytes == 4) static_cast<float*>(cb_vals)[dest] = static_cast<const float*>(vals)[e];
                else static_cast<uint16_t*>(cb_vals)[dest] = static_cast<const uint16_t*>(vals)[e];
            }
        }
    }
    if constexpr (!SCATTER) {
#pragma unroll
        for (int b = 0; b < kMaxColBlocks; ++b)
            if (lane == b && b < C) tile_counts[b * ntiles + tile] = running[b];
    }
}

template <typename E>
__global__ __launch_bounds__(kWG) void cb_values_kernel(const E* __restrict__ vals, const int32_t* __restrict__ cb_src,
                                                        E* __restrict__ cb_vals, int nnz) {
    // a slot the regrouping left unfilled (an entry dropped for a column outside the matrix, which only a caller who
    // skipped the validation can have) keeps the -1 it was cleared to
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; k < nnz; k += static_cast<int64_t>(gridDim.x) * kWG) {
        const int src = cb_src[k];
        if (src >= 0 && src < nnz) cb_vals[k] = vals[src];
    }
}

}  // namespace

int32_t column_block_tiles(int32_t nnz) { return ceil_div(nnz, kCbTile); }

hipError_t launch_column_block_count(const MatrixView& A, int shift, int C, int32_t* tile_counts, hipStream_t st) {
    const int ntiles = column_block_tiles(A.nnz);
    if (ntiles <= 0) return hipSuccess;
    if (C > kMaxColBlocks) return hipErrorInvalidValue;
    hipLaunchKernelGGL(cb_tile_kernel<false>, dim3(ntiles), dim3(64), 0, st, A.rowptr, A.colidx, A.vals, A.bf16 ? 2 : 4, A.m,
                       A.nnz, shift, C, ntiles, tile_counts, nullptr, nullptr, nullptr, nullptr, nullptr);
    return hipGetLastError();
}

hipError_t launch_column_block_scatter(const MatrixView& A, int shift, int C, const int32_t* tile_base, int32_t* cb_row,
                                       int32_t* cb_col, int32_t* cb_src, void* cb_vals, hipStream_t st) {
    const int ntiles = column_block_tiles(A.nnz);
    if (ntiles <= 0) return hipSuccess;
    if (C > kMaxColBlocks) return hipErrorInvalidValue;
    hipLaunchKernelGGL(cb_tile_kernel<true>, dim3(ntiles), dim3(64), 0, st, A.rowptr, A.colidx, A.vals, A.bf16 ? 2 : 4, A.m,
                       A.nnz, shift, C, ntiles, nullptr, tile_base, cb_row, cb_col, cb_src, cb_vals);
    return hipGetLastError();
}

hipError_t launch_column_block_values(const MatrixView& A, const int32_t* cb_src, void* cb_vals, hipStream_t st) {
    if (A.nnz <= 0) return hipSuccess;
    int grid = ceil_div(A.nnz, kWG);
    if (grid > 8192) grid = 8192;
    if (A.bf16)
        hipLaunchKernelGGL(cb_values_kernel<uint16_t>, dim3(grid), dim3(kWG), 0, st, static_cast<const uint16_t*>(A.vals), cb_src,
                           static_cast<uint16_t*>(cb_vals), A.nnz);
    else
        hipLaunchKernelGGL(cb_values_kernel<float>, dim3(grid), dim3(kWG), 0, st, static_cast<const float*>(A.vals), cb_src,
                           static_cast<float*>(cb_vals), A.nnz);
    return hipGetLastError();
}

}  // namespace spmv
