// The sliced ELL plan (gfx950): an analysis-time copy of the matrix in the ELL storage of the paper's App. C task 14
// (fixed width, col_id -1 marks padding), applied slice by slice.  A slice is 64 consecutive rows, as wide as its
// longest row, stored column by column: slot slice_ptr[s] + j*64 + i holds entry j of the slice's i-th row.  One
// wavefront takes a slice, lane i its i-th row: every load of the wavefront is one contiguous, aligned stretch
// (256 bytes of columns, 256 or 128 of values), no row offsets are read and nothing is reduced across lanes.
// x is gathered from memory as in the row-wise kernels.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"

namespace spmv {
namespace {

constexpr int kSellUnroll = 4;  // slots of a row in flight per lane

template <typename T>
__global__ __launch_bounds__(kWG) void spmv_sell_kernel(const int32_t* __restrict__ slice_ptr, const int32_t* __restrict__ sell_col,
                                                        const typename T::elem* __restrict__ sell_val,
                                                        const typename T::elem* __restrict__ x, float* y, int m, int ns,
                                                        float alpha, float beta) {
    const int lane = threadIdx.x & 63;
    // four slices per workgroup; the workgroups of a die walk through a contiguous stretch of slices
    const int s = xcd_remap(blockIdx.x, gridDim.x) * (kWG / 64) + (threadIdx.x >> 6);
    if (s >= ns) return;
    const int base = slice_ptr[s];
    const int width = (slice_ptr[s + 1] - base) >> 6;
    const int32_t* col = sell_col + base + lane;
    const typename T::elem* val = sell_val + base + lane;
    float acc = 0.f;
    int j = 0;
    for (; j + kSellUnroll <= width; j += kSellUnroll) {
        int c[kSellUnroll];
        float v[kSellUnroll], xv[kSellUnroll];
#pragma unroll
        for (int u = 0; u < kSellUnroll; ++u) {
            c[u] = __builtin_nontemporal_load(col + (j + u) * 64);
            v[u] = widen(__builtin_nontemporal_load(val + (j + u) * 64));
        }
#pragma unroll
        for (int u = 0; u < kSellUnroll; ++u) xv[u] = widen(x[c[u] >= 0 ? c[u] : 0]);  // a slice has slots only if the matrix has entries, so x[0] exists
#pragma unroll
        for (int u = 0; u < kSellUnroll; ++u) acc += c[u] >= 0 ? v[u] * xv[u] : 0.f;  // padding adds nothing whatever x[0] holds
    }
    for (; j < width; ++j) {
        const int c = __builtin_nontemporal_load(col + j * 64);
        const float v = widen(__builtin_nontemporal_load(val + j * 64));
        const float xv = widen(x[c >= 0 ? c : 0]);
        acc += c >= 0 ? v * xv : 0.f;
    }
    const int r = s * 64 + lane;
    if (r < m) y[r] = epilogue(acc, alpha, beta, y, r);
}

// Fills the slots of slice s (one wavefront per slice, lane i its i-th row): column, source position, value; -1, -1, 0
// where the row has no such entry.
template <typename E>
__global__ __launch_bounds__(kWG) void sell_fill_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                        const E* __restrict__ vals, const int32_t* __restrict__ slice_ptr, int m,
                                                        int ns, int32_t* __restrict__ sell_col, int32_t* __restrict__ sell_src,
                                                        E* __restrict__ sell_val) {
    const int lane = threadIdx.x & 63;
    const int s = blockIdx.x * (kWG / 64) + (threadIdx.x >> 6);
    if (s >= ns) return;
    const int base = slice_ptr[s];
    const int width = (slice_ptr[s + 1] - base) >> 6;
    const int r = s * 64 + lane;
    int k0 = 0, len = 0;
    if (r < m) {
        k0 = rowptr[r];
        len = rowptr[r + 1] - k0;
    }
    for (int j = 0; j < width; ++j) {
        const bool live = j < len;
        const int slot = base + j * 64 + lane;
        sell_col[slot] = live ? colidx[k0 + j] : -1;
        sell_src[slot] = live ? k0 + j : -1;
        sell_val[slot] = live ? vals[k0 + j] : E(0);
    }
}

template <typename E>
__global__ __launch_bounds__(kWG) void sell_values_kernel(const E* __restrict__ vals, const int32_t* __restrict__ sell_src,
                                                          E* __restrict__ sell_val, int64_t slots, int nnz) {
    for (int64_t s = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; s < slots; s += static_cast<int64_t>(gridDim.x) * kWG) {
        const int k = sell_src[s];
        if (k >= 0 && k < nnz) sell_val[s] = vals[k];
    }
}

}  // namespace

hipError_t launch_sell_fill(const MatrixView& A, const int32_t* slice_ptr, int32_t ns, int32_t* sell_col, int32_t* sell_src,
                            void* sell_val, hipStream_t st) {
    if (ns <= 0) return hipSuccess;
    const dim3 grid(ceil_div(ns, kWG / 64));
    if (A.bf16)
        hipLaunchKernelGGL(sell_fill_kernel<uint16_t>, grid, dim3(kWG), 0, st, A.rowptr, A.colidx, static_cast<const uint16_t*>(A.vals),
                           slice_ptr, A.m, ns, sell_col, sell_src, static_cast<uint16_t*>(sell_val));
    else
        hipLaunchKernelGGL(sell_fill_kernel<float>, grid, dim3(kWG), 0, st, A.rowptr, A.colidx, static_cast<const float*>(A.vals),
                           slice_ptr, A.m, ns, sell_col, sell_src, static_cast<float*>(sell_val));
    return hipGetLastError();
}

hipError_t launch_sell_values(const MatrixView& A, const int32_t* sell_src, void* sell_val, int64_t slots, hipStream_t st) {
    if (slots <= 0) return hipSuccess;
    int64_t g = (slots + kWG - 1) / kWG;
    const dim3 grid(static_cast<unsigned>(g > 8192 ? 8192 : g));
    if (A.bf16)
        hipLaunchKernelGGL(sell_values_kernel<uint16_t>, grid, dim3(kWG), 0, st, static_cast<const uint16_t*>(A.vals), sell_src,
                           static_cast<uint16_t*>(sell_val), slots, A.nnz);
    else
        hipLaunchKernelGGL(sell_values_kernel<float>, grid, dim3(kWG), 0, st, static_cast<const float*>(A.vals), sell_src,
                           static_cast<float*>(sell_val), slots, A.nnz);
    return hipGetLastError();
}

hipError_t launch_sell(const MatrixView& A, const int32_t* slice_ptr, int32_t ns, const int32_t* sell_col, const void* sell_val,
                       const void* x, float* y, Scalars s, hipStream_t st) {
    if (ns <= 0) return hipSuccess;
    const dim3 grid(ceil_div(ns, kWG / 64));
    if (A.bf16)
        hipLaunchKernelGGL(spmv_sell_kernel<BF16>, grid, dim3(kWG), 0, st, slice_ptr, sell_col, static_cast<const uint16_t*>(sell_val),
                           static_cast<const uint16_t*>(x), y, A.m, ns, s.alpha, s.beta);
    else
        hipLaunchKernelGGL(spmv_sell_kernel<F32>, grid, dim3(kWG), 0, st, slice_ptr, sell_col, static_cast<const float*>(sell_val),
                           static_cast<const float*>(x), y, A.m, ns, s.alpha, s.beta);
    return hipGetLastError();
}

const char* sell_kernel_name() { return "spmv_sell_kernel"; }

}  // namespace spmv
