// spmv_csr_run_static: the merge-path product for callers that cannot allocate (code under HIP graph
// capture, tight serving loops).  No handle, no analysis step, no hipMalloc: the merge-path splits are found on the
// device, and the splits and the carries of cut rows live in one fixed array in device memory that the library
// keeps for as long as it is loaded.
#include <hip/hip_runtime.h>

#include <mutex>

#include "analysis.h"
#include "device_common.h"
#include "kernels.h"
#include "spmv_mi355.h"

namespace {

// Layout of the array for P chunks (P <= kStaticMaxChunks):
//   int32 desc[2 * (kStaticMaxChunks + 1)]   pairs (rows finished, entries taken) at every split
//   int32 carry_row[kStaticMaxChunks]
//   float carry_val[kStaticMaxChunks]
constexpr int64_t kStaticMaxChunks = SPMV_STATIC_MAX_ITEMS / spmv::kDefaultItemsPerChunk;
constexpr size_t kScratchBytes = 4 * (2 * (kStaticMaxChunks + 1) + 2 * kStaticMaxChunks);
static_assert(SPMV_STATIC_MAX_ITEMS % spmv::kDefaultItemsPerChunk == 0, "whole chunks");
static_assert(kScratchBytes <= (size_t{2} << 20), "the fixed array stays at 2 MiB");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Every device holds its own copy of the array at its own address; the address is looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_of_current_device(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

// Merge-path split p (p = 0..P): after d = min(p * ipc, m + nnz) steps of the path over (row ends, entry positions)
// i rows are finished, i being the first row count in the feasible window with rowptr[i+1] + i > d - 1.
__global__ __launch_bounds__(256) void static_splits_kernel(const int32_t* __restrict__ rowptr, int m, int nnz, int ipc, int P,
                                                            int32_t* __restrict__ desc) {
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p > P) return;
    const int64_t T = static_cast<int64_t>(m) + nnz;
    const int64_t d = static_cast<int64_t>(p) * ipc < T ? static_cast<int64_t>(p) * ipc : T;
    int64_t lo = d - nnz > 0 ? d - nnz : 0;
    int64_t hi = d < m ? d : m;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (static_cast<int64_t>(rowptr[mid + 1]) + mid > d - 1)
            hi = mid;
        else
            lo = mid + 1;
    }
    desc[2 * p] = static_cast<int32_t>(lo);
    desc[2 * p + 1] = static_cast<int32_t>(d - lo);
}

}  // namespace

extern "C" spmv_status_t spmv_csr_run_static(int64_t m, int64_t n, int64_t nnz, const int32_t* rowptr, const int32_t* colidx,
                                             const void* vals, spmv_dtype_t dtype, const void* x, float* y, float alpha,
                                             float beta, void* stream) {
    if (m < 0 || n < 0 || nnz < 0) return SPMV_ERR_INVALID_ARG;
    if (dtype != SPMV_F32 && dtype != SPMV_BF16) return SPMV_ERR_INVALID_ARG;
    if (m + nnz > SPMV_STATIC_MAX_ITEMS) return SPMV_ERR_UNSUPPORTED;  // the fixed array holds no more chunks
    if (m == 0) return SPMV_OK;
    if (!rowptr || !y) return SPMV_ERR_INVALID_ARG;
    if (nnz > 0 && (!colidx || !vals || !x || n == 0)) return SPMV_ERR_INVALID_ARG;
    const uintptr_t esz = dtype == SPMV_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(rowptr) % 4 || reinterpret_cast<uintptr_t>(colidx) % 4 ||
        reinterpret_cast<uintptr_t>(vals) % esz || reinterpret_cast<uintptr_t>(x) % esz || reinterpret_cast<uintptr_t>(y) % 4)
        return SPMV_ERR_UNSUPPORTED;

    void* base = nullptr;
    if (spmv::note_hip_error(scratch_of_current_device(&base))) return SPMV_ERR_HIP;
    int32_t* desc = static_cast<int32_t*>(base);
    int32_t* carry_row = desc + 2 * (kStaticMaxChunks + 1);
    float* carry_val = reinterpret_cast<float*>(carry_row + kStaticMaxChunks);

    spmv::MatrixView A{};
    A.m = static_cast<int32_t>(m);
    A.n = static_cast<int32_t>(n);
    A.nnz = static_cast<int32_t>(nnz);
    A.rowptr = rowptr;
    A.colidx = colidx;
    A.vals = vals;
    A.bf16 = dtype == SPMV_BF16;
    A.vec_ok = reinterpret_cast<uintptr_t>(colidx) % 16 == 0 && reinterpret_cast<uintptr_t>(vals) % 16 == 0;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int ipc = spmv::kDefaultItemsPerChunk;
    const int P = static_cast<int>((m + nnz + ipc - 1) / ipc);  // >= 1 and <= kStaticMaxChunks
    hipLaunchKernelGGL(static_splits_kernel, dim3((P + 1 + 255) / 256), dim3(256), 0, st, rowptr, A.m, A.nnz, ipc, P, desc);
    if (spmv::note_hip_error(hipGetLastError())) return SPMV_ERR_HIP;
    // every chunk writes its carry (row -1 when it cuts no row), so nothing in the array has to start at zero
    if (spmv::note_hip_error(spmv::launch_merge(A, desc, P, ipc, carry_row, carry_val, x, y, spmv::Scalars{alpha, beta}, st)))
        return SPMV_ERR_HIP;
    return SPMV_OK;
}
