// gfx950 kernel for the sparse-times-dense product C <- alpha*A*B + beta*C (paper App. C task 13).
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"

namespace spmv {
namespace {

constexpr int kSpmmWG = 1024;  // 16 wavefronts per workgroup (one workgroup per CU: its B slice fills the LDS)
constexpr int kSpmmKT = 16;    // columns of B and C a workgroup owns (4 lanes x float4 per row)
constexpr int kSpmmNB = 2048;  // rows of B held in LDS at a time (2048 x 16 floats = 128 KB)

// ------------------------------------------------------------------------------------------
// C <- alpha*A*B + beta*C with A in CSR (FP32), B (n x K) and C (m x K) dense, row-major
// (paper App. C task 13).  Every stored entry a_ij adds a_ij * B[j, :] to C[i, :], so the
// operation reads a K-wide row of B per entry: nnz * K * 4 bytes in all, far more than B itself
// or than C.  Those reads are kept on chip: a workgroup owns kSpmmKT = 16 columns of B and C,
// copies that slice of B (up to kSpmmNB = 2048 rows: 128 KB) into LDS once and then walks over
// all its rows of A.  Four lanes (a DPP quad) serve a row, one float4 of the slice each; a
// wavefront serves 16 rows at a time.  The quad reads its row's entries straight from memory,
// lane q taking entries q, q+4, ..: neighbouring quads hold neighbouring rows, so a load
// instruction of the wavefront covers one contiguous stretch of colidx / vals.  An entry is then
// handed to the other three lanes with a quad broadcast, and each lane adds value * B-row piece
// out of LDS.  Rows and entries of the next group are fetched while the current one is multiplied.
// B wider than the LDS block is taken in several passes over A, accumulating into C.
struct SpmmArgs {
    const int32_t* rowptr;
    const int32_t* colidx;
    const float* vals;
    const float* B;
    float* C;
    int64_t ldb, ldc;
    int32_t m, n, K, nnz;
    int32_t row_splits;  // gridDim.y: each takes an equal share of the rows
    int32_t vec_ok;      // B and C 16-byte aligned, ldb and ldc multiples of 4
    float alpha, beta;
};

template <int S>
__device__ __forceinline__ int quad_bcast(int v) {  // every lane gets the value of lane S of its quad
    return __builtin_amdgcn_update_dpp(0, v, S * 0x55, 0xF, 0xF, true);
}

__global__ __launch_bounds__(kSpmmWG) void spmm_csr_kernel(const SpmmArgs a) {
    constexpr int KT = kSpmmKT, NB = kSpmmNB, RPW = 16, WAVES = kSpmmWG / 64;
    constexpr int U = 8;  // entries per lane and chunk: a chunk covers 32 entries of a row
    static_assert(KT == 16, "four lanes per row, one float4 each");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* Bs = reinterpret_cast<float*>(smem_raw);  // [NB + 1][KT]; row NB stays zero
    const unsigned char* const Bq = smem_raw + 16 * (threadIdx.x & 3);  // this lane's float4 of row 0
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane & 3;      // which float4 of the slice, and which entries of the row (q, q+4, ..)
    const int rsub = lane >> 2;  // which of the wavefront's 16 rows

    const int k0 = blockIdx.x * KT;
    const int kw = a.K - k0 < KT ? a.K - k0 : KT;  // live columns of this slice
    const int row_lo = static_cast<int>(static_cast<int64_t>(a.m) * blockIdx.y / a.row_splits);
    const int row_hi = static_cast<int>(static_cast<int64_t>(a.m) * (blockIdx.y + 1) / a.row_splits);
    const bool full4 = a.vec_ok && 4 * q + 4 <= kw;  // this lane's float4 lies wholly inside the slice

    if (a.nnz == 0) {  // C <- beta*C; the main path below may then assume that A has entries
        for (int r = row_lo + tid / 4; r < row_hi; r += kSpmmWG / 4) {
            float* dst = a.C + static_cast<size_t>(r) * a.ldc + k0 + 4 * q;
            for (int t = 0; t < 4; ++t)
                if (4 * q + t < kw) dst[t] = a.beta != 0.f ? a.beta * dst[t] : 0.f;
        }
        return;
    }
    if (tid < KT) Bs[NB * KT + tid] = 0.f;  // the row that entries without a partner in this block point to

    // Group number gi of a wavefront -> first row.  Every workgroup walks over all rows of A;
    // starting each at a different place keeps them from asking for the same lines together.
    const int n_groups = (row_hi - row_lo + RPW - 1) / RPW;
    const int rot = static_cast<int>((static_cast<int64_t>(blockIdx.x) * n_groups) / gridDim.x);
    auto base_of = [&](int gi) {
        if (gi >= n_groups) return row_hi;
        int g = gi + rot;
        if (g >= n_groups) g -= n_groups;
        return row_lo + g * RPW;
    };

    for (int cb0 = 0; cb0 < a.n; cb0 += NB) {
        const int nbk = a.n - cb0 < NB ? a.n - cb0 : NB;  // rows of B in this block
        if (cb0 > 0) __syncthreads();                     // the previous block is no longer read
        for (int idx = tid; idx < nbk * 4; idx += kSpmmWG) {
            const int j = idx >> 2, qq = idx & 3;
            const float* src = a.B + static_cast<size_t>(cb0 + j) * a.ldb + k0 + 4 * qq;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (a.vec_ok && 4 * qq + 4 <= kw) {
                v = *reinterpret_cast<const f32x4*>(src);
            } else {
                for (int t = 0; t < 4; ++t)
                    if (4 * qq + t < kw) v[t] = src[t];
            }
            *reinterpret_cast<f32x4*>(Bs + j * KT + 4 * qq) = v;
        }
        __syncthreads();

        // (first entry, length) of this lane's row in group gi; length 0 past the end
        auto load_row = [&](int gi, int& rs, int& len) {
            const int r = base_of(gi) + rsub;
            const bool live = r < row_hi;
            rs = a.rowptr[live ? r : 0];
            const int re = a.rowptr[live ? r + 1 : 0];
            len = live ? re - rs : 0;
        };
        // entries c0 + q, c0 + q + 4, .. of the row: LDS offset of the B row (in floats) and value.
        // The loads are unconditional (no branch, so all are in flight together); a lane past its
        // row's end reads the last entry of the array and then points at the zero row.
        auto load_chunk = [&](int rs, int len, int c0, int* col, float* val) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = c0 + q + 4 * u;
                const unsigned k = t < len ? rs + t : a.nnz - 1;  // unsigned: base + 32-bit offset addressing
                col[u] = a.colidx[k];
                val[u] = a.vals[k];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = c0 + q + 4 * u;
                const int c = col[u] - cb0;
                const bool ok = t < len && static_cast<unsigned>(c) < static_cast<unsigned>(nbk);
                col[u] = (ok ? c : NB) * (KT * 4);  // byte offset of the B row in the LDS block
                val[u] = ok ? val[u] : 0.f;
            }
        };

        int gi = wave;
        int rs, len, rs_n, len_n;
        load_row(gi, rs, len);
        load_row(gi + WAVES, rs_n, len_n);
        int col[U], coln[U];
        float val[U], valn[U];
        load_chunk(rs, len, 0, col, val);
        while (gi < n_groups) {
            // the next group's first chunk and the rows of the group after it: in flight during the multiply
            load_chunk(rs_n, len_n, 0, coln, valn);
            int rs_nn, len_nn;
            load_row(gi + 2 * WAVES, rs_nn, len_nn);

            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
            for (int c0 = 0;; c0 += 4 * U) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (!__builtin_amdgcn_ballot_w64(c0 + 4 * u < len)) break;  // no row of the wavefront reaches this far
                    const int cc[4] = {quad_bcast<0>(col[u]), quad_bcast<1>(col[u]), quad_bcast<2>(col[u]),
                                       quad_bcast<3>(col[u])};
                    const int vbits = __float_as_int(val[u]);
                    const float vv[4] = {__int_as_float(quad_bcast<0>(vbits)), __int_as_float(quad_bcast<1>(vbits)),
                                         __int_as_float(quad_bcast<2>(vbits)), __int_as_float(quad_bcast<3>(vbits))};
                    f32x4 b[4];
#pragma unroll
                    for (int s = 0; s < 4; ++s) b[s] = *reinterpret_cast<const f32x4*>(Bq + cc[s]);
#pragma unroll
                    for (int s = 0; s < 4; ++s) acc += vv[s] * b[s];
                }
                if (!__builtin_amdgcn_ballot_w64(c0 + 4 * U < len)) break;
                load_chunk(rs, len, c0 + 4 * U, col, val);  // rows longer than a chunk: fetched on demand
            }

            const int r = base_of(gi) + rsub;
            if (r < row_hi && 4 * q < kw) {
                float* dst = a.C + static_cast<size_t>(r) * a.ldc + k0 + 4 * q;
                const bool first = cb0 == 0;
                const bool reads_c = !first || a.beta != 0.f;
                const float scale_c = first ? a.beta : 1.f;
                if (full4) {
                    f32x4 out = a.alpha * acc;
                    if (reads_c) out += scale_c * *reinterpret_cast<const f32x4*>(dst);
                    *reinterpret_cast<f32x4*>(dst) = out;
                } else {
                    for (int t = 0; t < 4; ++t)
                        if (4 * q + t < kw) dst[t] = a.alpha * acc[t] + (reads_c ? scale_c * dst[t] : 0.f);
                }
            }
            gi += WAVES;
            rs = rs_n;
            len = len_n;
            rs_n = rs_nn;
            len_n = len_nn;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                col[u] = coln[u];
                val[u] = valn[u];
            }
        }
    }
}

}  // namespace

hipError_t launch_spmm(const MatrixView& A, const float* B, int64_t ldb, float* C, int64_t ldc, int32_t K, Scalars s,
                       hipStream_t st) {
    if (A.m <= 0 || K <= 0) return hipSuccess;
    if (A.bf16) return hipErrorInvalidValue;
    SpmmArgs a{};
    a.rowptr = A.rowptr;
    a.colidx = A.colidx;
    a.vals = static_cast<const float*>(A.vals);
    a.B = B;
    a.C = C;
    a.ldb = ldb;
    a.ldc = ldc;
    a.m = A.m;
    a.n = A.n;
    a.K = K;
    a.nnz = A.nnz;
    a.alpha = s.alpha;
    a.beta = s.beta;
    a.vec_ok = (reinterpret_cast<uintptr_t>(B) % 16 == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && ldb % 4 == 0 &&
                ldc % 4 == 0)
                   ? 1
                   : 0;
    const int slices = ceil_div(K, kSpmmKT);
    // one workgroup fits a CU (its B slice takes most of the LDS): aim at one per CU or more
    int splits = slices >= 256 ? 1 : ceil_div(256, slices);
    const int max_splits = ceil_div(A.m, 16);
    if (splits > max_splits) splits = max_splits;
    a.row_splits = splits;
    const size_t lds = sizeof(float) * (kSpmmNB + 1) * kSpmmKT;  // the B block and one zero row
    static thread_local bool allowed = false;
    if (!allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(spmm_csr_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return e;
        allowed = true;
    }
    hipLaunchKernelGGL(spmm_csr_kernel, dim3(slices, splits), dim3(kSpmmWG), lds, st, a);
    return hipGetLastError();
}

const char* spmm_kernel_name() { return "spmm_csr_kernel"; }

}  // namespace spmv
