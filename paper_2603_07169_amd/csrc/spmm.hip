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

// acc += (val of lane S of the quad) * b: the quad broadcast rides on the multiply-add itself.
// All 64 lanes are active wherever this is used.
template <int S>
__device__ __forceinline__ void fma_quad(float& acc, float val, float b) {
    if constexpr (S == 0)
        asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[0,0,0,0] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(val), "v"(b));
    else if constexpr (S == 1)
        asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[1,1,1,1] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(val), "v"(b));
    else if constexpr (S == 2)
        asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[2,2,2,2] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(val), "v"(b));
    else
        asm("v_fmac_f32_dpp %0, %1, %2 quad_perm:[3,3,3,3] row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(val), "v"(b));
}

// SINGLE: B has at most kSpmmNB rows, so one block holds all of it and cb0 is 0 throughout.
template <bool SINGLE>
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

    for (int cb0 = 0; cb0 < (SINGLE ? 1 : a.n); cb0 += NB) {
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

        // (first entry, length) of this lane's row in group gi.  A lane past the last row takes the last
        // row again (and stores nothing): two unconditional loads and no select, so nothing here
        // tempts the compiler into a branch with a wait behind it.
        auto load_row = [&](int gi, int& rs, int& len) {
            int r = base_of(gi) + rsub;
            r = r < row_hi ? r : row_hi - 1;
            const int32_t* rp = a.rowptr + (r > 0 ? r : 0);
            rs = rp[0];
            len = rp[1] - rs;
        };
        // A chunk is entries c0 + q, c0 + q + 4, .. (U of them) of the lane's row.  issue() only
        // requests them, so the loads stay in flight while something else is multiplied; a lane
        // reads on past the end of its row (into the next rows) and finish() sorts that out.
        // Where every lane's last read lies inside the arrays (all but the last rows of the matrix)
        // the loads share one address and differ in their immediate offsets.
        auto issue = [&](int rs, int c0, int (&col)[U], float (&val)[U]) {
            const int kq = rs + c0 + q;
            if (!__builtin_amdgcn_ballot_w64(kq + 4 * (U - 1) >= a.nnz)) {
                const int32_t* cp = a.colidx + kq;
                const float* vp = a.vals + kq;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    col[u] = cp[4 * u];
                    val[u] = vp[4 * u];
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int k = kq + 4 * u < a.nnz ? kq + 4 * u : a.nnz - 1;
                    col[u] = a.colidx[k];
                    val[u] = a.vals[k];
                }
            }
        };
        // Column -> byte offset of the B row in the LDS block.  Entries past the row's end, or with a
        // column outside this block, point at the zero row; the former also get the value 0 (they
        // belong to another row, whose value need not be finite).
        auto finish = [&](int len, int c0, int (&col)[U], float (&val)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool live = c0 + q + 4 * u < len;
                unsigned c = static_cast<unsigned>(col[u] - (SINGLE ? 0 : cb0));  // a column before the block wraps to a huge number
                c = c < static_cast<unsigned>(NB) ? c : static_cast<unsigned>(NB);
                c = live ? c : static_cast<unsigned>(NB);
                col[u] = static_cast<int>(c * (KT * 4));
                val[u] = live ? val[u] : 0.f;
            }
        };

        int gi = wave;
        int rs, len, rs_n, len_n;
        load_row(gi, rs, len);
        load_row(gi + WAVES, rs_n, len_n);
        int col[U], coln[U];
        float val[U], valn[U];
        issue(rs, 0, col, val);
        finish(len, 0, col, val);
        while (gi < n_groups) {
            // the next group's first chunk and the rows of the group after it: in flight during the multiply
            issue(rs_n, 0, coln, valn);
            int rs_nn, len_nn;
            load_row(gi + 2 * WAVES, rs_nn, len_nn);

            float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
            for (int c0 = 0;; c0 += 4 * U) {
#pragma unroll
                for (int u = 0; u < U; u += 2) {
                    if (!__builtin_amdgcn_ballot_w64(c0 + 4 * u < len)) break;  // no row of the wavefront reaches this far
                    // eight entries of the row: two from each lane of the quad
                    f32x4 b[8];
                    b[0] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<0>(col[u]));
                    b[1] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<1>(col[u]));
                    b[2] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<2>(col[u]));
                    b[3] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<3>(col[u]));
                    b[4] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<0>(col[u + 1]));
                    b[5] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<1>(col[u + 1]));
                    b[6] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<2>(col[u + 1]));
                    b[7] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<3>(col[u + 1]));
#define SPMM_FMA4(S, V, BV) \
    fma_quad<S>(acc0, V, BV[0]); fma_quad<S>(acc1, V, BV[1]); fma_quad<S>(acc2, V, BV[2]); fma_quad<S>(acc3, V, BV[3]);
                    SPMM_FMA4(0, val[u], b[0]) SPMM_FMA4(1, val[u], b[1]) SPMM_FMA4(2, val[u], b[2]) SPMM_FMA4(3, val[u], b[3])
                    SPMM_FMA4(0, val[u + 1], b[4]) SPMM_FMA4(1, val[u + 1], b[5]) SPMM_FMA4(2, val[u + 1], b[6])
                    SPMM_FMA4(3, val[u + 1], b[7])
#undef SPMM_FMA4
                }
                if (!__builtin_amdgcn_ballot_w64(c0 + 4 * U < len)) break;
                issue(rs, c0 + 4 * U, col, val);  // rows longer than a chunk: fetched on demand
                finish(len, c0 + 4 * U, col, val);
            }

            // What the next round needs is settled before C is touched: nothing that is loaded is
            // then still awaited when the loop comes round, and the store below stays in flight.
            finish(len_n, 0, coln, valn);
            asm volatile("" : "+v"(rs_nn), "+v"(len_nn));

            const int r = base_of(gi) + rsub;
            if (r < row_hi && 4 * q < kw) {
                float* dst = a.C + static_cast<size_t>(r) * a.ldc + k0 + 4 * q;
                const bool first = cb0 == 0;
                const bool reads_c = !first || a.beta != 0.f;
                const float scale_c = first ? a.beta : 1.f;
                const f32x4 acc = {acc0, acc1, acc2, acc3};
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
        for (const void* k : {reinterpret_cast<const void*>(spmm_csr_kernel<true>),
                              reinterpret_cast<const void*>(spmm_csr_kernel<false>)}) {
            hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return e;
        }
        allowed = true;
    }
    if (A.n <= kSpmmNB)
        hipLaunchKernelGGL(spmm_csr_kernel<true>, dim3(slices, splits), dim3(kSpmmWG), lds, st, a);
    else
        hipLaunchKernelGGL(spmm_csr_kernel<false>, dim3(slices, splits), dim3(kSpmmWG), lds, st, a);
    return hipGetLastError();
}

const char* spmm_kernel_name() { return "spmm_csr_kernel"; }

}  // namespace spmv
