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
// wavefront serves 16 rows at a time, for as long as the longest of them lasts: the rows can be
// handed out in an order that puts rows of like length side by side (built at analysis time on
// request).  The quad reads its row's entries straight from memory, 16 bytes per lane and load;
// an entry is then handed to the other three lanes with a quad broadcast that rides on the
// multiply-add, and each lane adds value * B-row piece out of LDS.  Row ids, row bounds and
// entries of the coming groups are fetched while the current one is multiplied.
// B wider than the LDS block is taken in several passes over A, accumulating into C.
struct SpmmArgs {
    const int32_t* rowptr;
    const int32_t* colidx;
    const void* vals;     // float or bf16 bit patterns (the kernel's storage type)
    const int32_t* rows;  // row order (SORTED kernels), else unused
    const void* B;        // same storage type as vals
    float* C;
    int64_t ldb, ldc;
    int32_t m, n, K, nnz;
    int32_t row_splits;  // split y takes every row_splits-th group of 16 rows, from group y on
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

// 4-byte aligned vectors of four: a row's entries start anywhere in colidx / vals.
typedef int32_t i32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2_a2 __attribute__((ext_vector_type(2), aligned(2)));

__device__ __forceinline__ f32x4 widen4(u32x2_t b) {  // four bf16 values, little-endian pairs
    return f32x4{__uint_as_float(b[0] << 16), __uint_as_float(b[0] & 0xFFFF0000u), __uint_as_float(b[1] << 16),
                 __uint_as_float(b[1] & 0xFFFF0000u)};
}
// Four consecutive stored values from element k on (any alignment the element type allows), as floats.
__device__ __forceinline__ f32x4 load4_any(const float* p, int64_t k) { return *reinterpret_cast<const f32x4_a4*>(p + k); }
__device__ __forceinline__ f32x4 load4_any(const uint16_t* p, int64_t k) { return widen4(*reinterpret_cast<const u32x2_a2*>(p + k)); }
// Four consecutive values from a 16-byte (float) or 8-byte (bf16) aligned address.
__device__ __forceinline__ f32x4 load4_aligned(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ f32x4 load4_aligned(const uint16_t* p) { return widen4(*reinterpret_cast<const u32x2_t*>(p)); }

// Copies rows cb0 .. cb0+nbk-1 of the slice of B (columns k0 .. k0+kw-1) to the LDS block Bs[row][16] as floats.
template <typename E>
__device__ __forceinline__ void stage_b_block(const E* B, int64_t ldb, int cb0, int nbk, int k0, int kw, bool vec_ok, float* Bs,
                                              int tid) {
    for (int idx = tid; idx < nbk * 4; idx += kSpmmWG) {
        const int j = idx >> 2, qq = idx & 3;
        const E* src = B + static_cast<size_t>(cb0 + j) * ldb + k0 + 4 * qq;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        if (vec_ok && 4 * qq + 4 <= kw) {
            v = load4_aligned(src);
        } else {
            for (int t = 0; t < 4; ++t)
                if (4 * qq + t < kw) v[t] = widen(src[t]);
        }
        *reinterpret_cast<f32x4*>(Bs + j * kSpmmKT + 4 * qq) = v;
    }
}

// SINGLE: B has at most kSpmmNB rows, so one block holds all of it and cb0 is 0 throughout.
// SORTED: the wavefronts take their rows from a.rows (rows of like length side by side) instead
// of in natural order.
template <typename T, bool SINGLE, bool SORTED>
__global__ __launch_bounds__(kSpmmWG) void spmm_csr_kernel(const SpmmArgs a) {
    using E = typename T::elem;
    const E* const a_vals = static_cast<const E*>(a.vals);
    constexpr int KT = kSpmmKT, NB = kSpmmNB, RPW = 16, WAVES = kSpmmWG / 64;
    constexpr int U = 8;  // entries per lane and chunk: a chunk covers 32 entries of a row
    static_assert(KT == 16, "four lanes per row, one float4 each");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* Bs = reinterpret_cast<float*>(smem_raw);  // [NB + 1][KT]; row NB stays zero
    const unsigned char* const Bq = smem_raw + 16 * (threadIdx.x & 3);  // this lane's float4 of row 0
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane & 3;      // which float4 of the slice, and which entries of the row (4q .. 4q+3, 16+4q .. 16+4q+3)
    const int rsub = lane >> 2;  // which of the wavefront's 16 rows

    // Workgroup ids are handed to the 8 dies round-robin.  Die j takes a contiguous run of
    // (slice, split) pairs, so that the slices whose pieces of a row of C lie side by side are
    // written through the same L2.
    const int n_slices = (a.K + KT - 1) / KT;
    int pair;
    {
        const int nb = gridDim.x, per = nb / kXcds, rem = nb % kXcds;
        const int die = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
        pair = die * per + (die < rem ? die : rem) + slot;
    }
    const int slice = pair % n_slices, split = pair / n_slices;
    const int k0 = slice * KT;
    const int kw = a.K - k0 < KT ? a.K - k0 : KT;  // live columns of this slice
    const bool full4 = a.vec_ok && 4 * q + 4 <= kw;  // this lane's float4 lies wholly inside the slice

    if (a.nnz == 0) {  // C <- beta*C; the main path below may then assume that A has entries
        const int row_lo = static_cast<int>(static_cast<int64_t>(a.m) * split / a.row_splits);
        const int row_hi = static_cast<int>(static_cast<int64_t>(a.m) * (split + 1) / a.row_splits);
        for (int r = row_lo + tid / 4; r < row_hi; r += kSpmmWG / 4) {
            float* dst = a.C + static_cast<size_t>(r) * a.ldc + k0 + 4 * q;
            for (int t = 0; t < 4; ++t)
                if (4 * q + t < kw) dst[t] = a.beta != 0.f ? a.beta * dst[t] : 0.f;
        }
        return;
    }
    if (tid < KT) Bs[NB * KT + tid] = 0.f;  // the row that entries without a partner in this block point to

    // Rows are dealt out in groups of 16 positions of the row order.  Workgroup (slice, split y of S)
    // takes the groups y, y + S, y + 2S, ..: with the rows sorted by length every split gets its
    // share of the long ones.  Its wavefronts take those in turn.  All slices walk through the
    // rows in the same order, so a row of C is written, piece by piece, within a short time.
    const int S = a.row_splits, y = split;
    const int total_groups = (a.m + RPW - 1) / RPW;
    const int n_groups = total_groups > y ? (total_groups - y + S - 1) / S : 0;
    auto pos_of = [&](int j) {  // position of this lane's row in the wavefront's j-th group; m or more: none
        if (j >= n_groups) return a.m;
        return (y + S * j) * RPW + rsub;
    };
    // A lane without a row takes the last row again (and stores nothing): no select on loaded
    // values anywhere, so nothing tempts the compiler into a branch with a wait behind it.
    auto load_id = [&](int j) {
        int p = pos_of(j);
        p = p < a.m ? p : a.m - 1;
        return SORTED ? a.rows[p] : p;
    };
    auto load_row = [&](int r, int& rs, int& len) {  // first entry and length of row r
        const int32_t* rp = a.rowptr + r;
        rs = rp[0];
        len = rp[1] - rs;
    };

    for (int cb0 = 0; cb0 < (SINGLE ? 1 : a.n); cb0 += NB) {
        const int nbk = a.n - cb0 < NB ? a.n - cb0 : NB;  // rows of B in this block
        if (cb0 > 0) __syncthreads();                     // the previous block is no longer read
        stage_b_block(static_cast<const E*>(a.B), a.ldb, cb0, nbk, k0, kw, a.vec_ok != 0, Bs, tid);
        __syncthreads();

        // A chunk is 32 consecutive entries of the lane's row from entry c0 on; lane q of the quad
        // holds entries 4q .. 4q+3 (slots 0..3) and 16+4q .. 16+4q+3 (slots 4..7) of it, two 16-byte
        // loads per array.  issue() only requests them, so the loads stay in flight while something
        // else is multiplied; a lane reads on past the end of its row (into the next rows) and
        // finish() sorts that out.  Only near the end of the arrays (the last rows of the matrix)
        // are the reads clamped one by one.
        auto issue = [&](int rs, int c0, int (&col)[U], float (&val)[U]) {
            const int kq = rs + c0 + 4 * q;
            if (!__builtin_amdgcn_ballot_w64(kq + 20 > a.nnz)) {
                const i32x4_a4 ca = *reinterpret_cast<const i32x4_a4*>(a.colidx + kq);
                const i32x4_a4 cb = *reinterpret_cast<const i32x4_a4*>(a.colidx + kq + 16);
                const f32x4 va = load4_any(a_vals, kq);
                const f32x4 vb = load4_any(a_vals, kq + 16);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    col[e] = ca[e];
                    col[4 + e] = cb[e];
                    val[e] = va[e];
                    val[4 + e] = vb[e];
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int t = kq + 16 * (u >> 2) + (u & 3);
                    const int k = t < a.nnz ? t : a.nnz - 1;
                    col[u] = a.colidx[k];
                    val[u] = widen(a_vals[k]);
                }
            }
        };
        // Column -> byte offset of the B row in the LDS block.  Entries past the row's end, or with a
        // column outside this block, point at the zero row; the former also get the value 0 (they
        // belong to another row, whose value need not be finite).
        auto finish = [&](int len, int c0, int (&col)[U], float (&val)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool live = c0 + 16 * (u >> 2) + 4 * q + (u & 3) < len;
                unsigned c = static_cast<unsigned>(col[u] - (SINGLE ? 0 : cb0));  // a column before the block wraps to a huge number
                c = c < static_cast<unsigned>(NB) ? c : static_cast<unsigned>(NB);
                c = live ? c : static_cast<unsigned>(NB);
                col[u] = static_cast<int>(c * (KT * 4));
                val[u] = live ? val[u] : 0.f;
            }
        };

        // Three stages in flight: row ids three groups ahead, row bounds two ahead, entries one ahead.
        int gi = wave;
        int r = load_id(gi), r_n = load_id(gi + WAVES), r_nn = load_id(gi + 2 * WAVES);
        int rs, len, rs_n, len_n;
        load_row(r, rs, len);
        load_row(r_n, rs_n, len_n);
        int col[U], coln[U];
        float val[U], valn[U];
        issue(rs, 0, col, val);
        finish(len, 0, col, val);
        while (gi < n_groups) {
            issue(rs_n, 0, coln, valn);
            int rs_nn, len_nn;
            load_row(r_nn, rs_nn, len_nn);
            int r_nnn = load_id(gi + 3 * WAVES);

            float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
            for (int c0 = 0;; c0 += 4 * U) {
                // Step st takes entries c0 + 4 st .. c0 + 4 st + 3 of every row: slots 4 (st / 4) .. + 3
                // of lane st % 4 of the quad.  Two steps per trip.
#define SPMM_STEP_LOADS(B0, ST)                                                                                  \
    B0[0] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<(ST) % 4>(col[4 * ((ST) / 4) + 0]));                \
    B0[1] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<(ST) % 4>(col[4 * ((ST) / 4) + 1]));                \
    B0[2] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<(ST) % 4>(col[4 * ((ST) / 4) + 2]));                \
    B0[3] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<(ST) % 4>(col[4 * ((ST) / 4) + 3]));
#define SPMM_STEP_FMAS(B0, ST)                                                 \
    _Pragma("unroll") for (int e = 0; e < 4; ++e) {                            \
        fma_quad<(ST) % 4>(acc0, val[4 * ((ST) / 4) + e], B0[e][0]);           \
        fma_quad<(ST) % 4>(acc1, val[4 * ((ST) / 4) + e], B0[e][1]);           \
        fma_quad<(ST) % 4>(acc2, val[4 * ((ST) / 4) + e], B0[e][2]);           \
        fma_quad<(ST) % 4>(acc3, val[4 * ((ST) / 4) + e], B0[e][3]);           \
    }
#define SPMM_TWO_STEPS(ST)                                                                     \
    if (__builtin_amdgcn_ballot_w64(c0 + 4 * (ST) < len)) {                                    \
        f32x4 b0[4], b1[4];                                                                    \
        SPMM_STEP_LOADS(b0, ST) SPMM_STEP_LOADS(b1, (ST) + 1)                                  \
        SPMM_STEP_FMAS(b0, ST) SPMM_STEP_FMAS(b1, (ST) + 1)                                    \
    } else {                                                                                   \
        break;                                                                                 \
    }
                do {  // left by the first pair of steps that no row of the wavefront reaches
                    SPMM_TWO_STEPS(0) SPMM_TWO_STEPS(2) SPMM_TWO_STEPS(4) SPMM_TWO_STEPS(6)
                } while (false);
#undef SPMM_TWO_STEPS
#undef SPMM_STEP_FMAS
#undef SPMM_STEP_LOADS
                if (!__builtin_amdgcn_ballot_w64(c0 + 4 * U < len)) break;
                issue(rs, c0 + 4 * U, col, val);  // rows longer than a chunk: fetched on demand
                finish(len, c0 + 4 * U, col, val);
            }

            // What the next round needs is settled before C is touched: nothing that is loaded is
            // then still awaited when the loop comes round, and the store below stays in flight.
            finish(len_n, 0, coln, valn);
            asm volatile("" : "+v"(rs_nn), "+v"(len_nn), "+v"(r_nnn));

            if (pos_of(gi) < a.m && 4 * q < kw) {
                float* dst = a.C + static_cast<size_t>(r) * a.ldc + k0 + 4 * q;
                const bool first = cb0 == 0;
                const bool reads_c = !first || a.beta != 0.f;
                const float scale_c = first ? a.beta : 1.f;
                const f32x4 acc = {acc0, acc1, acc2, acc3};
                if (full4) {
                    f32x4 out = a.alpha * acc;
                    if (reads_c) out += scale_c * *reinterpret_cast<const f32x4*>(dst);
                    __builtin_nontemporal_store(out, reinterpret_cast<f32x4*>(dst));  // written once, not read again soon
                } else {
                    for (int t = 0; t < 4; ++t)
                        if (4 * q + t < kw) dst[t] = a.alpha * acc[t] + (reads_c ? scale_c * dst[t] : 0.f);
                }
            }
            gi += WAVES;
            r = r_n;
            r_n = r_nn;
            r_nn = r_nnn;
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

// ------------------------------------------------------------------------------------------
// The same product from a packed copy of A (built at analysis time on request).  The rows are
// taken in the length-sorted order; group g (16 rows) is stored as ceil(longest row / 16) blocks,
// a block being what one load of the wavefront fetches: lane (row rsub, quad lane q) owns the four
// slots of the entries ranked 16b + 4q .. 16b + 4q + 3 in its row's order (below), columns and values in arrays of their
// own.  The order inside a row deals the entries out by column residue modulo 4, turned by the row's position: B's rows
// lie 64 bytes apart in LDS, four to a cycle of the banks, and the 16 rows a wavefront reads at once then fall on the
// four quarters in turn (bank-conflict cycles -44 % against storage order).  Slots past a row's end hold the value 0
// and a column that maps to the zero row.  Against
// reading CSR directly: every load is aligned and fully coalesced, columns take 2 bytes while
// n <= 32768, no row bounds are fetched, no entry needs a validity test, and the number of steps
// of a group is a scalar from its descriptor.
struct SpmmPackedArgs {
    const int32_t* desc;  // pairs (first block, steps of 4 entries) per group, one closing pair
    const void* pcol;     // [blocks + 1][64 lanes][4]: uint16 or int32; the last block is padding only
    const float* pval;    // [blocks + 1][64][4]
    const int32_t* rows;  // [m] the row order
    const void* B;        // float or bf16 bit patterns
    float* C;
    int64_t ldb, ldc;
    int32_t m, n, K, num_groups;
    int32_t row_splits, vec_ok;
    float alpha, beta;
};

// Column number a padding slot holds: the zero row itself when all of B fits one block, else a
// number no block of B contains.
template <typename CT>
__host__ __device__ inline CT packed_pad_column(int n) {
    return n <= kSpmmNB ? static_cast<CT>(kSpmmNB) : static_cast<CT>(-1);
}

template <typename CT, typename E>
__global__ __launch_bounds__(64) void spmm_pack_kernel(const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colidx,
                                                       const E* __restrict__ vals, const int32_t* __restrict__ rows,
                                                       const int32_t* __restrict__ desc, int m, int n, CT* __restrict__ pcol,
                                                       float* __restrict__ pval) {
    const int g = blockIdx.x, lane = threadIdx.x, rsub = lane >> 2, q = lane & 3;
    const int first = desc[2 * g], nblocks = desc[2 * g + 2] - first;
    const int pos = 16 * g + rsub;
    int rs = 0, len = 0;
    if (pos < m) {
        const int r = rows[pos];
        rs = rowptr[r];
        len = rowptr[r + 1] - rs;
    }
    const CT pad = packed_pad_column<CT>(n);
    // padding first: the slots past the row's end
    for (int b = 0; b < nblocks; ++b) {
        const size_t slot0 = (static_cast<size_t>(first + b) * 64 + lane) * 4;
        for (int e = 0; e < 4; ++e) {
            if (16 * b + 4 * q + e >= len) {
                pcol[slot0 + e] = pad;
                pval[slot0 + e] = 0.f;
            }
        }
    }
    // The row's entries, one lane per row.  Entry e, the j-th of the row's entries with its column residue, has the key
    // 4 j + d with d = (column - pos) mod 4; its rank is the number of entries with a smaller key: of the entries with
    // difference dd, those numbered below j (and number j itself when dd < d), as far as there are any.
    if (q == 0 && len > 0) {
        int cnt[4] = {0, 0, 0, 0};
        for (int k = 0; k < len; ++k) ++cnt[(colidx[rs + k] - pos) & 3];
        int seen[4] = {0, 0, 0, 0};
        for (int k = 0; k < len; ++k) {
            const int c = colidx[rs + k];
            const int d = (c - pos) & 3;
            const int j = seen[d]++;
            int t = 0;
#pragma unroll
            for (int dd = 0; dd < 4; ++dd) {
                const int below = j + (dd < d ? 1 : 0);
                t += cnt[dd] < below ? cnt[dd] : below;
            }
            const size_t slot = ((static_cast<size_t>(first + (t >> 4)) * 64 + 4 * rsub + ((t >> 2) & 3)) * 4) + (t & 3);
            pcol[slot] = static_cast<CT>(c);
            pval[slot] = widen(vals[rs + k]);
        }
    }
}

// One block of the packed copy as a lane holds it.
template <typename CT>
struct PackedBlock;
template <>
struct PackedBlock<uint16_t> {
    unsigned c01, c23;  // four 16-bit columns
    f32x4 v;
    // block: the same in every lane (a scalar base address), lane: the only per-lane part of the address
    __device__ __forceinline__ void load(const void* pcol, const float* pval, int block, int lane) {
        const uint16_t* cb = static_cast<const uint16_t*>(pcol) + static_cast<size_t>(block) * 256;
        const float* vb = pval + static_cast<size_t>(block) * 256;
        const uint2 c = *reinterpret_cast<const uint2*>(cb + static_cast<unsigned>(4 * lane));
        c01 = c.x;
        c23 = c.y;
        v = *reinterpret_cast<const f32x4*>(vb + static_cast<unsigned>(4 * lane));
    }
    __device__ __forceinline__ unsigned col(int e) const {
        const unsigned w = e < 2 ? c01 : c23;
        return (e & 1) ? w >> 16 : w & 0xFFFFu;
    }
    __device__ __forceinline__ void touch() { asm volatile("" : "+v"(c01), "+v"(c23), "+v"(v)); }
};
template <>
struct PackedBlock<int32_t> {
    i32x4 c;
    f32x4 v;
    __device__ __forceinline__ void load(const void* pcol, const float* pval, int block, int lane) {
        c = *reinterpret_cast<const i32x4*>(static_cast<const int32_t*>(pcol) + static_cast<size_t>(block) * 256 + static_cast<unsigned>(4 * lane));
        v = *reinterpret_cast<const f32x4*>(pval + static_cast<size_t>(block) * 256 + static_cast<unsigned>(4 * lane));
    }
    __device__ __forceinline__ unsigned col(int e) const { return static_cast<unsigned>(c[e]); }
    __device__ __forceinline__ void touch() { asm volatile("" : "+v"(c), "+v"(v)); }
};

template <typename T, bool SINGLE, typename CT>
__global__ __launch_bounds__(kSpmmWG) void spmm_packed_kernel(const SpmmPackedArgs a) {
    using E = typename T::elem;
    constexpr int KT = kSpmmKT, NB = kSpmmNB, RPW = 16, WAVES = kSpmmWG / 64;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* Bs = reinterpret_cast<float*>(smem_raw);  // [NB + 1][KT]; row NB stays zero
    const unsigned char* const Bq = smem_raw + 16 * (threadIdx.x & 3);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // the same in every lane: what depends on it alone stays in scalar registers
    const int q = lane & 3, rsub = lane >> 2;

    // die-aware numbering of the (slice, split) pairs, as in spmm_csr_kernel
    const int n_slices = (a.K + KT - 1) / KT;
    int pair;
    {
        const int nb = gridDim.x, per = nb / kXcds, rem = nb % kXcds;
        const int die = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
        pair = die * per + (die < rem ? die : rem) + slot;
    }
    const int slice = pair % n_slices, split = pair / n_slices;
    const int k0 = slice * KT;
    const int kw = a.K - k0 < KT ? a.K - k0 : KT;
    const bool full4 = a.vec_ok && 4 * q + 4 <= kw;
    if (tid < KT) Bs[NB * KT + tid] = 0.f;

    const int S = a.row_splits, y = split;
    const int n_groups = a.num_groups > y ? (a.num_groups - y + S - 1) / S : 0;  // this workgroup's
    // (first block, steps) of the wavefront's j-th group; past the end: the closing pair (all blocks, 0)
    auto load_desc = [&](int j, int& first, int& nsteps) {
        const int g = j < n_groups ? y + S * j : a.num_groups;
        first = a.desc[2 * g];
        nsteps = a.desc[2 * g + 1];
    };

    for (int cb0 = 0; cb0 < (SINGLE ? 1 : a.n); cb0 += NB) {
        const int nbk = a.n - cb0 < NB ? a.n - cb0 : NB;
        if (cb0 > 0) __syncthreads();
        stage_b_block(static_cast<const E*>(a.B), a.ldb, cb0, nbk, k0, kw, a.vec_ok != 0, Bs, tid);
        __syncthreads();

        // column -> byte offset of the B row in the LDS block; padding and columns of other blocks -> zero row
        auto offsets = [&](const PackedBlock<CT>& blk, int (&off)[4]) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                unsigned c = blk.col(e);
                if constexpr (!SINGLE) {
                    c -= static_cast<unsigned>(cb0);  // a column before the block wraps to a huge number
                    c = c < static_cast<unsigned>(NB) ? c : static_cast<unsigned>(NB);
                }
                off[e] = static_cast<int>(c * (KT * 4));
            }
        };

        int j = wave;
        int first, nsteps, first_n, nsteps_n;  // first_n, nsteps_n: as loaded (vector registers), one group ahead
        load_desc(j, first, nsteps);
        load_desc(j + WAVES, first_n, nsteps_n);
        first = __builtin_amdgcn_readfirstlane(first);
        nsteps = __builtin_amdgcn_readfirstlane(nsteps);
        PackedBlock<CT> cur;
        cur.load(a.pcol, a.pval, first, lane);
        while (j < n_groups) {
            // the next group's pair arrived a group ago; as scalars, block numbers and step counts cost no vector work
            const int first_nu = __builtin_amdgcn_readfirstlane(first_n);
            const int nsteps_nu = __builtin_amdgcn_readfirstlane(nsteps_n);
            const int pos = (y + S * j) * RPW + rsub;
            const int r = a.rows[pos < a.m ? pos : a.m - 1];
            float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
            const int nblocks = nsteps > 0 ? (nsteps + 3) / 4 : 1;  // a group of empty rows: one pass that multiplies nothing
            for (int b = 0; b < nblocks; ++b) {
                // the next block of the wavefront's stream: the group's next one, else the next group's first
                const int next_block = b + 1 < nblocks ? first + b + 1 : first_nu;
                PackedBlock<CT> nxt;
                nxt.load(a.pcol, a.pval, next_block, lane);
                const int steps = nsteps - 4 * b;  // steps of this block still to do (4 or more: all four)
                int off[4];
                offsets(cur, off);
#define SPMM_STEP_LOADS(B0, J)                                                   \
    B0[0] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<J>(off[0]));         \
    B0[1] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<J>(off[1]));         \
    B0[2] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<J>(off[2]));         \
    B0[3] = *reinterpret_cast<const f32x4*>(Bq + quad_bcast<J>(off[3]));
#define SPMM_STEP_FMAS(B0, J)                          \
    _Pragma("unroll") for (int e = 0; e < 4; ++e) {    \
        fma_quad<J>(acc0, cur.v[e], B0[e][0]);         \
        fma_quad<J>(acc1, cur.v[e], B0[e][1]);         \
        fma_quad<J>(acc2, cur.v[e], B0[e][2]);         \
        fma_quad<J>(acc3, cur.v[e], B0[e][3]);         \
    }
                // step J takes the four slots of lane J of every quad.  All LDS reads of the block go out
                // first, so the multiply-adds of the early steps run while the later rows arrive.
                {
                    f32x4 b0[4], b1[4], b2[4], b3[4];
                    switch (steps >= 4 ? 4 : steps) {
                        case 4:
                            SPMM_STEP_LOADS(b0, 0) SPMM_STEP_LOADS(b1, 1) SPMM_STEP_LOADS(b2, 2) SPMM_STEP_LOADS(b3, 3)
                            SPMM_STEP_FMAS(b0, 0) SPMM_STEP_FMAS(b1, 1) SPMM_STEP_FMAS(b2, 2) SPMM_STEP_FMAS(b3, 3)
                            break;
                        case 3:
                            SPMM_STEP_LOADS(b0, 0) SPMM_STEP_LOADS(b1, 1) SPMM_STEP_LOADS(b2, 2)
                            SPMM_STEP_FMAS(b0, 0) SPMM_STEP_FMAS(b1, 1) SPMM_STEP_FMAS(b2, 2)
                            break;
                        case 2:
                            SPMM_STEP_LOADS(b0, 0) SPMM_STEP_LOADS(b1, 1) SPMM_STEP_FMAS(b0, 0) SPMM_STEP_FMAS(b1, 1)
                            break;
                        case 1:
                            SPMM_STEP_LOADS(b0, 0) SPMM_STEP_FMAS(b0, 0)
                            break;
                        default:
                            break;
                    }
                }
#undef SPMM_STEP_FMAS
#undef SPMM_STEP_LOADS
                nxt.touch();  // arrived before anything is stored: the loop never waits behind a store
                cur = nxt;
            }

            if (pos < a.m && 4 * q < kw) {
                float* dst = a.C + static_cast<size_t>(r) * a.ldc + k0 + 4 * q;
                const bool first_pass = cb0 == 0;
                const bool reads_c = !first_pass || a.beta != 0.f;
                const float scale_c = first_pass ? a.beta : 1.f;
                const f32x4 acc = {acc0, acc1, acc2, acc3};
                if (full4) {
                    f32x4 out = a.alpha * acc;
                    if (reads_c) out += scale_c * *reinterpret_cast<const f32x4*>(dst);
                    __builtin_nontemporal_store(out, reinterpret_cast<f32x4*>(dst));  // written once, not read again soon
                } else {
                    for (int t = 0; t < 4; ++t)
                        if (4 * q + t < kw) dst[t] = a.alpha * acc[t] + (reads_c ? scale_c * dst[t] : 0.f);
                }
            }
            j += WAVES;
            first = first_nu;
            nsteps = nsteps_nu;
            load_desc(j + WAVES, first_n, nsteps_n);
        }
    }
}

}  // namespace

namespace {

// 128-bit (float) or 64-bit (bf16) accesses to B, 128-bit ones to C: base addresses and leading dimensions must allow them.
bool spmm_vec_ok(bool bf16, const void* B, int64_t ldb, const float* C, int64_t ldc) {
    return reinterpret_cast<uintptr_t>(B) % (bf16 ? 8 : 16) == 0 && reinterpret_cast<uintptr_t>(C) % 16 == 0 && ldb % 4 == 0 &&
           ldc % 4 == 0;
}

template <typename K>
hipError_t allow_lds(K kernel, size_t lds) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
}

template <typename T>
hipError_t launch_spmm_t(const SpmmArgs& a, bool single, bool sorted, dim3 grid, size_t lds, hipStream_t st) {
    static thread_local bool allowed = false;
    if (!allowed) {
        hipError_t e = allow_lds(spmm_csr_kernel<T, true, true>, lds);
        if (e == hipSuccess) e = allow_lds(spmm_csr_kernel<T, true, false>, lds);
        if (e == hipSuccess) e = allow_lds(spmm_csr_kernel<T, false, true>, lds);
        if (e == hipSuccess) e = allow_lds(spmm_csr_kernel<T, false, false>, lds);
        if (e != hipSuccess) return e;
        allowed = true;
    }
    const dim3 block(kSpmmWG);
    if (sorted) {
        if (single) hipLaunchKernelGGL((spmm_csr_kernel<T, true, true>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((spmm_csr_kernel<T, false, true>), grid, block, lds, st, a);
    } else {
        if (single) hipLaunchKernelGGL((spmm_csr_kernel<T, true, false>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((spmm_csr_kernel<T, false, false>), grid, block, lds, st, a);
    }
    return hipGetLastError();
}

template <typename T>
hipError_t launch_spmm_packed_t(const SpmmPackedArgs& a, bool col16, bool single, dim3 grid, size_t lds, hipStream_t st) {
    static thread_local bool allowed = false;
    if (!allowed) {
        hipError_t e = allow_lds(spmm_packed_kernel<T, true, uint16_t>, lds);
        if (e == hipSuccess) e = allow_lds(spmm_packed_kernel<T, false, uint16_t>, lds);
        if (e == hipSuccess) e = allow_lds(spmm_packed_kernel<T, false, int32_t>, lds);
        if (e != hipSuccess) return e;
        allowed = true;
    }
    const dim3 block(kSpmmWG);
    if (col16) {
        if (single) hipLaunchKernelGGL((spmm_packed_kernel<T, true, uint16_t>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((spmm_packed_kernel<T, false, uint16_t>), grid, block, lds, st, a);
    } else {
        hipLaunchKernelGGL((spmm_packed_kernel<T, false, int32_t>), grid, block, lds, st, a);
    }
    return hipGetLastError();
}

template <typename CT>
hipError_t launch_spmm_pack_t(const MatrixView& A, const int32_t* rows, const int32_t* desc, int32_t num_groups, CT* pcol, float* pval,
                              hipStream_t st) {
    if (A.bf16)
        hipLaunchKernelGGL((spmm_pack_kernel<CT, uint16_t>), dim3(num_groups), dim3(64), 0, st, A.rowptr, A.colidx,
                           static_cast<const uint16_t*>(A.vals), rows, desc, A.m, A.n, pcol, pval);
    else
        hipLaunchKernelGGL((spmm_pack_kernel<CT, float>), dim3(num_groups), dim3(64), 0, st, A.rowptr, A.colidx,
                           static_cast<const float*>(A.vals), rows, desc, A.m, A.n, pcol, pval);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_spmm(const MatrixView& A, const int32_t* rows, const void* B, int64_t ldb, float* C, int64_t ldc,
                       int32_t K, Scalars s, hipStream_t st) {
    if (A.m <= 0 || K <= 0) return hipSuccess;
    SpmmArgs a{};
    a.rowptr = A.rowptr;
    a.colidx = A.colidx;
    a.vals = A.vals;
    a.rows = rows;
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
    a.vec_ok = spmm_vec_ok(A.bf16, B, ldb, C, ldc) ? 1 : 0;
    const int slices = ceil_div(K, kSpmmKT);
    // one workgroup fits a CU (its B slice takes most of the LDS): aim at one per CU or more
    int splits = slices >= 256 ? 1 : ceil_div(256, slices);
    const int max_splits = ceil_div(A.m, 16);
    if (splits > max_splits) splits = max_splits;
    a.row_splits = splits;
    const size_t lds = sizeof(float) * (kSpmmNB + 1) * kSpmmKT;  // the B block and one zero row
    const dim3 grid(slices * splits);
    const bool single = A.n <= kSpmmNB;
    return A.bf16 ? launch_spmm_t<BF16>(a, single, rows != nullptr, grid, lds, st)
                  : launch_spmm_t<F32>(a, single, rows != nullptr, grid, lds, st);
}

hipError_t launch_spmm_pack(const MatrixView& A, const int32_t* rows, const int32_t* desc, int32_t num_groups, bool col16,
                            void* pcol, float* pval, hipStream_t st) {
    if (num_groups <= 0) return hipSuccess;
    return col16 ? launch_spmm_pack_t(A, rows, desc, num_groups, static_cast<uint16_t*>(pcol), pval, st)
                 : launch_spmm_pack_t(A, rows, desc, num_groups, static_cast<int32_t*>(pcol), pval, st);
}

hipError_t launch_spmm_packed(const MatrixView& A, const PackedRows& P, const void* B, int64_t ldb, float* C, int64_t ldc,
                              int32_t K, Scalars s, hipStream_t st) {
    if (A.m <= 0 || K <= 0) return hipSuccess;
    SpmmPackedArgs a{};
    a.desc = P.desc;
    a.pcol = P.pcol;
    a.pval = P.pval;
    a.rows = P.rows;
    a.B = B;
    a.C = C;
    a.ldb = ldb;
    a.ldc = ldc;
    a.m = A.m;
    a.n = A.n;
    a.K = K;
    a.num_groups = P.num_groups;
    a.alpha = s.alpha;
    a.beta = s.beta;
    a.vec_ok = spmm_vec_ok(A.bf16, B, ldb, C, ldc) ? 1 : 0;
    const int slices = ceil_div(K, kSpmmKT);
    int splits = slices >= 256 ? 1 : ceil_div(256, slices);
    if (splits > P.num_groups) splits = P.num_groups;
    a.row_splits = splits;
    const size_t lds = sizeof(float) * (kSpmmNB + 1) * kSpmmKT;
    const dim3 grid(slices * splits);
    return A.bf16 ? launch_spmm_packed_t<BF16>(a, P.col16, A.n <= kSpmmNB, grid, lds, st)
                  : launch_spmm_packed_t<F32>(a, P.col16, A.n <= kSpmmNB, grid, lds, st);
}

const char* spmm_kernel_name() { return "spmm_csr_kernel"; }
const char* spmm_packed_kernel_name() { return "spmm_packed_kernel"; }

}  // namespace spmv
