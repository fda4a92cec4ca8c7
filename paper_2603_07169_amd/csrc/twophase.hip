// The two-pass plan for matrices whose columns are spread over more of x than any cache holds
// (gfx950).  Neither pass gathers from memory:
//
//   multiply  The entries are kept regrouped by blocks of 2^s columns.  A workgroup copies one
//             block of x to LDS, streams a piece of that block's entries (16-bit column within the
//             block, value), takes x out of LDS and writes the products, four at a time, to where
//             the second pass wants them.
//   reduce    The products are kept grouped by merge-path chunk (a contiguous stretch of the CSR
//             entry list plus the rows that end in it).  A workgroup streams its chunk's products,
//             drops each into LDS at its CSR position within the chunk (16-bit), and then runs the
//             row phase of the tile kernels over them: teams of lanes add up one row each, the
//             piece of a row that the chunk cuts off leaves as a carry.
//
// A tile is the set of entries that share a column block and a chunk.  Its entries keep their CSR
// order, and every tile is padded to a multiple of four entries (value 0, column = the zero slot
// after the x block, position 0xFFFF = dropped), so that a group of four consecutive slots never
// straddles two tiles: one 32-bit number per group says where its four products go.
// The regrouping is done once, at analysis time, on the device (the kernels in the second half).
#include <cstring>

#include <hip/hip_runtime.h>
#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>

#include "device_common.h"
#include "kernels.h"
#include "row_phase.h"

namespace spmv {
namespace {

typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTpMulWG = 1024;  // the x block takes 64 KB of LDS: two workgroups per compute unit, if a lane stays within 64 registers
constexpr int kTpMulGroups = 2;  // groups a lane of the multiply pass has in flight (4 and 8 need more registers: one workgroup per unit)
constexpr int kTpRedWG = 512;
constexpr int kTpRedGroups = 4;

__device__ __forceinline__ void load_vals4(const float* vals, int g, float (&v)[4]) {
    const f32x4 vv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(vals) + g);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = vv[i];
}
__device__ __forceinline__ void load_vals4(const uint16_t* vals, int g, float (&v)[4]) {
    const u32x2 vv = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(vals) + g);
    v[0] = __uint_as_float(vv[0] << 16);
    v[1] = __uint_as_float(vv[0] & 0xFFFF0000u);
    v[2] = __uint_as_float(vv[1] << 16);
    v[3] = __uint_as_float(vv[1] & 0xFFFF0000u);
}

// One workgroup per piece: groups [piece_g[i], piece_g[i+1]) of column block piece_c[i].
template <typename T, int U>
__global__ __launch_bounds__(kTpMulWG) void tp_multiply_kernel(const int32_t* __restrict__ piece_c,
                                                               const int32_t* __restrict__ piece_g,
                                                               const uint16_t* __restrict__ tp_col,
                                                               const typename T::elem* __restrict__ tp_val,
                                                               const int32_t* __restrict__ tp_dst,
                                                               const typename T::elem* __restrict__ x, int n, int shift,
                                                               float* __restrict__ prod) {
    extern __shared__ __align__(16) float xs[];  // 2^shift x values, then four zeros
    const int tid = threadIdx.x;
    // a column block's pieces on one die: its block of x then crosses the fabric once, not once per die
    const int piece = xcd_remap(blockIdx.x, gridDim.x);
    const int c = piece_c[piece];
    const int g0 = piece_g[piece], g1 = piece_g[piece + 1];
    const int width = 1 << shift;
    const int64_t first = static_cast<int64_t>(c) << shift;
    const int have = n - first < width ? static_cast<int>(n - first) : width;  // columns of this block that exist
    // the piece's first U groups per lane are asked for before the block of x, so that the two overlap
    u16x4 cc[U];
    float v[U][4];
    int d[U];
    auto fetch = [&](int gb) {
#pragma unroll
        for (int u = 0; u < U; ++u) {  // past the end: the piece's last group again, not stored
            const int g = gb + u * kTpMulWG < g1 ? gb + u * kTpMulWG : g1 - 1;
            cc[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x4*>(tp_col) + g);
            load_vals4(tp_val, g, v[u]);
            d[u] = __builtin_nontemporal_load(tp_dst + g);
        }
    };
    if (g0 < g1) fetch(g0 + tid);
    if (have == width && reinterpret_cast<uintptr_t>(x) % 16 == 0) {  // a whole block from an aligned x: 16 bytes per lane and trip
        if constexpr (sizeof(typename T::elem) == 4) {
            for (int i = 4 * tid; i < width; i += 4 * kTpMulWG)
                *reinterpret_cast<f32x4*>(xs + i) = *reinterpret_cast<const f32x4*>(x + first + i);
        } else {
            for (int i = 8 * tid; i < width; i += 8 * kTpMulWG) {
                const u32x4 b = *reinterpret_cast<const u32x4*>(x + first + i);
                f32x4 lo, hi;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    lo[2 * j] = __uint_as_float(b[j] << 16);
                    lo[2 * j + 1] = __uint_as_float(b[j] & 0xFFFF0000u);
                    hi[2 * j] = __uint_as_float(b[2 + j] << 16);
                    hi[2 * j + 1] = __uint_as_float(b[2 + j] & 0xFFFF0000u);
                }
                *reinterpret_cast<f32x4*>(xs + i) = lo;
                *reinterpret_cast<f32x4*>(xs + i + 4) = hi;
            }
        }
    } else {
        for (int i = tid; i < width; i += kTpMulWG) xs[i] = i < have ? widen(x[first + i]) : 0.f;
    }
    if (tid < 4) xs[width + tid] = 0.f;
    __syncthreads();
    for (int gb = g0 + tid; gb < g1; gb += U * kTpMulWG) {
        if (gb != g0 + tid) fetch(gb);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            f32x4 p;
#pragma unroll
            for (int i = 0; i < 4; ++i) p[i] = v[u][i] * xs[cc[u][i]];
            if (gb + u * kTpMulWG < g1) reinterpret_cast<f32x4*>(prod)[d[u]] = p;
        }
    }
}

struct TpReduceArgs {
    const int32_t* chunk_desc;  // [2*(P+1)] pairs (rows finished, entries taken) at each split
    const int32_t* chunk_g;     // [P+1] first group of each chunk's stretch of tp_pos / prod
    const uint16_t* tp_pos;
    const float* prod;
    const int32_t* rowptr;
    float* y;
    int32_t* carry_row;
    float* carry_val;
    int32_t nparts;
    float alpha, beta;
};

// One workgroup per chunk.  LDS: the chunk's products at their CSR positions, then the segment
// bounds, then the rows' old y.
template <int WG, int U>
__global__ __launch_bounds__(WG) void tp_reduce_kernel(const TpReduceArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int deferred[kMaxDeferred];
    __shared__ int n_deferred;
    const int tid = threadIdx.x;
    const int part = blockIdx.x;
    const int r0 = a.chunk_desc[2 * part];
    const int k0 = a.chunk_desc[2 * part + 1];
    const int nr = a.chunk_desc[2 * part + 2] - r0;
    const int k1 = a.chunk_desc[2 * part + 3];
    const int g0 = a.chunk_g[part], g1 = a.chunk_g[part + 1];
    const int ent = k1 - k0;
    const int nseg = nr + 1;
    float* vals_l = reinterpret_cast<float*>(smem_raw);
    int* seg = reinterpret_cast<int*>(vals_l + ((ent + 3) & ~3));
    float* y0_l = reinterpret_cast<float*>(seg + nseg + 1);

    auto bound = [&](int v) {
        v = v < k0 ? k0 : v;
        v = v > k1 ? k1 : v;
        return v - k0;
    };
    for (int i = tid; i <= nr; i += WG) seg[i] = bound(a.rowptr[r0 + i]);
    if (tid == 0) {
        seg[nseg] = ent;
        n_deferred = 0;
    }
    if (a.beta != 0.f)
        for (int i = tid; i < nr; i += WG) y0_l[i] = a.y[r0 + i];
    for (int gb = g0 + tid; gb < g1; gb += U * WG) {
        u16x4 pos[U];
        f32x4 pp[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = gb + u * WG < g1 ? gb + u * WG : g1 - 1;
            pos[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x4*>(a.tp_pos) + g);
            pp[u] = reinterpret_cast<const f32x4*>(a.prod)[g];  // written a moment ago: a plain load finds much of it still cached
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (gb + u * WG < g1) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (pos[u][i] != 0xFFFF) vals_l[pos[u][i]] = pp[u][i];
            }
    }
    __syncthreads();
    const RowOut o{a.y, y0_l, a.carry_row, a.carry_val, a.alpha, a.beta};
    tile_rows<true, WG>(static_cast<const NoGather*>(nullptr), vals_l, static_cast<const float*>(nullptr), seg, nr, r0, part,
                        ent, o, deferred, &n_deferred, tid);
}

// ---------------------------------------------------------------------------- analysis time
// key[k] = column block of entry k, idx[k] = k.
__global__ __launch_bounds__(kWG) void tp_keys_kernel(const int32_t* __restrict__ colidx, int nnz, int shift, int C,
                                                      uint16_t* __restrict__ key, uint32_t* __restrict__ idx) {
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; k < nnz; k += static_cast<int64_t>(gridDim.x) * kWG) {
        unsigned c = static_cast<unsigned>(colidx[k]) >> shift;
        if (c >= static_cast<unsigned>(C)) c = C - 1;  // only possible when the caller skipped validation
        key[k] = static_cast<uint16_t>(c);
        idx[k] = static_cast<uint32_t>(k);
    }
}

// chunk_at[k] = the chunk whose stretch of the entry list holds position k.  One workgroup per chunk.
__global__ __launch_bounds__(kWG) void tp_chunk_fill_kernel(const int32_t* __restrict__ chunk_desc, int32_t* __restrict__ chunk_at) {
    const int p = blockIdx.x;
    const int k1 = chunk_desc[2 * p + 3];
    for (int k = chunk_desc[2 * p + 1] + threadIdx.x; k < k1; k += kWG) chunk_at[k] = p;
}

// chunk_of[q] = chunk of the q-th entry in (column block, CSR position) order.
__global__ __launch_bounds__(kWG) void tp_chunk_of_kernel(const uint32_t* __restrict__ idx, int nnz, const int32_t* __restrict__ chunk_at,
                                                          int32_t* __restrict__ chunk_of) {
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; q < nnz; q += static_cast<int64_t>(gridDim.x) * kWG)
        chunk_of[q] = chunk_at[idx[q]];
}

// In that order the tile number c*P + p never decreases, so a tile is a run: first[t] = where it starts,
// last[t] = where it ends (both stay 0 for a tile without entries).  No counters, no atomics.
__global__ __launch_bounds__(kWG) void tp_runs_kernel(const uint16_t* __restrict__ key, const int32_t* __restrict__ chunk_of, int nnz,
                                                      int P, int32_t* __restrict__ first, int32_t* __restrict__ last) {
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; q < nnz; q += static_cast<int64_t>(gridDim.x) * kWG) {
        const int t = key[q] * P + chunk_of[q];
        const int before = q > 0 ? key[q - 1] * P + chunk_of[q - 1] : -1;
        const int after = q + 1 < nnz ? key[q + 1] * P + chunk_of[q + 1] : -1;
        if (t != before) first[t] = static_cast<int32_t>(q);
        if (t != after) last[t] = static_cast<int32_t>(q + 1);
    }
}

// padded[t] = the tile's entries rounded up to whole groups of four slots.
__global__ __launch_bounds__(kWG) void tp_pad_kernel(const int32_t* __restrict__ first, const int32_t* __restrict__ last, int T,
                                                     int32_t* __restrict__ padded) {
    for (int t = blockIdx.x * kWG + threadIdx.x; t < T; t += gridDim.x * kWG) padded[t] = (last[t] - first[t] + 3) & ~3;
}

// One lane per chunk p walks down its column of the (c, p) table: within[c*P + p] = slots of chunk p in the column
// blocks before c, in_chunk[p] = the chunk's slots (in_chunk[P] = 0 closes the list for the scan that follows).
__global__ __launch_bounds__(kWG) void tp_chunk_columns_kernel(const int32_t* __restrict__ padded, int C, int P,
                                                               int32_t* __restrict__ within, int32_t* __restrict__ in_chunk) {
    const int p = blockIdx.x * kWG + threadIdx.x;
    if (p > P) return;
    int run = 0;
    if (p < P)
        for (int c = 0; c < C; ++c) {
            const int64_t t = static_cast<int64_t>(c) * P + p;
            within[t] = run;
            run += padded[t];
        }
    in_chunk[p] = run;
}

// block_first[c] = first slot of column block c in the multiply order (block_first[C] = all slots);
// chunk_g[p] = first group of chunk p in the reduce order (chunk_g[P] = all groups).
__global__ __launch_bounds__(kWG) void tp_starts_kernel(const int32_t* __restrict__ base1, const int32_t* __restrict__ padded, int C,
                                                        int P, const int32_t* __restrict__ chunk_first,
                                                        int32_t* __restrict__ block_first, int32_t* __restrict__ chunk_g) {
    const int i = blockIdx.x * kWG + threadIdx.x;
    const int64_t T = static_cast<int64_t>(C) * P;
    if (i <= C) block_first[i] = i < C ? base1[static_cast<int64_t>(i) * P] : base1[T - 1] + padded[T - 1];
    if (i <= P) chunk_g[i] = chunk_first[i] >> 2;
}

struct TpPlaceArgs {
    const uint16_t* key;
    const uint32_t* idx;
    const int32_t* chunk_of;
    const int32_t* first;        // [C*P] where tile t starts in the sorted order (t = c*P + p)
    const int32_t* base1;        // [C*P] slots before tile t in (c, p) order
    const int32_t* within;       // [C*P] slots of t's chunk in the column blocks before t's
    const int32_t* chunk_first;  // [P+1] slots before each chunk in (p, c) order
    const int32_t* chunk_desc;
    const int32_t* colidx;
    const void* vals;
    int32_t nnz, P, shift, elem_bytes;
    uint16_t* tp_col;
    void* tp_val;
    int32_t* tp_src;
    int32_t* tp_dst;
    uint16_t* tp_pos;
};

__global__ __launch_bounds__(kWG) void tp_place_kernel(const TpPlaceArgs a) {
    for (int64_t q = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; q < a.nnz; q += static_cast<int64_t>(gridDim.x) * kWG) {
        const int k = static_cast<int>(a.idx[q]);
        const int c = a.key[q];
        const int p = a.chunk_of[q];
        const int64_t t = static_cast<int64_t>(c) * a.P + p;
        const int o = static_cast<int>(q) - a.first[t];
        const int s1 = a.base1[t] + o;
        const int s2 = a.chunk_first[p] + a.within[t] + o;
        a.tp_col[s1] = static_cast<uint16_t>(static_cast<unsigned>(a.colidx[k]) & ((1u << a.shift) - 1u));
        if (a.elem_bytes == 4) static_cast<float*>(a.tp_val)[s1] = static_cast<const float*>(a.vals)[k];
        else static_cast<uint16_t*>(a.tp_val)[s1] = static_cast<const uint16_t*>(a.vals)[k];
        a.tp_src[s1] = k;
        a.tp_pos[s2] = static_cast<uint16_t>(k - a.chunk_desc[2 * p + 1]);
        if ((o & 3) == 0) a.tp_dst[s1 >> 2] = s2 >> 2;
    }
}

template <typename E>
__global__ __launch_bounds__(kWG) void tp_values_kernel(const E* __restrict__ vals, const int32_t* __restrict__ tp_src,
                                                        E* __restrict__ tp_val, int slots) {
    for (int64_t s = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; s < slots; s += static_cast<int64_t>(gridDim.x) * kWG) {
        const int k = tp_src[s];
        if (k >= 0) tp_val[s] = vals[k];
    }
}

__global__ __launch_bounds__(kWG) void tp_fill16_kernel(uint16_t* __restrict__ p, int64_t count, uint16_t v) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; i < count; i += static_cast<int64_t>(gridDim.x) * kWG)
        p[i] = v;
}

int capped_grid(int64_t items) {
    const int64_t g = (items + kWG - 1) / kWG;
    return static_cast<int>(g > 8192 ? 8192 : (g < 1 ? 1 : g));
}

template <typename K>
hipError_t allow_lds(K kernel, size_t lds, size_t* allowed) {
    if (lds <= 64 * 1024 || lds <= *allowed) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(lds));
    if (e == hipSuccess) *allowed = lds;
    return e;
}

}  // namespace

size_t two_phase_reduce_lds(int32_t entries, int32_t rows) {
    return sizeof(float) * static_cast<size_t>((entries + 3) & ~3) + (sizeof(int) + sizeof(float)) * static_cast<size_t>(rows + 2);
}

hipError_t launch_two_phase(const TwoPhase& t, const MatrixView& A, const void* x, float* y, Scalars s, hipStream_t st) {
    const size_t lds1 = sizeof(float) * ((size_t{1} << t.shift) + 4);
    hipError_t e;
    if (t.num_pieces > 0) {
        if (A.bf16) {
            auto k = tp_multiply_kernel<BF16, kTpMulGroups>;
            static thread_local size_t allowed = 0;
            if ((e = allow_lds(k, lds1, &allowed)) != hipSuccess) return e;
            hipLaunchKernelGGL(k, dim3(t.num_pieces), dim3(kTpMulWG), lds1, st, t.piece_c, t.piece_g, t.tp_col,
                               static_cast<const uint16_t*>(t.tp_val), t.tp_dst, static_cast<const uint16_t*>(x), A.n, t.shift,
                               t.prod);
        } else {
            auto k = tp_multiply_kernel<F32, kTpMulGroups>;
            static thread_local size_t allowed = 0;
            if ((e = allow_lds(k, lds1, &allowed)) != hipSuccess) return e;
            hipLaunchKernelGGL(k, dim3(t.num_pieces), dim3(kTpMulWG), lds1, st, t.piece_c, t.piece_g, t.tp_col,
                               static_cast<const float*>(t.tp_val), t.tp_dst, static_cast<const float*>(x), A.n, t.shift, t.prod);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const TpReduceArgs a{t.chunk_desc, t.chunk_g, t.tp_pos, t.prod, A.rowptr, y, t.carry_row, t.carry_val, t.num_chunks,
                         s.alpha,      s.beta};
    auto k = tp_reduce_kernel<kTpRedWG, kTpRedGroups>;
    static thread_local size_t allowed = 0;
    if ((e = allow_lds(k, t.reduce_lds, &allowed)) != hipSuccess) return e;
    hipLaunchKernelGGL(k, dim3(t.num_chunks), dim3(kTpRedWG), t.reduce_lds, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    return launch_merge_fixup(t.carry_row, t.carry_val, t.num_chunks, y, s.alpha, st);
}

size_t two_phase_sort_bytes(int32_t nnz, int bits) {
    size_t bytes = 0;
    if (rocprim::radix_sort_pairs(nullptr, bytes, static_cast<const uint16_t*>(nullptr), static_cast<uint16_t*>(nullptr),
                                  static_cast<const uint32_t*>(nullptr), static_cast<uint32_t*>(nullptr),
                                  static_cast<size_t>(nnz), 0, bits, nullptr) != hipSuccess)
        return 0;
    return bytes < 16 ? 16 : bytes;
}

hipError_t launch_two_phase_sort(const MatrixView& A, int shift, int C, int bits, void* temp, size_t temp_bytes,
                                 uint16_t* key_in, uint16_t* key_out, uint32_t* idx_in, uint32_t* idx_out, hipStream_t st) {
    hipLaunchKernelGGL(tp_keys_kernel, dim3(capped_grid(A.nnz)), dim3(kWG), 0, st, A.colidx, A.nnz, shift, C, key_in, idx_in);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // a stable sort by column block alone: the CSR positions stay ascending inside a block, and
    // with them the chunks
    return rocprim::radix_sort_pairs(temp, temp_bytes, key_in, key_out, idx_in, idx_out, static_cast<size_t>(A.nnz), 0, bits,
                                     st);
}

size_t two_phase_scan_bytes(int64_t tiles) {
    size_t bytes = 0;
    if (rocprim::exclusive_scan(nullptr, bytes, static_cast<const int32_t*>(nullptr), static_cast<int32_t*>(nullptr), int32_t{0},
                                static_cast<size_t>(tiles), rocprim::plus<int32_t>(), nullptr) != hipSuccess)
        return 0;
    return bytes < 16 ? 16 : bytes;
}

hipError_t launch_two_phase_tables(const TwoPhaseTables& w, const uint16_t* key, const uint32_t* idx, int32_t nnz,
                                   const int32_t* chunk_desc, int32_t C, int32_t P, void* temp, size_t temp_bytes,
                                   int32_t* chunk_g, hipStream_t st) {
    const int64_t T = static_cast<int64_t>(C) * P;
    hipError_t e;
    if ((e = hipMemsetAsync(w.first, 0, sizeof(int32_t) * T, st)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(w.last, 0, sizeof(int32_t) * T, st)) != hipSuccess) return e;
    hipLaunchKernelGGL(tp_chunk_fill_kernel, dim3(P), dim3(kWG), 0, st, chunk_desc, w.chunk_at);
    hipLaunchKernelGGL(tp_chunk_of_kernel, dim3(capped_grid(nnz)), dim3(kWG), 0, st, idx, nnz, w.chunk_at, w.chunk_of);
    hipLaunchKernelGGL(tp_runs_kernel, dim3(capped_grid(nnz)), dim3(kWG), 0, st, key, w.chunk_of, nnz, P, w.first, w.last);
    hipLaunchKernelGGL(tp_pad_kernel, dim3(capped_grid(T)), dim3(kWG), 0, st, w.first, w.last, static_cast<int>(T), w.padded);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    size_t bytes = temp_bytes;
    if ((e = rocprim::exclusive_scan(temp, bytes, w.padded, w.base1, int32_t{0}, static_cast<size_t>(T), rocprim::plus<int32_t>(),
                                     st)) != hipSuccess)
        return e;
    hipLaunchKernelGGL(tp_chunk_columns_kernel, dim3(ceil_div(P + 1, kWG)), dim3(kWG), 0, st, w.padded, C, P, w.within, w.in_chunk);
    bytes = temp_bytes;
    if ((e = rocprim::exclusive_scan(temp, bytes, w.in_chunk, w.chunk_first, int32_t{0}, static_cast<size_t>(P) + 1,
                                     rocprim::plus<int32_t>(), st)) != hipSuccess)
        return e;
    hipLaunchKernelGGL(tp_starts_kernel, dim3(ceil_div((C > P ? C : P) + 1, kWG)), dim3(kWG), 0, st, w.base1, w.padded, C, P,
                       w.chunk_first, w.block_first, chunk_g);
    return hipGetLastError();
}

hipError_t launch_two_phase_place(const MatrixView& A, int shift, int32_t P, const uint16_t* key, const uint32_t* idx,
                                  const TwoPhaseTables& w, const int32_t* chunk_desc, int64_t slots, uint16_t* tp_col, void* tp_val,
                                  int32_t* tp_src, int32_t* tp_dst, uint16_t* tp_pos, hipStream_t st) {
    // padding first: column = the zero slot after the x block, value 0, no source, position "dropped"
    hipLaunchKernelGGL(tp_fill16_kernel, dim3(capped_grid(slots)), dim3(kWG), 0, st, tp_col, slots,
                       static_cast<uint16_t>(1u << shift));
    hipLaunchKernelGGL(tp_fill16_kernel, dim3(capped_grid(slots)), dim3(kWG), 0, st, tp_pos, slots, static_cast<uint16_t>(0xFFFF));
    hipError_t e = hipMemsetAsync(tp_val, 0, static_cast<size_t>(slots) * (A.bf16 ? 2 : 4), st);
    if (e != hipSuccess) return e;
    if ((e = hipMemsetAsync(tp_src, 0xFF, static_cast<size_t>(slots) * 4, st)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(tp_dst, 0, static_cast<size_t>(slots), st)) != hipSuccess) return e;
    const TpPlaceArgs a{key, idx, w.chunk_of, w.first, w.base1, w.within, w.chunk_first, chunk_desc, A.colidx, A.vals, A.nnz,
                        P,   shift, A.bf16 ? 2 : 4, tp_col, tp_val, tp_src, tp_dst, tp_pos};
    hipLaunchKernelGGL(tp_place_kernel, dim3(capped_grid(A.nnz)), dim3(kWG), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_two_phase_values(const MatrixView& A, const int32_t* tp_src, void* tp_val, int64_t slots, hipStream_t st) {
    if (slots <= 0) return hipSuccess;
    if (A.bf16)
        hipLaunchKernelGGL(tp_values_kernel<uint16_t>, dim3(capped_grid(slots)), dim3(kWG), 0, st,
                           static_cast<const uint16_t*>(A.vals), tp_src, static_cast<uint16_t*>(tp_val), static_cast<int>(slots));
    else
        hipLaunchKernelGGL(tp_values_kernel<float>, dim3(capped_grid(slots)), dim3(kWG), 0, st, static_cast<const float*>(A.vals),
                           tp_src, static_cast<float*>(tp_val), static_cast<int>(slots));
    return hipGetLastError();
}

}  // namespace spmv
