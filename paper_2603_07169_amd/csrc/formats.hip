// gfx950 kernels for y <- alpha*A*x + beta*y with A in COO, CSC and ELL storage (paper App. C
// tasks 8, 10, 14).
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "kernels.h"
#include "row_phase.h"

namespace spmv {
namespace {

constexpr int kCscLdsRows = 16384;  // CSC: up to this many rows a workgroup keeps a private y in LDS (64 KB)

// ------------------------------------------------------------------------------------------
// y <- alpha*A*x + beta*y for A in the other storage layouts of the benchmark (App. C tasks 8,
// 10, 14).  ELL rows are independent and are reduced like CSR rows.  COO and CSC entries arrive
// grouped by nothing (COO) or by column (CSC), so their contributions are added to y with
// hardware float atomics after y has been scaled by beta in a kernel of its own; sums therefore
// depend on the order in which the atomics land (results agree to rounding, not bit for bit).
__global__ __launch_bounds__(kWG) void scale_y_kernel(float* __restrict__ y, int m, float beta) {
    for (int i = blockIdx.x * kWG + threadIdx.x; i < m; i += gridDim.x * kWG) y[i] = beta == 0.f ? 0.f : beta * y[i];
}

// Four consecutive entries per lane and trip.  A lane first sums the runs of equal row numbers
// among its own four; runs that lie wholly inside go to y with one hardware float atomic each.
// Its last run (its only one, if all four rows agree) may go on in the next lanes and its first may
// continue the previous lane's: those are joined across the wavefront with a segmented scan over
// the lanes' last-run sums, so a row held by consecutive entries (the whole row, for row-sorted
// input) costs one atomic per wavefront it touches instead of one per entry.
// shift: the arrays are read in aligned groups of four starting `shift` (0..3) entries before
// `row`; vec: those groups may be fetched with one 16-byte (8-byte for bf16 values) load each.
template <typename T>
__global__ __launch_bounds__(kWG) void spmv_coo_kernel(const int32_t* __restrict__ row, const int32_t* __restrict__ col,
                                                       const typename T::elem* __restrict__ vals,
                                                       const typename T::elem* __restrict__ x, float* y, int nnz,
                                                       int shift, int vec, float alpha) {
    using E = typename T::elem;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x) >> 6;
    const int64_t n_waves = (static_cast<int64_t>(gridDim.x) * kWG) >> 6;
    const int64_t n_groups = (static_cast<int64_t>(nnz) + shift + 3) / 4;
    for (int64_t gbase = wave * 64; gbase < n_groups; gbase += n_waves * 64) {  // the same trip count for all lanes of a wavefront
        const int64_t e0_64 = 4 * (gbase + lane) - shift;  // first of this lane's four entries; < 0 or >= nnz: none
        int r[4];
        float p[4];
        if (vec && e0_64 >= 0 && e0_64 + 3 < nnz) {
            const int e0 = static_cast<int>(e0_64);
            const i32x4 rv = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(row + e0));
            const i32x4 cv = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(col + e0));
            float v[4];
            if constexpr (sizeof(E) == 4) {
                const f32x4 vv = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(vals + e0));
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = vv[i];
            } else {
                typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
                const u32x2 vv = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(vals + e0));
                v[0] = __uint_as_float(vv[0] << 16);
                v[1] = __uint_as_float(vv[0] & 0xFFFF0000u);
                v[2] = __uint_as_float(vv[1] << 16);
                v[3] = __uint_as_float(vv[1] & 0xFFFF0000u);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                r[i] = rv[i];
                p[i] = alpha * (v[i] * widen(x[cv[i]]));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t e = e0_64 + i;
                const bool live = e >= 0 && e < nnz;
                r[i] = live ? row[e] : -1;
                p[i] = live ? alpha * (widen(vals[e]) * widen(x[col[e]])) : 0.f;
            }
        }
        // runs inside the lane: the first is kept as the head, the last as the tail, others go out at once
        const int head_row = r[0];
        float head_sum = 0.f;
        bool single = true;  // no row change seen yet: the run in hand is still the first
        int tail_row = r[0];
        float tail_sum = p[0];
#pragma unroll
        for (int i = 1; i < 4; ++i) {
            if (r[i] != tail_row) {
                if (single) {
                    head_sum = tail_sum;
                    single = false;
                } else if (tail_row >= 0) {
                    unsafeAtomicAdd(y + tail_row, tail_sum);
                }
                tail_row = r[i];
                tail_sum = p[i];
            } else {
                tail_sum += p[i];
            }
        }
        // chains of last runs: a lane joins the chain of the lane before it when all its entries have that lane's last row
        const int prev_tail_row = __shfl_up(tail_row, 1, 64);
        const int next_head_row = __shfl_down(head_row, 1, 64);
        const bool follows = lane > 0 && head_row == prev_tail_row;
        float chain = tail_sum;
        bool head = !(single && follows);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const float cc = __shfl_up(chain, d, 64);
            const int hh = __shfl_up(static_cast<int>(head), d, 64);
            if (lane >= d && !head) {
                chain += cc;
                head = hh != 0;
            }
        }
        const float chain_before = __shfl_up(chain, 1, 64);
        if (!single && head_row >= 0) unsafeAtomicAdd(y + head_row, follows ? head_sum + chain_before : head_sum);
        if (tail_row >= 0 && (lane == 63 || next_head_row != tail_row)) unsafeAtomicAdd(y + tail_row, chain);
    }
}

// A team of G lanes per column: its entries all multiply the same x[j] and go to different rows.
template <typename T, int G>
__global__ __launch_bounds__(kWG) void spmv_csc_kernel(const int32_t* __restrict__ col_offsets,
                                                       const int32_t* __restrict__ row,
                                                       const typename T::elem* __restrict__ vals,
                                                       const typename T::elem* __restrict__ x, float* y, int n, float alpha) {
    const int64_t j64 = (static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x) / G;
    const int tl = threadIdx.x % G;
    if (j64 >= n) return;
    const int j = static_cast<int>(j64);
    const float xj = alpha * widen(x[j]);
    const int e1 = col_offsets[j + 1];
    for (int e = col_offsets[j] + tl; e < e1; e += G) unsafeAtomicAdd(y + row[e], widen(vals[e]) * xj);
}

// The same for matrices with few rows, where the atomics of thousands of columns would queue up
// on the same few addresses of y: a workgroup adds its columns into a private copy of y in LDS
// and sends every row's total to memory once.  Few workgroups, so few atomics per address.
// gridDim.y workgroups share a stretch of columns, each with its own stretch of the rows.
constexpr int kCscLdsWG = 512;      // lanes of a workgroup of spmv_csc_lds_kernel
constexpr int kCscLdsBlocks = 128;  // most workgroups it is launched with
template <typename T, int G>
__global__ __launch_bounds__(kCscLdsWG) void spmv_csc_lds_kernel(const int32_t* __restrict__ col_offsets,
                                                           const int32_t* __restrict__ row,
                                                           const typename T::elem* __restrict__ vals,
                                                           const typename T::elem* __restrict__ x, float* y, int m, int n,
                                                           float alpha) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float* ly = reinterpret_cast<float*>(smem_raw);  // [hi - lo]
    // blockIdx.y: the stretch of rows this workgroup adds up; entries of other rows are read and passed over
    const int lo = static_cast<int>(static_cast<int64_t>(m) * blockIdx.y / gridDim.y);
    const int hi = static_cast<int>(static_cast<int64_t>(m) * (blockIdx.y + 1) / gridDim.y);
    for (int i = threadIdx.x; i < hi - lo; i += kCscLdsWG) ly[i] = 0.f;
    __syncthreads();
    const int tl = threadIdx.x % G;
    for (int j = (blockIdx.x * kCscLdsWG + threadIdx.x) / G; j < n; j += gridDim.x * (kCscLdsWG / G)) {
        const float xj = alpha * widen(x[j]);
        const int e1 = col_offsets[j + 1];
        for (int e = col_offsets[j] + tl; e < e1; e += G) {
            const int r = row[e];
            if (r >= lo && r < hi) atomicAdd(ly + (r - lo), widen(vals[e]) * xj);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < hi - lo; i += kCscLdsWG) {
        const float v = ly[i];
        if (v != 0.f) unsafeAtomicAdd(y + lo + i, v);
    }
}

// A team of G lanes per row of `width` slots; a slot with col_id -1 is padding.
template <typename T, int G>
__global__ __launch_bounds__(kWG) void spmv_ell_kernel(const int32_t* __restrict__ col_ids,
                                                       const typename T::elem* __restrict__ vals,
                                                       const typename T::elem* __restrict__ x, float* y, int m, int width,
                                                       float alpha, float beta) {
    // m * G can pass 2^32 lanes: 64-bit lane number
    const int64_t i64 = (static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x) / G;
    const int tl = threadIdx.x % G;
    const bool live = i64 < m;
    const int i = static_cast<int>(i64);
    float acc = 0.f;
    if (live) {
        const size_t base = static_cast<size_t>(i) * width;
        for (int s = tl; s < width; s += G) {
            const int c = col_ids[base + s];
            if (c >= 0) acc += widen(vals[base + s]) * widen(x[c]);
        }
    }
    acc = group_sum<G>(acc);  // every lane of the wavefront takes part
    if (live && tl == 0) y[i] = epilogue(acc, alpha, beta, y, i);
}


// ELL rows of moderate width, the CSR tile kernel's way: a workgroup copies the slots of a run of
// rows (a contiguous stretch of col_ids / vals, since the layout is row-major) to LDS with 128-bit
// non-temporal loads, turning padding slots into (column 0, value 0) on the way, and then runs the
// shared row phase on them, rows being segments of equal length `width`.  Against a team of lanes
// reading its row straight from memory this keeps the global reads fully coalesced whatever the
// width, and issues the x gathers with neighbouring lanes on neighbouring rows.
// rows_per_tile is a multiple of 8, so a tile's first slot is 16-byte aligned in both arrays.
template <typename T>
__global__ __launch_bounds__(kWG, 8) void spmv_ell_tile_kernel(const int32_t* __restrict__ col_ids,
                                                               const typename T::elem* __restrict__ vals,
                                                               const typename T::elem* __restrict__ x, float* y, int m,
                                                               int width, int rows_per_tile, float alpha, float beta,
                                                               int vec_ok) {
    using E = typename T::elem;
    constexpr int VEC = T::VEC;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int deferred[kMaxDeferred];
    __shared__ int n_deferred;
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * rows_per_tile;
    const int nr = m - r0 < rows_per_tile ? m - r0 : rows_per_tile;
    const size_t k0 = static_cast<size_t>(r0) * width;
    const int span = nr * width;
    const int slots = (span + VEC - 1) & ~(VEC - 1);
    int* cols_l = reinterpret_cast<int*>(smem_raw);
    E* vals_l = reinterpret_cast<E*>(smem_raw + sizeof(int) * slots);
    int* seg = reinterpret_cast<int*>(smem_raw + (sizeof(int) + sizeof(E)) * slots);  // nr + 1 bounds
    float* y0_l = reinterpret_cast<float*>(seg + nr + 1);                             // nr old values of y

    const float y0v = (beta != 0.f && tid < nr) ? y[r0 + tid] : 0.f;
    const int whole = vec_ok ? span & ~(VEC - 1) : 0;  // slots of the tile that whole vectors cover
    for (int off = tid * VEC; off < whole; off += kWG * VEC) {
        i32x4 c[VEC / 4];
#pragma unroll
        for (int v = 0; v < VEC / 4; ++v)
            c[v] = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(col_ids + k0 + off) + v);
        if constexpr (VEC == 4) {
            f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(vals + k0 + off));
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = c[0][i] < 0 ? 0.f : a[i];
                c[0][i] = c[0][i] < 0 ? 0 : c[0][i];
            }
            *reinterpret_cast<f32x4*>(vals_l + off) = a;
            *reinterpret_cast<i32x4*>(cols_l + off) = c[0];
        } else {
            u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vals + k0 + off));
#pragma unroll
            for (int i = 0; i < 4; ++i) {  // dword i holds elements 2i (low half) and 2i+1
                const int lo = c[i / 2][2 * (i % 2)], hi = c[i / 2][2 * (i % 2) + 1];
                a[i] &= (lo < 0 ? 0xFFFF0000u : 0xFFFFFFFFu) & (hi < 0 ? 0x0000FFFFu : 0xFFFFFFFFu);
            }
#pragma unroll
            for (int v = 0; v < 2; ++v)
#pragma unroll
                for (int i = 0; i < 4; ++i) c[v][i] = c[v][i] < 0 ? 0 : c[v][i];
            *reinterpret_cast<u32x4*>(vals_l + off) = a;
            *reinterpret_cast<i32x4*>(cols_l + off) = c[0];
            *reinterpret_cast<i32x4*>(cols_l + off + 4) = c[1];
        }
    }
    for (int off = whole + tid; off < span; off += kWG) {  // what no whole vector covers (everything, if unaligned)
        const int c = col_ids[k0 + off];
        cols_l[off] = c < 0 ? 0 : c;
        vals_l[off] = c < 0 ? E(0) : vals[k0 + off];
    }
    if (tid == 0) n_deferred = 0;
    for (int i = tid; i <= nr; i += kWG) seg[i] = i * width;
    if (tid < nr) y0_l[tid] = y0v;
    if (beta != 0.f)
        for (int i = tid + kWG; i < nr; i += kWG) y0_l[i] = y[r0 + i];
    __syncthreads();

    const RowOut o{y, y0_l, nullptr, nullptr, alpha, beta};
    tile_rows<false, kWG>(cols_l, vals_l, x, seg, nr, r0, 0, span, o, deferred, &n_deferred, tid);
}

}  // namespace

namespace {

int lanes_for_length(int64_t len) {  // smallest power of two G in [2, 64] with 8*G >= len
    int G = 2;
    while (G < 64 && 8 * G < len) G <<= 1;
    return G;
}

template <typename T>
hipError_t launch_coo_t(int32_t m, int32_t nnz, const int32_t* row, const int32_t* col, const void* vals, const void* x,
                        float* y, Scalars s, hipStream_t st) {
    using E = typename T::elem;
    int grid = ceil_div(m, kWG);
    hipLaunchKernelGGL(scale_y_kernel, dim3(grid > 2048 ? 2048 : grid), dim3(kWG), 0, st, y, m, s.beta);
    if (nnz > 0) {
        // the caller's arrays start where they start: whole-vector loads only if all three are aligned as they are
        const bool vec = reinterpret_cast<uintptr_t>(row) % 16 == 0 && reinterpret_cast<uintptr_t>(col) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(vals) % (4 * sizeof(E)) == 0;
        grid = ceil_div(nnz, 4 * kWG);
        hipLaunchKernelGGL((spmv_coo_kernel<T>), dim3(grid > 8192 ? 8192 : grid), dim3(kWG), 0, st, row, col,
                           static_cast<const E*>(vals), static_cast<const E*>(x), y, nnz, 0, vec ? 1 : 0, s.alpha);
    }
    return hipGetLastError();
}

template <typename T, int G>
hipError_t launch_csc_tg(int32_t m, int32_t n, int32_t nnz, const int32_t* col_offsets, const int32_t* row, const void* vals,
                         const void* x, float* y, Scalars s, hipStream_t st) {
    using E = typename T::elem;
    const int grid = ceil_div(m, kWG);
    hipLaunchKernelGGL(scale_y_kernel, dim3(grid > 2048 ? 2048 : grid), dim3(kWG), 0, st, y, m, s.beta);
    if (n <= 0) return hipGetLastError();
    const int blocks = ceil_div(static_cast<int64_t>(n) * G, kWG);
    if (m <= kCscLdsRows) {
        // A private y per workgroup.  A compute unit retires one LDS float atomic every 1.3 ns whatever the workgroup's
        // size (integer ones every 0.5 ns), so the time to add the entries falls with the number of workgroups, while each
        // workgroup sends one global atomic per row at the end: measured 57 / 31 / 18 / 13 / 15 us with 16 / 32 / 64 / 128 /
        // 256 workgroups on the benchmark's 2048 x 32768 shape (256, 512 or 1024 lanes each: the same).  Up to 2^20 entries
        // entries in columns of eight or more, a second workgroup per stretch of columns takes the other half of the rows:
        // both read every entry of the stretch, each adds half of them, and no row gets more atomics than before
        // (13 -> 10.5 us; with 1.3 entries per column the walk over the columns is what takes the time, and doubling it
        // costs 13.5 -> 15.4 us).
        const int lds_blocks = ceil_div(static_cast<int64_t>(n) * G, kCscLdsWG);
        const int col_blocks = lds_blocks > kCscLdsBlocks ? kCscLdsBlocks : lds_blocks;
        const int parts = (nnz <= (1 << 20) && nnz >= 8 * static_cast<int64_t>(n) && m >= 2) ? 2 : 1;
        hipLaunchKernelGGL((spmv_csc_lds_kernel<T, G>), dim3(col_blocks, parts), dim3(kCscLdsWG), sizeof(float) * (m / parts + 1), st,
                           col_offsets, row, static_cast<const E*>(vals), static_cast<const E*>(x), y, m, n, s.alpha);
    } else {
        hipLaunchKernelGGL((spmv_csc_kernel<T, G>), dim3(blocks), dim3(kWG), 0, st, col_offsets, row,
                           static_cast<const E*>(vals), static_cast<const E*>(x), y, n, s.alpha);
    }
    return hipGetLastError();
}

template <typename T, int G>
hipError_t launch_ell_tg(int32_t m, int32_t width, const int32_t* col_ids, const void* vals, const void* x, float* y,
                         Scalars s, hipStream_t st) {
    using E = typename T::elem;
    hipLaunchKernelGGL((spmv_ell_kernel<T, G>), dim3(ceil_div(static_cast<int64_t>(m) * G, kWG)), dim3(kWG), 0, st,
                       col_ids, static_cast<const E*>(vals), static_cast<const E*>(x), y, m, width, s.alpha, s.beta);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_scale_y(float* y, int32_t m, float beta, hipStream_t st) {
    if (m <= 0) return hipSuccess;
    const int grid = ceil_div(m, kWG);
    hipLaunchKernelGGL(scale_y_kernel, dim3(grid > 2048 ? 2048 : grid), dim3(kWG), 0, st, y, m, beta);
    return hipGetLastError();
}

hipError_t launch_coo_accumulate(bool bf16, int32_t nnz, const int32_t* row, const int32_t* col, const void* vals,
                                 const void* x, float* y, float alpha, hipStream_t st) {
    if (nnz <= 0) return hipSuccess;
    // The arrays are stretches of the library's own allocations, all three starting the same number of
    // entries into theirs: the (up to three) entries before `row` that complete its first aligned
    // group of four may be read, and are ignored.
    const int shift = static_cast<int>((reinterpret_cast<uintptr_t>(row) / 4) % 4);
    const size_t esz = bf16 ? 2 : 4;
    const bool vec = (reinterpret_cast<uintptr_t>(row) - 4 * shift) % 16 == 0 &&
                     (reinterpret_cast<uintptr_t>(col) - 4 * shift) % 16 == 0 &&
                     (reinterpret_cast<uintptr_t>(vals) - esz * shift) % (4 * esz) == 0;
    int grid = ceil_div(static_cast<int64_t>(nnz) + shift, 4 * kWG);
    if (grid > 8192) grid = 8192;
    if (bf16)
        hipLaunchKernelGGL((spmv_coo_kernel<BF16>), dim3(grid), dim3(kWG), 0, st, row, col, static_cast<const uint16_t*>(vals),
                           static_cast<const uint16_t*>(x), y, nnz, vec ? shift : 0, vec ? 1 : 0, alpha);
    else
        hipLaunchKernelGGL((spmv_coo_kernel<F32>), dim3(grid), dim3(kWG), 0, st, row, col, static_cast<const float*>(vals),
                           static_cast<const float*>(x), y, nnz, vec ? shift : 0, vec ? 1 : 0, alpha);
    return hipGetLastError();
}

hipError_t launch_coo(bool bf16, int32_t m, int32_t nnz, const int32_t* row, const int32_t* col, const void* vals,
                      const void* x, float* y, Scalars s, hipStream_t st) {
    if (m <= 0) return hipSuccess;
    return bf16 ? launch_coo_t<BF16>(m, nnz, row, col, vals, x, y, s, st)
                : launch_coo_t<F32>(m, nnz, row, col, vals, x, y, s, st);
}

hipError_t launch_csc(bool bf16, int32_t m, int32_t n, int32_t nnz, const int32_t* col_offsets, const int32_t* row,
                      const void* vals, const void* x, float* y, Scalars s, hipStream_t st) {
    if (m <= 0) return hipSuccess;
#define SPMV_CSC_CASE(G) \
    case G: return bf16 ? launch_csc_tg<BF16, G>(m, n, nnz, col_offsets, row, vals, x, y, s, st) \
                        : launch_csc_tg<F32, G>(m, n, nnz, col_offsets, row, vals, x, y, s, st);
    switch (lanes_for_length(n > 0 ? (nnz + n - 1) / n : 0)) {
        SPMV_CSC_CASE(2) SPMV_CSC_CASE(4) SPMV_CSC_CASE(8) SPMV_CSC_CASE(16) SPMV_CSC_CASE(32) SPMV_CSC_CASE(64)
    }
#undef SPMV_CSC_CASE
    return hipErrorInvalidValue;
}

namespace {

constexpr int kEllTileSlots = 4096;    // most slots a workgroup of the ELL tile kernel stages
constexpr int kEllTileMaxWidth = 64;  // widest rows that kernel is used for

template <typename T>
hipError_t launch_ell_tile(int32_t m, int32_t width, const int32_t* col_ids, const void* vals, const void* x, float* y,
                           Scalars s, hipStream_t st) {
    using E = typename T::elem;
    int rows = kEllTileSlots / width;
    rows = rows > kWG ? kWG : rows & ~7;
    const bool vec_ok = reinterpret_cast<uintptr_t>(col_ids) % 16 == 0 && reinterpret_cast<uintptr_t>(vals) % 16 == 0;
    const size_t lds = (sizeof(int) + sizeof(E)) * static_cast<size_t>(rows * width + T::VEC) +
                       (sizeof(int) + sizeof(float)) * static_cast<size_t>(rows + 2);
    hipLaunchKernelGGL((spmv_ell_tile_kernel<T>), dim3(ceil_div(m, rows)), dim3(kWG), lds, st, col_ids,
                       static_cast<const E*>(vals), static_cast<const E*>(x), y, m, width, rows, s.alpha, s.beta,
                       vec_ok ? 1 : 0);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ell(bool bf16, int32_t m, int32_t width, const int32_t* col_ids, const void* vals, const void* x,
                      float* y, Scalars s, hipStream_t st) {
    if (m <= 0) return hipSuccess;
    // Rows of up to 64 slots go through LDS: read directly they would get teams of at most 8 lanes,
    // whose loads fall into many short pieces.  Wider rows get teams of 16 to 64 lanes, which read
    // 64 to 256 contiguous bytes at a time as it is (measured: width 390, 2048 rows: 3.9 us direct
    // against 5.0 us through LDS; width 27, 2 M rows: 114 us against 85 us).
    if (width >= 1 && width <= kEllTileMaxWidth)
        return bf16 ? launch_ell_tile<BF16>(m, width, col_ids, vals, x, y, s, st)
                    : launch_ell_tile<F32>(m, width, col_ids, vals, x, y, s, st);
#define SPMV_ELL_CASE(G) \
    case G: return bf16 ? launch_ell_tg<BF16, G>(m, width, col_ids, vals, x, y, s, st) \
                        : launch_ell_tg<F32, G>(m, width, col_ids, vals, x, y, s, st);
    switch (lanes_for_length(width)) {
        SPMV_ELL_CASE(2) SPMV_ELL_CASE(4) SPMV_ELL_CASE(8) SPMV_ELL_CASE(16) SPMV_ELL_CASE(32) SPMV_ELL_CASE(64)
    }
#undef SPMV_ELL_CASE
    return hipErrorInvalidValue;
}

}  // namespace spmv
