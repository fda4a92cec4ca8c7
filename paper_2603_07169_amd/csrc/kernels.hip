// gfx950 kernels for y <- alpha*A*x + beta*y with A in CSR (values / col_indices / row_offsets,
// paper App. C task 12), FP32 or bf16 storage, FP32 products and sums.
//
// SpMV moves 8 (FP32) or 6 (bf16) bytes per stored entry for 2 flops, so every kernel is built
// around reading vals/colidx exactly once, as wide and as coalesced as the row layout allows:
//   spmv_scalar_kernel  one lane per row                     (short rows; the naive baseline)
//   spmv_vector_kernel  G = 2..64 lanes per row, DPP/ds_swizzle/permlane reduction
//   spmv_tile_kernel    a workgroup copies a contiguous entry range (a row block, or a merge-path
//                       chunk whose cut-off tail leaves as a carry) to LDS with 128-bit loads and
//                       lets teams of lanes take one row each, gathering x through the caches
//   spmv_window_kernel  the same with the block's window of x in LDS and 16-bit window positions
//                       in place of the column indices (built by window_build_kernel at analysis)
//   merge_fixup_kernel  adds the carries of cut rows to y, in chunk order, without atomics
// No matrix cores: nothing here is a dense contraction.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "device_common.h"
#include "kernels.h"
#include "row_phase.h"

namespace spmv {
namespace {

// ------------------------------------------------------------------------------------------
// 128-bit streaming loads.  vals/colidx are read once: mark them non-temporal so they do not
// push x out of the caches.
__device__ __forceinline__ i32x4 load_idx4(const int32_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(p));
}
__device__ __forceinline__ f32x4 load_val4(const float* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
}
__device__ __forceinline__ u32x4 load_val8(const uint16_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// Products of VEC consecutive entries starting at k (k multiple of VEC, k + VEC <= nnz, arrays
// 16-byte aligned).
__device__ __forceinline__ void products_vec(const int32_t* colidx, const float* vals, const float* x, int k,
                                             float (&p)[4], int /*n*/, bool /*x_group_ok*/) {
    const f32x4 v = load_val4(vals + k);
    const i32x4 c = load_idx4(colidx + k);
    p[0] = v[0] * x[c[0]];
    p[1] = v[1] * x[c[1]];
    p[2] = v[2] * x[c[2]];
    p[3] = v[3] * x[c[3]];
}
// bf16: the eight x operands often sit together (a run of consecutive columns).  One aligned
// 16-byte load fetches the 8-column group around the first column; columns inside that group
// are served from registers, the others are gathered one by one, and a gather instruction is
// skipped altogether when no lane of the wavefront needs it.  x_group_ok: x is 16-byte aligned.
__device__ __forceinline__ void products_vec(const int32_t* colidx, const uint16_t* vals, const uint16_t* x, int k,
                                             float (&p)[8], int n, bool x_group_ok) {
    const u32x4 v = load_val8(vals + k);
    const i32x4 c0 = load_idx4(colidx + k);
    const i32x4 c1 = load_idx4(colidx + k + 4);
    const int c[8] = {c0[0], c0[1], c0[2], c0[3], c1[0], c1[1], c1[2], c1[3]};
    const int g = c[0] & ~7;
    const bool group = x_group_ok && g + 8 <= n;
    u32x4 w = {0u, 0u, 0u, 0u};
    if (group) w = *reinterpret_cast<const u32x4*>(x + g);
    unsigned lone[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        lone[i] = 0;
        if (!(group && static_cast<unsigned>(c[i] - g) < 8u)) lone[i] = x[c[i]];
    }
    float xs[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned d = static_cast<unsigned>(c[i] - g);
        if (group && d < 8u) {
            const unsigned word = (d & 4u) ? ((d & 2u) ? w[3] : w[2]) : ((d & 2u) ? w[1] : w[0]);
            xs[i] = __uint_as_float((d & 1u) ? (word & 0xFFFF0000u) : (word << 16));
        } else {
            xs[i] = __uint_as_float(lone[i] << 16);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // little-endian: the low half of dword i is entry 2i, the high half entry 2i+1
        p[2 * i] = __uint_as_float(v[i] << 16) * xs[2 * i];
        p[2 * i + 1] = __uint_as_float(v[i] & 0xFFFF0000u) * xs[2 * i + 1];
    }
}

template <typename E>
__device__ __forceinline__ float product_one(const int32_t* colidx, const E* vals, const E* x, int k) {
    return widen(vals[k]) * widen(x[colidx[k]]);
}

// Partial dot product of entries [k0, k1) taken by lane `lane` of a team of G lanes.
// Long enough ranges are split into an unaligned head (< VEC entries), an aligned body read
// with 128-bit loads, and a tail (< VEC entries).
template <typename T, int G>
__device__ __forceinline__ float team_dot(const int32_t* colidx, const typename T::elem* vals,
                                          const typename T::elem* x, int k0, int k1, int lane, bool vec_ok, int n,
                                          bool x_group_ok) {
    constexpr int VEC = T::VEC;
    float acc = 0.f;
    if constexpr (G >= 16) {
        if (vec_ok && k1 - k0 >= 2 * VEC) {
            const int ka = (k0 + VEC - 1) & ~(VEC - 1);
            if (k0 + lane < ka) acc += product_one(colidx, vals, x, k0 + lane);
            const int nvec = (k1 - ka) / VEC;
            for (int v = lane; v < nvec; v += G) {
                float p[VEC];
                products_vec(colidx, vals, x, ka + v * VEC, p, n, x_group_ok);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc += p[i];
            }
            const int kt = ka + nvec * VEC;
            if (kt + lane < k1) acc += product_one(colidx, vals, x, kt + lane);
            return acc;
        }
    }
    for (int k = k0 + lane; k < k1; k += G) acc += product_one(colidx, vals, x, k);
    return acc;
}

// ------------------------------------------------------------------------------------------
// One lane per row.
template <typename T>
__global__ __launch_bounds__(kWG) void spmv_scalar_kernel(const int32_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ colidx,
                                                          const typename T::elem* __restrict__ vals,
                                                          const typename T::elem* __restrict__ x, float* y,
                                                          const int32_t* __restrict__ rows, int count, float alpha,
                                                          float beta) {
    const int i = blockIdx.x * kWG + threadIdx.x;
    if (i >= count) return;
    const int r = rows ? rows[i] : i;
    const int k1 = rowptr[r + 1];
    float acc = 0.f;
    for (int k = rowptr[r]; k < k1; ++k) acc += product_one(colidx, vals, x, k);
    y[r] = epilogue(acc, alpha, beta, y, r);
}

// G lanes per row.
template <typename T, int G>
__global__ __launch_bounds__(kWG) void spmv_vector_kernel(const int32_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ colidx,
                                                          const typename T::elem* __restrict__ vals,
                                                          const typename T::elem* __restrict__ x, float* y,
                                                          const int32_t* __restrict__ rows, int count, float alpha,
                                                          float beta, int vec_ok, int n, int x_group_ok) {
    const int team = static_cast<int>((static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x) / G);
    const int lane = threadIdx.x % G;
    const bool live = team < count;
    int r = 0, k0 = 0, k1 = 0;
    if (live) {
        r = rows ? rows[team] : team;
        k0 = rowptr[r];
        k1 = rowptr[r + 1];
    }
    float acc = team_dot<T, G>(colidx, vals, x, k0, k1, lane, vec_ok != 0, n, x_group_ok != 0);
    acc = group_sum<G>(acc);  // every lane of the wave takes part, also those without a row
    if (live && lane == 0) y[r] = epilogue(acc, alpha, beta, y, r);
}

// ------------------------------------------------------------------------------------------
struct TileArgs {
    // what a workgroup needs before its first vector load comes first, in one stretch
    int32_t nparts, x_cap, tile_cap, nnz;
    const int32_t* xv_pad;     // window kernel: [nparts * x_cap] first element of each 16-byte x vector of a block, -1 padded
    const uint16_t* lidx8;     // window kernel, grouped positions: [nnz/8] lidx[8g], the first of every aligned group of eight
    const uint16_t* lidx;      // window kernel: [nnz, padded to a multiple of 8] position of each entry's x value in the block's window
    const int32_t* run_desc;   // pattern kernel: [8 * nparts] the runs of every row block (packed; word 7 = number of runs, 0: no pattern)
    const uint16_t* pat_pad;   // pattern kernel: [nparts * pt_cap] the blocks' pattern lists at a fixed stride
    int32_t pt_cap;            // pattern kernel: entries per block in pat_pad (a multiple of 8)
    const int32_t* part_desc;  // [2*(nparts+1)] pairs (row, entry): first row and first entry of each row block, or rows
                               // finished and entries taken at each merge-path split
    const int32_t* rowptr;
    const void* vals;
    const void* x;
    float* y;
    int32_t n, m;
    float alpha, beta;
    int32_t vec_ok;            // colidx and vals are 16-byte aligned
    int32_t x_vec_ok;          // x is 16-byte aligned
    const int32_t* colidx;
    int32_t* carry_row;        // merge path only, [nparts]
    float* carry_val;          // merge path only, [nparts]
};

// A single row longer than a tile: the whole workgroup strides over it.
template <typename T, int WG>
__device__ __forceinline__ void long_row(const TileArgs& a, int r, int k0, int k1, float* wave_part, int tid) {
    using E = typename T::elem;
    float acc = team_dot<T, WG>(a.colidx, static_cast<const E*>(a.vals), static_cast<const E*>(a.x), k0, k1, tid,
                                a.vec_ok != 0, a.n, reinterpret_cast<uintptr_t>(a.x) % 16 == 0);
    acc = group_sum<64>(acc);
    if ((tid & 63) == 0) wave_part[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) {
        float s = wave_part[0];
        for (int w = 1; w < WG / 64; ++w) s += wave_part[w];
        a.y[r] = epilogue(s, a.alpha, a.beta, a.y, r);
    }
}

// One workgroup per tile.  A tile is a contiguous entry range [k0, k1) together with the rows
// r0 .. r0+nr-1 whose last entry lies in it, plus (merge path only) the leading piece of row
// r0+nr that the range cuts off, which leaves as a carry.
//   1. The tile's slice of colidx/vals is copied to LDS as it is, with 128-bit loads from an
//      aligned origin (element-wise when the arrays are not 16-byte aligned, and for the last
//      few entries of the array that no whole vector covers).  The bounds of the tile's
//      segments, relative to that origin, go to LDS as well.
//   2. Teams of G lanes (G from the tile's mean row length) take one row each, read its
//      entries back from LDS, gather x and accumulate; a DPP/swizzle reduction closes the
//      row.  Rows far longer than the mean are set aside and taken by whole wavefronts.
// Streaming the matrix through LDS keeps its global reads perfectly coalesced while the x
// gathers are issued row-wise, where neighbouring lanes touch neighbouring columns.
template <typename T, bool MERGE, int WG>
__global__ __launch_bounds__(WG, 8) void spmv_tile_kernel(const TileArgs a) {
    using E = typename T::elem;
    constexpr int VEC = T::VEC;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int deferred[kMaxDeferred];
    __shared__ int n_deferred;
    __shared__ float wave_part[WG / 64];

    const int tid = threadIdx.x;
    const int part = xcd_remap(blockIdx.x, a.nparts);
    const E* vals = static_cast<const E*>(a.vals);
    const E* x = static_cast<const E*>(a.x);

    const int r0 = a.part_desc[2 * part];  // one 16-byte scalar load: (r0, k0, r1, k1)
    const int k0 = a.part_desc[2 * part + 1];
    const int nr = a.part_desc[2 * part + 2] - r0;
    const int k1 = a.part_desc[2 * part + 3];

    if constexpr (!MERGE) {
        if (k1 - k0 > a.tile_cap) {
            long_row<T, WG>(a, r0, k0, k1, wave_part, tid);
            return;
        }
    }

    const int nseg = nr + (MERGE ? 1 : 0);
    const int k0a = k0 & ~(VEC - 1);
    const int span = k1 - k0a;
    const int slots = (span + VEC - 1) & ~(VEC - 1);  // whole vectors are stored
    int* cols_l = reinterpret_cast<int*>(smem_raw);
    E* vals_l = reinterpret_cast<E*>(smem_raw + sizeof(int) * slots);
    int* seg = reinterpret_cast<int*>(smem_raw + (sizeof(int) + sizeof(E)) * slots);  // nseg + 1 entries

    float* y0_l = reinterpret_cast<float*>(seg + nseg + 1);  // nr entries

    // row bounds and (beta != 0) old y of the first WG rows: issued ahead of the entry stream,
    // stored to LDS after it, so that neither costs a memory round trip of its own
    const int rp0 = a.rowptr[r0 + (tid < nr ? tid : nr)];
    const int rp_nr = MERGE ? a.rowptr[r0 + nr] : k1;  // same address in every lane; row blocks end at k1
    const float* const y_src = (a.beta != 0.f && tid < nr) ? a.y + r0 + tid : reinterpret_cast<const float*>(a.rowptr);
    const float y0v = *y_src;
    auto clamp_bound = [&](int v) {
        v = v < k0 ? k0 : v;
        v = v > k1 ? k1 : v;
        return v - k0a;
    };

    // ---- 1. stage the tile's entries: two vectors per lane and trip, all loads before any store
    if (a.vec_ok) {
        const int nnz_vec = a.nnz & ~(VEC - 1);  // entries reachable by whole vectors
        for (int off0 = tid * VEC; off0 < span; off0 += 2 * WG * VEC) {
            const int off1 = off0 + WG * VEC;
            const int kA = k0a + off0, kB = k0a + off1;
            const bool vecA = kA < nnz_vec;
            const bool vecB = off1 < span && kB < nnz_vec;
            if constexpr (VEC == 4) {
                f32x4 vA, vB;
                i32x4 cA, cB;
                if (vecA) {
                    vA = load_val4(reinterpret_cast<const float*>(vals) + kA);
                    cA = load_idx4(a.colidx + kA);
                }
                if (vecB) {
                    vB = load_val4(reinterpret_cast<const float*>(vals) + kB);
                    cB = load_idx4(a.colidx + kB);
                }
                if (vecA) {
                    *reinterpret_cast<f32x4*>(vals_l + off0) = vA;
                    *reinterpret_cast<i32x4*>(cols_l + off0) = cA;
                }
                if (vecB) {
                    *reinterpret_cast<f32x4*>(vals_l + off1) = vB;
                    *reinterpret_cast<i32x4*>(cols_l + off1) = cB;
                }
            } else {
                u32x4 vA, vB;
                i32x4 cA, cA2, cB, cB2;
                if (vecA) {
                    vA = load_val8(reinterpret_cast<const uint16_t*>(vals) + kA);
                    cA = load_idx4(a.colidx + kA);
                    cA2 = load_idx4(a.colidx + kA + 4);
                }
                if (vecB) {
                    vB = load_val8(reinterpret_cast<const uint16_t*>(vals) + kB);
                    cB = load_idx4(a.colidx + kB);
                    cB2 = load_idx4(a.colidx + kB + 4);
                }
                if (vecA) {
                    *reinterpret_cast<u32x4*>(vals_l + off0) = vA;
                    *reinterpret_cast<i32x4*>(cols_l + off0) = cA;
                    *reinterpret_cast<i32x4*>(cols_l + off0 + 4) = cA2;
                }
                if (vecB) {
                    *reinterpret_cast<u32x4*>(vals_l + off1) = vB;
                    *reinterpret_cast<i32x4*>(cols_l + off1) = cB;
                    *reinterpret_cast<i32x4*>(cols_l + off1 + 4) = cB2;
                }
            }
            // the last few entries of the array that no whole vector covers
            if (!vecA)
                for (int i = 0; i < VEC; ++i)
                    if (kA + i < a.nnz) {
                        vals_l[off0 + i] = vals[kA + i];
                        cols_l[off0 + i] = a.colidx[kA + i];
                    }
            if (!vecB && off1 < span)
                for (int i = 0; i < VEC; ++i)
                    if (kB + i < a.nnz) {
                        vals_l[off1 + i] = vals[kB + i];
                        cols_l[off1 + i] = a.colidx[kB + i];
                    }
        }
    } else {
        for (int off = (k0 - k0a) + tid; off < span; off += WG) {
            vals_l[off] = vals[k0a + off];
            cols_l[off] = a.colidx[k0a + off];
        }
    }
    if (tid == 0) n_deferred = 0;
    if (tid < nr) seg[tid] = clamp_bound(rp0);
    if (tid == 0) seg[nr] = clamp_bound(rp_nr);
    if (tid < nr) y0_l[tid] = y0v;
    for (int i = tid + WG; i < nr; i += WG) seg[i] = clamp_bound(a.rowptr[r0 + i]);
    if (a.beta != 0.f)
        for (int i = tid + WG; i < nr; i += WG) y0_l[i] = a.y[r0 + i];
    if (MERGE && tid == 0) seg[nseg] = k1 - k0a;
    __syncthreads();

    // ---- 2. rows
    const RowOut o{a.y, y0_l, a.carry_row, a.carry_val, a.alpha, a.beta};
    tile_rows<MERGE, WG>(cols_l, vals_l, x, seg, nr, r0, part, k1 - k0, o, deferred, &n_deferred, tid);
}

// First elements of the x vectors a lane fetches for block `part` (-1: none; lanes from x_cap on read the start of lidx
// instead and must not use what they get).  after: 0, possibly obtained from a value the loads are to follow.
template <int WG, int XPL>
__device__ __forceinline__ void load_x_addresses(const TileArgs& a, int part, int tid, int after, int (&xs)[XPL]) {
#pragma unroll
    for (int u = 0; u < XPL; ++u) {
        const int i = tid + u * WG;
        const int32_t* src = i < a.x_cap ? a.xv_pad + part * a.x_cap + i + after : reinterpret_cast<const int32_t*>(a.lidx);
        xs[u] = *src;  // a lane beyond x_cap holds something else than an address: the users test i < x_cap first
    }
}

// Row blocks with x served from LDS.  The analysis has listed, for every row block, the
// distinct aligned 16-byte vectors of x that its entries touch (xv_pad: one fixed-size slice per
// block, so a lane knows where its vector's address is before any descriptor has arrived) and
// has replaced each entry's 32-bit column by a 16-bit position in that list (lidx).  A workgroup
//   1. copies its block's x vectors to LDS (one 128-bit load per vector, coalesced wherever
//      the block's columns are contiguous) together with the block's slice of vals and lidx,
//   2. runs the same row phase as the tile kernel, every operand now coming out of LDS.
// Per entry the matrix stream shrinks from value + 4 bytes to value + 2 bytes, and the row
// phase issues no global load at all.  A block that is one over-long row takes the global path.
// XPL: x vectors a lane fetches (x_cap <= XPL*WG); NG: 8-entry groups a lane stages in the
// first, branch-free round (blocks of up to NG*WG*8 - 7 entries need no second round).
// GROUPED: the analysis found every aligned group of eight entries at eight consecutive window
// positions (rows made of aligned runs of columns): one 16-bit position per group is read instead
// of eight, and the other seven are counted up from it.
// One row block of the window kernel.  xs: with XPL == 1 the x vector addresses, already requested by the caller
// (they need only the block number, so they go out before the block's descriptor has arrived); with larger windows
// the x gathers that follow them keep the address units busy for long, and measured best when they start after the
// entry stream has been requested, so there the addresses are fetched here, with the stream.
template <typename T, int WG, int XPL, int NG, bool GROUPED>
__device__ __forceinline__ void window_block(const TileArgs& a, int part, int (&xs)[XPL]) {
    using E = typename T::elem;
    constexpr int XE = 16 / sizeof(E);  // elements per x vector
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int deferred[kMaxDeferred];
    __shared__ int n_deferred;
    __shared__ float wave_part[WG / 64];

    const int tid = threadIdx.x;
    const E* vals = static_cast<const E*>(a.vals);
    const E* x = static_cast<const E*>(a.x);
    const uint16_t* const dummy = a.lidx;

    const int r0 = a.part_desc[2 * part];  // one 16-byte scalar load: (r0, k0, r1, k1)
    const int k0 = a.part_desc[2 * part + 1];
    const int nr = a.part_desc[2 * part + 2] - r0;
    const int k1 = a.part_desc[2 * part + 3];
    // A block that is one over-long row stages nothing (span 0) and is taken from global memory
    // after the barrier: no branch stands between the kernel's start and its loads.
    const bool long_block = k1 - k0 > a.tile_cap;

    const int k0a = k0 & ~7;  // lidx vectors hold 8 entries
    const int span = long_block ? 0 : k1 - k0a;
    const int slots = (span + 7) & ~7;
    E* xbuf = reinterpret_cast<E*>(smem_raw);  // x_cap vectors
    E* vals_l = reinterpret_cast<E*>(smem_raw + 16 * a.x_cap);
    uint16_t* lidx_l = reinterpret_cast<uint16_t*>(smem_raw + 16 * a.x_cap + sizeof(E) * slots);
    int* seg = reinterpret_cast<int*>(smem_raw + 16 * a.x_cap + (sizeof(E) + sizeof(uint16_t)) * slots);  // nr + 1
    float* y0_l = reinterpret_cast<float*>(seg + nr + 1);                                                   // nr

    // Every load of the common path below is unconditional, in straight-line code: a lane with
    // nothing to fetch reads the start of lidx instead (always allocated, 16-byte aligned, at
    // least 16 bytes).  Without branches around the loads the compiler can wait for the oldest
    // loads only, so the order of issue is also the order of use:
    //   x vector addresses -> row bounds -> entry stream -> x vectors (need the addresses)
    //   -> LDS stores of the stream (while the x vectors are in flight) -> LDS stores of x.
    if constexpr (XPL > 1) {
        // a zero the compiler cannot see through, produced from the descriptor: the address loads
        // then really wait for it instead of being scheduled back to the top
        int zero;
        asm volatile("s_mov_b32 %0, 0" : "=s"(zero) : "s"(k1));
        load_x_addresses<WG, XPL>(a, part, tid, zero, xs);
    }
    const int rp0 = a.rowptr[r0 + (tid < nr ? tid : nr)];  // bound nr is k1: no load needed for it
    const float* const y_src = (a.beta != 0.f && tid < nr) ? a.y + r0 + tid : reinterpret_cast<const float*>(dummy);
    const float y0v = *y_src;

    // A group is 8 consecutive entries: one 128-bit vector of lidx, one (bf16) or two (binary32)
    // of vals.  Groups that reach past the last whole vector of the arrays, and everything when
    // vals is not 16-byte aligned, are copied element by element afterwards.
    struct Group {
        u32x4 v0, v1, l;
        bool live, vec;
    };
    const int nnz_vec = a.vec_ok ? a.nnz & ~7 : 0;
    auto load_group = [&](int off, Group& g) {
        const int k = k0a + off;
        g.live = off < span;
        g.vec = g.live && k < nnz_vec;
        const uint16_t* vp = g.vec ? reinterpret_cast<const uint16_t*>(vals + k) : dummy;
        const uint16_t* lp = g.vec ? a.lidx + k : dummy;
        g.v0 = load_val8(vp);
        if constexpr (sizeof(E) == 4) g.v1 = load_val8(g.vec ? vp + 8 : dummy);
        if constexpr (GROUPED) {
            const unsigned both = static_cast<unsigned>(*(g.vec ? a.lidx8 + (k >> 3) : dummy)) * 0x10001u;  // the position in both halves
            g.l = u32x4{both + 0x00010000u, both + 0x00030002u, both + 0x00050004u, both + 0x00070006u};
        } else {
            g.l = load_val8(lp);
        }
    };
    auto store_group = [&](int off, const Group& g) {
        if (g.vec) {
            *reinterpret_cast<u32x4*>(vals_l + off) = g.v0;
            if constexpr (sizeof(E) == 4) *reinterpret_cast<u32x4*>(vals_l + off + 4) = g.v1;
            *reinterpret_cast<u32x4*>(lidx_l + off) = g.l;
        } else if (g.live) {
            const int k = k0a + off;
            for (int i = 0; i < 8; ++i)
                if (k + i >= k0 && k + i < k1) {
                    vals_l[off + i] = vals[k + i];
                    lidx_l[off + i] = a.lidx[k + i];
                }
        }
    };

    Group g[NG];
#pragma unroll
    for (int u = 0; u < NG; ++u) load_group((tid + u * WG) * 8, g[u]);

    // the instruction scheduler must not pull the address arithmetic of the x vectors (and the
    // wait for xs that it needs) ahead of the stream loads
    __builtin_amdgcn_sched_barrier(0);
    u32x4 xv[XPL];
    bool xvec[XPL];
#pragma unroll
    for (int u = 0; u < XPL; ++u) {
        xs[u] = tid + u * WG < a.x_cap ? xs[u] : -1;
        xvec[u] = xs[u] >= 0 && a.x_vec_ok && xs[u] + XE <= a.n;
        const E* src = xvec[u] ? x + xs[u] : reinterpret_cast<const E*>(dummy);
        xv[u] = *reinterpret_cast<const u32x4*>(src);
    }

    __builtin_amdgcn_sched_barrier(0);
    if (tid == 0) n_deferred = 0;
    if (tid < nr) seg[tid] = rp0 - k0a;
    if (tid == 0) seg[nr] = k1 - k0a;
    if (tid < nr) y0_l[tid] = y0v;
#pragma unroll
    for (int u = 0; u < NG; ++u) store_group((tid + u * WG) * 8, g[u]);
#pragma unroll
    for (int u = 0; u < XPL; ++u) {
        const int i = tid + u * WG;
        if (xvec[u]) {
            *reinterpret_cast<u32x4*>(xbuf + i * XE) = xv[u];
        } else if (xs[u] >= 0) {
            for (int e = 0; e < XE; ++e) xbuf[i * XE + e] = xs[u] + e < a.n ? x[xs[u] + e] : E(0);
        }
    }
    // what the fixed-size first round did not cover (blocks of more than WG rows or NG*WG*8 entries)
    for (int i = tid + WG; i < nr; i += WG) seg[i] = a.rowptr[r0 + i] - k0a;
    if (a.beta != 0.f)
        for (int i = tid + WG; i < nr; i += WG) y0_l[i] = a.y[r0 + i];
    for (int off = (tid + NG * WG) * 8; off < span; off += WG * 8) {
        Group h;
        load_group(off, h);
        store_group(off, h);
    }
    __syncthreads();

    // ---- 2. rows
    if (long_block) {
        long_row<T, WG>(a, r0, k0, k1, wave_part, tid);
        return;
    }
    const RowOut o{a.y, y0_l, a.carry_row, a.carry_val, a.alpha, a.beta};
    tile_rows<false, WG>(lidx_l, vals_l, xbuf, seg, nr, r0, part, k1 - k0, o, deferred, &n_deferred, tid);
}

template <typename T, int WG, int XPL, int NG, bool GROUPED>
__global__ __launch_bounds__(WG, (XPL == 4 && NG == 2) ? 4 : 8) void spmv_window_kernel(const TileArgs a) {
    const int part = xcd_remap(blockIdx.x, a.nparts);
    int xs[XPL];
    if constexpr (XPL == 1) load_x_addresses<WG, XPL>(a, part, threadIdx.x, 0, xs);
    window_block<T, WG, XPL, NG, GROUPED>(a, part, xs);
}

// The window kernel for matrices whose window positions follow row patterns (stencils).  The analysis has cut the
// rows of a block into at most four runs; inside a run every row has the same number of entries, and the window
// position of its j-th entry is  base + (row's place in the run) * stride + pat[j]  (run_desc: eight words per block,
// one scalar load; pat_pad: the blocks' pattern lists, a few dozen 16-bit numbers each, at a fixed stride).  Such a block
// is served without its position stream and without its row offsets: what is read per entry is the value alone.
// A block without a pattern (word 7 of its descriptor is 0) is taken by window_block as it is.
// Packing of run_desc: words 0-1 the runs' row counts, words 3-4 their bases, words 5-6 their strides (signed), 16 bits
// each; word 2 their row lengths, 8 bits each.
template <int G, typename E>
__device__ __forceinline__ float pattern_dot(const E* vals, const E* xbuf, const uint16_t* pat, int slot, int pos0, int len,
                                             int tl) {
    // the lane's entries j = tl, tl + G, ..: four at a time, then two, then one
    float acc = 0.f;
    int cnt = (len - tl + G - 1) / G;
    vals += slot + tl;
    pat += tl;
    auto batch = [&](auto B_) {
        constexpr int B = decltype(B_)::value;
        unsigned c[B];
        E xv[B], av[B];
#pragma unroll
        for (int u = 0; u < B; ++u) c[u] = static_cast<unsigned>(pos0) + pat[u * G];
#pragma unroll
        for (int u = 0; u < B; ++u) xv[u] = xbuf[c[u]];
#pragma unroll
        for (int u = 0; u < B; ++u) av[u] = vals[u * G];
#pragma unroll
        for (int u = 0; u < B; ++u) acc += widen(av[u]) * widen(xv[u]);
        vals += B * G;
        pat += B * G;
        cnt -= B;
    };
    while (cnt >= 4) batch(std::integral_constant<int, 4>{});
    if (cnt >= 2) batch(std::integral_constant<int, 2>{});
    if (cnt >= 1) batch(std::integral_constant<int, 1>{});
    return acc;
}

struct RunTable {
    int n;          // runs in the block, 1..4
    int cut[3];     // rows before run 1, 2, 3 (INT_MAX for a run that does not exist)
    int len[4];     // entries per row
    int slot[4];    // staged slot of entry 0 of row `row` of the block = slot[r] + row * len[r]
    int pos[4];     // window position of that entry = pos[r] + row * stride[r]
    int stride[4];
    int tab[4];     // where the run's pattern starts in the block's list
};

template <int WG, int G, typename E>
__device__ __forceinline__ void pattern_rows_g(const E* vals_l, const E* xbuf, const uint16_t* pat_l, const float* y0_l,
                                               const RunTable& rt, int nr, int r0, float* y, float alpha, float beta, int tid) {
    constexpr int teams = WG / G;
    const int team = tid / G, tl = tid % G;
    for (int first = 0; first < nr; first += teams) {
        const int row = first + team;
        int len = rt.len[0], slot = rt.slot[0], pos = rt.pos[0], stride = rt.stride[0], tab = rt.tab[0];
        if (rt.n > 1) {  // uniform over the workgroup
#pragma unroll
            for (int r = 1; r < 4; ++r) {
                const bool in = row >= rt.cut[r - 1];
                len = in ? rt.len[r] : len;
                slot = in ? rt.slot[r] : slot;
                pos = in ? rt.pos[r] : pos;
                stride = in ? rt.stride[r] : stride;
                tab = in ? rt.tab[r] : tab;
            }
        }
        const bool live = row < nr;
        len = live ? len : 0;
        float acc = pattern_dot<G>(vals_l, xbuf, pat_l + tab, slot + row * len, pos + row * stride, len, tl);
        acc = group_sum<G>(acc);  // every lane takes part
        if (live && tl == 0) y[r0 + row] = epilogue(acc, alpha, beta, y0_l, row);
    }
}

template <typename T, int WG, int XPL, int NG>
__device__ __forceinline__ void pattern_block(const TileArgs& a, int part, int (&xs)[XPL], const int32_t* rd, int r0, int k0,
                                              int r1, int k1) {
    using E = typename T::elem;
    constexpr int XE = 16 / sizeof(E);
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int tid = threadIdx.x;
    const E* vals = static_cast<const E*>(a.vals);
    const E* x = static_cast<const E*>(a.x);
    const uint16_t* const dummy = a.lidx;

    // the block's pattern list needs only the block number
    const int pt_vecs = a.pt_cap >> 3;
    const uint16_t* const pt_src = tid < pt_vecs ? a.pat_pad + static_cast<int64_t>(part) * a.pt_cap + 8 * tid : dummy;
    const u32x4 ptab = *reinterpret_cast<const u32x4*>(pt_src);

    const int nr = r1 - r0;
    if constexpr (XPL > 1) {
        int zero;
        asm volatile("s_mov_b32 %0, 0" : "=s"(zero) : "s"(k1));
        load_x_addresses<WG, XPL>(a, part, tid, zero, xs);
    }
    const float* const y_src = (a.beta != 0.f && tid < nr) ? a.y + r0 + tid : reinterpret_cast<const float*>(dummy);
    const float y0v = *y_src;

    const int k0a = k0 & ~7;
    const int span = k1 - k0a;
    const int slots = (span + 7) & ~7;
    E* xbuf = reinterpret_cast<E*>(smem_raw);
    E* vals_l = reinterpret_cast<E*>(smem_raw + 16 * a.x_cap);
    uint16_t* pat_l = reinterpret_cast<uint16_t*>(smem_raw + 16 * a.x_cap + sizeof(E) * slots);
    float* y0_l = reinterpret_cast<float*>(smem_raw + 16 * a.x_cap + sizeof(E) * slots + 2 * a.pt_cap);

    // the entry stream is the values alone: groups of eight, all loads unconditional (see window_block)
    struct Group {
        u32x4 v0, v1;
        bool live, vec;
    };
    const int nnz_vec = a.vec_ok ? a.nnz & ~7 : 0;
    auto load_group = [&](int off, Group& g) {
        const int k = k0a + off;
        g.live = off < span;
        g.vec = g.live && k < nnz_vec;
        const uint16_t* vp = g.vec ? reinterpret_cast<const uint16_t*>(vals + k) : dummy;
        g.v0 = load_val8(vp);
        if constexpr (sizeof(E) == 4) g.v1 = load_val8(g.vec ? vp + 8 : dummy);
    };
    auto store_group = [&](int off, const Group& g) {
        if (g.vec) {
            *reinterpret_cast<u32x4*>(vals_l + off) = g.v0;
            if constexpr (sizeof(E) == 4) *reinterpret_cast<u32x4*>(vals_l + off + 4) = g.v1;
        } else if (g.live) {
            const int k = k0a + off;
            for (int i = 0; i < 8; ++i)
                if (k + i >= k0 && k + i < k1) vals_l[off + i] = vals[k + i];
        }
    };
    Group g[NG];
#pragma unroll
    for (int u = 0; u < NG; ++u) load_group((tid + u * WG) * 8, g[u]);

    __builtin_amdgcn_sched_barrier(0);
    u32x4 xv[XPL];
    bool xvec[XPL];
#pragma unroll
    for (int u = 0; u < XPL; ++u) {
        xs[u] = tid + u * WG < a.x_cap ? xs[u] : -1;
        xvec[u] = xs[u] >= 0 && a.x_vec_ok && xs[u] + XE <= a.n;
        const E* src = xvec[u] ? x + xs[u] : reinterpret_cast<const E*>(dummy);
        xv[u] = *reinterpret_cast<const u32x4*>(src);
    }
    __builtin_amdgcn_sched_barrier(0);

    // the runs, unpacked with scalar arithmetic while the loads are in flight
    RunTable rt;
    rt.n = rd[7];
    const int rows[4] = {rd[0] & 0xFFFF, static_cast<int>(static_cast<unsigned>(rd[0]) >> 16), rd[1] & 0xFFFF,
                         static_cast<int>(static_cast<unsigned>(rd[1]) >> 16)};
    const int base[4] = {rd[3] & 0xFFFF, static_cast<int>(static_cast<unsigned>(rd[3]) >> 16), rd[4] & 0xFFFF,
                         static_cast<int>(static_cast<unsigned>(rd[4]) >> 16)};
    const int stride[4] = {static_cast<int16_t>(rd[5] & 0xFFFF), rd[5] >> 16, static_cast<int16_t>(rd[6] & 0xFFFF), rd[6] >> 16};
    int row_first = 0, entry_first = k0 - k0a, tab = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int len = (rd[2] >> (8 * r)) & 0xFF;
        rt.len[r] = len;
        rt.slot[r] = entry_first - row_first * len;
        rt.pos[r] = base[r] - row_first * stride[r];
        rt.stride[r] = stride[r];
        rt.tab[r] = tab;
        row_first += rows[r];
        entry_first += rows[r] * len;
        tab += len;
        if (r < 3) rt.cut[r] = r + 1 < rt.n ? row_first : 0x7FFFFFFF;
    }

    if (tid < pt_vecs) *reinterpret_cast<u32x4*>(pat_l + 8 * tid) = ptab;
    if (tid < nr) y0_l[tid] = y0v;
#pragma unroll
    for (int u = 0; u < NG; ++u) store_group((tid + u * WG) * 8, g[u]);
#pragma unroll
    for (int u = 0; u < XPL; ++u) {
        const int i = tid + u * WG;
        if (xvec[u]) {
            *reinterpret_cast<u32x4*>(xbuf + i * XE) = xv[u];
        } else if (xs[u] >= 0) {
            for (int e = 0; e < XE; ++e) xbuf[i * XE + e] = xs[u] + e < a.n ? x[xs[u] + e] : E(0);
        }
    }
    // what the fixed-size first round did not cover (blocks of more than WG rows or NG*WG*8 entries)
    if (a.beta != 0.f)
        for (int i = tid + WG; i < nr; i += WG) y0_l[i] = a.y[r0 + i];
    for (int off = (tid + NG * WG) * 8; off < span; off += WG * 8) {
        Group h;
        load_group(off, h);
        store_group(off, h);
    }
    __syncthreads();

    // Lanes per row: as many as fill the workgroup in one sweep over the block's rows (what is in LDS is then taken by
    // the most lanes at once: measured 35 us on the 27-point stencil with two lanes for each of its 128 rows, 58 us
    // with one, 38 us with four), but at least four entries for every lane.
    const int tile_nnz = k1 - k0;
    int G = 1;
    while (G < 16 && 2 * G * nr <= WG && 8 * G * nr <= tile_nnz) G <<= 1;
    switch (G) {
        case 1: pattern_rows_g<WG, 1>(vals_l, xbuf, pat_l, y0_l, rt, nr, r0, a.y, a.alpha, a.beta, tid); break;
        case 2: pattern_rows_g<WG, 2>(vals_l, xbuf, pat_l, y0_l, rt, nr, r0, a.y, a.alpha, a.beta, tid); break;
        case 4: pattern_rows_g<WG, 4>(vals_l, xbuf, pat_l, y0_l, rt, nr, r0, a.y, a.alpha, a.beta, tid); break;
        case 8: pattern_rows_g<WG, 8>(vals_l, xbuf, pat_l, y0_l, rt, nr, r0, a.y, a.alpha, a.beta, tid); break;
        default: pattern_rows_g<WG, 16>(vals_l, xbuf, pat_l, y0_l, rt, nr, r0, a.y, a.alpha, a.beta, tid); break;
    }
}

template <typename T, int WG, int XPL, int NG>
__global__ __launch_bounds__(WG, (XPL == 4 && NG == 2) ? 4 : 8) void spmv_pattern_kernel(const TileArgs a) {
    const int part = xcd_remap(blockIdx.x, a.nparts);
    int xs[XPL];
    if constexpr (XPL == 1) load_x_addresses<WG, XPL>(a, part, threadIdx.x, 0, xs);
    const int32_t* rd = a.run_desc + 8 * static_cast<int64_t>(part);
    const int runs = rd[7];
    const int r0 = a.part_desc[2 * part], k0 = a.part_desc[2 * part + 1];  // with the runs: one wait for both scalar loads
    const int r1 = a.part_desc[2 * part + 2], k1 = a.part_desc[2 * part + 3];
    if (runs == 0)
        window_block<T, WG, XPL, NG, false>(a, part, xs);
    else
        pattern_block<T, WG, XPL, NG>(a, part, xs, rd, r0, k0, r1, k1);
}

// Builds the x windows of row blocks (one workgroup of 256 lanes per block; analysis time).
// keys = colidx >> shift of the block's entries.  Where they span few enough values, a bitmap in LDS gives the
// distinct keys and every key's rank without sorting; otherwise the keys (those that repeat their predecessor's are left out
// at once) are sorted in LDS (bitonic network over the next power of two) and duplicates dropped.  count pass (fill == 0): nv[b] = number of distinct keys.
// fill pass: xv_start[xv_ptr[b] + j] = xv_pad[b * x_cap + j] = j-th key << shift (the rest of the
// block's xv_pad slice is -1), and for every entry
// lidx[k] = rank of its key * 2^shift + colidx[k] mod 2^shift.  A block with more than tile_cap
// entries (one over-long row) gets nv = 0 and lidx = 0.  The fill pass is only launched when
// every nv[b] <= kMaxXVectors.
__global__ __launch_bounds__(256) void window_build_kernel(const int32_t* __restrict__ block_nz,
                                                           const int32_t* __restrict__ colidx, int tile_cap, int shift,
                                                           int fill, int32_t* __restrict__ nv,
                                                           const int32_t* __restrict__ xv_ptr,
                                                           int32_t* __restrict__ xv_start, int32_t* __restrict__ xv_pad,
                                                           int x_cap, uint16_t* __restrict__ lidx) {
    __shared__ uint32_t keys[kMaxTileEntries];  // the keys to sort, or one bit per possible key
    __shared__ uint32_t uniq[kMaxXVectors];
    __shared__ int counts[256];
    __shared__ int chunk_base[kMaxTileEntries / 64 + 1];
    __shared__ uint16_t word_rank[kMaxTileEntries];  // bitmap path: distinct keys below each word
    __shared__ uint32_t key_lo, key_hi;
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int k0 = block_nz[b], k1 = block_nz[b + 1];
    const int cnt = k1 - k0;
    if (cnt > tile_cap || cnt > kMaxTileEntries || cnt == 0) {
        if (!fill && tid == 0) nv[b] = 0;
        if (fill) {
            for (int i = tid; i < cnt; i += 256) lidx[k0 + i] = 0;
            for (int i = tid; i < x_cap; i += 256) xv_pad[b * x_cap + i] = -1;
        }
        return;
    }
    // Keys that span at most 32 * kMaxTileEntries values (a stencil's neighbouring grid lines, a band, a matrix of
    // moderate width) need no sort: one bit per possible key in LDS, ranks from the population counts below a bit.
    {
        uint32_t lo = 0xFFFFFFFFu, hi = 0;
        for (int i = tid; i < cnt; i += 256) {
            const uint32_t key = static_cast<uint32_t>(colidx[k0 + i]) >> shift;
            lo = key < lo ? key : lo;
            hi = key > hi ? key : hi;
        }
        if (tid == 0) {
            key_lo = 0xFFFFFFFFu;
            key_hi = 0;
        }
        __syncthreads();
        atomicMin(&key_lo, lo);
        atomicMax(&key_hi, hi);
        __syncthreads();
    }
    const uint32_t kmin = key_lo;
    const uint32_t range = key_hi - kmin + 1;
    constexpr uint32_t kBitmapKeys = 32u * kMaxTileEntries;
    if (!fill && range > kBitmapKeys && range <= 16u * kBitmapKeys) {
        // counting alone over a wider span of keys: the bitmap slides over it, a window of keys at a time
        int mine = 0;
        for (uint32_t first = kmin; first - kmin < range; first += kBitmapKeys) {
            for (int w = tid; w < kMaxTileEntries; w += 256) keys[w] = 0;
            __syncthreads();
            for (int i = tid; i < cnt; i += 256) {
                const uint32_t rel = (static_cast<uint32_t>(colidx[k0 + i]) >> shift) - first;  // a key below the window wraps to a huge number
                if (rel < kBitmapKeys) atomicOr(&keys[rel >> 5], 1u << (rel & 31));
            }
            __syncthreads();
            for (int w = tid; w < kMaxTileEntries; w += 256) mine += __popc(keys[w]);
            __syncthreads();
        }
        counts[tid] = mine;
        __syncthreads();
        if (tid == 0) {
            int total = 0;
            for (int t = 0; t < 256; ++t) total += counts[t];
            nv[b] = total;
        }
        return;
    }
    if (range <= kBitmapKeys) {
        const int nwords = static_cast<int>((range + 31) >> 5);
        for (int w = tid; w < nwords; w += 256) keys[w] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < cnt; i0 += 256) {
            const int i = i0 + tid;
            const uint32_t rel = i < cnt ? (static_cast<uint32_t>(colidx[k0 + i]) >> shift) - kmin : 0xFFFFFFFFu;
            const uint32_t before = __shfl_up(rel, 1);  // the entry before: the same key again needs no second atomic
            if (i < cnt && ((tid & 63) == 0 || before != rel)) atomicOr(&keys[rel >> 5], 1u << (rel & 31));
        }
        __syncthreads();
        const int per = (nwords + 255) / 256;  // each lane owns `per` consecutive words
        const int w0 = tid * per < nwords ? tid * per : nwords, w1 = w0 + per < nwords ? w0 + per : nwords;
        int mine = 0;
        for (int w = w0; w < w1; ++w) mine += __popc(keys[w]);
        // distinct keys in the words of the lanes before this one, and in all
        int incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if ((tid & 63) >= d) incl += up;
        }
        if ((tid & 63) == 63) counts[tid >> 6] = incl;
        __syncthreads();
        int pre = incl - mine, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const int c = counts[w];
            pre += w < (tid >> 6) ? c : 0;
            total += c;
        }
        if (!fill) {
            if (tid == 0) nv[b] = total;
            return;
        }
        if (total > kMaxXVectors) return;  // not reached: the host launches the fill pass only when all fit
        const int v0 = xv_ptr[b];
        for (int w = w0; w < w1; ++w) {
            word_rank[w] = static_cast<uint16_t>(pre);
            uint32_t bits = keys[w];
            while (bits) {
                const int bit = __ffs(bits) - 1;
                bits &= bits - 1;
                const int32_t first = static_cast<int32_t>((kmin + 32u * w + bit) << shift);
                xv_start[v0 + pre] = first;
                xv_pad[b * x_cap + pre] = first;
                ++pre;
            }
        }
        for (int i = total + tid; i < x_cap; i += 256) xv_pad[b * x_cap + i] = -1;
        __syncthreads();
        const uint32_t low = (1u << shift) - 1u;
        for (int i = tid; i < cnt; i += 256) {
            const uint32_t c = static_cast<uint32_t>(colidx[k0 + i]);
            const uint32_t rel = (c >> shift) - kmin;
            const uint32_t rank = word_rank[rel >> 5] + __popc(keys[rel >> 5] & ((1u << (rel & 31)) - 1u));
            lidx[k0 + i] = static_cast<uint16_t>((rank << shift) + (c & low));
        }
        return;
    }
    // Only an entry whose key differs from its predecessor's can bring a new key: those are
    // compacted into keys[] (order kept), which for rows made of runs of consecutive columns leaves
    // a fraction of the entries to sort.  Two sweeps over colidx: count per run of 64 entries, place.
    const int lane = tid & 63, wv = tid >> 6;
    const int nchunk = (cnt + 63) / 64;  // <= kMaxTileEntries / 64 = 128
    auto first_of_run = [&](int i, uint32_t* key) {
        if (i >= cnt) return false;
        *key = static_cast<uint32_t>(colidx[k0 + i]) >> shift;
        return i == 0 || (static_cast<uint32_t>(colidx[k0 + i - 1]) >> shift) != *key;
    };
    for (int c = wv; c < nchunk; c += 4) {
        uint32_t key = 0;
        const unsigned long long mask = __builtin_amdgcn_ballot_w64(first_of_run(c * 64 + lane, &key));
        if (lane == 0) chunk_base[c] = __popcll(mask);
    }
    __syncthreads();
    int mine = 0, before = 0;
    if (tid < nchunk) {
        mine = chunk_base[tid];
        for (int q = 0; q < tid; ++q) before += chunk_base[q];
    }
    __syncthreads();
    if (tid < nchunk) chunk_base[tid] = before;
    if (tid == nchunk - 1) chunk_base[nchunk] = before + mine;
    __syncthreads();
    for (int c = wv; c < nchunk; c += 4) {
        uint32_t key = 0;
        const bool f = first_of_run(c * 64 + lane, &key);
        const unsigned long long mask = __builtin_amdgcn_ballot_w64(f);
        if (f) keys[chunk_base[c] + __popcll(mask & ((1ull << lane) - 1ull))] = key;
    }
    const int kept = chunk_base[nchunk];
    int P = 256;
    while (P < kept) P <<= 1;
    for (int i = kept + tid; i < P; i += 256) keys[i] = 0xFFFFFFFFu;
    __syncthreads();
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < P; i += 256) {
                const int l = i ^ j;
                if (l > i) {
                    const uint32_t lo = keys[i], hi = keys[l];
                    const bool up = (i & k) == 0;
                    if (up ? lo > hi : lo < hi) {
                        keys[i] = hi;
                        keys[l] = lo;
                    }
                }
            }
            __syncthreads();
        }
    // distinct keys: each lane owns P/256 consecutive sorted slots
    const int C = P / 256;
    const int base = tid * C;
    int heads = 0;
    for (int i = base; i < base + C; ++i) {
        const uint32_t key = keys[i];
        if (key != 0xFFFFFFFFu && (i == 0 || keys[i - 1] != key)) ++heads;
    }
    counts[tid] = heads;
    __syncthreads();
    int pre = 0, total = 0;
    for (int t = 0; t < 256; ++t) {
        const int c = counts[t];
        pre += t < tid ? c : 0;
        total += c;
    }
    if (!fill) {
        if (tid == 0) nv[b] = total;
        return;
    }
    if (total > kMaxXVectors) return;  // not reached: the host launches the fill pass only when all fit
    for (int i = base; i < base + C; ++i) {
        const uint32_t key = keys[i];
        if (key != 0xFFFFFFFFu && (i == 0 || keys[i - 1] != key)) uniq[pre++] = key;
    }
    __syncthreads();
    const int v0 = xv_ptr[b];
    for (int i = tid; i < total; i += 256) xv_start[v0 + i] = static_cast<int32_t>(uniq[i] << shift);
    for (int i = tid; i < x_cap; i += 256) xv_pad[b * x_cap + i] = i < total ? static_cast<int32_t>(uniq[i] << shift) : -1;
    const uint32_t low = (1u << shift) - 1u;
    for (int i = tid; i < cnt; i += 256) {
        const uint32_t c = static_cast<uint32_t>(colidx[k0 + i]);
        const uint32_t key = c >> shift;
        int lo = 0, hi = total;  // first position with uniq[pos] >= key
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (uniq[mid] < key) lo = mid + 1;
            else hi = mid;
        }
        lidx[k0 + i] = static_cast<uint16_t>((static_cast<uint32_t>(lo) << shift) + (c & low));
    }
}

// Finds the row patterns of the window positions (one workgroup of 256 lanes per row block; analysis time).
// Row i of the block has base_i = lidx of its first entry (0 when empty) and rel_i = its positions minus base_i.
// A run takes the next row when rel repeats and, from its third row on, the bases keep the step of its first two rows.
// The block is patterned when it is staged, no row exceeds kMaxPatternLen entries, no rel is negative and there are at
// most kMaxPatternRuns runs.  fill == 0: packs the runs into run_desc[8b .. 8b+7] (word 7 = runs, 0 when not patterned).
// fill == 1 (same inputs, pat_pad allocated with stride pt_cap): writes the list, zero padded.
__global__ __launch_bounds__(256) void pattern_build_kernel(const int32_t* __restrict__ block_desc, const int32_t* __restrict__ rowptr,
                                                            const uint16_t* __restrict__ lidx, int tile_cap, int fill,
                                                            int32_t* __restrict__ run_desc, uint16_t* __restrict__ pat_pad, int pt_cap) {
    __shared__ int base_s[kMaxRowsPerBlock];
    __shared__ unsigned char len_s[kMaxRowsPerBlock], same_s[kMaxRowsPerBlock], flag_s[kMaxRowsPerBlock];
    __shared__ int bad;
    __shared__ int run_first[kMaxPatternRuns + 1], run_stride[kMaxPatternRuns];
    const int tid = threadIdx.x, b = blockIdx.x;
    const int r0 = block_desc[2 * b], k0 = block_desc[2 * b + 1], r1 = block_desc[2 * b + 2], k1 = block_desc[2 * b + 3];
    const int nr = r1 - r0;
    if (tid == 0) bad = (k1 - k0 > tile_cap || nr > kMaxRowsPerBlock) ? 1 : 0;
    __syncthreads();
    if (fill) {  // the runs were found and packed by the first pass: the lists are written from them
        const int32_t* d = run_desc + 8 * static_cast<int64_t>(b);
        uint16_t* out = pat_pad + static_cast<int64_t>(b) * pt_cap;
        const int runs = d[7];
        int row = 0, at = 0;
        for (int r = 0; r < runs; ++r) {
            const int rows = (static_cast<uint32_t>(d[r >> 1]) >> (16 * (r & 1))) & 0xFFFF;
            const int len = (static_cast<uint32_t>(d[2]) >> (8 * r)) & 0xFF;
            const int base = (static_cast<uint32_t>(d[3 + (r >> 1)]) >> (16 * (r & 1))) & 0xFFFF;
            const int ka = rowptr[r0 + row];
            for (int j = tid; j < len; j += 256) out[at + j] = static_cast<uint16_t>(lidx[ka + j] - base);
            row += rows;
            at += len;
        }
        for (int j = at + tid; j < pt_cap; j += 256) out[j] = 0;
        return;
    }
    if (!bad) {
        for (int i = tid; i < nr; i += 256) {
            const int ka = rowptr[r0 + i], len = rowptr[r0 + i + 1] - ka;
            if (len > kMaxPatternLen) {
                bad = 1;
                continue;
            }
            const int base = len > 0 ? lidx[ka] : 0;
            bool same = false;
            if (i > 0) {
                const int pa = rowptr[r0 + i - 1];
                if (ka - pa == len) {
                    same = true;
                    const int pbase = len > 0 ? lidx[pa] : 0;
                    for (int j = 1; j < len; ++j) same &= lidx[ka + j] - base == lidx[pa + j] - pbase;
                }
            }
            bool negative = false;
            for (int j = 1; j < len; ++j) negative |= lidx[ka + j] < base;
            if (negative) bad = 1;
            base_s[i] = base;
            len_s[i] = static_cast<unsigned char>(len);
            same_s[i] = same ? 1 : 0;
        }
    }
    __syncthreads();
    // What row i does to the runs, as far as it can be said without knowing them: 1 = starts a run (its positions
    // differ from the row before), 2 = repeats them but with another step than the row before (joins only as a run's
    // second row), 0 = repeats positions and step.
    if (!bad)
        for (int i = tid; i < nr; i += 256) {
            int f = same_s[i] ? 0 : 1;
            if (f == 0 && i >= 2 && base_s[i] - base_s[i - 1] != base_s[i - 1] - base_s[i - 2]) f = 2;
            flag_s[i] = static_cast<unsigned char>(f);
        }
    __syncthreads();
    if (tid == 0) {
        int runs = 0;
        if (!bad) {
            bool prev_started = false;
            for (int i = 0; i < nr; ++i) {
                const int f = flag_s[i];
                const bool starts = f == 1 || (f == 2 && !prev_started);
                if (starts) {
                    if (runs == kMaxPatternRuns) {
                        runs = 0;
                        break;
                    }
                    run_first[runs] = i;
                    ++runs;
                }
                prev_started = starts;
            }
            run_first[runs] = nr;
            for (int r = 0; r < runs; ++r)  // the step of a run is that of its first two rows
                run_stride[r] = run_first[r + 1] - run_first[r] >= 2 ? base_s[run_first[r] + 1] - base_s[run_first[r]] : 0;
        }
        {
            int rows[4] = {0, 0, 0, 0}, len[4] = {0, 0, 0, 0}, base[4] = {0, 0, 0, 0}, stride[4] = {0, 0, 0, 0};
            for (int r = 0; r < runs; ++r) {
                rows[r] = run_first[r + 1] - run_first[r];
                len[r] = len_s[run_first[r]];
                base[r] = base_s[run_first[r]];
                stride[r] = run_stride[r] & 0xFFFF;
            }
            int32_t* d = run_desc + 8 * static_cast<int64_t>(b);
            d[0] = rows[0] | rows[1] << 16;
            d[1] = rows[2] | rows[3] << 16;
            d[2] = len[0] | len[1] << 8 | len[2] << 16 | len[3] << 24;
            d[3] = base[0] | base[1] << 16;
            d[4] = base[2] | base[3] << 16;
            d[5] = stride[0] | stride[1] << 16;
            d[6] = stride[2] | stride[3] << 16;
            d[7] = runs;
        }
    }
}

// *max_table = the longest pattern list of a patterned block, *covered = the entries of the patterned blocks (both
// cleared by the caller).  A pass of its own over the packed runs: one atomic per wavefront instead of two per block
// on the same two addresses.
__global__ __launch_bounds__(256) void pattern_totals_kernel(const int32_t* __restrict__ block_desc, const int32_t* __restrict__ run_desc,
                                                             int nb, int32_t* max_table, unsigned long long* covered) {
    int table = 0;
    unsigned long long entries = 0;
    for (int b = blockIdx.x * 256 + threadIdx.x; b < nb; b += gridDim.x * 256) {
        const int32_t* d = run_desc + 8 * static_cast<int64_t>(b);
        if (d[7] > 0) {
            const uint32_t lens = static_cast<uint32_t>(d[2]);
            const int t = static_cast<int>((lens & 0xFF) + ((lens >> 8) & 0xFF) + ((lens >> 16) & 0xFF) + (lens >> 24));
            table = t > table ? t : table;
            entries += static_cast<unsigned long long>(block_desc[2 * b + 3] - block_desc[2 * b + 1]);
        }
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_xor(table, d);
        table = t > table ? t : table;
        entries += __shfl_xor(entries, d);
    }
    if ((threadIdx.x & 63) == 0 && entries > 0) {
        atomicMax(max_table, table);
        atomicAdd(covered, entries);
    }
}

// Adds the carries of rows that were cut by chunk boundaries.  Chunks that cut the same row
// are consecutive; the thread of the first of them sums the run in chunk order.
__global__ __launch_bounds__(kWG) void merge_fixup_kernel(const int32_t* __restrict__ carry_row,
                                                          const float* __restrict__ carry_val, int P, float* y,
                                                          float alpha) {
    const int p = blockIdx.x * kWG + threadIdx.x;
    if (p >= P) return;
    const int r = carry_row[p];
    if (r < 0) return;
    if (p > 0 && carry_row[p - 1] == r) return;
    float s = 0.f;
    for (int q = p; q < P && carry_row[q] == r; ++q) s += carry_val[q];
    y[r] += alpha * s;
}

// lidx8[g] = lidx[8g] for every whole aligned group of eight entries; *flag = 1 if some group's positions are not
// eight consecutive numbers (then lidx8 is of no use).
__global__ __launch_bounds__(kWG) void lidx_groups_kernel(const uint16_t* __restrict__ lidx, int groups, uint16_t* __restrict__ lidx8,
                                                          int32_t* flag) {
    bool bad = false;
    for (int g = blockIdx.x * kWG + threadIdx.x; g < groups; g += gridDim.x * kWG) {
        const u32x4 l = *reinterpret_cast<const u32x4*>(lidx + 8 * static_cast<int64_t>(g));
        const unsigned both = (l[0] & 0xFFFFu) * 0x10001u;
        bad = bad || l[0] != both + 0x00010000u || l[1] != both + 0x00030002u || l[2] != both + 0x00050004u ||
              l[3] != both + 0x00070006u;
        lidx8[g] = static_cast<uint16_t>(l[0] & 0xFFFFu);
    }
    if (bad) *flag = 1;
}

__global__ __launch_bounds__(kWG) void validate_columns_kernel(const int32_t* __restrict__ colidx, int nnz, int n,
                                                               int32_t* flag) {
    bool bad = false;
    for (int64_t k = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; k < nnz;
         k += static_cast<int64_t>(gridDim.x) * kWG) {
        const int c = colidx[k];
        bad |= (c < 0) | (c >= n);
    }
    if (bad) *flag = 1;
}

__global__ __launch_bounds__(64) void reduce_selftest_kernel(const float* in, float* out) {
    const int l = threadIdx.x;
    const float v = in[l];
    out[0 * 64 + l] = group_sum<1>(v);
    out[1 * 64 + l] = group_sum<2>(v);
    out[2 * 64 + l] = group_sum<4>(v);
    out[3 * 64 + l] = group_sum<8>(v);
    out[4 * 64 + l] = group_sum<16>(v);
    out[5 * 64 + l] = group_sum<32>(v);
    out[6 * 64 + l] = group_sum<64>(v);
    for (int gi = 0; gi < 7; ++gi) out[(7 + gi) * 64 + l] = group_sum_rt(v, 1 << gi);
}


template <typename T>
hipError_t launch_scalar_t(const MatrixView& A, const int32_t* rows, int32_t count, const void* x, float* y, Scalars s,
                           hipStream_t st) {
    using E = typename T::elem;
    hipLaunchKernelGGL((spmv_scalar_kernel<T>), dim3(ceil_div(count, kWG)), dim3(kWG), 0, st, A.rowptr, A.colidx,
                       static_cast<const E*>(A.vals), static_cast<const E*>(x), y, rows, count, s.alpha, s.beta);
    return hipGetLastError();
}

template <typename T, int G>
hipError_t launch_vector_tg(const MatrixView& A, const int32_t* rows, int32_t count, const void* x, float* y,
                            Scalars s, hipStream_t st) {
    using E = typename T::elem;
    const int grid = ceil_div(static_cast<int64_t>(count) * G, kWG);
    hipLaunchKernelGGL((spmv_vector_kernel<T, G>), dim3(grid), dim3(kWG), 0, st, A.rowptr, A.colidx,
                       static_cast<const E*>(A.vals), static_cast<const E*>(x), y, rows, count, s.alpha, s.beta,
                       A.vec_ok ? 1 : 0, A.n, reinterpret_cast<uintptr_t>(x) % 16 == 0 ? 1 : 0);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_vector_t(const MatrixView& A, int lanes, const int32_t* rows, int32_t count, const void* x, float* y,
                           Scalars s, hipStream_t st) {
    switch (lanes) {
        case 2: return launch_vector_tg<T, 2>(A, rows, count, x, y, s, st);
        case 4: return launch_vector_tg<T, 4>(A, rows, count, x, y, s, st);
        case 8: return launch_vector_tg<T, 8>(A, rows, count, x, y, s, st);
        case 16: return launch_vector_tg<T, 16>(A, rows, count, x, y, s, st);
        case 32: return launch_vector_tg<T, 32>(A, rows, count, x, y, s, st);
        case 64: return launch_vector_tg<T, 64>(A, rows, count, x, y, s, st);
        default: return hipErrorInvalidValue;
    }
}

TileArgs tile_args(const MatrixView& A, const void* x, float* y, Scalars s) {
    TileArgs a{};
    a.rowptr = A.rowptr;
    a.colidx = A.colidx;
    a.vals = A.vals;
    a.x = x;
    a.y = y;
    a.m = A.m;
    a.n = A.n;
    a.nnz = A.nnz;
    a.alpha = s.alpha;
    a.beta = s.beta;
    a.vec_ok = A.vec_ok ? 1 : 0;
    return a;
}

}  // namespace

hipError_t launch_scalar(const MatrixView& A, const int32_t* rows, int32_t count, const void* x, float* y, Scalars s,
                         hipStream_t st) {
    if (count <= 0) return hipSuccess;
    return A.bf16 ? launch_scalar_t<BF16>(A, rows, count, x, y, s, st) : launch_scalar_t<F32>(A, rows, count, x, y, s, st);
}

hipError_t launch_vector(const MatrixView& A, int lanes, const int32_t* rows, int32_t count, const void* x, float* y,
                         Scalars s, hipStream_t st) {
    if (count <= 0) return hipSuccess;
    return A.bf16 ? launch_vector_t<BF16>(A, lanes, rows, count, x, y, s, st)
                  : launch_vector_t<F32>(A, lanes, rows, count, x, y, s, st);
}

namespace {

// LDS bytes of a tile kernel launch: staged colidx + vals for `entries` entries (plus alignment
// slack) and `bounds` segment bounds.
template <typename T>
size_t tile_lds_bytes(int entries, int bounds) {
    return (sizeof(int) + sizeof(typename T::elem)) * static_cast<size_t>(entries + 2 * T::VEC) +
           (sizeof(int) + sizeof(float)) * static_cast<size_t>(bounds + 2);
}

template <typename T>
size_t merge_lds_bytes(int items) {
    const size_t per_entry = sizeof(int) + sizeof(typename T::elem);
    const size_t per_row = sizeof(int) + sizeof(float);
    return (per_entry > per_row ? per_entry : per_row) * static_cast<size_t>(items + 2 * T::VEC) + 4 * per_row;
}

template <typename T, bool MERGE, int WG>
hipError_t launch_tiles_wg(const TileArgs& a, size_t lds, hipStream_t st) {
    auto kernel = spmv_tile_kernel<T, MERGE, WG>;
    if (lds > 64 * 1024) {
        // beyond the default limit the kernel has to be told once (per process) how much it may get
        static thread_local size_t allowed = 0;
        if (lds > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return e;
            allowed = lds;
        }
    }
    hipLaunchKernelGGL(kernel, dim3(a.nparts), dim3(WG), lds, st, a);
    return hipGetLastError();
}

template <typename T, bool MERGE>
hipError_t launch_tiles(const TileArgs& a, size_t lds, hipStream_t st) {
    return launch_tiles_wg<T, MERGE, 256>(a, lds, st);
}

template <typename T, int XPL, int NG, bool GROUPED>
hipError_t launch_window_g(const TileArgs& a, size_t lds, hipStream_t st) {
    auto kernel = spmv_window_kernel<T, 256, XPL, NG, GROUPED>;
    if (lds > 64 * 1024) {
        static thread_local size_t allowed = 0;
        if (lds > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return e;
            allowed = lds;
        }
    }
    hipLaunchKernelGGL(kernel, dim3(a.nparts), dim3(256), lds, st, a);
    return hipGetLastError();
}

template <typename T, int XPL, int NG>
hipError_t launch_pattern_g(const TileArgs& a, size_t lds, hipStream_t st) {
    auto kernel = spmv_pattern_kernel<T, 256, XPL, NG>;
    if (lds > 64 * 1024) {
        static thread_local size_t allowed = 0;
        if (lds > allowed) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e != hipSuccess) return e;
            allowed = lds;
        }
    }
    hipLaunchKernelGGL(kernel, dim3(a.nparts), dim3(256), lds, st, a);
    return hipGetLastError();
}

// Picks the instantiation whose fixed first round of loads just covers the blocks.
template <typename T, int XPL, int NG>
hipError_t launch_window_k(const TileArgs& a, size_t lds, hipStream_t st) {
    if (a.run_desc) return launch_pattern_g<T, XPL, NG>(a, lds, st);
    return a.lidx8 ? launch_window_g<T, XPL, NG, true>(a, lds, st) : launch_window_g<T, XPL, NG, false>(a, lds, st);
}

template <typename T>
hipError_t launch_window_t(const TileArgs& a, int staged_max, size_t lds, hipStream_t st) {
    const bool one_group = staged_max + 7 <= 256 * 8;  // a block's span starts up to 7 entries early
    if (a.x_cap <= 256)
        return one_group ? launch_window_k<T, 1, 1>(a, lds, st) : launch_window_k<T, 1, 2>(a, lds, st);
    if (a.x_cap <= 512)
        return one_group ? launch_window_k<T, 2, 1>(a, lds, st) : launch_window_k<T, 2, 2>(a, lds, st);
    return one_group ? launch_window_k<T, 4, 1>(a, lds, st) : launch_window_k<T, 4, 2>(a, lds, st);
}

}  // namespace

hipError_t launch_adaptive(const MatrixView& A, const int32_t* block_desc, int32_t nb,
                           int32_t block_nnz, int32_t rows_max, const void* x, float* y, Scalars s, hipStream_t st) {
    if (nb <= 0) return hipSuccess;
    TileArgs a = tile_args(A, x, y, s);
    a.part_desc = block_desc;
    a.nparts = nb;
    a.tile_cap = block_nnz;
    // a block stages at most block_nnz entries and has at most rows_max rows
    if (A.bf16) return launch_tiles<BF16, false>(a, tile_lds_bytes<BF16>(block_nnz, rows_max), st);
    return launch_tiles<F32, false>(a, tile_lds_bytes<F32>(block_nnz, rows_max), st);
}

hipError_t launch_windowed(const MatrixView& A, const int32_t* block_desc, int32_t nb,
                           int32_t block_nnz, int32_t staged_max, int32_t rows_max, const XWindows& w, const void* x,
                           float* y, Scalars s, hipStream_t st) {
    if (nb <= 0) return hipSuccess;
    if (w.max_vectors > kMaxXVectors || block_nnz > kMaxTileEntries || staged_max > block_nnz)
        return hipErrorInvalidValue;
    TileArgs a = tile_args(A, x, y, s);
    a.part_desc = block_desc;
    a.nparts = nb;
    a.tile_cap = block_nnz;
    a.xv_pad = w.xv_pad;
    a.lidx = w.lidx;
    a.lidx8 = w.run_desc ? nullptr : w.lidx8;
    a.run_desc = w.run_desc;
    a.pat_pad = w.pat_pad;
    a.pt_cap = w.run_desc ? w.pt_cap : 0;
    if (w.run_desc && (w.pt_cap < 8 || w.pt_cap % 8 != 0 || w.pt_cap > kMaxPatternRuns * kMaxPatternLen || !w.pat_pad))
        return hipErrorInvalidValue;
    a.x_cap = w.max_vectors > 0 ? w.max_vectors : 1;
    a.x_vec_ok = reinterpret_cast<uintptr_t>(x) % 16 == 0 ? 1 : 0;
    const size_t esz = A.bf16 ? 2 : 4;
    const size_t lds = 16 * static_cast<size_t>(a.x_cap) + (esz + 2) * static_cast<size_t>(staged_max + 16) +
                       (sizeof(int) + sizeof(float)) * static_cast<size_t>(rows_max + 2) + 2 * static_cast<size_t>(a.pt_cap);
    if (A.bf16) return launch_window_t<BF16>(a, staged_max, lds, st);
    return launch_window_t<F32>(a, staged_max, lds, st);
}

hipError_t launch_window_build(const MatrixView& A, const int32_t* block_nz, int32_t nb, int32_t block_nnz, bool fill,
                               int32_t* nv, const int32_t* xv_ptr, int32_t* xv_start, int32_t* xv_pad, int32_t x_cap,
                               uint16_t* lidx, hipStream_t st) {
    if (nb <= 0) return hipSuccess;
    const int shift = A.bf16 ? 3 : 2;
    hipLaunchKernelGGL(window_build_kernel, dim3(nb), dim3(256), 0, st, block_nz, A.colidx, block_nnz, shift,
                       fill ? 1 : 0, nv, xv_ptr, xv_start, xv_pad, x_cap, lidx);
    return hipGetLastError();
}

hipError_t launch_pattern_build(const int32_t* block_desc, int32_t nb, const int32_t* rowptr, const uint16_t* lidx, int32_t block_nnz,
                                bool fill, int32_t* run_desc, int32_t* max_table, unsigned long long* covered, uint16_t* pat_pad,
                                int32_t pt_cap, hipStream_t st) {
    if (nb <= 0) return hipSuccess;
    hipLaunchKernelGGL(pattern_build_kernel, dim3(nb), dim3(256), 0, st, block_desc, rowptr, lidx, block_nnz, fill ? 1 : 0, run_desc,
                       pat_pad, pt_cap);
    if (!fill) {
        const int grid = nb < 256 * 64 ? (nb + 255) / 256 : 64;
        hipLaunchKernelGGL(pattern_totals_kernel, dim3(grid), dim3(256), 0, st, block_desc, static_cast<const int32_t*>(run_desc), nb,
                           max_table, covered);
    }
    return hipGetLastError();
}

hipError_t launch_merge(const MatrixView& A, const int32_t* chunk_desc, int32_t P,
                        int32_t items_per_chunk, int32_t* carry_row, float* carry_val, const void* x, float* y,
                        Scalars s, hipStream_t st) {
    if (P <= 0) return hipSuccess;
    TileArgs a = tile_args(A, x, y, s);
    a.part_desc = chunk_desc;
    a.carry_row = carry_row;
    a.carry_val = carry_val;
    a.nparts = P;
    a.tile_cap = items_per_chunk;
    // entries + finished rows of a chunk add up to at most items_per_chunk; size for whichever of
    // the two needs more LDS per item (an entry: colidx + value; a row: bound + old y)
    hipError_t e;
    if (A.bf16)
        e = launch_tiles<BF16, true>(a, merge_lds_bytes<BF16>(items_per_chunk), st);
    else
        e = launch_tiles<F32, true>(a, merge_lds_bytes<F32>(items_per_chunk), st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(merge_fixup_kernel, dim3(ceil_div(P, kWG)), dim3(kWG), 0, st, carry_row, carry_val, P, y, s.alpha);
    return hipGetLastError();
}

hipError_t launch_merge_fixup(const int32_t* carry_row, const float* carry_val, int32_t P, float* y, float alpha,
                              hipStream_t st) {
    if (P <= 0) return hipSuccess;
    hipLaunchKernelGGL(merge_fixup_kernel, dim3(ceil_div(P, kWG)), dim3(kWG), 0, st, carry_row, carry_val, P, y, alpha);
    return hipGetLastError();
}

hipError_t launch_lidx_groups(const uint16_t* lidx, int32_t groups, uint16_t* lidx8, int32_t* flag, hipStream_t st) {
    if (groups <= 0) return hipSuccess;
    const int grid = ceil_div(groups, kWG);
    hipLaunchKernelGGL(lidx_groups_kernel, dim3(grid > 8192 ? 8192 : grid), dim3(kWG), 0, st, lidx, groups, lidx8, flag);
    return hipGetLastError();
}

hipError_t launch_validate_columns(const MatrixView& A, int32_t* flag, hipStream_t st) {
    if (A.nnz <= 0) return hipSuccess;
    int grid = ceil_div(A.nnz, kWG);
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(validate_columns_kernel, dim3(grid), dim3(kWG), 0, st, A.colidx, A.nnz, A.n, flag);
    return hipGetLastError();
}

hipError_t launch_reduce_selftest(const float* in, float* out, hipStream_t st) {
    hipLaunchKernelGGL(reduce_selftest_kernel, dim3(1), dim3(64), 0, st, in, out);
    return hipGetLastError();
}

const char* scalar_kernel_name() { return "spmv_scalar_kernel"; }
const char* vector_kernel_name() { return "spmv_vector_kernel"; }
const char* tile_kernel_name() { return "spmv_tile_kernel"; }
const char* window_kernel_name() { return "spmv_window_kernel"; }
const char* pattern_kernel_name() { return "spmv_pattern_kernel"; }

}  // namespace spmv
