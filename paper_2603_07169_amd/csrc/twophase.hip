// The two-pass plan for matrices whose columns are spread over more of x than any cache holds
// (gfx950).  Neither pass gathers from memory:
//
//   multiply  The entries are kept regrouped by blocks of 2^s columns.  A workgroup copies one
//             block of x to LDS, streams a piece of that block's entries (16-bit column within the
//             block, value), takes x out of LDS and writes the products where the entries lie:
//             every store of the pass is one contiguous run.
//   reduce    One workgroup per merge-path chunk (a contiguous stretch of the CSR entry list plus
//             the rows that end in it).  It fetches its chunk's products, four at a time, from
//             where the first pass left them (a tile's products lie together, and the tiles of
//             neighbouring chunks are neighbours, so the chunks a die works on at one time share
//             their cache lines), drops each into LDS at its CSR position within the chunk
//             (16-bit), and then runs the row phase of the tile kernels over them: teams of lanes
//             add up one row each, the piece of a row that the chunk cuts off leaves as a carry
//             (chunks cut only rows of more than SPMV_TP_SNAP entries; where no row is cut the
//             fix-up kernel that adds the carries is not launched).
//
// A tile is the set of entries that share a column block and a chunk.  Its entries keep their CSR
// order, and every tile is padded to a multiple of four entries (value 0, column = the zero slot
// after the x block, position 0xFFFF = dropped), so that a group of four consecutive slots never
// straddles two tiles: one 32-bit number per group of the reduce order says which four products it is.
// The regrouping is done once, at analysis time, on the device (the kernels in the second half).
#include <cstring>

#include <hip/hip_runtime.h>

#include "analysis.h"
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
    auto fetch = [&](int gb) {
#pragma unroll
        for (int u = 0; u < U; ++u) {  // past the end: the piece's last group again, not stored
            const int g = gb + u * kTpMulWG < g1 ? gb + u * kTpMulWG : g1 - 1;
            cc[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x4*>(tp_col) + g);
            load_vals4(tp_val, g, v[u]);
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
            if (gb + u * kTpMulWG < g1) reinterpret_cast<f32x4*>(prod)[gb + u * kTpMulWG] = p;
        }
    }
}

// The multiply pass on a group-aligned matrix: a slot stands for a group of eight entries, its "column" is the number of
// the aligned run of eight x values within the block, its value eight stored numbers; the product written is the dot
// product of the two.  The block of x in LDS: 2^shift runs of eight (64 KB: bf16 runs as they are stored, binary32 runs as
// two vectors of four), then one run of zeros for the padding slots.
__device__ __forceinline__ float dot8(const u32x4 v, const u32x4 xv) {  // eight bf16 pairs
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        acc += __uint_as_float(v[j] << 16) * __uint_as_float(xv[j] << 16);
        acc += __uint_as_float(v[j] & 0xFFFF0000u) * __uint_as_float(xv[j] & 0xFFFF0000u);
    }
    return acc;
}
__device__ __forceinline__ float dot8(const f32x4 v0, const f32x4 v1, const f32x4 x0, const f32x4 x1) {
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) acc += v0[j] * x0[j];
#pragma unroll
    for (int j = 0; j < 4; ++j) acc += v1[j] * x1[j];
    return acc;
}

template <typename T>
__global__ __launch_bounds__(kTpMulWG) void tp_multiply_group_kernel(const int32_t* __restrict__ piece_c,
                                                                     const int32_t* __restrict__ piece_g,
                                                                     const uint16_t* __restrict__ tp_col,
                                                                     const typename T::elem* __restrict__ tp_val,
                                                                     const typename T::elem* __restrict__ x, int n, int shift,
                                                                     float* __restrict__ prod) {
    using E = typename T::elem;
    constexpr int VPR = sizeof(E) == 2 ? 1 : 2;  // 16-byte vectors per run of eight
    extern __shared__ __align__(16) u32x4 xs_raw[];  // (2^shift + 1) * VPR vectors
    const int tid = threadIdx.x;
    const int piece = xcd_remap(blockIdx.x, gridDim.x);
    const int c = piece_c[piece];
    const int g0 = piece_g[piece], g1 = piece_g[piece + 1];
    const int runs = 1 << shift;
    const int64_t first = (static_cast<int64_t>(c) << shift) * 8;  // first column of the block
    // the block of x: whole aligned runs where x allows 16-byte loads and the run lies inside the matrix
    const bool x_vec = reinterpret_cast<uintptr_t>(x) % 16 == 0;
    for (int r = tid; r <= runs; r += kTpMulWG) {
        const int64_t col = first + 8 * static_cast<int64_t>(r);
        if (r < runs && x_vec && col + 8 <= n) {
#pragma unroll
            for (int v = 0; v < VPR; ++v) xs_raw[r * VPR + v] = *reinterpret_cast<const u32x4*>(x + col + (8 / VPR) * v);
        } else {
            E tmp[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) tmp[e] = (r < runs && col + e < n) ? x[col + e] : E(0);
#pragma unroll
            for (int v = 0; v < VPR; ++v) xs_raw[r * VPR + v] = *reinterpret_cast<const u32x4*>(tmp + (8 / VPR) * v);
        }
    }
    __syncthreads();
    // One slot per lane and trip, U trips in flight: neighbouring lanes read neighbouring 16-byte (32-byte) value runs and
    // write neighbouring products.
    constexpr int U = 2;
    const u32x4* vals = reinterpret_cast<const u32x4*>(tp_val);
    const int s0 = 4 * g0, s1 = 4 * g1;
    for (int sb = s0 + tid; sb < s1; sb += U * kTpMulWG) {
        u32x4 v[U][VPR];
        int cc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {  // past the end: the piece's last slot again, not stored
            const int sl = sb + u * kTpMulWG < s1 ? sb + u * kTpMulWG : s1 - 1;
#pragma unroll
            for (int i = 0; i < VPR; ++i) v[u][i] = __builtin_nontemporal_load(vals + static_cast<int64_t>(sl) * VPR + i);
            cc[u] = __builtin_nontemporal_load(tp_col + sl);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int sl = sb + u * kTpMulWG;
            float p;
            if constexpr (VPR == 1) {
                p = dot8(v[u][0], xs_raw[cc[u]]);
            } else {
                p = dot8(__builtin_bit_cast(f32x4, v[u][0]), __builtin_bit_cast(f32x4, v[u][1]),
                         __builtin_bit_cast(f32x4, xs_raw[2 * cc[u]]), __builtin_bit_cast(f32x4, xs_raw[2 * cc[u] + 1]));
            }
            if (sl < s1) prod[sl] = p;
        }
    }
}

struct TpReduceArgs {
    const int32_t* chunk_desc;  // [2*(P+1)] pairs (rows finished, entries taken) at each split
    const int32_t* chunk_g;     // [P+1] first group of each chunk's stretch of tp_pos / prod
    const int32_t* tp_from;     // [groups] the group of prod that each group of the reduce order is
    const uint16_t* tp_pos;
    const float* prod;
    const int32_t* rowptr;
    float* y;
    int32_t* carry_row;
    float* carry_val;
    int32_t nparts;
    int32_t row_shift;  // 0, or 3 when a slot stands for a group of eight entries: rowptr is then counted in groups
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
    // a die works through a contiguous stretch of chunks: the lines their tiles share are fetched into one L2
    const int part = xcd_remap(blockIdx.x, gridDim.x);
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
    for (int i = tid; i <= nr; i += WG) seg[i] = bound(a.rowptr[r0 + i] >> a.row_shift);
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
            // written a moment ago: a plain load finds much of it still cached
            pp[u] = reinterpret_cast<const f32x4*>(a.prod)[__builtin_nontemporal_load(a.tp_from + g)];
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
// A tile is the set of entries that share a column block c and a chunk p.  A chunk is a contiguous stretch of the
// CSR entry list, so everything is derived chunk by chunk from colidx as it lies: one workgroup counts its chunk's
// entries per column block, prefix sums over the (c, p) table give every tile its slots in both orders, and one
// workgroup per chunk then ranks its entries (CSR order kept inside a tile) and writes them out.  No sort over the
// whole matrix and no gather.

constexpr int kTpBinSpan = 2048;  // column blocks a workgroup handles per pass over its chunk (more: several passes)
constexpr int kTpScanBlock = 4096;  // elements per workgroup of the prefix sums

__device__ __forceinline__ unsigned column_block_of(int col, int shift, int C) {
    const unsigned c = static_cast<unsigned>(col) >> shift;
    return c < static_cast<unsigned>(C) ? c : static_cast<unsigned>(C - 1);  // beyond n only when the caller skipped validation
}

// padded[c*P + p] = slots of tile (c, p): its entries rounded up to whole groups of four.  One workgroup per chunk.
__global__ __launch_bounds__(kWG) void tp_count_kernel(const int32_t* __restrict__ colidx, const int32_t* __restrict__ chunk_desc,
                                                       int shift, int C, int P, int32_t* __restrict__ padded) {
    __shared__ int cnt[kTpBinSpan];
    const int p = blockIdx.x, tid = threadIdx.x;
    const int k0 = chunk_desc[2 * p + 1], k1 = chunk_desc[2 * p + 3];
    for (int lo = 0; lo < C; lo += kTpBinSpan) {
        const int span = C - lo < kTpBinSpan ? C - lo : kTpBinSpan;
        for (int i = tid; i < span; i += kWG) cnt[i] = 0;
        __syncthreads();
        for (int k = k0 + tid; k < k1; k += kWG) {
            const unsigned b = column_block_of(colidx[k], shift, C) - static_cast<unsigned>(lo);
            if (b < static_cast<unsigned>(span)) atomicAdd(&cnt[b], 1);
        }
        __syncthreads();
        for (int i = tid; i < span; i += kWG) padded[static_cast<int64_t>(lo + i) * P + p] = (cnt[i] + 3) & ~3;
        __syncthreads();
    }
}

// Exclusive prefix sums of 32-bit counts, three launches: sums of blocks of kTpScanBlock elements, their prefix sums
// (one workgroup), the elements themselves.  count may be anything up to 2^31 - 1.
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(v, d);
        if (lane >= d) v += up;
    }
    return v;
}
// Exclusive prefix of v over the workgroup's kWG lanes (in lane order) and the workgroup's total; wave_sums: kWG/64 ints of LDS.
__device__ __forceinline__ int block_exclusive_scan(int v, int* wave_sums, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int incl = wave_inclusive_scan(v, lane);
    __syncthreads();  // wave_sums may still be read from the call before
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWG / 64; ++w) {
        const int sw = wave_sums[w];
        before += w < wave ? sw : 0;
        all += sw;
    }
    *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(kWG) void tp_scan_sums_kernel(const int32_t* __restrict__ in, int64_t count, int32_t* __restrict__ sums) {
    __shared__ int wave_sums[kWG / 64];
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kTpScanBlock;
    int v = 0;
    for (int i = threadIdx.x; i < kTpScanBlock; i += kWG)
        if (base + i < count) v += in[base + i];
    int total;
    block_exclusive_scan(v, wave_sums, &total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kWG) void tp_scan_top_kernel(int32_t* __restrict__ sums, int nblocks) {
    __shared__ int wave_sums[kWG / 64];
    const int per = (nblocks + kWG - 1) / kWG;  // consecutive block sums per lane
    const int first = threadIdx.x * per;
    int v = 0;
    for (int i = first; i < first + per && i < nblocks; ++i) v += sums[i];
    int total;
    int run = block_exclusive_scan(v, wave_sums, &total);
    for (int i = first; i < first + per && i < nblocks; ++i) {
        const int x = sums[i];
        sums[i] = run;
        run += x;
    }
}

__global__ __launch_bounds__(kWG) void tp_scan_apply_kernel(const int32_t* __restrict__ in, int64_t count, const int32_t* __restrict__ sums,
                                                            int32_t* __restrict__ out) {
    __shared__ int wave_sums[kWG / 64];
    constexpr int PER = kTpScanBlock / kWG;  // consecutive elements per lane
    const int64_t base = static_cast<int64_t>(blockIdx.x) * kTpScanBlock + static_cast<int64_t>(threadIdx.x) * PER;
    int x[PER];
    int v = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        x[j] = base + j < count ? in[base + j] : 0;
        v += x[j];
    }
    int total;
    int run = sums[blockIdx.x] + block_exclusive_scan(v, wave_sums, &total);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (base + j < count) out[base + j] = run;
        run += x[j];
    }
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
    const int32_t* base1;        // [C*P] slots before tile t in the multiply order (t = c*P + p)
    const int32_t* within;       // [C*P] slots of t's chunk in the column blocks before t's
    const int32_t* chunk_first;  // [P+1] slots before each chunk in the reduce order
    const int32_t* chunk_desc;
    const int32_t* colidx;
    const void* vals;
    int32_t C, P, shift, elem_bytes;  // elem_bytes 0: a slot stands for a group of entries, no value is placed here
    int32_t span_cap;  // min(C, kTpBinSpan): the LDS tables' size
    uint16_t* tp_col;
    void* tp_val;
    int32_t* tp_src;
    int32_t* tp_from;
    uint16_t* tp_pos;
};

// One workgroup per chunk.  Per pass over a range of column blocks: every wavefront counts its quarter of the chunk's
// entries per block; prefix sums over (block, wavefront) give each wavefront its first place in each block's run;
// the wavefronts then walk through their quarters 64 entries at a time, in CSR order, ranking the lanes that share a
// block with ballots, and drop every entry at its place in an LDS copy sorted by (block, CSR position); the copy is
// written out run by run, so the stores of a tile are coalesced.
__global__ __launch_bounds__(kWG) void tp_place_kernel(const TpPlaceArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int wave_sums[kWG / 64];
    __shared__ int n_staged;
    constexpr int WAVES = kWG / 64;
    int* cntw = reinterpret_cast<int*>(smem_raw);                           // [WAVES][span_cap]
    int* lstart = cntw + WAVES * a.span_cap;                                 // [span_cap + 1], padded to a multiple of four
    int* tile1 = lstart + ((a.span_cap + 4) & ~3);                           // [span_cap] the tile's first slot in the multiply order, less lstart
    int* tile2 = tile1 + a.span_cap;                                         // [span_cap] the same in the reduce order
    uint32_t* sval = reinterpret_cast<uint32_t*>(tile2 + a.span_cap);        // [kTwoPhaseItems] value bits
    uint16_t* spos = reinterpret_cast<uint16_t*>(sval + kTwoPhaseItems);     // CSR position within the chunk
    uint16_t* scol = spos + kTwoPhaseItems;                                  // column within the block
    uint16_t* sblk = scol + kTwoPhaseItems;                                  // block within the pass's range
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned long long below = (1ull << lane) - 1ull;
    const int p = blockIdx.x;
    const int k0 = a.chunk_desc[2 * p + 1], k1 = a.chunk_desc[2 * p + 3];
    const int quarter = (((k1 - k0 + WAVES - 1) / WAVES) + 63) & ~63;
    const int q0 = k0 + wave * quarter < k1 ? k0 + wave * quarter : k1;
    const int q1 = q0 + quarter < k1 ? q0 + quarter : k1;
    const unsigned col_mask = (1u << a.shift) - 1u;
    const int slot2 = a.chunk_first[p];

    // the wavefront's quarter, 64 entries per round, fetched once and in one go (a lane past the quarter's end reads
    // the chunk's last entry again and never uses it): the passes below then run out of registers
    constexpr int ROUNDS = kTwoPhaseItems / kWG;
    int cols[ROUNDS];
    uint32_t vbits[ROUNDS];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        cols[r] = 0;
        vbits[r] = 0;
    }
    if (k0 < k1) {
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            int k = q0 + r * 64 + lane;
            k = k < k1 ? k : k1 - 1;
            cols[r] = a.colidx[k];
            if (a.elem_bytes == 4) vbits[r] = static_cast<const uint32_t*>(a.vals)[k];
            else if (a.elem_bytes == 2) vbits[r] = static_cast<const uint16_t*>(a.vals)[k];  // 0: the values are placed by a pass of their own
        }
    }

    for (int lo = 0; lo < a.C; lo += kTpBinSpan) {
        const int span = a.C - lo < kTpBinSpan ? a.C - lo : kTpBinSpan;
        int nbits = 0;
        while ((1 << nbits) < span) ++nbits;
        for (int i = tid; i < WAVES * a.span_cap; i += kWG) cntw[i] = 0;
        __syncthreads();
        int* mine_cnt = cntw + wave * a.span_cap;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const unsigned b = column_block_of(cols[r], a.shift, a.C) - static_cast<unsigned>(lo);
            if (q0 + r * 64 + lane < q1 && b < static_cast<unsigned>(span)) atomicAdd(&mine_cnt[b], 1);
        }
        __syncthreads();
        // per block: the wavefronts' counts become their first places inside the block's run; lstart = the runs' starts
        constexpr int PER = kTpBinSpan / kWG;  // consecutive blocks per lane
        int tot[PER];
        int v = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int b = tid * PER + j;
            int run = 0;
            if (b < span) {
#pragma unroll
                for (int w = 0; w < WAVES; ++w) {
                    const int c = cntw[w * a.span_cap + b];
                    cntw[w * a.span_cap + b] = run;
                    run += c;
                }
            }
            tot[j] = run;
            v += run;
        }
        int total;
        int run = block_exclusive_scan(v, wave_sums, &total);
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int b = tid * PER + j;
            if (b < span) lstart[b] = run;
            run += tot[j];
        }
        if (tid == 0) {
            lstart[span] = total;
            n_staged = total;
        }
        __syncthreads();
        // where each block's run goes (one gather per block instead of two per entry)
        for (int b = tid; b < span; b += kWG) {
            const int64_t t = static_cast<int64_t>(lo + b) * a.P + p;
            tile1[b] = a.base1[t] - lstart[b];
            tile2[b] = slot2 + a.within[t] - lstart[b];
        }
        // rank and stage, wavefront by wavefront over its own quarter, 64 entries at a time in CSR order
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            if (q0 + r * 64 >= q1) break;
            const int k = q0 + r * 64 + lane;
            const unsigned b = column_block_of(cols[r], a.shift, a.C) - static_cast<unsigned>(lo);
            const bool mine = k < q1 && b < static_cast<unsigned>(span);
            unsigned long long same = __builtin_amdgcn_ballot_w64(mine);  // lanes of this round in the same block as this one
            for (int bit = 0; bit < nbits; ++bit) {
                const bool one = (b >> bit) & 1u;
                const unsigned long long with_one = __builtin_amdgcn_ballot_w64(one);
                same &= one ? with_one : ~with_one;
            }
            if (mine) {
                const int i = lstart[b] + mine_cnt[b] + __popcll(same & below);
                sval[i] = vbits[r];
                spos[i] = static_cast<uint16_t>(k - k0);
                scol[i] = static_cast<uint16_t>(static_cast<unsigned>(cols[r]) & col_mask);
                sblk[i] = static_cast<uint16_t>(b);
            }
            __builtin_amdgcn_wave_barrier();
            if (mine && (same & below) == 0) mine_cnt[b] += __popcll(same);  // the first lane of each block moves its wavefront's place on
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        const int n = n_staged;
        for (int i = tid; i < n; i += kWG) {
            const int b = sblk[i];
            const int o = i - lstart[b];
            const int s1 = tile1[b] + i;
            const int s2 = tile2[b] + i;
            a.tp_col[s1] = scol[i];
            if (a.elem_bytes == 4) static_cast<uint32_t*>(a.tp_val)[s1] = sval[i];
            else if (a.elem_bytes == 2) static_cast<uint16_t*>(a.tp_val)[s1] = static_cast<uint16_t>(sval[i]);
            a.tp_src[s1] = k0 + spos[i];
            a.tp_pos[s2] = spos[i];
            if ((o & 3) == 0) a.tp_from[s2 >> 2] = s1 >> 2;
        }
        __syncthreads();
    }
}

// Group-aligned?  gcol[g] = colidx[8g] / 8 for every group of eight entries; *flag is set when a group does not start
// at a multiple of eight columns or its columns are not eight consecutive numbers.
__global__ __launch_bounds__(kWG) void tp_groups_kernel(const int32_t* __restrict__ colidx, int ngroups, int32_t* __restrict__ gcol,
                                                        int32_t* flag) {
    bool bad = false;
    for (int64_t g = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; g < ngroups; g += static_cast<int64_t>(gridDim.x) * kWG) {
        const int32_t* c = colidx + 8 * g;
        const int c0 = c[0];
        bad = bad || (c0 & 7) != 0;
#pragma unroll
        for (int i = 1; i < 8; ++i) bad = bad || c[i] != c0 + i;
        gcol[g] = c0 >> 3;
    }
    if (__builtin_amdgcn_ballot_w64(bad) != 0 && (threadIdx.x & 63) == 0) *flag = 1;  // plain store: every writer writes 1
}

// tp_val[8s + e] = vals[8 tp_src[s] + e] for the slots that hold a group (tp_src[s] >= 0).
template <typename E>
__global__ __launch_bounds__(kWG) void tp_group_values_kernel(const E* __restrict__ vals, const int32_t* __restrict__ tp_src,
                                                              E* __restrict__ tp_val, int64_t slots, int ngroups) {
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kWG + threadIdx.x; i < 8 * slots; i += static_cast<int64_t>(gridDim.x) * kWG) {
        const int g = tp_src[i >> 3];
        if (g >= 0 && g < ngroups) tp_val[i] = vals[8 * static_cast<int64_t>(g) + (i & 7)];
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
    hipError_t e;
    if (t.num_pieces > 0 && t.group == 8) {
        // a slot is a group of eight entries: the block of x as 2^shift aligned runs of eight, and one run of zeros
        const size_t lds1 = (A.bf16 ? 16 : 32) * ((size_t{1} << t.shift) + 1);
        if (A.bf16) {
            auto k = tp_multiply_group_kernel<BF16>;
            static thread_local size_t allowed = 0;
            if ((e = allow_lds(k, lds1, &allowed)) != hipSuccess) return e;
            hipLaunchKernelGGL(k, dim3(t.num_pieces), dim3(kTpMulWG), lds1, st, t.piece_c, t.piece_g, t.tp_col,
                               static_cast<const uint16_t*>(t.tp_val), static_cast<const uint16_t*>(x), A.n, t.shift,
                               t.prod);
        } else {
            auto k = tp_multiply_group_kernel<F32>;
            static thread_local size_t allowed = 0;
            if ((e = allow_lds(k, lds1, &allowed)) != hipSuccess) return e;
            hipLaunchKernelGGL(k, dim3(t.num_pieces), dim3(kTpMulWG), lds1, st, t.piece_c, t.piece_g, t.tp_col,
                               static_cast<const float*>(t.tp_val), static_cast<const float*>(x), A.n, t.shift, t.prod);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else if (t.num_pieces > 0) {
        const size_t lds1 = sizeof(float) * ((size_t{1} << t.shift) + 4);
        if (A.bf16) {
            auto k = tp_multiply_kernel<BF16, kTpMulGroups>;
            static thread_local size_t allowed = 0;
            if ((e = allow_lds(k, lds1, &allowed)) != hipSuccess) return e;
            hipLaunchKernelGGL(k, dim3(t.num_pieces), dim3(kTpMulWG), lds1, st, t.piece_c, t.piece_g, t.tp_col,
                               static_cast<const uint16_t*>(t.tp_val), static_cast<const uint16_t*>(x), A.n, t.shift,
                               t.prod);
        } else {
            auto k = tp_multiply_kernel<F32, kTpMulGroups>;
            static thread_local size_t allowed = 0;
            if ((e = allow_lds(k, lds1, &allowed)) != hipSuccess) return e;
            hipLaunchKernelGGL(k, dim3(t.num_pieces), dim3(kTpMulWG), lds1, st, t.piece_c, t.piece_g, t.tp_col,
                               static_cast<const float*>(t.tp_val), static_cast<const float*>(x), A.n, t.shift, t.prod);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const TpReduceArgs a{t.chunk_desc, t.chunk_g, t.tp_from, t.tp_pos, t.prod, A.rowptr, y, t.carry_row, t.carry_val, t.num_chunks,
                         t.group == 8 ? 3 : 0, s.alpha, s.beta};
    auto k = tp_reduce_kernel<kTpRedWG, kTpRedGroups>;
    static thread_local size_t allowed = 0;
    if ((e = allow_lds(k, t.reduce_lds, &allowed)) != hipSuccess) return e;
    hipLaunchKernelGGL(k, dim3(t.num_chunks), dim3(kTpRedWG), t.reduce_lds, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // no chunk cuts a row (rows of up to kTwoPhaseSnap entries are kept whole): every carry is empty
    if (!t.carries) return hipSuccess;
    return launch_merge_fixup(t.carry_row, t.carry_val, t.num_chunks, y, s.alpha, st);
}

hipError_t launch_two_phase_groups(const int32_t* colidx, int32_t ngroups, int32_t* gcol, int32_t* flag, hipStream_t st) {
    if (ngroups <= 0) return hipSuccess;
    hipLaunchKernelGGL(tp_groups_kernel, dim3(capped_grid(ngroups)), dim3(kWG), 0, st, colidx, ngroups, gcol, flag);
    return hipGetLastError();
}

int64_t two_phase_scan_blocks(int64_t count) { return (count + kTpScanBlock - 1) / kTpScanBlock; }

namespace {
// out[i] = in[0] + .. + in[i-1] for i < count; sums: two_phase_scan_blocks(count) ints of scratch.
hipError_t exclusive_scan(const int32_t* in, int64_t count, int32_t* sums, int32_t* out, hipStream_t st) {
    if (count <= 0) return hipSuccess;
    const int nblocks = static_cast<int>(two_phase_scan_blocks(count));
    hipLaunchKernelGGL(tp_scan_sums_kernel, dim3(nblocks), dim3(kWG), 0, st, in, count, sums);
    hipLaunchKernelGGL(tp_scan_top_kernel, dim3(1), dim3(kWG), 0, st, sums, nblocks);
    hipLaunchKernelGGL(tp_scan_apply_kernel, dim3(nblocks), dim3(kWG), 0, st, in, count, static_cast<const int32_t*>(sums), out);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_two_phase_tables(const MatrixView& A, int shift, int32_t C, int32_t P, const int32_t* chunk_desc,
                                   const TwoPhaseTables& w, int32_t* chunk_g, hipStream_t st) {
    const int64_t T = static_cast<int64_t>(C) * P;
    hipError_t e;
    hipLaunchKernelGGL(tp_count_kernel, dim3(P), dim3(kWG), 0, st, A.colidx, chunk_desc, shift, C, P, w.padded);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = exclusive_scan(w.padded, T, w.scan_sums, w.base1, st)) != hipSuccess) return e;
    hipLaunchKernelGGL(tp_chunk_columns_kernel, dim3(ceil_div(P + 1, kWG)), dim3(kWG), 0, st, w.padded, C, P, w.within, w.in_chunk);
    if ((e = exclusive_scan(w.in_chunk, static_cast<int64_t>(P) + 1, w.scan_sums, w.chunk_first, st)) != hipSuccess) return e;
    hipLaunchKernelGGL(tp_starts_kernel, dim3(ceil_div((C > P ? C : P) + 1, kWG)), dim3(kWG), 0, st, w.base1, w.padded, C, P,
                       w.chunk_first, w.block_first, chunk_g);
    return hipGetLastError();
}

hipError_t launch_two_phase_place(const MatrixView& A, int shift, int32_t C, int32_t P, const TwoPhaseTables& w,
                                  const int32_t* chunk_desc, int64_t slots, int group, uint16_t* tp_col, void* tp_val,
                                  int32_t* tp_src, int32_t* tp_from, uint16_t* tp_pos, hipStream_t st) {
    // padding first: column = the zero slot after the x block, value 0, no source, position "dropped"
    hipLaunchKernelGGL(tp_fill16_kernel, dim3(capped_grid(slots)), dim3(kWG), 0, st, tp_col, slots,
                       static_cast<uint16_t>(1u << shift));
    hipLaunchKernelGGL(tp_fill16_kernel, dim3(capped_grid(slots)), dim3(kWG), 0, st, tp_pos, slots, static_cast<uint16_t>(0xFFFF));
    hipError_t e = hipMemsetAsync(tp_val, 0, static_cast<size_t>(slots) * group * (A.bf16 ? 2 : 4), st);
    if (e != hipSuccess) return e;
    if ((e = hipMemsetAsync(tp_src, 0xFF, static_cast<size_t>(slots) * 4, st)) != hipSuccess) return e;
    if ((e = hipMemsetAsync(tp_from, 0, static_cast<size_t>(slots), st)) != hipSuccess) return e;
    const int span_cap = C < kTpBinSpan ? C : kTpBinSpan;
    // group > 1: A is the matrix of groups (colidx = the groups' columns); the values follow in a pass of their own
    const TpPlaceArgs a{w.base1, w.within, w.chunk_first, chunk_desc, A.colidx, A.vals, C,      P,     shift,
                        group > 1 ? 0 : (A.bf16 ? 2 : 4), span_cap, tp_col, tp_val, tp_src, tp_from, tp_pos};
    const size_t lds = sizeof(int) * (static_cast<size_t>(kWG / 64 + 2) * span_cap + ((span_cap + 4) & ~3)) +
                       static_cast<size_t>(kTwoPhaseItems) * (sizeof(uint32_t) + 3 * sizeof(uint16_t));
    static thread_local size_t allowed = 0;
    if ((e = allow_lds(tp_place_kernel, lds, &allowed)) != hipSuccess) return e;
    hipLaunchKernelGGL(tp_place_kernel, dim3(P), dim3(kWG), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_two_phase_values(const MatrixView& A, const int32_t* tp_src, void* tp_val, int64_t slots, int group,
                                   hipStream_t st) {
    if (slots <= 0) return hipSuccess;
    if (group == 8) {
        const int ngroups = A.nnz / 8;
        if (A.bf16)
            hipLaunchKernelGGL(tp_group_values_kernel<uint16_t>, dim3(capped_grid(8 * slots)), dim3(kWG), 0, st,
                               static_cast<const uint16_t*>(A.vals), tp_src, static_cast<uint16_t*>(tp_val), slots, ngroups);
        else
            hipLaunchKernelGGL(tp_group_values_kernel<float>, dim3(capped_grid(8 * slots)), dim3(kWG), 0, st,
                               static_cast<const float*>(A.vals), tp_src, static_cast<float*>(tp_val), slots, ngroups);
        return hipGetLastError();
    }
    if (A.bf16)
        hipLaunchKernelGGL(tp_values_kernel<uint16_t>, dim3(capped_grid(slots)), dim3(kWG), 0, st,
                           static_cast<const uint16_t*>(A.vals), tp_src, static_cast<uint16_t*>(tp_val), static_cast<int>(slots));
    else
        hipLaunchKernelGGL(tp_values_kernel<float>, dim3(capped_grid(slots)), dim3(kWG), 0, st, static_cast<const float*>(A.vals),
                           tp_src, static_cast<float*>(tp_val), static_cast<int>(slots));
    return hipGetLastError();
}

}  // namespace spmv
