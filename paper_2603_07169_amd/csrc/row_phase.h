// The row phase of the tile kernels: the entries of a tile sit in LDS and teams of lanes take one
// row (segment) each.  Shared by the CSR tile kernels and the ELL kernel.  Internal linkage.
#pragma once
#include "device_common.h"

namespace spmv {
namespace {

constexpr int kMaxDeferred = 136;  // segments far longer than the tile's mean that can be set aside per tile

// Column type of a tile whose staged values are finished products: nothing is gathered, the row
// phase only adds.  cols and x are then null pointers that are never read.
struct NoGather {};

// B entries of one segment for one lane of a team of G lanes: staged slots j, j+G, .., j+(B-1)G.
// Three bursts of independent accesses, each issued back to back: column indices out of LDS,
// x out of memory, matrix values out of LDS.  G and B are compile-time so that every LDS
// access is the lane's base address plus an immediate offset, and nothing is predicated:
// the row phase is bound by instruction issue, so instructions per entry are what counts.
template <int B, int G, typename I, typename E>
__device__ __forceinline__ float gather_batch(const I* cols, const E* vals, const E* x, int j) {
    unsigned c[B];
    E xv[B];
    E av[B];
#pragma unroll
    for (int u = 0; u < B; ++u) c[u] = static_cast<unsigned>(cols[j + u * G]);
#pragma unroll
    for (int u = 0; u < B; ++u) xv[u] = x[c[u]];
#pragma unroll
    for (int u = 0; u < B; ++u) av[u] = vals[j + u * G];
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < B; ++u) acc += widen(av[u]) * widen(xv[u]);
    return acc;
}

template <int B, int G>
__device__ __forceinline__ float gather_batch(const NoGather*, const float* vals, const float*, int j) {
    float p[B];
#pragma unroll
    for (int u = 0; u < B; ++u) p[u] = vals[j + u * G];
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < B; ++u) acc += p[u];
    return acc;
}

// Partial dot product of the staged entries [b, e) of one segment, taken by lane `tl` of a team
// of G lanes: entry j of the segment goes to lane j mod G.  Neighbouring teams work on
// neighbouring rows, so for banded or stencil-like rows the lanes of a gather instruction fall
// into a handful of cache lines.  The lane's entries are taken in batches of 8, then 4, 2, 1.
template <int G, typename I, typename E>
__device__ __forceinline__ float segment_dot(const I* cols, const E* vals, const E* x, int b, int e, int tl) {
    float acc = 0.f;
    int j = b + tl;
    int cnt = (e - j + G - 1) / G;  // entries this lane takes (<= 0 when the segment is shorter than the team)
    for (; cnt >= 8; cnt -= 8, j += 8 * G) acc += gather_batch<8, G>(cols, vals, x, j);
    if (cnt >= 4) {
        acc += gather_batch<4, G>(cols, vals, x, j);
        j += 4 * G;
        cnt -= 4;
    }
    if (cnt >= 2) {
        acc += gather_batch<2, G>(cols, vals, x, j);
        j += 2 * G;
        cnt -= 2;
    }
    if (cnt >= 1) acc += gather_batch<1, G>(cols, vals, x, j);
    return acc;
}

// Where the row phase of a tile sends its results.
struct RowOut {
    float* y;
    const float* y0;  // LDS: y0[i] = old y of row r0+i when beta != 0 (fetched while the tile was loading)
    int32_t* carry_row;
    float* carry_val;
    float alpha, beta;
};

// Row phase of a tile whose entries sit in LDS (cols[], vals[]); seg[i] .. seg[i+1] bounds the
// slots of segment i.  cols[] indexes x[]: global column numbers into the x vector in memory,
// or 16-bit positions into the tile's x window in LDS.  Segments 0 .. nr-1 are the rows r0 .. r0+nr-1 and go to y.  With MERGE
// there is one more segment, the piece of row r0+nr that the chunk cuts off: its sum is the
// chunk's carry (no carry when it is empty).  Teams of G lanes take one segment each;
// segments longer than defer_len are set aside and taken by whole wavefronts afterwards.
// Entered by the whole workgroup with *n_deferred == 0; contains one barrier.
template <bool MERGE, int WG, int G, typename I, typename E>
__device__ __forceinline__ void tile_rows_g(const I* cols, const E* vals, const E* x, const int* seg, int nr, int r0,
                                            int part, const RowOut& o, int* deferred, int* n_deferred, int tid) {
    const int nseg = nr + (MERGE ? 1 : 0);
    constexpr int defer_len = 32 * G > 64 ? 32 * G : 64;
    constexpr int teams = WG / G;
    const int team = tid / G;
    const int tl = tid % G;

    auto emit = [&](int i, float s, int len) {
        if (i < nr) {
            o.y[r0 + i] = epilogue(s, o.alpha, o.beta, o.y0, i);
        } else {
            o.carry_row[part] = len > 0 ? r0 + nr : -1;
            o.carry_val[part] = s;
        }
    };

    for (int base = 0; base < nseg; base += teams) {
        const int i = base + team;
        float acc = 0.f;
        bool mine = false;
        int len = 0;
        if (i < nseg) {
            const int b = seg[i], e = seg[i + 1];
            len = e - b;
            if (len <= defer_len) {
                mine = true;
                acc = segment_dot<G>(cols, vals, x, b, e, tl);
            } else if (tl == 0) {
                deferred[atomicAdd(n_deferred, 1)] = i;
            }
        }
        acc = group_sum<G>(acc);  // every lane takes part
        if (mine && tl == 0) emit(i, acc, len);
    }
    __syncthreads();

    const int nd = *n_deferred;
    const int lane = tid & 63;
    for (int d = tid >> 6; d < nd; d += WG / 64) {
        const int i = deferred[d];
        const int b = seg[i], e = seg[i + 1];
        float acc = segment_dot<64>(cols, vals, x, b, e, lane);
        acc = group_sum<64>(acc);
        if (lane == 0) emit(i, acc, e - b);
    }
}

// Lanes per row from the tile's mean segment length: the largest power of two G <= 64 with
// 16*G <= mean + 15.  Small teams keep the lanes of a gather on
// neighbouring rows, which is what makes the gathers of banded matrices coalesce.
template <bool MERGE, int WG, typename I, typename E>
__device__ __forceinline__ void tile_rows(const I* cols, const E* vals, const E* x, const int* seg, int nr, int r0,
                                          int part, int tile_nnz, const RowOut& o, int* deferred, int* n_deferred,
                                          int tid) {
    const int nseg = nr + (MERGE ? 1 : 0);
    // With mean = floor(tile_nnz / nseg):  k < mean  <=>  (k + 1) * nseg <= tile_nnz  and
    // k > mean  <=>  k * nseg > tile_nnz, so the choice needs no division.
    int G = 1;
    while (G < 64 && nseg > 0 && (16 * G + 1) * nseg <= tile_nnz) G <<= 1;
    if (sizeof(I) == 2 && nseg > 0 && tile_nnz >= 64 * nseg) {
        // x comes out of LDS (16-bit window positions) and mean >= 64: long rows get about four
        // entries per lane.  Fewer rows then share a wavefront, and rows whose length is a multiple
        // of the 128-byte bank cycle would otherwise have all their teams on the same LDS banks.
        G = 64;
        while (4 * G * nseg > tile_nnz) G >>= 1;
    }
    switch (G) {
        case 1: tile_rows_g<MERGE, WG, 1>(cols, vals, x, seg, nr, r0, part, o, deferred, n_deferred, tid); break;
        case 2: tile_rows_g<MERGE, WG, 2>(cols, vals, x, seg, nr, r0, part, o, deferred, n_deferred, tid); break;
        case 4: tile_rows_g<MERGE, WG, 4>(cols, vals, x, seg, nr, r0, part, o, deferred, n_deferred, tid); break;
        case 8: tile_rows_g<MERGE, WG, 8>(cols, vals, x, seg, nr, r0, part, o, deferred, n_deferred, tid); break;
        case 16: tile_rows_g<MERGE, WG, 16>(cols, vals, x, seg, nr, r0, part, o, deferred, n_deferred, tid); break;
        case 32: tile_rows_g<MERGE, WG, 32>(cols, vals, x, seg, nr, r0, part, o, deferred, n_deferred, tid); break;
        default: tile_rows_g<MERGE, WG, 64>(cols, vals, x, seg, nr, r0, part, o, deferred, n_deferred, tid); break;
    }
}

}  // namespace
}  // namespace spmv
