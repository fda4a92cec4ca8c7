// Device-side helpers shared by the kernel files: storage types, cross-lane sums, the alpha/beta
// epilogue.  Everything has internal linkage.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace spmv {
namespace {

constexpr int kWG = 256;   // threads per workgroup = 4 wavefronts of 64
constexpr int kXcds = 8;   // accelerator dies; workgroup ids are dealt round-robin over them

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct F32 {
    using elem = float;
    static constexpr int VEC = 4;  // elements per 128-bit load of vals
};
struct BF16 {
    using elem = uint16_t;
    static constexpr int VEC = 8;
};

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(uint16_t b) { return __uint_as_float(static_cast<uint32_t>(b) << 16); }

// ------------------------------------------------------------------------------------------
// Cross-lane sums over aligned groups of G lanes; every lane of the group receives the total.
// Steps 1 and 2 permute inside a quad, 4 and 8 mirror a half row / a row of 16 (valid because
// the lanes being mirrored already agree), 16 swaps inside 32 lanes through the LDS crossbar
// (ds_swizzle, no memory touched), 32 swaps the two wave halves (v_permlane32_swap).
// All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float add_xor1(float v) { return v + dpp_move<0xB1>(v); }    // quad_perm [1,0,3,2]
__device__ __forceinline__ float add_xor2(float v) { return v + dpp_move<0x4E>(v); }    // quad_perm [2,3,0,1]
__device__ __forceinline__ float add_half_mirror(float v) { return v + dpp_move<0x141>(v); }
__device__ __forceinline__ float add_row_mirror(float v) { return v + dpp_move<0x140>(v); }
__device__ __forceinline__ float add_swap16(float v) {
    return v + __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));  // and 0x1f, xor 0x10
}
__device__ __forceinline__ float add_swap32(float v) {
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int G>
__device__ __forceinline__ float group_sum(float v) {
    if constexpr (G >= 2) v = add_xor1(v);
    if constexpr (G >= 4) v = add_xor2(v);
    if constexpr (G >= 8) v = add_half_mirror(v);
    if constexpr (G >= 16) v = add_row_mirror(v);
    if constexpr (G >= 32) v = add_swap16(v);
    if constexpr (G >= 64) v = add_swap32(v);
    return v;
}

// Same with G known only at run time (uniform over the workgroup).
__device__ __forceinline__ float group_sum_rt(float v, int G) {
    if (G >= 2) v = add_xor1(v);
    if (G >= 4) v = add_xor2(v);
    if (G >= 8) v = add_half_mirror(v);
    if (G >= 16) v = add_row_mirror(v);
    if (G >= 32) v = add_swap16(v);
    if (G >= 64) v = add_swap32(v);
    return v;
}

__device__ __forceinline__ float epilogue(float acc, float alpha, float beta, const float* y, int r) {
    return beta == 0.f ? alpha * acc : alpha * acc + beta * y[r];
}

// Workgroup ids are handed to the 8 dies round-robin (id % 8).  Each die has its own L2, so
// give die j one contiguous run of logical tiles: its x window then lives in one L2.
__device__ __forceinline__ int xcd_remap(int bid, int nb) {
    const int q = nb / kXcds, r = nb % kXcds;
    const int die = bid % kXcds, slot = bid / kXcds;
    return die * q + (die < r ? die : r) + slot;
}

inline int ceil_div(int64_t a, int64_t b) { return static_cast<int>((a + b - 1) / b); }

}  // namespace
}  // namespace spmv
