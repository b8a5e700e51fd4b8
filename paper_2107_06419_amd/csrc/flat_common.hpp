// Shared device-side vocabulary of the gfx950 attention kernels: vector types, the CDNA4 matrix
// instructions that both contractions run on, and the lane <-> matrix-element maps they imply.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flat {

typedef __bf16 bf16;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

// v_mfma_f32_32x32x16_bf16:  D[32x32] += A[32x16] * B[16x32], one wavefront.
//   A operand: lane l holds row (l % 32), contraction indices 8*(l/32) .. 8*(l/32)+7
//   B operand: lane l holds column (l % 32), contraction indices 8*(l/32) .. 8*(l/32)+7
//   C/D:       lane l holds column (l % 32); register r (0..15) is row 8*(r/4) + 4*(l/32) + (r%4)
__device__ __forceinline__ floatx16 mfma_bf16_32x32x16(bf16x8 a, bf16x8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// v_mfma_f32_32x32x2_f32:  D[32x32] += A[32x2] * B[2x32].
//   A: lane l holds row (l % 32), contraction index (l / 32);  B: column (l % 32), index (l / 32);
//   C/D as above.
__device__ __forceinline__ floatx16 mfma_f32_32x32x2(float a, float b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Row of the 32x32 accumulator tile held in register r of a lane in wave half `half` (= lane / 32).
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// ds_read_b64_tr_b16: within each group of 16 lanes, lane 4*j + q supplies the address of four
// consecutive 16-bit elements (row j, columns 4q..4q+3 of a 4 x 16 block); lane i receives the four
// elements of column i, one from each row j = 0..3.  It turns a row-major [contraction][column]
// tile in LDS into the "contraction index contiguous per lane" form an MFMA operand needs.
__device__ __forceinline__ bf16x4 lds_read_tr16(const void* lds_ptr) {
    typedef short4v __attribute__((address_space(3))) * lds_s4_ptr;
    short4v t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(uintptr_t)lds_ptr);
    return __builtin_bit_cast(bf16x4, t);
}

// Same, from a 32-bit LDS byte address.
__device__ __forceinline__ bf16x4 lds_read_tr16_at(int lds_addr) {
    typedef short4v __attribute__((address_space(3))) * lds_s4_ptr;
    short4v t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr)(uintptr_t)(uint32_t)lds_addr);
    return __builtin_bit_cast(bf16x4, t);
}

__device__ __forceinline__ bf16x8 concat(bf16x4 lo, bf16x4 hi) {
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    floatx2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // v_cvt_pk_bf16_f32, RNE
}

// Combine a value across the two halves of a wavefront (lanes l and l ^ 32).  v_permlane32_swap
// exchanges the upper half of one register with the lower half of another; fed the same value
// twice it returns {x[l % 32], x[l % 32 + 32]} in some order, and max / + do not care which.
__device__ __forceinline__ float halves_max(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
__device__ __forceinline__ float halves_sum(float x) {
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}

// XCD-aware remap of a 1-D grid.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs;
// this makes each XCD own a contiguous range of logical ids, so that the workgroups sharing one
// head's K/V also share one L2.
__device__ __forceinline__ int xcd_logical_block(int bid, int blocks_per_xcd) {
    return (bid & 7) * blocks_per_xcd + (bid >> 3);
}

}  // namespace flat
