// Device-side helpers shared by the gfx950 kernels: vector types, MFMA wrappers, LDS
// swizzles and the cross-half exchange of a 64-lane wavefront.
//
// MFMA orientation used everywhere in this library ("transposed" flash attention):
//   S^T[key][query] = K_tile (A operand) x Q^T (B operand)
//   O^T[d][query]   = V^T    (A operand) x P^T (B operand)
// With v_mfma_f32_32x32x16_bf16 lane l holds, of A, row (l%32) and 8 consecutive
// contraction indices starting at 8*(l/32); of B, column (l%32) and the same 8 contraction
// indices; of the 32x32 result, column (l%32) and rows 8*(r/4) + 4*(l/32) + r%4 for
// r = 0..15.  So every lane owns ONE query column: softmax statistics are per-lane
// scalars, and only one exchange between the two 32-lane halves is needed per row.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pulsecol {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

#define PULSECOL_LDS __attribute__((address_space(3)))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Row of the 32x32 MFMA result held in accumulator register r by a lane of half h.
__device__ __forceinline__ int acc_row(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// max / sum of a per-lane value with the lane 32 positions away (same query column).
__device__ __forceinline__ float half_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
    return fmaxf(__int_as_float(r[0]), __int_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
    return __int_as_float(r[0]) + __int_as_float(r[1]);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// 16-byte pieces of a K/V row are stored in LDS at piece ^ swizzle(row) so that
//  - K: 16 consecutive rows read at one logical piece (ds_read_b128) hit 16 distinct pieces;
//  - V: the transposing 8-byte reads (ds_read_b64_tr_b16) of 4 consecutive rows x 4
//       consecutive pieces hit 16 distinct pieces, and 8 distinct ones per 16 lanes.
template <int PIECES>
__device__ __forceinline__ int swizzle_k(int row) { return row & (PIECES - 1); }
template <int PIECES>
__device__ __forceinline__ int swizzle_v(int row) { return (((row & 3) << 2) | (row & 2)) & (PIECES - 1); }

// Transposing LDS read: within each group of 16 lanes, lane j supplies the address of 4
// consecutive bf16 (row j/4, columns 4*(j%4)..+3 of a 4x16 block); lane i receives column i
// of that block, i.e. the 4 row values.
__device__ __forceinline__ bf16x4 lds_read_tr(const void* generic_lds_ptr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((PULSECOL_LDS bf16x4*)generic_lds_ptr);
}

// Workgroup id -> (batch*head, query block) such that all query blocks of one head run on
// one XCD (hardware deals consecutive workgroup ids round-robin over the 8 XCDs, each with
// its own L2): the K/V rows a head gathers are then fetched into a single L2.
// The grid holds nqb * bh_pad workgroups, bh_pad = bh rounded up to a multiple of 8;
// returns false for the padding workgroups.
__device__ __forceinline__ bool xcd_tile(int wg, int nqb, int bh, int* out_bh, int* out_qb) {
    const int xcd = wg & 7;
    const int slot = wg >> 3;
    const int hh = slot / nqb;
    *out_qb = slot - hh * nqb;
    *out_bh = hh * 8 + xcd;
    return *out_bh < bh;
}

}  // namespace pulsecol
