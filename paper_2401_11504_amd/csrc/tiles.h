// MFMA tile helpers shared by the GEMM and attention kernels (gfx950).
//
// v_mfma_f32_32x32x16_bf16 operand layout (lane = 32*g + l32):
//   A fragment: row  i = l32, contraction slots k = 8g .. 8g+7   (8 bf16 = 16 bytes per lane)
//   B fragment: col  j = l32, contraction slots k = 8g .. 8g+7
//   D fragment: col  j = l32, rows i = 8*(v/4) + 4g + v%4 for v = 0..15
// Because the contraction is a sum, any permutation of the 16 slots is allowed as long as A and B
// use the same one.  A D fragment reused as a B operand (keeping j) supplies, for registers
// v = 8h .. 8h+7, the slot order  i = 16h + {4g..4g+3, 8+4g..8+4g+3}; the A operand is then read
// as two 4-slot pieces at i = 16h+4g and 16h+8+4g (load_a_tr below).
#pragma once
#include "common.h"

#define BK 64
#define LS 72  // LDS row stride (elements) of a 64-wide K-contiguous bf16 tile read with 16-byte accesses

__device__ __forceinline__ f32x16_t mfma32(bf16x8_t a, bf16x8_t b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16_t zero16() {
    f32x16_t z;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v] = 0.f;
    return z;
}

// A operand for a D-fragment-as-B product (contraction slots 16h + {4g..4g+3, 8+4g..8+4g+3}, see the top of this
// file) taken from the tile as it lies in memory, [k][n] row-major with n contiguous, by the LDS transpose read of
// gfx950 (ds_read_b64_tr_b16): within each group of 16 lanes, lane 4q + c receives element c of the four 8-byte rows
// that lanes q, q + 4, q + 8, q + 12 of the group point at.  Lane q + 4e therefore points at row k0 + e, columns
// n0 + 4q .. 4q + 3, and lane 4q + c ends up with column n0 + 4q + c of rows k0 .. k0 + 3: four consecutive contraction
// slots of one operand row, which is what the matrix unit wants.  Lane groups 0 / 1 cover columns n0 .. 15 /
// n0 + 16 .. 31 (l32), groups 2 / 3 the same columns for g = 1.  Used for both operands of a product, the slot
// permutation cancels, so the same read serves ordinary P^T Q products (gemm_tn).
// tr_lane_offset: the lane's share of the address, (4 g + e) * ld + 16 (G & 1) + 4 q, in elements.
#define LTR(DH) ((DH) + 32)  // row stride of a tile read this way: 4 consecutive rows x 64 bytes fall into 4 distinct bank ranges
__device__ __forceinline__ int tr_lane_offset(int lane, int ld) {
    const int G = lane >> 4, s = lane & 15, q = s & 3, e = s >> 2;
    return (4 * (G >> 1) + e) * ld + 16 * (G & 1) + 4 * q;
}
typedef __bf16 bf16x4v_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8_t load_a_tr(const bf16_t* tile, int ld, int lane_off, int n0, int k16) {
    typedef __attribute__((address_space(3))) bf16x4v_t* lds_ptr_t;
    const bf16_t* p = tile + lane_off + k16 * ld + n0;
    const bf16x4v_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr_t)(p));
    const bf16x4v_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_ptr_t)(p + 8 * ld));
    bf16x8_t a;
    a[0] = lo[0]; a[1] = lo[1]; a[2] = lo[2]; a[3] = lo[3];
    a[4] = hi[0]; a[5] = hi[1]; a[6] = hi[2]; a[7] = hi[3];
    return a;
}

// registers v = 8h .. 8h+7 of a D fragment, rounded to bf16, as a B operand
__device__ __forceinline__ bf16x8_t pack_b_from_d(const float* d, int h) {
    bf16x8_t b;
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = (__bf16)d[8 * h + e];
    return b;
}
