// Building blocks of the bf16 MFMA attention kernels (gfx950): 32x32x16 MFMA wrappers, the
// swizzled row-major LDS tile that every operand is staged in, and its two read patterns.
//
// MFMA v_mfma_f32_32x32x16_bf16, lane l (l32 = l % 32, g = l / 32):
//   A operand: row l32,  k-slots 8g .. 8g+7        B operand: column l32, k-slots 8g .. 8g+7
//   C/D:       column l32, 16 floats i -> row 8*(i/4) + 4g + i%4
//
// A tile is [rows][128 bf16] = 256 bytes per row = 16 chunks of 16 bytes; chunk c of row r is
// stored at chunk c ^ swz(r).  swz is a bijection on 16 consecutive rows (row-pattern reads of
// 16 lanes hit 16 different chunks) and moves rows r, r+1, r+2, r+3 to different 64-byte units
// (transposed reads of 4 rows x 32 bytes spread over the banks).
#pragma once
#include "common.h"

namespace lrsa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int TILE_ROW_BYTES = 256;  // head_dim 128 in bf16

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// byte offset of chunk `c` (16 bytes) of row `r`
__device__ __forceinline__ int tile_off(int r, int c) { return r * TILE_ROW_BYTES + ((c ^ swz(r)) << 4); }

// Operand with the tile's rows as MFMA rows/columns and head_dim as the contraction:
// lane takes row rb + l32, channels 16*kk + 8g .. +7  (one 16-byte LDS read).
__device__ __forceinline__ bf16x8 read_rows(const unsigned char* tile, int rb, int kk, int l32, int g) {
    return *reinterpret_cast<const bf16x8*>(tile + tile_off(rb + l32, kk * 2 + g));
}

// Operand with head_dim as MFMA rows and 16 tile rows as the contraction ("transposed" read):
// lane takes channel db*32 + l32 and the 8 k-slots of its half g, where slot j is tile row
// rb16 + 8*(j/4) + 4g + j%4 -- exactly the rows a C-layout accumulator hands over when its
// registers 8h .. 8h+7 are reused as the other operand.
// ds_read_b64_tr_b16 works per 16-lane group: lane i receives, as element e, element i%4 of the
// 8 bytes that lane 4e + i/4 of its group points at.  So source lane lam points at row
// 4g + lam/4 (+8 for the second read), channels dbase + 4*(lam%4) .. +3.
__device__ __forceinline__ bf16x8 read_cols(const unsigned char* tile, int rb16, int db, int lane) {
    const int lam = lane & 15, m = (lane >> 4) & 1, g = lane >> 5;
    const int ch = db * 32 + 16 * m + 4 * (lam & 3);  // first channel of the 8 bytes this lane points at
    const int r0 = rb16 + 4 * g + (lam >> 2);
    const int c = ch >> 3, within = (ch & 7) * 2;
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + tile_off(r0, c) + within));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + tile_off(r0 + 8, c) + within));
    union { s16x4 h[2]; bf16x8 v; } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
}

// registers i0 .. i0+7 of a C-layout accumulator as a bf16 operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int i0) {
    f32x8 t;
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = v[i0 + j];
    return __builtin_convertvector(t, bf16x8);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// position of stream entry j: the gather list (sink positions, then the flattened survivor
// lists) followed by the contiguous window that starts at cs
__device__ __forceinline__ int stream_pos(const Dims& D, const int32_t* idx_h, int j, int ng, int cs) {
    if (j < ng) return j < D.S ? j : idx_h[j - D.S];
    return cs + (j - ng);
}

}  // namespace lrsa
