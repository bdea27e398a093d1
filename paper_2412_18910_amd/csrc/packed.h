// Shared device helpers of the bf16 MFMA path: vector typedefs, the bf16 hi/lo split and
// the "packed" activation layout (B operand of v_mfma_f32_16x16x32_bf16):
//   Xp[kt][h][slot] (16 bytes each), h = 0 hi / 1 lo, slot = row*4 + (k%32)/8, holding
//   k = kt*32 + (slot%4)*8 .. +7 of that row.  MFMA lane (k-octet g, row m) reads slot m*4+g:
//   the rows of a tile are contiguous (64 bytes each), so a block of r rows touches only
//   ceil(r/2) cache lines per tile.
// The decode step has one block of 16 rows (k-tile stride 128 pieces).  The dense prompt
// pass keeps RB row-blocks side by side, Xp[kt][rb][h][slot] (k-tile stride RB*128), so the
// row-blocks a workgroup multiplies are contiguous for every k-tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ae {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// x0,x1 -> packed bf16 hi (round to nearest even) and packed bf16 of the remainders
__device__ __forceinline__ void split2(float x0, float x1, uint32_t &hi, uint32_t &lo) {
  bf16x2 h;
  h[0] = (__bf16)x0;
  h[1] = (__bf16)x1;
  hi = __builtin_bit_cast(uint32_t, h);
  bf16x2 l;
  l[0] = (__bf16)(x0 - __uint_as_float(hi << 16));
  l[1] = (__bf16)(x1 - __uint_as_float(hi & 0xffff0000u));
  lo = __builtin_bit_cast(uint32_t, l);
}

// Store 4 consecutive k-values (k0 % 4 == 0) of row m (0..15) of one row-block into a packed
// activation buffer; Xp points at the row-block's first tile, kts = k-tile stride in pieces.
__device__ __forceinline__ void packed_store4(u32x4 *Xp, int m, int k0, float a, float b, float c, float d,
                                              size_t kts = 128) {
  uint32_t h0, l0, h1, l1;
  split2(a, b, h0, l0);
  split2(c, d, h1, l1);
  const int kt = k0 >> 5, g = (k0 & 31) >> 3, half = (k0 & 7) >> 2;
  u32x2 *ph = reinterpret_cast<u32x2 *>(Xp + (size_t)kt * kts + m * 4 + g) + half;
  u32x2 *pl = reinterpret_cast<u32x2 *>(Xp + (size_t)kt * kts + 64 + m * 4 + g) + half;
  *ph = u32x2{h0, h1};
  *pl = u32x2{l0, l1};
}

__device__ __forceinline__ f32x4 mfma_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

}  // namespace ae
