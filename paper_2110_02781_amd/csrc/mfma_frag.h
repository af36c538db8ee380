// MFMA operand fragments out of LDS for v_mfma_f32_16x16x32_bf16: a lane (l16 = lane % 16, G = lane / 16) holds, for
// row / column l16 of its operand, the eight reduction elements 8*G .. 8*G+7 of a 32-element step.
#pragma once
#include "dev_common.h"

namespace ftp {

typedef float f4v_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s4v_t __attribute__((ext_vector_type(4)));

// operand stored with the reduction index contiguous: one 16-byte read
__device__ __forceinline__ bf16x8_t lds_frag(const bf16_t* p) {
  return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(p));
}
// operand stored with the reduction index as the ROW of a row-major LDS tile (leading dimension ld): rows r0 .. r0+7 of
// column c0 + l16 through the LDS transpose read.  Within a 16-lane group lane j hands in the address of row (j / 4)
// [+4 for the second read], columns c0 + 4 * (j % 4) .., and receives column c0 + j of four consecutive rows.
__device__ __forceinline__ bf16x8_t lds_frag_tr(const bf16_t* tile, int ld, int r0, int c0, int l16) {
  const bf16_t* p = tile + (r0 + (l16 >> 2)) * ld + c0 + 4 * (l16 & 3);
  const s4v_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4v_t __attribute__((address_space(3)))*)p);
  const s4v_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s4v_t __attribute__((address_space(3)))*)(p + 4 * ld));
  typedef short s8v_t __attribute__((ext_vector_type(8)));
  const s8v_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, v);
}

}  // namespace ftp
