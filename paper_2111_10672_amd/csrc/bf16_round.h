// float32 -> bfloat16, round to nearest with ties to even: gfx950 converts a pair in one instruction
// (v_cvt_pk_bf16_f32), which is what the conversion below compiles to.  Bit for bit the result of adding
// 0x7FFF + (bit 16) to the float32 pattern and keeping the upper half, for every finite input; a NaN stays a NaN.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace spb {

__device__ __forceinline__ uint32_t bf16_pack2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ uint16_t bf16_round(float v) { return (uint16_t)(bf16_pack2(v, 0.f) & 0xFFFFu); }

}  // namespace spb
