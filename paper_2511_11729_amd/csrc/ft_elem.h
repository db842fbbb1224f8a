// 16-bit element type of the finetune unit's activations, gradients and weight copies.
// It is IEEE half: with 10 mantissa bits the unit meets its parity bar at hidden 4096, which bfloat16's 7 bits do not;
// the price is the narrower exponent, which the GEMM epilogues guard (a clamped output raises the context's error flag)
// and the backward pass avoids by scaling dY to a fixed magnitude.
#pragma once
#include "device_utils.h"

namespace harli {
__device__ __forceinline__ unsigned short F2E(float f) { return f2h(f); }
__device__ __forceinline__ float E2F(unsigned short e) { return h2f(e); }
__device__ __forceinline__ unsigned PACK2(float lo, float hi) { return pack_h2(lo, hi); }
__device__ __forceinline__ void UNPACK8(const uint4& u, float* f) { unpack8h(u, f); }

// The same stores with a range check: `over` turns true when a value lay beyond the element's range (the store clamps it)
// or was not a number.  A kernel ends with elem_flag(over, flag), which raises bit 8 of the context's error word, so
// that harli_ctx_check reports activations or gradients that half cannot hold instead of silently clamped results.
__device__ __forceinline__ bool elem_over(float f) { return !(fabsf(f) <= 65504.f); }
__device__ __forceinline__ unsigned short F2EG(float f, bool& over) {
  over |= elem_over(f);
  return F2E(f);
}
__device__ __forceinline__ unsigned PACK2G(float lo, float hi, bool& over) {
  over = over || elem_over(lo) || elem_over(hi);
  return PACK2(lo, hi);
}
__device__ __forceinline__ void elem_flag(bool over, int* flag) {
  if (over && flag) atomicOr(flag, 8);
}

// host-side rounding of a float to the compute element (round to nearest even), for small tables built at set-up
inline unsigned short host_to_elem(float f) {
  const _Float16 h = static_cast<_Float16>(f);
  unsigned short u;
  __builtin_memcpy(&u, &h, 2);
  return u;
}
}  // namespace harli
