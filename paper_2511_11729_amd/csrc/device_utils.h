// Small device-side helpers shared by the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "common.h"

namespace harli {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float bf2f(unsigned short b) { return __uint_as_float(((unsigned)b) << 16); }

// round-to-nearest-even float -> bfloat16 bits
__device__ __forceinline__ unsigned short f2bf(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}

__device__ __forceinline__ unsigned pack_bf2(float lo, float hi) {
  return (unsigned)f2bf(lo) | ((unsigned)f2bf(hi) << 16);
}

// the 8 bf16 values of a 16-byte word, widened
__device__ __forceinline__ void unpack8(const uint4& u, float* f) {
  f[0] = __uint_as_float(u.x << 16);
  f[1] = __uint_as_float(u.x & 0xffff0000u);
  f[2] = __uint_as_float(u.y << 16);
  f[3] = __uint_as_float(u.y & 0xffff0000u);
  f[4] = __uint_as_float(u.z << 16);
  f[5] = __uint_as_float(u.z & 0xffff0000u);
  f[6] = __uint_as_float(u.w << 16);
  f[7] = __uint_as_float(u.w & 0xffff0000u);
}

// Byte offset of a KV page in the slab: the pool's 2-D grid (chunk, then the
// (layer, K/V) block row, then the page column).
__device__ __forceinline__ size_t kv_page_off(const KvGeom& g, int page, int layer, int kv) {
  int c = page / g.pages_per_block;
  int s = page - c * g.pages_per_block;
  return (size_t)g.small_pool_bytes + (size_t)c * g.chunk_bytes + (size_t)(2 * layer + kv) * g.block_bytes +
         (size_t)s * g.page_bytes;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace harli

// ---- 16-bit element abstraction of the finetune unit -------------------------------------------
// The finetune kernels compute on IEEE half operands: with bf16 operands (8 significand bits,
// unit round-off 2^-8) every GEMM input on the path from dY to an adapter gradient adds ~1.6e-3
// of relative noise, and at hidden 4096 the layer gradients end up 2e-2 away from the fp64
// oracle; half (11 bits) is 8x tighter at the same MFMA rate.  Frozen weights stored as bf16
// convert to half exactly over half's normal range.
namespace harli {
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

__device__ __forceinline__ unsigned short f2h(float f) {
  f = fminf(fmaxf(f, -65504.f), 65504.f);
  return __builtin_bit_cast(unsigned short, (_Float16)f);
}
__device__ __forceinline__ float h2f(unsigned short h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ __forceinline__ unsigned pack_h2(float lo, float hi) { return (unsigned)f2h(lo) | ((unsigned)f2h(hi) << 16); }
__device__ __forceinline__ void unpack8h(const uint4& u, float* f) {
  f[0] = h2f((unsigned short)(u.x & 0xffffu)); f[1] = h2f((unsigned short)(u.x >> 16));
  f[2] = h2f((unsigned short)(u.y & 0xffffu)); f[3] = h2f((unsigned short)(u.y >> 16));
  f[4] = h2f((unsigned short)(u.z & 0xffffu)); f[5] = h2f((unsigned short)(u.z >> 16));
  f[6] = h2f((unsigned short)(u.w & 0xffffu)); f[7] = h2f((unsigned short)(u.w >> 16));
}
}  // namespace harli
