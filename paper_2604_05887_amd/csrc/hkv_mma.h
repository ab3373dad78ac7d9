// 32x32 matrix-core tile update shared by the prefill kernels that contract query rows with key rows
// (window scoring of the compress pass, text-centric attention of the head classification).
#pragma once

#include "hkv_device.h"

namespace hkv {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

// One 32x32 tile update over a 16-byte piece of the head dimension.
// a: this lane's piece of key row (lane % 32); b: this lane's piece of query row (lane % 32);
// lanes 0-31 hold the first half of the piece pair, lanes 32-63 the second (same split in a and b).
__device__ __forceinline__ floatx16 mma_piece(const uint4& a, const uint4& b, floatx16 c, bf16_t) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ floatx16 mma_piece(const uint4& a, const uint4& b, floatx16 c, float) {
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(bits_to_float(a.x), bits_to_float(b.x), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(bits_to_float(a.y), bits_to_float(b.y), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(bits_to_float(a.z), bits_to_float(b.z), c, 0, 0, 0);
  c = __builtin_amdgcn_mfma_f32_32x32x2f32(bits_to_float(a.w), bits_to_float(b.w), c, 0, 0, 0);
  return c;
}

}  // namespace hkv
