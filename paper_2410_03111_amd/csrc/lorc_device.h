// Internal: device-side helpers shared by the HIP kernels (vector types, matrix-core wrappers, bf16 casts).
#ifndef LORC_DEVICE_H_
#define LORC_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lorc_layout.h"

namespace lorc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// D[32x32] += A[32x16] B[16x32].  Lane l supplies A[m = l%32][k = 8*(l/32) .. +7] and
// B[k = 8*(l/32) .. +7][n = l%32]; it receives D[m = 8*(j/4) + 4*(l/32) + j%4][n = l%32] in register j.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Same op with fp16 operands (11-bit significands): used where bf16 rounding of an intermediate would cost
// accuracy (scores), while the data read from memory stays bf16.
__device__ __forceinline__ f32x16 mfma32_f16(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// Row of the 32x32 accumulator block held in register j by a lane of half hf = lane / 32.
__device__ __forceinline__ constexpr int acc_row(int j, int hf) { return 8 * (j >> 2) + 4 * hf + (j & 3); }

__device__ __forceinline__ uint16_t bf16_bits(float f) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f)); }
__device__ __forceinline__ float bf16_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ bf16x8 load_frag(const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ f16x8 load_frag_f16(const uint16_t* p) { return *reinterpret_cast<const f16x8*>(p); }
__device__ __forceinline__ uint16_t f16_bits(float f) { return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f)); }

__device__ __forceinline__ bf16x8 zero_frag() {
  u32x4 z = {0u, 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, z);
}

}  // namespace lorc
#endif  // LORC_DEVICE_H_
