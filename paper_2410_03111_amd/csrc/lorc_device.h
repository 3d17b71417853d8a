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

// Buffer addressing for the loads that run next to the MFMA stream: a descriptor of the array (wave-uniform base,
// byte size; reads past the size return zero), a 32-bit lane offset and a scalar offset.  Such a load issues in a
// few cycles; one with 64-bit lane addresses holds the wave for about thirty, with its MFMAs queued behind it.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
// A pointer that is the same in every lane, moved to scalar registers whatever the compiler believes about it
// (a descriptor built from a pointer it takes for lane-dependent is applied once per distinct value, in a loop).
template <typename P>
__device__ __forceinline__ P* uniform_ptr(P* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<P*>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ bf16x8 buf_frag(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t wave_off) {
  return __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, wave_off, 0));
}
__device__ __forceinline__ uint16_t f16_bits(float f) { return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f)); }

// Cross-lane step of a reduction inside rows of 16 lanes, with DPP moves: quad swaps (STEP 0, 1), then row
// rotations by 4 and 8 (STEP 2, 3).  After the four steps every lane holds the result of its row.
template <int STEP>
__device__ __forceinline__ float half_wave_peer(float v) {
  static_assert(STEP >= 0 && STEP <= 3, "rows of 16 lanes");
  const int b = __builtin_bit_cast(int, v);
  if constexpr (STEP == 0) return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(b, 0xB1, 0xF, 0xF, false));   // lane ^ 1
  if constexpr (STEP == 1) return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(b, 0x4E, 0xF, 0xF, false));   // lane ^ 2
  if constexpr (STEP == 2) return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(b, 0x124, 0xF, 0xF, false));  // row_ror:4
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(b, 0x128, 0xF, 0xF, false));                           // row_ror:8
}

// A lane's value and the value of lane ^ 16 (row_pair) or lane ^ 32 (half_pair), in unspecified order, exchanged
// on the vector ALU by the row-swap instructions (no LDS round trip): for the last steps of reductions with a
// commutative operation.  (The elements of the builtins' result are copied to scalars before the bit cast: a bit
// cast applied to a vector element directly always takes element 0 with this toolchain.)
__device__ __forceinline__ float2 row_pair(float v) {
  const uint32_t a = __builtin_bit_cast(uint32_t, v);
  const auto r = __builtin_amdgcn_permlane16_swap(a, a, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  return make_float2(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}
__device__ __forceinline__ float2 half_pair(float v) {
  const uint32_t a = __builtin_bit_cast(uint32_t, v);
  const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  return make_float2(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}

// Index of the lane in its wavefront, from the hardware mask counters: two VALU ops, no register kept alive.
__device__ __forceinline__ int lane_id() { return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// Workgroup barrier for data exchanged through LDS only: waits for this wave's own LDS operations, then a bare
// barrier.  Unlike __syncthreads() it carries no memory fence, so global loads still in flight (prefetches into
// registers or straight into LDS) stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0); vector-memory and export counters untouched
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Immediate of s_waitcnt that waits until at most n vector-memory operations are outstanding and leaves the other
// counters alone (6-bit count split over bits 3:0 and 15:14).
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

__device__ __forceinline__ bf16x8 zero_frag() {
  u32x4 z = {0u, 0u, 0u, 0u};
  return __builtin_bit_cast(bf16x8, z);
}

}  // namespace lorc
#endif  // LORC_DEVICE_H_
