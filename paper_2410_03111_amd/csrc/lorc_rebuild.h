// Internal: the rank-r rebuild K^T (or V^T) = B^T C^T of one wave -- two 32-column blocks of the output
// (RoPE partners for keys) times NPB blocks of 32 cached positions -- shared by the decode and prefill kernels.
#ifndef LORC_REBUILD_H_
#define LORC_REBUILD_H_

#include "lorc_device.h"

namespace lorc {

constexpr double kTwoPi = 6.283185307179586476925286766559;

// acc[a][pb] += sum_ks  Bt_a[32 x 16](ks) * C[16 x 32](pb, ks),  ks < nks.
//   bt       : descriptor of the packed factor tiles (global memory);  s0, s1 : byte offsets of the two column
//              blocks in it (wave-uniform; k-step stride 1 KiB);  lane_off : 16 * lane;
//   ckl      : this lane's pointer into the latent tile in LDS, tiled [pb][ks][64 lanes][8].
// Software pipeline without register copies: two operand sets (A, B) of PF k-steps each.  While set A feeds the
// matrix cores, set B is loaded PF k-steps ahead, then the roles swap; the latent operands are read from LDS
// one k-step ahead in the same ping-pong fashion.  Scheduling barriers keep every load inside the k-step that
// issues it; the loop body has no branches, prefetch indices are clamped instead of guarded.
// SWAP: the two operands of every product change places (their register layouts are the same), which transposes the
// accumulators: a lane then owns one output column and its registers walk the positions.
template <int NPB, int PF, bool SWAP = false>
__device__ __forceinline__ void rebuild_pair(f32x16 (&acc)[2][NPB], __amdgpu_buffer_rsrc_t bt, uint32_t s0, uint32_t s1,
                                             uint32_t lane_off, const uint16_t* ckl, int nks) {
  constexpr uint32_t frag_stride = 1024;
  auto lds_frags = [&](int ks, bf16x8* c) {
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) c[pb] = load_frag(ckl + (size_t)(pb * nks + ks) * 512);
  };
  auto kstep = [&](const bf16x8& a0, const bf16x8& a1, const bf16x8* c) {
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) {
      acc[0][pb] = SWAP ? mfma32(c[pb], a0, acc[0][pb]) : mfma32(a0, c[pb], acc[0][pb]);
      acc[1][pb] = SWAP ? mfma32(c[pb], a1, acc[1][pb]) : mfma32(a1, c[pb], acc[1][pb]);
    }
  };
  const int nks_main = nks & ~(2 * PF - 1);
  if (nks_main > 0) {
    bf16x8 A0[PF], A1[PF], B0[PF], B1[PF], c0[NPB], c1[NPB];
    // The first operand set is requested in the order in which it is consumed, and the compiler must keep that
    // order: the wait it places at the top of the loop has to hold for the entry path too, so a prologue that
    // loads k-step 0 last turns the loop's partial waits into a full drain on every trip.
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      A0[u] = buf_frag(bt, lane_off, s0 + (uint32_t)(u) * frag_stride);
      A1[u] = buf_frag(bt, lane_off, s1 + (uint32_t)(u) * frag_stride);
      __builtin_amdgcn_sched_barrier(0);
    }
    lds_frags(0, c0);
    for (int ks0 = 0; ks0 < nks_main; ks0 += 2 * PF) {
#pragma unroll
      for (int u = 0; u < PF; ++u) {  // k-steps ks0 .. ks0+PF-1 on set A; set B loads for ks0+PF ..
        const int ks = ks0 + u;
        B0[u] = buf_frag(bt, lane_off, s0 + (uint32_t)(ks + PF) * frag_stride);
        B1[u] = buf_frag(bt, lane_off, s1 + (uint32_t)(ks + PF) * frag_stride);
        if (u & 1) {
          lds_frags(ks + 1, c0);
          kstep(A0[u], A1[u], c1);
        } else {
          lds_frags(ks + 1, c1);
          kstep(A0[u], A1[u], c0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int u = 0; u < PF; ++u) {  // k-steps ks0+PF .. ks0+2PF-1 on set B; set A loads for the next round
        const int ks = ks0 + PF + u;
        const int nxt = ks + PF < nks ? ks + PF : nks - 1;
        A0[u] = buf_frag(bt, lane_off, s0 + (uint32_t)(nxt) * frag_stride);
        A1[u] = buf_frag(bt, lane_off, s1 + (uint32_t)(nxt) * frag_stride);
        const int ksn = ks + 1 < nks ? ks + 1 : nks - 1;
        if (u & 1) {
          lds_frags(ksn, c0);
          kstep(B0[u], B1[u], c1);
        } else {
          lds_frags(ksn, c1);
          kstep(B0[u], B1[u], c0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  for (int ks = nks_main; ks < nks; ++ks) {  // ranks that are not a multiple of 32 * PF: unpipelined tail
    bf16x8 c[NPB];
    lds_frags(ks, c);
    kstep(buf_frag(bt, lane_off, s0 + (uint32_t)(ks) * frag_stride), buf_frag(bt, lane_off, s1 + (uint32_t)(ks) * frag_stride), c);
  }
}

// Reduce an angle given in fp64 to (-pi, pi] and evaluate it in fp32.
__device__ __forceinline__ float2 cos_sin_reduced(double angle) {
  angle -= kTwoPi * rint(angle / kTwoPi);
  float s, c;
  sincosf((float)angle, &s, &c);
  return make_float2(c, s);
}

__device__ __forceinline__ double rope_theta(int i, int head_dim, float base) {
  return exp2(-(2.0 * (double)i / (double)head_dim) * log2((double)base));
}

}  // namespace lorc
#endif  // LORC_REBUILD_H_
