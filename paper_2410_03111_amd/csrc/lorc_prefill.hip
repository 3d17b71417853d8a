// Causal prefill attention over the latent cache (Eq. 1 with the mask j <= i; GQA of Section 4.3; RoPE applied
// to rebuilt keys as in the Appendix on the adjusted position embedding).
//
// Two launches per call:
//   rebuild : one workgroup per (sequence, 64-position page).  K^T = B_k^T C_k^T per KV head on the matrix
//             cores (same pipeline as decode), rotated in registers, written once to scratch as fp16
//             K_rot[seq][pos][n]; then the page's V latents are re-tiled through LDS (their cache tiling is
//             made for contraction over positions, the rebuild contracts over the latent index) and
//             V^T = B_v^T C_v^T is written as fp16 Vt[seq][n][pos'] with positions permuted inside groups of 16
//             into the order in which the attention kernel's P accumulators serve as operands.
//   attend  : flash-style causal attention.  One workgroup per (sequence, 64-query block, KV head); each wave
//             owns one query head of the group.  S^T = K Q^T so that a lane owns one query column: row maxima
//             and sums need a single cross-lane exchange, the P^T accumulators are re-used in place as the
//             B operand of O^T += V^T P^T, and rescaling is a per-lane scalar.
#include <type_traits>

#include "lorc_device.h"
#include "lorc_kernels.h"
#include "lorc_rebuild.h"

namespace lorc {

constexpr float kNegInfP = -__builtin_huge_valf();


// V^T storage order inside a group of 16 positions: slot 8*hf + e holds position 8*(e/4) + 4*hf + e%4 (position q sits
// in slot 8*((q>>2)&1) + 4*(q>>3) + (q&3)), so that the 8 positions a lane of a value operand needs are 16 bytes.

// ------------------------------------------------------------------------------------------------ rebuild
// Ranks above kRebuildPartSteps * 16 do not fit LDS at once: the rank is then walked in parts (the accumulators of a
// pass stay in registers across the parts; every pass copies the parts again).
constexpr int kRebuildPartSteps = 64;  // k-steps of 16 latents per part: 64 positions x 1024 x 2 B = 128 KiB

template <int HD>
__global__ __launch_bounds__(256, 1) void prefill_rebuild_kernel(PrefillParams p) {
  constexpr int NPB = 2, T = 64, HALF = HD / 2, PF = 4;
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int seq = blockIdx.x / p.tiles_per_seq, tile = blockIdx.x % p.tiles_per_seq;
  const int len = p.cu_seqlens[seq + 1] - p.cu_seqlens[seq];
  const int pos0 = tile * T;
  if (pos0 >= len) return;
  const int r_k = p.r_k, r_v = p.r_v, n = p.h_kv * HD;
  const int rmax = r_k > r_v ? r_k : r_v;
  const int part_cap = (rmax >> 4) < kRebuildPartSteps ? (rmax >> 4) : kRebuildPartSteps;  // k-steps the LDS tile holds
  uint16_t* ck = reinterpret_cast<uint16_t*>(smem);
  float2* cs_base = reinterpret_cast<float2*>(smem + (size_t)T * part_cap * 16 * 2);

  const int id = p.block_table[(size_t)seq * p.max_pages + tile];
  const bool page_ok = id >= 0 && id < p.n_pages;
  const uint16_t* page = p.cache + (size_t)(page_ok ? id : 0) * p.page_elems;

  // k-steps [ks0, ks0 + steps) of the page's K latents -> LDS, tiled [position block][k-step][64 lanes][8] (a linear
  // copy per position block: the page tiling is the operand tiling)
  auto copy_k_part = [&](int ks0, int steps) {
    const int nks = r_k >> 4;
    const u32x4* src = reinterpret_cast<const u32x4*>(page);
    u32x4* dst = reinterpret_cast<u32x4*>(ck);
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int pb = 0; pb < NPB; ++pb)
      for (int c = tid; c < steps * 64; c += 256)
        dst[(size_t)pb * steps * 64 + c] = page_ok ? src[((size_t)pb * nks + ks0) * 64 + c] : z;
  };
  // V latents [16 ks0, 16 (ks0 + steps)): cache tile (lane = latent index, 8 consecutive positions) -> LDS in the
  // K-style tiling (lane = position, 8 consecutive latent indices); slots past the sequence are zeroed.
  auto copy_v_part = [&](int ks0, int steps) {
    const uint16_t* vpart = page + (size_t)kPage * r_k;
    const int f0 = (ks0 >> 1) * 4, f1 = ((ks0 + steps) >> 1) * 4;  // blocks of 32 latent indices x 16 positions
    for (int f = f0 + w; f < f1; f += 4) {
      const int nb = f >> 2, kp = f & 3;
      const u32x4 raw = page_ok ? *reinterpret_cast<const u32x4*>(vpart + ((size_t)f * 64 + lane) * 8) : u32x4{0u, 0u, 0u, 0u};
      const int j = nb * 32 + l32 - 16 * ks0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int slot = kp * 16 + 8 * hf + e;
        uint16_t v = (uint16_t)(raw[e >> 1] >> (16 * (e & 1)));
        if (pos0 + slot >= len) v = 0;
        ck[k_index(16 * steps, slot, j)] = v;
      }
    }
  };

  const int fbase = HD == 128 ? 32 * (w & 1) : 0;
  float cl[16], sl[16];
#pragma unroll
  for (int jj = 0; jj < 16; ++jj) {
    const float th = (float)rope_theta(fbase + acc_row(jj, hf), HD, p.rope_base);
    sincosf((float)l32 * th, &sl[jj], &cl[jj]);
  }
  if (tid < NPB * HALF) cs_base[tid] = cos_sin_reduced((double)(pos0 + 32 * (tid / HALF)) * rope_theta(tid % HALF, HD, p.rope_base));

  const int n_tasks = n / 64;
  const int n_pass = (n_tasks + 3) >> 2;
  // One pass = one task per wave (two column blocks x two position blocks), accumulated over the rank parts.
  auto rebuild_pass = [&](f32x16 (&acc)[2][NPB], bool active, int cb0, int cb1, const uint16_t* factor, int rank, bool keys,
                          bool first_pass) {
    const int nks = rank >> 4;
    const int n_parts = (nks + part_cap - 1) / part_cap;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[a][pb][j] = 0.f;
    for (int part = 0; part < n_parts; ++part) {
      const int ks0 = part * part_cap, steps = nks - ks0 < part_cap ? nks - ks0 : part_cap;
      if (n_parts > 1 || first_pass) {  // a rank that fits stays in LDS for all passes
        __syncthreads();
        if (keys) copy_k_part(ks0, steps);
        else copy_v_part(ks0, steps);
        __syncthreads();
      }
      if (active) {  // values with the operands swapped: a lane then owns a column of V^T and 8 consecutive storage slots
        if (keys)
          rebuild_pair<NPB, PF, false>(acc, make_rsrc(factor, (uint32_t)n * rank * 2u), (uint32_t)(cb0 * nks + ks0) * 1024u,
                                       (uint32_t)(cb1 * nks + ks0) * 1024u, (uint32_t)lane * 16u, ck + (size_t)lane * 8, steps);
        else
          rebuild_pair<NPB, PF, true>(acc, make_rsrc(factor, (uint32_t)n * rank * 2u), (uint32_t)(cb0 * nks + ks0) * 1024u,
                                      (uint32_t)(cb1 * nks + ks0) * 1024u, (uint32_t)lane * 16u, ck + (size_t)lane * 8, steps);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  uint16_t* krot = p.krot + ((size_t)seq * p.lp + pos0) * n;
  for (int ps = 0; ps < n_pass; ++ps) {
    const int task = ps * 4 + w;
    const bool active = task < n_tasks;
    const int g = HD == 128 ? task >> 1 : task, wh = HD == 128 ? task & 1 : 0;
    const int cb0 = HD == 128 ? g * 4 + wh : g * 2, cb1 = cb0 + (HD == 128 ? 2 : 1);
    f32x16 acc[2][NPB];
    rebuild_pass(acc, active, cb0, cb1, p.bk, r_k, true, ps == 0);
    if (active) {
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb) {
        uint16_t* row = krot + (size_t)(pb * 32 + l32) * n + g * HD + fbase;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint16_t lo[4], hi[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int jj = 4 * q4 + i;
            const float2 cb = cs_base[pb * HALF + fbase + acc_row(jj, hf)];
            const float cA = cb.x * cl[jj] - cb.y * sl[jj];
            const float sA = cb.y * cl[jj] + cb.x * sl[jj];
            const float x = acc[0][pb][jj], y = acc[1][pb][jj];
            lo[i] = f16_bits(x * cA - y * sA);
            hi[i] = f16_bits(y * cA + x * sA);
          }
          const int c0 = 8 * q4 + 4 * hf;  // first of 4 consecutive head-dim coordinates
          const u32x2 plo = {(uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16)};
          const u32x2 phi = {(uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16)};
          *reinterpret_cast<u32x2*>(row + c0) = plo;
          *reinterpret_cast<u32x2*>(row + c0 + HALF) = phi;
        }
      }
    }
  }

  uint16_t* vt = p.vt + (size_t)seq * n * p.lp + pos0;
  for (int ps = 0; ps < n_pass; ++ps) {
    const int task = ps * 4 + w;
    const bool active = task < n_tasks;
    const int g = HD == 128 ? task >> 1 : task, wh = HD == 128 ? task & 1 : 0;
    const int cb0 = HD == 128 ? g * 4 + wh : g * 2, cb1 = cb0 + (HD == 128 ? 2 : 1);
    f32x16 acc[2][NPB];
    rebuild_pass(acc, active, cb0, cb1, p.bv, r_v, false, ps == 0);
    if (active) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
          // accumulator rows = positions acc_row(jj, hf) of the block, lane = column: registers 8 u .. 8 u + 7 are the
          // positions that the storage order keeps in slots 8 hf .. 8 hf + 7 of the block's u-th group of 16
          uint16_t* dst = vt + (size_t)(g * HD + fbase + a * HALF + l32) * p.lp + pb * 32 + 8 * hf;
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            uint32_t w4[4];
#pragma unroll
            for (int c = 0; c < 4; ++c)
              w4[c] = (uint32_t)f16_bits(acc[a][pb][8 * u + 2 * c]) | ((uint32_t)f16_bits(acc[a][pb][8 * u + 2 * c + 1]) << 16);
            *reinterpret_cast<u32x4*>(dst + 16 * u) = u32x4{w4[0], w4[1], w4[2], w4[3]};
          }
        }
    }
  }
}

// ------------------------------------------------------------------------------------------------ uncompressed layers
// The rebuild launch for a layer whose pages hold the keys and values themselves (rank = n, no read-side factors):
// nothing to multiply.  One workgroup per (sequence, page); wave w takes position block w % 2 and the KV heads of
// parity w / 2.  Keys: a lane of a K operand block holds one position and 8 consecutive head-dim coordinates, its
// rotation partner the same lane and element four blocks further; rotated (angles reduced in fp64, hardware sine /
// cosine in turns), rounded to fp16 and written as 16-byte pieces of K_rot rows.  Values: a lane of a V operand
// block holds one column and 8 consecutive positions, which go to V^T in the permuted order the attention kernel
// reads (two 8-byte pieces).  Slots past the sequence and pages that are not cached are written as zeros.
__global__ __launch_bounds__(256, 2) void prefill_plain_gather_kernel(PrefillParams p) {
  constexpr int HD = 128, T = 64;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int seq = blockIdx.x / p.tiles_per_seq, tile = blockIdx.x % p.tiles_per_seq;
  const int len = p.cu_seqlens[seq + 1] - p.cu_seqlens[seq];
  const int pos0 = tile * T;
  if (pos0 >= len) return;
  const int n = p.h_kv * HD, pb = w & 1;
  const int id = p.block_table[(size_t)seq * p.max_pages + tile];
  const bool page_ok = id >= 0 && id < p.n_pages;
  const uint16_t* page = uniform_ptr(p.cache + (size_t)(page_ok ? id : 0) * p.page_elems);
  const __amdgpu_buffer_rsrc_t pr = make_rsrc(page, page_ok ? (uint32_t)kPage * 2u * n * 2u : 0u);  // K part, then V part

  float cs_c[4][8], cs_s[4][8];
  {
    const double pos = (double)(pos0 + 32 * pb + l32);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const double turns = pos * p.rope_tab[16 * kb + 8 * hf + e] * 0.15915494309189533576888;
        const float fr = (float)(turns - rint(turns));
        cs_c[kb][e] = __builtin_amdgcn_cosf(fr);
        cs_s[kb][e] = __builtin_amdgcn_sinf(fr);
      }
  }
  const int blocks_per_row = n >> 4;
  const bool k_live = pos0 + 32 * pb + l32 < len;
  uint16_t* krow = p.krot + ((size_t)seq * p.lp + pos0 + 32 * pb + l32) * n + 8 * hf;
  for (int g = w >> 1; g < p.h_kv; g += 2) {
    u32x4 raw[8];
#pragma unroll
    for (int kb = 0; kb < 8; ++kb)
      raw[kb] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(pr, lane * 16, (pb * blocks_per_row + g * 8 + kb) * 1024, 0));
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      uint16_t lo[8], hi[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = bf16_to_float((uint16_t)(raw[kb][e >> 1] >> (16 * (e & 1))));
        const float y = bf16_to_float((uint16_t)(raw[kb + 4][e >> 1] >> (16 * (e & 1))));
        lo[e] = k_live ? f16_bits(x * cs_c[kb][e] - y * cs_s[kb][e]) : (uint16_t)0;
        hi[e] = k_live ? f16_bits(y * cs_c[kb][e] + x * cs_s[kb][e]) : (uint16_t)0;
      }
      u32x4 plo, phi;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        plo[c] = (uint32_t)lo[2 * c] | ((uint32_t)lo[2 * c + 1] << 16);
        phi[c] = (uint32_t)hi[2 * c] | ((uint32_t)hi[2 * c + 1] << 16);
      }
      *reinterpret_cast<u32x4*>(krow + g * HD + 16 * kb) = plo;
      *reinterpret_cast<u32x4*>(krow + g * HD + 16 * kb + 64) = phi;
    }
  }
  // values: operand block (jb, kp) = columns 32 jb .. +31, positions 16 kp .. +15; wave w takes the blocks jb = w mod 4
  const uint32_t v_base = (uint32_t)kPage * n * 2u;
  uint16_t* vt = p.vt + (size_t)seq * n * p.lp + pos0;
  for (int jb = w; jb < (n >> 5); jb += 4) {
    u32x4 raw[4];
#pragma unroll
    for (int kp = 0; kp < 4; ++kp)
      raw[kp] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(pr, lane * 16, v_base + (jb * 4 + kp) * 1024, 0));
    const int col = jb * 32 + l32;
#pragma unroll
    for (int kp = 0; kp < 4; ++kp) {
      uint16_t h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const bool live = pos0 + kp * 16 + 8 * hf + e < len;
        h[e] = live ? f16_bits(bf16_to_float((uint16_t)(raw[kp][e >> 1] >> (16 * (e & 1))))) : (uint16_t)0;
      }
      // positions 8 hf + e of the group go to storage slots 4 hf + e (e < 4) and 8 + 4 hf + e - 4 (e >= 4)
      uint16_t* dst = vt + (size_t)col * p.lp + kp * 16;
      const u32x2 a = {(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
      const u32x2 b = {(uint32_t)h[4] | ((uint32_t)h[5] << 16), (uint32_t)h[6] | ((uint32_t)h[7] << 16)};
      *reinterpret_cast<u32x2*>(dst + 4 * hf) = a;
      *reinterpret_cast<u32x2*>(dst + 8 + 4 * hf) = b;
    }
  }
}

// ------------------------------------------------------------------------------------------------ attend
// Four waves per workgroup, each with one 32-query block of one query head, two workgroups per CU (each hides the
// other's softmax behind its matrix-core work).  The waves are dealt as (query sub-block, head of the group): groups
// of 4 or more heads take 4 heads x 1 sub-block (32 queries per workgroup), 2 heads x 2 sub-blocks, 1 head x 4
// sub-blocks (128 queries), so that every wave has work whatever the grouping and a K/V tile copied to LDS serves 128
// query rows.  (Eight waves and 256 rows per tile, which halves the copies from L2, measured 7 % slower.)
constexpr int kAttnWaves = 4;
__host__ __device__ inline int attn_heads_per_pass(int G) { return G >= 4 ? 4 : (G >= 2 ? 2 : 1); }

template <int HD>
__global__ __launch_bounds__(64 * kAttnWaves, kAttnWaves == 4 ? 2 : 1) void prefill_attn_kernel(PrefillParams p) {
  constexpr int KS = HD / 16, ND = HD / 32, BK = 64, NW = kAttnWaves;
  constexpr int NKF = 2 * KS, NVF = 4 * ND;  // K and V operand fragments per tile
  constexpr int RING = 8;                    // fragments in flight from LDS
  static_assert(NKF % RING == 0 && NVF % RING == 0, "fragment ring");
  // LDS tiles with one 16-byte pad chunk per row: K tile [kpos][d] rows of HD/8 + 1 chunks, V tile [d][kpos'] rows
  // of 9 chunks.  Padding (not XOR swizzling) keeps every operand address = one per-lane base + a compile-time
  // offset, and the 16 rows a quarter-wave reads start in 16 different bank groups.
  constexpr int KROW = HD / 8 + 1, VROW = BK / 8 + 1;          // chunks per padded row
  constexpr int KTILE = BK * KROW, VTILE = HD * VROW;           // chunks per tile
  constexpr int KINS = (KTILE + 63) / 64, VINS = (VTILE + 63) / 64;  // wave-wide 1 KiB copies per tile
  constexpr int KELE = KINS * 64 * 8, VELE = VINS * 64 * 8;     // elements reserved per stage
  extern __shared__ __align__(16) unsigned char smem_attn[];
  uint16_t* const sK = reinterpret_cast<uint16_t*>(smem_attn);          // [2][KELE]
  uint16_t* const sV = sK + 2 * KELE;                                   // [2][VELE]
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = p.h_kv * HD, G = p.G;
  const int NH = attn_heads_per_pass(G), BQW = 32 * (NW / NH);  // heads per pass; queries per workgroup
  const int wh = w % NH, wq = w / NH;                            // this wave's head of the pass and query sub-block
  const int g = blockIdx.x % p.h_kv;
  const int rest = blockIdx.x / p.h_kv;
  const int nqb = (p.lp + BQW - 1) / BQW;       // query blocks per sequence
  const int qb = nqb - 1 - rest % nqb;          // longest blocks first
  const int seq = rest / nqb;
  const int tok0 = p.cu_seqlens[seq];
  const int len = p.cu_seqlens[seq + 1] - tok0;
  if (qb * BQW >= len) return;
  const int q_last = qb * BQW + BQW - 1 < p.lp - 1 ? qb * BQW + BQW - 1 : p.lp - 1;
  const int t_wg = q_last / BK;                 // the last tile any wave of the workgroup needs
  const int qw0 = qb * BQW + wq * 32;           // this wave's first query
  const int t_w = qw0 / BK;                     // the tile that holds this wave's diagonal
  const int dq = qw0 - t_w * BK;                // offset of the wave's first query inside that tile
  const uint16_t* krot = p.krot + (size_t)seq * p.lp * n + g * HD;
  const uint16_t* vt = p.vt + ((size_t)seq * n + g * HD) * p.lp;
  const uint16_t* const kfrag = sK + (l32 * KROW + hf) * 8;  // + (mb*32*KROW + 2*ks)*8 : operand (mb, ks)
  const uint16_t* const vfrag = sV + (l32 * VROW + hf) * 8;  // + (db*32*VROW + 2*k4)*8 : operand (db, k4)

  // One K/V tile, global -> LDS directly (no staging registers).  A wave's 64 lanes fill 64 consecutive 16-byte
  // LDS chunks; each lane fetches the global chunk that belongs there (pad chunks re-fetch the row's first).
  constexpr int KI = (KINS + NW - 1) / NW, VI = (VINS + NW - 1) / NW;
  uint32_t koff[KI], voff[VI];  // this lane's source offsets (elements) inside a tile, fixed for the kernel
  static_assert(KI + VI <= NKF, "one copy per score MFMA");
#pragma unroll
  for (int i = 0; i < KI; ++i) {
    int L = (i * NW + w < KINS ? i * NW + w : KINS - 1) * 64 + lane;
    L = L < KTILE ? L : KTILE - 1;
    const int row = L / KROW, c = L % KROW;
    koff[i] = (uint32_t)row * n + (c < HD / 8 ? c : 0) * 8;
  }
#pragma unroll
  for (int i = 0; i < VI; ++i) {
    int L = (i * NW + w < VINS ? i * NW + w : VINS - 1) * 64 + lane;
    L = L < VTILE ? L : VTILE - 1;
    const int row = L / VROW, c = L % VROW;
    voff[i] = (uint32_t)row * p.lp + (c < BK / 8 ? c : 0) * 8;
  }
  // (buffer loads: descriptors of this sequence's rotated keys and of this head's value rows)
  const __amdgpu_buffer_rsrc_t k_rsrc = make_rsrc(krot, (uint32_t)(((size_t)p.lp * n - g * HD) * 2));
  const __amdgpu_buffer_rsrc_t v_rsrc = make_rsrc(vt, (uint32_t)((size_t)HD * p.lp * 2));
  auto tile_dma_one = [&](int t, int buf, int i) {  // copy i < KI + VI of this wave's share (branch-free: a copy past
                                                    // the tile's last one repeats the last one)
    const uint32_t ks_off = (uint32_t)t * BK * n * 2u, vs_off = (uint32_t)t * BK * 2u;
    if (i < KI) {
      const int ins = i * NW + w < KINS ? i * NW + w : KINS - 1;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(k_rsrc, (__attribute__((address_space(3))) void*)(sK + (size_t)buf * KELE + (size_t)ins * 512), 16,
                                               (int)(koff[i] * 2), (int)ks_off, 0, 0);
    } else {
      const int j = i - KI;
      const int ins = j * NW + w < VINS ? j * NW + w : VINS - 1;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(v_rsrc, (__attribute__((address_space(3))) void*)(sV + (size_t)buf * VELE + (size_t)ins * 512), 16,
                                               (int)(voff[j] * 2), (int)vs_off, 0, 0);
    }
  };
  auto tile_dma = [&](int t, int buf) {
#pragma unroll
    for (int i = 0; i < KI + VI; ++i) tile_dma_one(t, buf, i);
  };

  for (int hc = 0; hc < G; hc += NH) {
    const int hq = hc + wh;
    const bool active = hq < G && qw0 < len;
    const int h = g * G + hq;

    // Q operands (B operand: n = query, k = head-dim coordinate), rotated at the query's position and scaled.
    // The angle is reduced in fp64 turns and evaluated by the hardware sine and cosine (which take turns).
    f16x8 qf[KS];
    {
      const int qpos = qw0 + l32;
      const bool ok = active && qpos < len;
      const uint16_t* qrow = p.q + ((size_t)(tok0 + (ok ? qpos : 0)) * p.h_q + (active ? h : 0)) * HD;
      bf16x8 raw[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) raw[ks] = load_frag(qrow + ks * 16 + 8 * hf);
#pragma unroll
      for (int ks = 0; ks < KS / 2; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const double turns = (double)qpos * p.rope_tab[ks * 16 + 8 * hf + e] * 0.15915494309189533576888;
          const float fr = (float)(turns - rint(turns));
          const float c = __builtin_amdgcn_cosf(fr), sn = __builtin_amdgcn_sinf(fr);
          const float lo = (float)raw[ks][e], hi = (float)raw[ks + KS / 2][e];
          qf[ks][e] = static_cast<_Float16>(ok ? (lo * c - hi * sn) * p.q_scale : 0.f);
          qf[ks + KS / 2][e] = static_cast<_Float16>(ok ? (hi * c + lo * sn) * p.q_scale : 0.f);
        }
    }
    f32x16 o[ND];
#pragma unroll
    for (int a = 0; a < ND; ++a)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[a][j] = 0.f;
    // running maximum of the query's row (both halves of the wave agree on it) and this half's share of its sum
    float m_run = kNegInfP, l_half = 0.f;

    __syncthreads();  // previous head chunk is done with both stages
    tile_dma(0, 0);
    // One tile.  An in-order wave that asks LDS for an operand right before the MFMA that takes it pays the whole
    // LDS latency every time, so the operand reads run RING fragments ahead of the MFMAs: K fragment i + RING is
    // requested behind MFMA i, the first V fragments behind the last score MFMAs (they land under the softmax),
    // the rest behind the first value MFMAs.  The softmax itself touches no LDS (the row maximum crosses the
    // wave's halves on the vector ALU; the row sum is kept per half until the end).  The wave's share of the next
    // tile's copies is issued one copy per score MFMA rather than as a burst (a burst holds the wave, and its MFMAs,
    // in the issue of the loads); past the workgroup's last tile the copies repeat that tile into the idle stage.
    auto tile_step = [&](int t, auto diag_c) {  // the wave's diagonal tile is the only one that needs the mask
      const int buf = t & 1;
      const uint16_t* const kt = kfrag + buf * KELE;
      const uint16_t* const vtile = vfrag + buf * VELE;
      auto k_at = [&](int i) { return load_frag_f16(kt + ((i & 1) * 32 * KROW + 2 * (i >> 1)) * 8); };    // i = 2 ks + mb
      auto v_at = [&](int j) { return load_frag_f16(vtile + ((j % ND) * 32 * VROW + 2 * (j / ND)) * 8); };  // j = ND k4 + db
      f16x8 fr[RING];
#pragma unroll
      for (int i = 0; i < RING; ++i) fr[i] = k_at(i);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 s[2];
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      const int tn = t + 1 <= t_wg ? t + 1 : t_wg;  // (clamped: the copies are unconditional)
#pragma unroll
      for (int i = 0; i < NKF; ++i) {
        s[i & 1] = mfma32_f16(fr[i % RING], qf[i >> 1], i < 2 ? zero : s[i & 1]);
        fr[i % RING] = i + RING < NKF ? k_at(i + RING) : v_at(i + RING - NKF);
        if (i < KI + VI) tile_dma_one(tn, buf ^ 1, i);
      }
#pragma unroll
      for (int i = 0; i < NKF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
        if (i < KI + VI) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (decltype(diag_c)::value) {  // diagonal tile: key position must not exceed the query position
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int jj = 0; jj < 16; ++jj)
            if (mb * 32 + acc_row(jj, hf) > dq + l32) s[mb][jj] = kNegInfP;
      }
      float mx = kNegInfP;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) mx = fmaxf(mx, s[mb][jj]);
      {
        const float2 both = half_pair(mx);
        mx = fmaxf(both.x, both.y);
      }
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      f16x8 pf[4];
      float sum = 0.f;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          const float pv = __builtin_amdgcn_exp2f(s[mb][jj] - m_new);
          sum += pv;
          pf[mb * 2 + (jj >> 3)][jj & 7] = static_cast<_Float16>(pv);
        }
      l_half = l_half * alpha + sum;
      const bool moved = m_new > m_run;
      m_run = m_new;
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {  // some row's maximum moved
#pragma unroll
        for (int db = 0; db < ND; ++db)
#pragma unroll
          for (int jj = 0; jj < 16; ++jj) o[db][jj] *= alpha;
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NVF; ++j) {
        o[j % ND] = mfma32_f16(fr[j % RING], pf[j / ND], o[j % ND]);
        if (j + RING < NVF) fr[j % RING] = v_at(j + RING);
      }
#pragma unroll
      for (int j = 0; j < NVF - RING; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    // Every wave passes every hand-over of the workgroup's tiles; it computes on the tiles up to its own diagonal
    // (waves of the earlier sub-blocks are done before the workgroup's last tiles).
    const int t_mine = active ? t_w : -1;
    auto hand_over = [&](int t) {
      __builtin_amdgcn_s_waitcnt(0);   // this wave's part of tile t has landed (LDS-bound loads count as vector memory)
      __syncthreads();                 // tile t visible; everyone is done with the other stage
      if (t > t_mine && t + 1 <= t_wg) tile_dma(t + 1, (t + 1) & 1);  // a wave with no work on tile t: as a burst
    };
    for (int t = 0; t < t_mine; ++t) {
      hand_over(t);
      tile_step(t, std::false_type{});
    }
    if (active) {
      hand_over(t_w);
      tile_step(t_w, std::true_type{});
    }
    for (int t = t_mine + 1; t <= t_wg; ++t) hand_over(t);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no LDS-bound copy is left in flight when the wave ends

    if (active) {
      const int qpos = qw0 + l32;
      const float2 l_both = half_pair(l_half);
      const float l_run = l_both.x + l_both.y;
      if (qpos < len) {
        const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
        uint16_t* orow = p.out + ((size_t)(tok0 + qpos) * p.h_q + h) * HD;
#pragma unroll
        for (int db = 0; db < ND; ++db)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            uint16_t v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = bf16_bits(o[db][4 * q4 + i] * inv);
            const u32x2 pk = {(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16)};
            *reinterpret_cast<u32x2*>(orow + db * 32 + 8 * q4 + 4 * hf) = pk;
          }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------ host
static size_t align256p(size_t x) { return (x + 255) & ~(size_t)255; }

PrefillPlan make_prefill_plan(const lorc_layer_desc& d, int b, int max_seqlen) {
  PrefillPlan pl;
  pl.tiles_per_seq = (max_seqlen + kPage - 1) / kPage;
  if (pl.tiles_per_seq < 1) pl.tiles_per_seq = 1;
  pl.lp = pl.tiles_per_seq * kPage;
  const size_t n = (size_t)d.n_kv_heads * d.head_dim;
  size_t off = 0;
  pl.off_rope = off;
  off = align256p(off + 64 * sizeof(double));
  pl.off_krot = off;
  off = align256p(off + (size_t)b * pl.lp * n * 2);
  pl.off_vt = off;
  off = align256p(off + (size_t)b * pl.lp * n * 2);
  pl.total_bytes = off;
  return pl;
}

static size_t attn_lds_bytes(int hd) {  // two stages of padded K and V tiles, whole 1 KiB copies
  const int ktile = 64 * (hd / 8 + 1), vtile = hd * 9;
  return (size_t)2 * (((ktile + 63) / 64) + ((vtile + 63) / 64)) * 1024;
}

static int attn_grid(const PrefillParams& p) {  // one workgroup per (sequence, block of queries, KV head)
  const int bqw = 32 * (kAttnWaves / attn_heads_per_pass(p.G));
  return p.b * ((p.lp + bqw - 1) / bqw) * p.h_kv;
}

int set_kernel_attributes_prefill() {
  const void* kernels[] = {reinterpret_cast<const void*>(prefill_attn_kernel<128>),
                           reinterpret_cast<const void*>(prefill_attn_kernel<64>),
                           reinterpret_cast<const void*>(prefill_rebuild_kernel<128>),
                           reinterpret_cast<const void*>(prefill_rebuild_kernel<64>)};
  for (const void* k : kernels)
    if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return LORC_EHIP;
  return LORC_OK;
}

int launch_prefill(const PrefillParams& p, hipStream_t s, bool plain) {
  if (plain) {  // uncompressed layer: keys and values are gathered from the pages, then the same attention kernel
    if (p.head_dim != 128) return LORC_EUNSUPPORTED;
    const dim3 grid_g(p.b * p.tiles_per_seq), grid_att(attn_grid(p));
    if (int rc = launch_kernel(prefill_plain_gather_kernel, grid_g, dim3(256), 0, s, p)) return rc;
    return launch_kernel(prefill_attn_kernel<128>, grid_att, dim3(64 * kAttnWaves), attn_lds_bytes(128), s, p);
  }
  const int rmax = p.r_k > p.r_v ? p.r_k : p.r_v;
  const int part = rmax < kRebuildPartSteps * 16 ? rmax : kRebuildPartSteps * 16;  // ranks beyond that are walked in parts
  const size_t lds = (size_t)64 * part * 2 + (size_t)2 * (p.head_dim / 2) * 8;
  if (lds > 160 * 1024) return LORC_EUNSUPPORTED;
  const dim3 grid_r(p.b * p.tiles_per_seq), grid_a(attn_grid(p));
  if (p.head_dim == 128) {
    if (int rc = launch_kernel(prefill_rebuild_kernel<128>, grid_r, dim3(256), lds, s, p)) return rc;
    return launch_kernel(prefill_attn_kernel<128>, grid_a, dim3(64 * kAttnWaves), attn_lds_bytes(128), s, p);
  }
  if (int rc = launch_kernel(prefill_rebuild_kernel<64>, grid_r, dim3(256), lds, s, p)) return rc;
  return launch_kernel(prefill_attn_kernel<64>, grid_a, dim3(64 * kAttnWaves), attn_lds_bytes(64), s, p);
}

}  // namespace lorc

