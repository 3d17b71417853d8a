// Decode attention in three launches, for the shapes the single-pass split kernels do not take:
//   * wide layers: ranks above 1024 (Table 2's LLaMA-2-13B row: MHA, 40 heads, n = 5120 compressed to 2048).  A tile's
//     K latents no longer fit LDS and the latent-space output of all heads no longer fits one workgroup's registers,
//     so the rank is walked in parts and o_lat in column chunks;
//   * layers that Algorithm 1's threshold leaves uncompressed (Section 6.2): the cache pages hold the un-rotated
//     keys and the values themselves (rank = n, identity read-side factors that are never stored or multiplied).
//
//   scores : S[seq][h][t] = softmax_scale * log2(e) * <R(q_pos) q_h, R(t) k_t>   (Eq. 1; the Appendix on the adjusted
//            position embedding: keys are rotated when they are read).  Wide layers rebuild k_t = c_t B_k per KV head
//            on the matrix cores, the rank in parts of up to 512 that pass through LDS; uncompressed layers read k_t.
//   values : per (sequence, context split, column chunk): row maxima of the split's scores, P = exp2(S - m), row
//            sums, o = P C_v for the chunk's columns on the matrix cores; written as split partials (m, l, o / l) in
//            the format of the single-pass kernels.  Wide layers: all heads x 512 latent columns per workgroup (the
//            latent is joint across heads, Section 4.1).  Uncompressed layers: one KV head's group x its 128 columns.
//   merge  : the common merge kernel (wide: softmax-merge of the splits, then B_v; uncompressed: the merge alone).
#include "lorc_device.h"
#include "lorc_kernels.h"
#include "lorc_rebuild.h"

namespace lorc {

namespace {
constexpr float kNegInfW = -__builtin_huge_valf();
constexpr int kWideT = 64;           // positions per tile = one page
constexpr int kWidePartSteps = 32;   // k-steps (of 16 latents) of one rank part in LDS: 64 x 512 x 2 B = 64 KiB, two workgroups per CU
constexpr int kWideHeadsPerWg = 4;   // KV heads per workgroup of the wide scores kernel (one per wave)
constexpr int kWideMaxG = 8;

__host__ __device__ inline size_t wide_scores_lds_bytes(int r_k, int G) {
  const int part = r_k < kWidePartSteps * 16 ? r_k : kWidePartSteps * 16;
  size_t b = (size_t)kWideT * part * 2;              // one rank part of the tile's K latents
  b += (size_t)2 * 64 * 8;                           // rotation bases of the two position blocks
  b += (size_t)kWideHeadsPerWg * G * 128 * 2;        // rotated, scaled queries of the workgroup's heads (fp16)
  return b;
}
}  // namespace

// ------------------------------------------------------------------------------------------------ scores, wide
// One workgroup per (group of four KV heads, sequence, 64-position tile), the head group outermost in the block
// index: the workgroups in flight at one time work on the same four heads, whose B_k slice (4 x 128 columns x r_k)
// stays in the L2 caches while the latents stream past.  Wave w owns KV head 4 * group + w.  Two passes (the two
// halves of the head's rotation pairs: columns [32 wh, 32 wh + 32) and their partners 64 further), each walking the
// rank in parts: a part of the tile's K latents is copied to LDS, every wave accumulates its 2 x 2 blocks of K^T
// over the part's k-steps with B_k operands streamed from L2, and after the last part rotates the blocks and
// multiplies them with its head group's query rows (fp16 matrix-core op, accumulated over the two passes).
// Two workgroups share a CU: while one copies a part (direct global -> LDS loads) the other multiplies.
__global__ __launch_bounds__(256, 2) void wide_scores_kernel(DecodeParams p) {
  constexpr int HD = 128, HALF = 64, T = kWideT, NPB = 2, PF = 4;
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tiles = p.score_stride / T;
  const int per_group = p.b * tiles;
  const int hg = blockIdx.x / per_group, rem = blockIdx.x % per_group;
  const int seq = rem / tiles, tile = rem % tiles;
  int ctx = p.ctx_len[seq];
  ctx = ctx < 0 ? 0 : (ctx > p.max_ctx ? p.max_ctx : ctx);
  const int pos0 = tile * T;
  if (pos0 >= ctx) return;  // whole workgroup: nothing of this tile is attended to
  const int r_k = p.r_k, G = p.G, nks = r_k >> 4;
  const int part_steps = nks < kWidePartSteps ? nks : kWidePartSteps;
  const int n_parts = (nks + part_steps - 1) / part_steps;

  uint16_t* ck = reinterpret_cast<uint16_t*>(smem);
  float2* cs_base = reinterpret_cast<float2*>(smem + (size_t)T * part_steps * 16 * 2);
  _Float16* qrot = reinterpret_cast<_Float16*>(cs_base + NPB * HALF);  // [4 heads x G][HD]

  const int id = p.block_table[(size_t)seq * p.max_pages + tile];
  const bool page_ok = id >= 0 && id < p.n_pages;
  const uint16_t* page = uniform_ptr(p.cache + (size_t)(page_ok ? id : 0) * p.page_elems);
  const __amdgpu_buffer_rsrc_t page_rsrc = make_rsrc(page, (uint32_t)kPage * r_k * 2u);
  const int q_pos = p.q_pos[seq];

  // rotation bases of the tile's two position blocks, and the workgroup's query rows rotated at q_pos
  if (tid < NPB * HALF) cs_base[tid] = cos_sin_reduced((double)(pos0 + 32 * (tid / HALF)) * p.rope_tab[tid % HALF]);
  const int g0 = hg * kWideHeadsPerWg;
  for (int idx = tid; idx < kWideHeadsPerWg * G * HALF; idx += 256) {
    const int hl = idx / HALF, i = idx % HALF;
    const int h = g0 * G + hl;
    if (h < p.h_q) {
      const float2 cs = cos_sin_reduced((double)q_pos * p.rope_tab[i]);
      const uint16_t* qs = p.q + ((size_t)seq * p.h_q + h) * HD;
      const float lo = bf16_to_float(qs[i]) * p.q_scale, hi = bf16_to_float(qs[i + HALF]) * p.q_scale;
      qrot[hl * HD + i] = static_cast<_Float16>(lo * cs.x - hi * cs.y);
      qrot[hl * HD + i + HALF] = static_cast<_Float16>(hi * cs.x + lo * cs.y);
    }
  }

  const int g = g0 + w;
  const bool active = g < p.h_kv;
  const __amdgpu_buffer_rsrc_t bk_rsrc = make_rsrc(p.bk, (uint32_t)p.h_kv * HD * r_k * 2u);
  f32x16 S[NPB];
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
    for (int j = 0; j < 16; ++j) S[pb][j] = 0.f;

  for (int wh = 0; wh < 2; ++wh) {
    const int fbase = 32 * wh;
    const int cb0 = g * 4 + wh, cb1 = cb0 + 2;
    f32x16 acc[2][NPB];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[a][pb][j] = 0.f;
    for (int part = 0; part < n_parts; ++part) {
      const int ks0 = part * part_steps;
      const int steps = nks - ks0 < part_steps ? nks - ks0 : part_steps;
      if (!(n_parts == 1 && wh == 1)) {  // a single part stays in LDS for the second pass
        __syncthreads();                 // the previous part's operand reads are over
        if (page_ok) {                   // 1 KiB per instruction, the LDS image being the page's own tiling
          for (int pb = 0; pb < NPB; ++pb)
            for (int blk = w; blk < steps; blk += 4)
              __builtin_amdgcn_raw_ptr_buffer_load_lds(page_rsrc, (__attribute__((address_space(3))) void*)(ck + (size_t)(pb * steps + blk) * 512),
                                                       16, lane * 16, (pb * nks + ks0 + blk) * 1024, 0, 0);
        } else {
          const u32x4 z = {0u, 0u, 0u, 0u};
          u32x4* dst = reinterpret_cast<u32x4*>(ck);
          for (int c = tid; c < NPB * steps * 64; c += 256) dst[c] = z;
        }
      }
      __syncthreads();                   // (its fence also waits for the copies)
      if (active)
        rebuild_pair<NPB, PF>(acc, bk_rsrc, (uint32_t)(cb0 * nks + ks0) * 1024u, (uint32_t)(cb1 * nks + ks0) * 1024u,
                              (uint32_t)lane * 16u, ck + (size_t)lane * 8, steps);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (active) {
      // Query operands (m = query head of the group, k = 16 head-dim coordinates) in the order in which the rotated
      // K^T accumulators serve as B operands: element e of operand s4 is coordinate 16 (s4 & 1) + 8 (e >> 2) + 4 hf
      // + (e & 3) of half s4 >> 1 of the head, + 32 wh.
      f16x8 qf[4];
      {
        const bool qreal = l32 < G && g * G + l32 < p.h_q;
        const _Float16* qh = qrot + (size_t)(w * G + (qreal ? l32 : 0)) * HD + fbase + 4 * hf;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          const _Float16* src = qh + HALF * (s4 >> 1) + 16 * (s4 & 1);
          const u32x2 lo = *reinterpret_cast<const u32x2*>(src), hi = *reinterpret_cast<const u32x2*>(src + 8);
          const u32x4 v = {qreal ? lo[0] : 0u, qreal ? lo[1] : 0u, qreal ? hi[0] : 0u, qreal ? hi[1] : 0u};
          qf[s4] = __builtin_bit_cast(f16x8, v);
        }
      }
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb) {
        f16x8 kf[4];
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          const int fi = fbase + acc_row(jj, hf);
          const float2 cb = cs_base[pb * HALF + fi];
          const float2 cl = p.lane_cs[l32 * HALF + fi];
          const float cA = cb.x * cl.x - cb.y * cl.y;
          const float sA = cb.y * cl.x + cb.x * cl.y;
          const float x = acc[0][pb][jj], y = acc[1][pb][jj];
          kf[jj >> 3][jj & 7] = static_cast<_Float16>(x * cA - y * sA);
          kf[2 + (jj >> 3)][jj & 7] = static_cast<_Float16>(y * cA + x * sA);
        }
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) S[pb] = mfma32_f16(qf[s4], kf[s4], S[pb]);
      }
    }
  }
  if (active) {
#pragma unroll
    for (int jr = 0; jr < 4; ++jr) {  // rows 0 .. 7 of the score block hold the group's (at most eight) heads
      const int m = acc_row(jr, hf);
      const int h = g * G + m;
      if (m < G && h < p.h_q) {
        float* row = p.scores + ((size_t)seq * p.h_q + h) * p.score_stride + pos0;
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) row[pb * 32 + l32] = S[pb][jr];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------ scores, uncompressed
// One workgroup per (sequence, 64-position tile).  Wave w takes position block w % 2 and the KV heads of parity
// w / 2.  A lane of a K operand block holds one position and 8 consecutive head-dim coordinates, and the rotation
// partner of a block sits four blocks further in the same lane and element: the keys are rotated in registers
// (angles per position and frequency worked out once per tile and shared by all heads; reduced in fp64, evaluated
// by the hardware sine / cosine, which take turns), rounded to fp16 and multiplied with the group's query rows.
__global__ __launch_bounds__(256, 2) void plain_scores_kernel(DecodeParams p) {
  constexpr int HD = 128, HALF = 64, T = kWideT;
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tiles = p.score_stride / T;
  const int seq = blockIdx.x / tiles, tile = blockIdx.x % tiles;
  int ctx = p.ctx_len[seq];
  ctx = ctx < 0 ? 0 : (ctx > p.max_ctx ? p.max_ctx : ctx);
  const int pos0 = tile * T;
  if (pos0 >= ctx) return;
  const int G = p.G, n = p.h_kv * HD;
  _Float16* qrot = reinterpret_cast<_Float16*>(smem);  // [h_q][HD]

  const int id = p.block_table[(size_t)seq * p.max_pages + tile];
  const bool page_ok = id >= 0 && id < p.n_pages;
  const uint16_t* page = uniform_ptr(p.cache + (size_t)(page_ok ? id : 0) * p.page_elems);
  // a page that is not cached reads as zeros through a descriptor of size zero
  const __amdgpu_buffer_rsrc_t kr = make_rsrc(page, page_ok ? (uint32_t)kPage * n * 2u : 0u);
  const int q_pos = p.q_pos[seq];

  for (int idx = tid; idx < p.h_q * HALF; idx += 256) {
    const int h = idx / HALF, i = idx % HALF;
    const float2 cs = cos_sin_reduced((double)q_pos * p.rope_tab[i]);
    const uint16_t* qs = p.q + ((size_t)seq * p.h_q + h) * HD;
    const float lo = bf16_to_float(qs[i]) * p.q_scale, hi = bf16_to_float(qs[i + HALF]) * p.q_scale;
    qrot[h * HD + i] = static_cast<_Float16>(lo * cs.x - hi * cs.y);
    qrot[h * HD + i + HALF] = static_cast<_Float16>(hi * cs.x + lo * cs.y);
  }
  const int pb = w & 1;
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
  __syncthreads();

  const int blocks_per_row = n >> 4;  // 1 KiB operand blocks per 32 positions
  for (int g = w >> 1; g < p.h_kv; g += 2) {
    u32x4 raw[8];
#pragma unroll
    for (int kb = 0; kb < 8; ++kb)
      raw[kb] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(kr, lane * 16, (pb * blocks_per_row + g * 8 + kb) * 1024, 0));
    f16x8 kf[8];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = bf16_to_float((uint16_t)(raw[kb][e >> 1] >> (16 * (e & 1))));
        const float y = bf16_to_float((uint16_t)(raw[kb + 4][e >> 1] >> (16 * (e & 1))));
        kf[kb][e] = static_cast<_Float16>(x * cs_c[kb][e] - y * cs_s[kb][e]);
        kf[kb + 4][e] = static_cast<_Float16>(y * cs_c[kb][e] + x * cs_s[kb][e]);
      }
    f32x16 S;
#pragma unroll
    for (int j = 0; j < 16; ++j) S[j] = 0.f;
    const bool qreal = l32 < G;
    const _Float16* qh = qrot + (size_t)(g * G + (qreal ? l32 : 0)) * HD + 8 * hf;
#pragma unroll
    for (int kb = 0; kb < 8; ++kb) {
      const u32x4 qv = *reinterpret_cast<const u32x4*>(qh + 16 * kb);
      const u32x4 v = {qreal ? qv[0] : 0u, qreal ? qv[1] : 0u, qreal ? qv[2] : 0u, qreal ? qv[3] : 0u};
      S = mfma32_f16(__builtin_bit_cast(f16x8, v), kf[kb], S);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int m = acc_row(j, hf);
      if (m < G) p.scores[((size_t)seq * p.h_q + g * G + m) * p.score_stride + pos0 + 32 * pb + l32] = S[j];
    }
  }
}

// ------------------------------------------------------------------------------------------------ scores, absorbed query
// Models without positional rotation (Section 4.1, Eq. 7): S[h][t] = scale * <q_lat[h], c_k[t]> on the cached K
// latents themselves.  One workgroup per (sequence, 64-position tile).  Wave w takes position block w % 2 and the
// k-steps of parity w / 2, for all QB blocks of 32 heads: a K operand block (k = 16 latent indices, n = 32 positions:
// the page tiling) is read once, by one wave; the query operands (m = head, k = 16 latent indices: 16 contiguous
// bytes of a q_lat row per lane) come from L2.  The two parities meet in LDS.
template <int QB>
__global__ __launch_bounds__(256, 2) void absorbed_scores_kernel(DecodeParams p) {
  constexpr int T = kWideT, U = 4;
  __shared__ float xs[2][QB][16][64];  // [position block][row block][accumulator register][lane]
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tiles = p.score_stride / T;
  const int seq = blockIdx.x / tiles, tile = blockIdx.x % tiles;
  int ctx = p.ctx_len[seq];
  ctx = ctx < 0 ? 0 : (ctx > p.max_ctx ? p.max_ctx : ctx);
  const int pos0 = tile * T;
  if (pos0 >= ctx) return;
  const int r_k = p.r_k, nks = r_k >> 4, pb = w & 1, par = w >> 1;
  const int id = p.block_table[(size_t)seq * p.max_pages + tile];
  const bool page_ok = id >= 0 && id < p.n_pages;
  const uint16_t* page = uniform_ptr(p.cache + (size_t)(page_ok ? id : 0) * p.page_elems);
  const __amdgpu_buffer_rsrc_t kr = make_rsrc(page, page_ok ? (uint32_t)kPage * r_k * 2u : 0u);  // not cached: zeros
  // rows past the last head read row 0 and are not written
  const __amdgpu_buffer_rsrc_t qr = make_rsrc(p.q + (size_t)seq * p.h_q * r_k, (uint32_t)p.h_q * r_k * 2u);
  uint32_t qoff[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int h = qb * 32 + l32;
    qoff[qb] = (uint32_t)((h < p.h_q ? h : 0) * r_k + 8 * hf) * 2u;
  }
  f32x16 S[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int j = 0; j < 16; ++j) S[qb][j] = 0.f;
  const int my_steps = (nks - par + 1) >> 1;  // k-steps par, par + 2, ...
  for (int i0 = 0; i0 < my_steps; i0 += U) {
    bf16x8 kf[U], qf[U][QB];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int i = i0 + u < my_steps ? i0 + u : my_steps - 1;  // clamped: the repeats are not multiplied
      const int ks = par + 2 * i;
      kf[u] = buf_frag(kr, (uint32_t)lane * 16u, (uint32_t)(pb * nks + ks) * 1024u);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) qf[u][qb] = buf_frag(qr, qoff[qb], (uint32_t)ks * 32u);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (i0 + u < my_steps)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) S[qb] = mfma32(qf[u][qb], kf[u], S[qb]);
  }
  if (par == 1) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int j = 0; j < 16; ++j) xs[pb][qb][j][lane] = S[qb][j];
  }
  __syncthreads();
  if (par == 0) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int h = qb * 32 + acc_row(j, hf);
        if (h < p.h_q)
          p.scores[((size_t)seq * p.h_q + h) * p.score_stride + pos0 + 32 * pb + l32] = (S[qb][j] + xs[pb][qb][j][lane]) * p.q_scale;
      }
  }
}

// ------------------------------------------------------------------------------------------------ values
// QB: blocks of 32 score rows; NB: blocks of 32 output columns per wave.
//   wide  (PLAIN = false): rows = all query heads, columns = latent indices [512 chunk, 512 chunk + 512) of C_v;
//   plain (PLAIN = true) : rows = the G heads of KV head `chunk`, columns = that head's 128 value coordinates.
// Grid: (sequence, split, chunk).  The split's row maxima are taken first (the scores are there already), so the
// weights need no rescaling afterwards; P goes to LDS in A-operand order (bf16), the value operands come straight
// from the page tiling (a wave-wide 1 KiB block is one B operand: k = 16 positions, n = 32 columns).
template <int QB, int NB, bool PLAIN>
__global__ __launch_bounds__(256, QB == 1 ? 2 : 1) void latent_pv_kernel(DecodeParams p) {
  constexpr int T = kWideT, KP = T / 16;
  __shared__ __align__(16) uint16_t pbuf[2][QB * KP * 512];
  __shared__ float m_s[QB * 32], l_s[QB * 32];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nc = PLAIN ? p.h_kv : p.v_chunks;
  const int chunk = blockIdx.x % nc, ss = blockIdx.x / nc;
  const int split = ss % p.n_splits, seq = ss / p.n_splits;
  int ctx = p.ctx_len[seq];
  ctx = ctx < 0 ? 0 : (ctx > p.max_ctx ? p.max_ctx : ctx);
  const int R = PLAIN ? p.G : p.h_q;                        // real rows
  const int head0 = PLAIN ? chunk * p.G : 0;                // head of row 0
  const int r_k = p.r_k, r_v = p.r_v;
  const int t_begin = split * p.tiles_per_split * T;
  int t_end = t_begin + p.tiles_per_split * T;
  if (t_end > ctx) t_end = ctx;
  const int out_w = PLAIN ? 128 : r_v;                      // width of a partial row
  const int nblk = r_v >> 5;                                // 32-column blocks of the value part
  const size_t part_row0 = ((size_t)seq * p.n_splits + split) * p.h_q + head0;

  // this thread's share of a tile's scores: row tid / 4, sixteen positions
  const int prow = tid >> 2, pseg = tid & 3;
  const bool prow_real = prow < QB * 32 && prow < R;
  const float* srow = p.scores + ((size_t)seq * p.h_q + head0 + (prow_real ? prow : 0)) * p.score_stride;
  const int tile_begin = t_begin / T, tile_end = (t_end + T - 1) / T;  // empty split: tile_end <= tile_begin

  // ---- 1. row maxima over the split (same thread layout as the weights below; the loads of several tiles are
  //         independent and in flight together)
  {
    float mx = kNegInfW;
    if (prow_real) {
#pragma unroll 4
      for (int tile = tile_begin; tile < tile_end; ++tile) {
        const int tb = tile * T + pseg * 16;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x4 s4 = *reinterpret_cast<const f32x4*>(srow + tb + q4 * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) mx = fmaxf(mx, tb + q4 * 4 + e < t_end ? s4[e] : kNegInfW);
        }
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 1));
    mx = fmaxf(mx, __shfl_xor(mx, 2));
    if (tid < QB * 32 * 4 && pseg == 0) m_s[prow] = mx;
  }
  __syncthreads();

  f32x16 o[QB][NB];
#pragma unroll
  for (int a = 0; a < QB; ++a)
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[a][i][j] = 0.f;

  const float pm = prow < QB * 32 ? m_s[prow] : 0.f;
  float lsum = 0.f;

  // column blocks of this wave (clamped: blocks past the rank are computed on repeated data and never written)
  int jb[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int b_ = PLAIN ? chunk * 4 + w : chunk * 16 + w * NB + i;
    jb[i] = b_ < nblk ? b_ : nblk - 1;
  }
  // Page ids are fetched two tiles ahead and a tile's value operands one tile ahead, and inside a tile the scores
  // are requested before the next tile's operands: the in-order load counter then lets the weights wait for the
  // scores alone while the operands (the HBM stream) stay in flight across the tile's work.
  auto page_id = [&](int tile) {
    const int tc = tile < tile_end ? tile : tile_end - 1;
    return p.block_table[(size_t)seq * p.max_pages + (tc > 0 ? tc : 0)];
  };
  auto v_load = [&](bf16x8 (&v)[NB][KP], int id_raw) {
    const int id = __builtin_amdgcn_readfirstlane(id_raw);
    const bool ok = id >= 0 && id < p.n_pages;
    const uint16_t* vpart = uniform_ptr(p.cache + (size_t)(ok ? id : 0) * p.page_elems + (size_t)kPage * r_k);
    const __amdgpu_buffer_rsrc_t vr = make_rsrc(vpart, ok ? (uint32_t)kPage * r_v * 2u : 0u);  // not cached: zeros, nothing fetched
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int kp = 0; kp < KP; ++kp) v[i][kp] = buf_frag(vr, (uint32_t)lane * 16u, (uint32_t)(jb[i] * KP + kp) * 1024u);
  };

  bf16x8 v[NB][KP], v_next[NB][KP];
  int id_next = 0;
  if (tile_begin < tile_end) {
    const int id0 = page_id(tile_begin);
    id_next = page_id(tile_begin + 1);
    v_load(v_next, id0);
  }
  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int pos0 = tile * T, buf = (tile - tile_begin) & 1;
    f32x4 s4[4];  // threads without a row read row 0 (unconditional: a fixed number of loads in flight)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) s4[q4] = *reinterpret_cast<const f32x4*>(srow + pos0 + pseg * 16 + q4 * 4);
    const int id_after = page_id(tile + 2);
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int kp = 0; kp < KP; ++kp) v[i][kp] = v_next[i][kp];
    v_load(v_next, id_next);  // tile + 1 (past the end: the last page again, never multiplied)
    id_next = id_after;
    if (pos0 + T > t_end) {
      // Ragged last tile: slots past the context hold whatever the pool held before (possibly NaN patterns); P is
      // zero there, but 0 * NaN is not, so those elements of the value operands are cleared.  Element e of operand
      // kp is position 16 kp + 8 hf + e.
#pragma unroll
      for (int kp = 0; kp < KP; ++kp) {
        int nv = t_end - pos0 - kp * 16 - 8 * hf;
        nv = nv < 0 ? 0 : (nv > 8 ? 8 : nv);
        const uint32_t vmask = (1u << nv) - 1u;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          u32x4 raw = __builtin_bit_cast(u32x4, v[i][kp]);
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t two = (vmask >> (2 * c)) & 3u;
            raw[c] &= (two & 1u ? 0x0000ffffu : 0u) | (two & 2u ? 0xffff0000u : 0u);
          }
          v[i][kp] = __builtin_bit_cast(bf16x8, raw);
        }
      }
    }
    // ---- 2. weights of the tile
    if (tid < QB * 32 * 4) {
      float pv[16];
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int t = pos0 + pseg * 16 + q4 * 4 + e;
          const float pe = (prow_real && t < t_end) ? exp2f(s4[q4][e] - pm) : 0.f;
          pv[q4 * 4 + e] = pe;
          lsum += pe;
        }
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        u32x4 pk;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          pk[c] = (uint32_t)bf16_bits(pv[half * 8 + 2 * c]) | ((uint32_t)bf16_bits(pv[half * 8 + 2 * c + 1]) << 16);
        const int qb = prow >> 5, m = prow & 31;
        *reinterpret_cast<u32x4*>(&pbuf[buf][(size_t)((qb * KP + pseg) * 64 + m + 32 * half) * 8]) = pk;
      }
    }
    __syncthreads();  // P of this tile is complete; the buffer of the tile before the previous one is free again
    // ---- 3. o += P V
#pragma unroll
    for (int kp = 0; kp < KP; ++kp) {
      bf16x8 a[QB];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) a[qb] = load_frag(&pbuf[buf][(size_t)((qb * KP + kp) * 64 + lane) * 8]);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int i = 0; i < NB; ++i) o[qb][i] = mfma32(a[qb], v[i][kp], o[qb][i]);
    }
  }

  // ---- 4. row sums, partials
  lsum += __shfl_xor(lsum, 1);
  lsum += __shfl_xor(lsum, 2);
  if (tid < QB * 32 * 4 && pseg == 0) l_s[prow] = lsum;
  __syncthreads();
  if ((PLAIN || chunk == 0) && tid < QB * 32 && tid < R) {
    float* ml = p.part_ml + (part_row0 + tid) * 2;
    ml[0] = m_s[tid];
    ml[1] = l_s[tid];
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int b_ = PLAIN ? chunk * 4 + w : chunk * 16 + w * NB + i;
      if (b_ >= nblk) continue;
      const int col = (PLAIN ? w * 32 : b_ * 32) + l32;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int r = qb * 32 + acc_row(j, hf);
        if (r < R) {
          const float l = l_s[r];
          p.part_o[(part_row0 + r) * out_w + col] = f16_bits(l > 0.f ? o[qb][i][j] / l : 0.f);
        }
      }
    }
}

// ------------------------------------------------------------------------------------------------ host
static size_t align256w(size_t x) { return (x + 255) & ~(size_t)255; }

bool wide_shape_ok(const lorc_layer_desc& d) {
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.head_dim == 128 && G <= kWideMaxG && d.n_q_heads <= 64 && d.rank_k <= kWideMaxRank && d.rank_v <= kWideMaxRank &&
         wide_scores_lds_bytes(d.rank_k, G) <= 160 * 1024;
}

bool plain_shape_ok(const lorc_layer_desc& d) {
  const int n = d.n_kv_heads * d.head_dim, G = d.n_q_heads / d.n_kv_heads;
  return d.head_dim == 128 && d.rank_k == n && d.rank_v == n && G <= 32 && d.n_q_heads <= 64;
}

// Splits for the value kernel: enough workgroups for about two per CU, each walking at least four tiles.
DecodePlan make_wide_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus, bool plain) {
  DecodePlan pl{};
  pl.tile = kWideT;
  pl.occupancy = 1;
  pl.stationary = 0;
  pl.wide = plain ? 2 : 1;
  int n_tiles = (max_ctx + kWideT - 1) / kWideT;
  if (n_tiles < 1) n_tiles = 1;
  pl.score_stride = n_tiles * kWideT;
  pl.v_chunks = plain ? d.n_kv_heads : (d.rank_v + 511) / 512;
  // uncompressed layers: a workgroup streams only one head's 16 KiB per tile, so many more of them are kept in flight
  const long want = (plain ? 8L : 2L) * (n_cus > 0 ? n_cus : 256);
  long ns = (want + (long)b * pl.v_chunks - 1) / ((long)b * pl.v_chunks);
  if (ns > (n_tiles + 3) / 4) ns = (n_tiles + 3) / 4;
  if (ns < 1) ns = 1;
  if (ns > 512) ns = 512;
  pl.tiles_per_split = (int)((n_tiles + ns - 1) / ns);
  pl.n_splits = (n_tiles + pl.tiles_per_split - 1) / pl.tiles_per_split;
  const int out_w = plain ? d.head_dim : d.rank_v;
  size_t off = 0;
  pl.off_ml = off;
  off = align256w(off + (size_t)b * pl.n_splits * d.n_q_heads * 2 * 4);
  pl.off_o = off;
  off = align256w(off + (size_t)b * pl.n_splits * d.n_q_heads * out_w * 2);
  pl.off_scores = off;
  off = align256w(off + (size_t)b * d.n_q_heads * pl.score_stride * 4);
  pl.total_bytes = off;
  return pl;
}

int set_kernel_attributes_decode_wide() {
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(wide_scores_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
    return LORC_EHIP;
  return LORC_OK;
}

bool wide_absorbed_shape_ok(const lorc_layer_desc& d) {
  return d.n_q_heads <= 64 && d.rank_v <= kWideMaxRank;
}

// The two streaming launches; the caller records its events around them and runs the merge.
int launch_decode_wide(const DecodeParams& p, const DecodePlan& plan, hipStream_t s) {
  const int tiles = plan.score_stride / kWideT;
  const int qb = (p.h_q + 31) / 32;
  if (plan.wide == 3) {  // absorbed query: scores on the latents, then the same value kernel
    const dim3 grid(p.b * p.n_splits * p.v_chunks);
    if (qb == 1) {
      if (int rc = launch_kernel(absorbed_scores_kernel<1>, dim3(p.b * tiles), dim3(256), 0, s, p)) return rc;
      return launch_kernel(latent_pv_kernel<1, 4, false>, grid, dim3(256), 0, s, p);
    }
    if (int rc = launch_kernel(absorbed_scores_kernel<2>, dim3(p.b * tiles), dim3(256), 0, s, p)) return rc;
    return launch_kernel(latent_pv_kernel<2, 4, false>, grid, dim3(256), 0, s, p);
  }
  if (plan.wide == 2) {
    const size_t lds = (size_t)p.h_q * 128 * 2;
    if (int rc = launch_kernel(plain_scores_kernel, dim3(p.b * tiles), dim3(256), lds, s, p)) return rc;
    return launch_kernel(latent_pv_kernel<1, 1, true>, dim3(p.b * p.n_splits * p.h_kv), dim3(256), 0, s, p);
  }
  const size_t lds = wide_scores_lds_bytes(p.r_k, p.G);
  if (lds > 160 * 1024 || p.G > kWideMaxG) return LORC_EUNSUPPORTED;
  const int groups = (p.h_kv + kWideHeadsPerWg - 1) / kWideHeadsPerWg;
  if (int rc = launch_kernel(wide_scores_kernel, dim3(groups * p.b * tiles), dim3(256), lds, s, p)) return rc;
  const dim3 grid(p.b * p.n_splits * p.v_chunks);
  if (qb == 1) return launch_kernel(latent_pv_kernel<1, 4, false>, grid, dim3(256), 0, s, p);
  return launch_kernel(latent_pv_kernel<2, 4, false>, grid, dim3(256), 0, s, p);
}

}  // namespace lorc
