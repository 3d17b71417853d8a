// Decode attention over the latent cache (Eq. 1 on cached latents; GQA of Section 4.3; RoPE applied at read
// time to the rebuilt keys, as the cache holds un-rotated latents).
//
// Two launches per call:
//   split    : one workgroup per (sequence, context split).  Per tile of T positions it copies the K latents
//              into LDS once, and for every KV head rebuilds K^T = B_k^T C_k^T on the matrix cores (B_k tiles
//              stream from L2, the latent tile is reused by all heads), rotates it in registers, takes
//              scores against the group's query heads, keeps an online softmax per head, and accumulates
//              o_lat += P C_v in latent space with the V latents loaded straight from the cache
//   merge    : combine the splits' (m, l, o_lat) and apply the value up-projection o = o_lat B_v
#include <type_traits>

#include "lorc_device.h"
#include "lorc_kernels.h"
#include "lorc_rebuild.h"

namespace lorc {

constexpr float kNegInf = -__builtin_huge_valf();

// N independent reductions over the 32 lanes of each wavefront half, walked step by step together so that their
// dependency chains overlap.
template <int N, class Op>
__device__ __forceinline__ void half_wave_reduce(float (&v)[N], Op op) {
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = op(v[i], half_wave_peer<0>(v[i]));
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = op(v[i], half_wave_peer<1>(v[i]));
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = op(v[i], half_wave_peer<2>(v[i]));
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = op(v[i], half_wave_peer<3>(v[i]));
#pragma unroll
  for (int i = 0; i < N; ++i) {  // the half's two rows
    const float2 rows = row_pair(v[i]);
    v[i] = op(rows.x, rows.y);
  }
}

__host__ __device__ inline size_t decode_lds_bytes(int T, int QB, int G, int r_k, int half) {
  size_t b = (size_t)T * r_k * 2;        // K latent tile
  b += (size_t)2 * G * T * 4;            // partner exchange of partial scores
  b += (size_t)QB * 32 * T * 2 + 128;    // P operands + one scrap element per lane
  b += (size_t)3 * QB * 32 * 4;          // alpha, running max, running sum
  b += (size_t)(T / 32) * half * 8;      // per-tile rotation bases
  b += (size_t)QB * 32 * half * 2 * 2;   // rotated, scaled queries of the sequence (fp16)
  return b;
}


// ------------------------------------------------------------------------------------------------ split
// JR = accumulator registers of a score block that can hold real query heads (rows 4*hf + j, j < JR <= 4
// covers G <= 8; JR = 16 covers G <= 32).
template <int HD, int NPB, int QB, int NBW, int JR, int OCC>
__global__ __launch_bounds__(256, OCC) void decode_split_kernel(DecodeParams p) {
  constexpr int T = 32 * NPB, HALF = HD / 2, KP = T / 16, PAGES = T / kPage;
  constexpr int PF = 4;  // B_k operand prefetch depth (k-steps)
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index as a scalar: keeps per-wave addresses in SGPRs
  const int seq = blockIdx.x / p.n_splits, split = blockIdx.x % p.n_splits;
  const int r_k = p.r_k, r_v = p.r_v, G = p.G, nks = r_k >> 4;
  auto my_tid = [&]() {
    int l = lane_id();
    asm volatile("" : "+v"(l));
    return l + (w << 6);
  };

  uint16_t* ck = reinterpret_cast<uint16_t*>(smem);
  float* xbuf = reinterpret_cast<float*>(smem + (size_t)T * r_k * 2);
  uint16_t* pbuf = reinterpret_cast<uint16_t*>(xbuf + 2 * G * T);
  float* alpha = reinterpret_cast<float*>(pbuf + QB * 32 * T + 64);  // 64 scrap elements follow the P operands
  float* m_run = alpha + QB * 32;
  float* l_run = m_run + QB * 32;
  float2* cs_base = reinterpret_cast<float2*>(l_run + QB * 32);
  _Float16* qrot = reinterpret_cast<_Float16*>(cs_base + NPB * HALF);  // [h_q][HD]
  // Everything the set-up needs from memory is requested here, before any of it is used, so that it costs one
  // round trip: the context length, the page ids of the split's first tile (speculatively: whether the tile
  // exists depends on the context length), the query position and this thread's share of the query rows, the
  // rotation tables.
  const int tile_begin = split * p.tiles_per_split;
  const int ctx_raw = p.ctx_len[seq];
  int ids0[PAGES];
#pragma unroll
  for (int pg = 0; pg < PAGES; ++pg) {
    const int pi = (tile_begin * T) / kPage + pg;
    ids0[pg] = pi < p.max_pages ? p.block_table[(size_t)seq * p.max_pages + pi] : -1;
  }
  const int q_pos = p.q_pos[seq];
  const double theta_t = p.rope_tab[tid % HALF];
  constexpr int QI = QB * 32 * HALF / 256;  // (head, frequency) pairs of the query per thread
  uint16_t q_lo[QI], q_hi[QI];
  {
    const uint16_t* qsrc = p.q + (size_t)seq * p.h_q * HD;
#pragma unroll
    for (int u = 0; u < QI; ++u) {
      const int idx = tid + 256 * u, h = idx / HALF, i = idx % HALF;
      const int hc = h < p.h_q ? h : p.h_q - 1;  // unconditional loads (rows past the last head repeat it, unused)
      q_lo[u] = qsrc[hc * HD + i];
      q_hi[u] = qsrc[hc * HD + i + HALF];
    }
  }
  // Per-lane rotation constants: (cos, sin)((lane % 32) * theta_i) for the 16 frequencies this lane's
  // accumulator rows carry.  The wave's half of the head (HD = 128) is fixed: task % 2 == wave % 2.
  const int fbase = HD == 128 ? 32 * (w & 1) : 0;
  float cl[16], sl[16];
#pragma unroll
  for (int jj = 0; jj < 16; ++jj) {
    const float2 t = p.lane_cs[l32 * HALF + fbase + acc_row(jj, hf)];
    cl[jj] = t.x;
    sl[jj] = t.y;
  }

  // All of the above has to be here before the first tile is requested: the tile's loads are counted in the same
  // in-order counter and their number is not known at compile time, so any later wait for one of the values
  // above would turn into a wait for the whole tile.
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  int ctx = ctx_raw;
  ctx = ctx < 0 ? 0 : (ctx > p.max_ctx ? p.max_ctx : ctx);
  int tile_end = tile_begin + p.tiles_per_split;
  const int n_tiles = (ctx + T - 1) / T;
  if (tile_end > n_tiles) tile_end = n_tiles;

  // Pages of a tile (nullptr = not cached) and the copy of their K latents into LDS.  The copy is made of direct
  // global -> LDS loads, 1 KiB per instruction, the LDS image being the page's own tiling; it is issued while the
  // previous tile still has its softmax and P C_v phases to run, and waited for at the top of the tile.
  // Page ids of a tile are fetched one tile ahead (a vector load: its latency hides behind the tile's work) and
  // turned into pointers when the tile's K latents are requested.
  auto fetch_ids = [&](int tile_, int (&ids)[PAGES]) {
    const int valid_ = ctx - tile_ * T;
#pragma unroll
    for (int pg = 0; pg < PAGES; ++pg) {
      ids[pg] = -1;
      if (tile_ < tile_end && pg * kPage < valid_) ids[pg] = p.block_table[(size_t)seq * p.max_pages + (tile_ * T) / kPage + pg];
    }
  };
  auto ids_to_pages = [&](const int (&ids)[PAGES], const uint16_t* (&pp)[PAGES]) {
#pragma unroll
    for (int pg = 0; pg < PAGES; ++pg) {
      const int id = __builtin_amdgcn_readfirstlane(ids[pg]);
      pp[pg] = id >= 0 && id < p.n_pages ? p.cache + (size_t)id * p.page_elems : nullptr;
    }
  };
  // Waves blk0, blk0 + stride, ... of the issuing set each take every stride-th KiB block.
  auto issue_k_tile = [&](int tile_, const uint16_t* const (&pp)[PAGES], int blk0, int stride) {
    const int valid_ = ctx - tile_ * T;
    const int n_kib = r_k >> 3;  // 64 * r_k * 2 bytes per page / 1024
    int lo = lane_id(), zero = 0;  // recomputed / opaque: nothing derived from them is carried in registers
    asm volatile("" : "+v"(lo), "+v"(zero));
#pragma unroll
    for (int pg = 0; pg < PAGES; ++pg) {
      uint16_t* dst = ck + (size_t)pg * kPage * r_k;
      if (pp[pg] != nullptr) {
        const __amdgpu_buffer_rsrc_t pr = make_rsrc(pp[pg], (uint32_t)kPage * r_k * 2u);
        for (int blk = blk0; blk < n_kib; blk += stride)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(pr, (__attribute__((address_space(3))) void*)(dst + (size_t)blk * 512), 16, lo * 16,
                                                   blk * 1024, 0, 2);
      } else if (pg * kPage < valid_) {
        const u32x4 z = {(uint32_t)zero, (uint32_t)zero, (uint32_t)zero, (uint32_t)zero};
        for (int c = blk0 * 64 + lo; c < 8 * r_k; c += stride * 64) reinterpret_cast<u32x4*>(dst)[c] = z;
      }
    }
  };

  // One 1 KiB operand block of a page's V latents (used once: streamed past the caches).  For a page that is not
  // cached the load is still issued, through a descriptor of size zero: it fetches nothing and returns zeros; the
  // caller masks what it reads all the same.
  auto v_operand = [&](const uint16_t* page, int kib, int lane_) {
    const __amdgpu_buffer_rsrc_t vr = make_rsrc((page != nullptr ? page : p.cache) + (size_t)kPage * r_k, page != nullptr ? (uint32_t)kPage * r_v * 2u : 0u);
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(vr, lane_ * 16, kib * 1024, 2));
  };

  // One-page tiles: the first tile's K latents are requested into registers right here (sixteen 1 KiB blocks per
  // wave, a fixed count; blocks past the rank and pages that are not cached come back as zeros without a fetch),
  // travel while the set-up below runs, and are written to LDS where the set-up's own LDS traffic is over.
  // Later tiles come by direct global -> LDS loads, which the set-up's LDS reads would have to wait for.
  constexpr int KST = PAGES == 1 ? 16 : 1;
  static_assert(PAGES != 1 || kStreamMaxRank / 8 <= 4 * 16 * 2, "blocks per page against the staging registers");
  const uint16_t* page_ptr[PAGES];
#pragma unroll
  for (int pg = 0; pg < PAGES; ++pg) page_ptr[pg] = nullptr;
  u32x4 kstage[KST];
  const bool stage_first = PAGES == 1 && (r_k >> 3) <= 4 * KST;  // every block of the page has a register
  if (stage_first && tile_begin < tile_end) {
    if (0 >= ctx - tile_begin * T) ids0[0] = -1;
    ids_to_pages(ids0, page_ptr);
    const __amdgpu_buffer_rsrc_t pr = make_rsrc(page_ptr[0] != nullptr ? page_ptr[0] : p.cache, page_ptr[0] != nullptr ? (uint32_t)kPage * r_k * 2u : 0u);
    int lo = lane_id();
    asm volatile("" : "+v"(lo));
#pragma unroll
    for (int u = 0; u < KST; ++u) kstage[u] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(pr, lo * 16, (w + 4 * u) * 1024, 2));
  }

  // Set-up work that needs the thread index comes before the first tile is requested, so that nothing derived
  // from it has to be kept (or reloaded, which would wait for the tile) across the request.
  const int tq = my_tid();
  if (tq < QB * 32) {
    alpha[tq] = 0.f;
    m_run[tq] = kNegInf;
    l_run[tq] = 0.f;
  }
  for (int i = tq; i < QB * 32 * T / 2; i += 256) reinterpret_cast<uint32_t*>(pbuf)[i] = 0u;
  // Queries of this sequence: rotated at q_pos, scaled (softmax scale x log2 e) and rounded to fp16 once, kept in
  // LDS; the score operands of every pass are gathered from there.  cs_base is free until the first tile.
  if (tq < HALF) {
    double a = (double)q_pos * theta_t;
    a -= kTwoPi * rint(a / kTwoPi);
    float sn, cs;
    sincosf((float)a, &sn, &cs);
    cs_base[tq] = make_float2(cs, sn);
  }
  int q_dst[QI], q_cs[QI];  // where this thread's query pairs go, and which rotation they take
  float q_lf[QI], q_hf[QI];  // the pairs, scaled (their first use is here, before the tile request, on purpose)
#pragma unroll
  for (int u = 0; u < QI; ++u) {
    const int idx = tq + 256 * u, h = idx / HALF, i = idx % HALF;
    q_dst[u] = h < p.h_q ? h * HD + i : -1;
    q_cs[u] = i;
    q_lf[u] = bf16_to_float(q_lo[u]) * p.q_scale;
    q_hf[u] = bf16_to_float(q_hi[u]) * p.q_scale;
    asm volatile("" : "+v"(q_lf[u]), "+v"(q_hf[u]));  // pins the computation (and its wait) here
  }

  lds_barrier();
#pragma unroll
  for (int u = 0; u < QI; ++u) {
    if (q_dst[u] >= 0) {
      const float2 cs = cs_base[q_cs[u]];
      qrot[q_dst[u]] = static_cast<_Float16>(q_lf[u] * cs.x - q_hf[u] * cs.y);
      qrot[q_dst[u] + HALF] = static_cast<_Float16>(q_hf[u] * cs.x + q_lf[u] * cs.y);
    }
  }
  lds_barrier();

  // First tile.  By direct-to-LDS loads it is requested only now: an LDS read that follows such a load in program
  // order waits for it (the compiler cannot tell the two apart), so the set-up's LDS traffic has to be over first.
  if (stage_first) {
    if (tile_begin < tile_end) {
      int lo = lane_id();
      asm volatile("" : "+v"(lo));
#pragma unroll
      for (int u = 0; u < KST; ++u)
        if (w + 4 * u < (r_k >> 3)) reinterpret_cast<u32x4*>(ck)[(size_t)(w + 4 * u) * 64 + lo] = kstage[u];
    }
  } else if (tile_begin < tile_end) {
#pragma unroll
    for (int pg = 0; pg < PAGES; ++pg)
      if (pg * kPage >= ctx - tile_begin * T) ids0[pg] = -1;  // page past the context: not part of the tile
    ids_to_pages(ids0, page_ptr);
    issue_k_tile(tile_begin, page_ptr, w, 4);
  }

  f32x16 o[QB][NBW];
#pragma unroll
  for (int a = 0; a < QB; ++a)
#pragma unroll
    for (int b = 0; b < NBW; ++b)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[a][b][j] = 0.f;

  const int n_pass = (p.n_tasks + 3) >> 2;
  const __amdgpu_buffer_rsrc_t bk_rsrc = make_rsrc(p.bk, (uint32_t)p.h_kv * HD * r_k * 2u);

  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int pos0 = tile * T;
    const int valid = (ctx - pos0) < T ? (ctx - pos0) : T;
    const uint16_t* next_ptr[PAGES];
#pragma unroll
    for (int pg = 0; pg < PAGES; ++pg) next_ptr[pg] = nullptr;
    int next_ids[PAGES];
    fetch_ids(tile + 1, next_ids);

    // ---- 1. rotation bases of the tile; the tile's K latents (requested earlier) must have landed
    const int tt = my_tid();
    if (tt < NPB * HALF) {
      double a = (double)(pos0 + 32 * (tt / HALF)) * p.rope_tab[tt % HALF];
      a -= kTwoPi * rint(a / kTwoPi);
      float s, c;
      sincosf((float)a, &s, &c);
      cs_base[tt] = make_float2(c, s);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    lds_barrier();

    // The V operands of the first group of latent blocks and the next tile's K latents are requested as soon as
    // the last head has been rebuilt (the K tile in LDS is dead from then on), and arrive while the softmax and
    // the P C_v product of this tile run.
    constexpr int NG = NBW < 4 ? NBW : 4;
    u32x4 vraw0[NG][KP];
    auto request_ahead = [&]() {
      if (tile + 1 < tile_end) {
        ids_to_pages(next_ids, next_ptr);
        // HD = 128: the odd waves have no softmax to run, they issue the whole tile
        if (HD != 128) issue_k_tile(tile + 1, next_ptr, w, 4);
        else if (w & 1) issue_k_tile(tile + 1, next_ptr, w >> 1, 2);
      }
      int lo = lane_id();
      asm volatile("" : "+v"(lo));
#pragma unroll
      for (int i = 0; i < NG; ++i) {
        const int nb = w + 4 * i;
        const int nbc = nb * 32 < r_v ? nb : w;  // clamp: blocks past r_v are loaded but never used
#pragma unroll
        for (int kp = 0; kp < KP; ++kp) vraw0[i][kp] = v_operand(page_ptr[kp >> 2], nbc * 4 + (kp & 3), lo);
      }
    };

    // ---- 2. per KV head: rebuild K^T, rotate, score, softmax bookkeeping
    auto head_pass = [&](int ps, auto last_tag) {
      constexpr bool kLast = decltype(last_tag)::value;  // the tile's last pass: peeled, it starts the loads ahead
      const int task = ps * 4 + w;
      const bool active = task < p.n_tasks;
      const int g = HD == 128 ? task >> 1 : task;
      const int wh = HD == 128 ? task & 1 : 0;
      float sr[NPB][JR];  // scores of the real query-head rows

      if (active) {
        const int cb0 = HD == 128 ? g * 4 + wh : g * 2;
        const int cb1 = cb0 + (HD == 128 ? 2 : 1);

        f32x16 acc[2][NPB];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[a][pb][j] = 0.f;

        rebuild_pair<NPB, PF>(acc, bk_rsrc, (uint32_t)(cb0 * nks) * 1024u, (uint32_t)(cb1 * nks) * 1024u, (uint32_t)lane * 16u, ck + (size_t)lane * 8, nks);
        __builtin_amdgcn_sched_barrier(0);
        // rotate (pair = same register of the two accumulator blocks), round to fp16, score
        // Score A operands (m = query head of the group, k = 16 head-dim coordinates), in the order in which
        // the rotated K^T accumulators are re-used as B operands: element e of operand s4 is coordinate
        // 16*(s4 & 1) + 8*(e >> 2) + 4*hf + (e & 3) of half s4 >> 1 of the head (+ 32*wh for HD = 128).
        f16x8 qf[4];
        {
          const bool qreal = l32 < G;
          const _Float16* qh = qrot + (size_t)(g * G + (qreal ? l32 : 0)) * HD + (HD == 128 ? 32 * wh : 0) + 4 * hf;
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
            const float2 cb = cs_base[pb * HALF + fbase + acc_row(jj, hf)];
            const float cA = cb.x * cl[jj] - cb.y * sl[jj];
            const float sA = cb.y * cl[jj] + cb.x * sl[jj];
            const float x = acc[0][pb][jj], y = acc[1][pb][jj];
            kf[jj >> 3][jj & 7] = static_cast<_Float16>(x * cA - y * sA);
            kf[2 + (jj >> 3)][jj & 7] = static_cast<_Float16>(y * cA + x * sA);
          }
          f32x16 sa;
#pragma unroll
          for (int j = 0; j < 16; ++j) sa[j] = 0.f;
#pragma unroll
          for (int s4 = 0; s4 < 4; ++s4) sa = mfma32_f16(qf[s4], kf[s4], sa);
#pragma unroll
          for (int jr = 0; jr < JR; ++jr) sr[pb][jr] = sa[jr];
          __builtin_amdgcn_sched_barrier(0);  // keep one position block in flight: bounds live registers
        }
      }
      if (HD == 128) {
        // the two waves of a head each hold half of the head-dim contraction
        float* xb = xbuf + (size_t)(w >> 1) * G * T;
        if (active && wh == 1) {
#pragma unroll
          for (int jr = 0; jr < JR; ++jr) {
            const int m = acc_row(jr, hf);
            if (m < G) {
#pragma unroll
              for (int pb = 0; pb < NPB; ++pb) xb[m * T + pb * 32 + l32] = sr[pb][jr];
            }
          }
        }
        __syncthreads();
        if constexpr (kLast) request_ahead();
        if (active && wh == 0) {
#pragma unroll
          for (int jr = 0; jr < JR; ++jr) {
            const int m = acc_row(jr, hf);
            if (m < G) {
#pragma unroll
              for (int pb = 0; pb < NPB; ++pb) sr[pb][jr] += xb[m * T + pb * 32 + l32];
            }
          }
        }
      }
      if (active && wh == 0) {
        // Online softmax for the JR head rows this lane may hold; the rows are walked together so that their
        // cross-lane reductions (independent dependency chains) overlap instead of running back to back.
        // Lanes whose register is not a query head of the group do the same arithmetic on harmless values and
        // store to a scrap slot: no per-row branches.  The lane index is recomputed here, so that the LDS addresses
        // below are rebuilt on the spot instead of being carried (spilled) across the rebuild loop.
        int lid = lane_id();
        asm volatile("" : "+v"(lid));
        const int lq = lid & 31, hq = lid >> 5;
        const int lane_t = (lq >> 4) * 512 + ((lq >> 3) & 1) * 256 + (lq & 7);  // position part of the P operand index
        float mx[JR], m_old[JR], sum[JR];
        int hterm[JR];
        bool real[JR];
#pragma unroll
        for (int jr = 0; jr < JR; ++jr) {
          const int row = 8 * (jr >> 2) + 4 * hq + (jr & 3);
          real[jr] = row < G;
          const int h = real[jr] ? g * G + row : 0;
          hterm[jr] = (h >> 5) * (KP * 512) + (h & 31) * 8 + lane_t;
          mx[jr] = kNegInf;
#pragma unroll
          for (int pb = 0; pb < NPB; ++pb) {
            if (pb * 32 + lq >= valid) sr[pb][jr] = kNegInf;
            mx[jr] = fmaxf(mx[jr], sr[pb][jr]);
          }
          const float mo = m_run[h];
          m_old[jr] = real[jr] ? mo : 0.f;
        }
        half_wave_reduce<JR>(mx, [](float x, float y) { return fmaxf(x, y); });
        const int scrap = QB * 32 * T + (hq * 32 + lq);  // past the P operands: one element per lane
#pragma unroll
        for (int jr = 0; jr < JR; ++jr) {
          const float m_new = fmaxf(m_old[jr], mx[jr]);
          mx[jr] = m_new;
          sum[jr] = 0.f;
#pragma unroll
          for (int pb = 0; pb < NPB; ++pb) {
            const float pv = __builtin_amdgcn_exp2f(sr[pb][jr] - m_new);  // arguments <= 0: no range fix-up needed
            sum[jr] += pv;
            pbuf[real[jr] ? hterm[jr] + pb * 1024 : scrap] = bf16_bits(pv);
          }
        }
        half_wave_reduce<JR>(sum, [](float x, float y) { return x + y; });
        // lane jr of each half files the running state of register jr's row
        float s_new = mx[0], s_old = m_old[0], s_sum = sum[0];
#pragma unroll
        for (int jr = 1; jr < JR; ++jr) {
          s_new = lq == jr ? mx[jr] : s_new;
          s_old = lq == jr ? m_old[jr] : s_old;
          s_sum = lq == jr ? sum[jr] : s_sum;
        }
        const int srow = 8 * (lq >> 2) + 4 * hq + (lq & 3);
        if (lq < JR && srow < G) {
          const int h = g * G + srow;
          const float a = __builtin_amdgcn_exp2f(s_old - s_new);
          m_run[h] = s_new;
          l_run[h] = l_run[h] * a + s_sum;
          alpha[h] = a;
        }
      }
      if (HD == 128) lds_barrier();
    };
    for (int ps = 0; ps + 1 < n_pass; ++ps) head_pass(ps, std::false_type{});
    head_pass(n_pass - 1, std::true_type{});
    lds_barrier();
    if (HD != 128) request_ahead();  // no barrier inside the passes: only here is the K tile known to be dead

    // ---- 3. o_lat = alpha * o_lat + P C_v : wave w owns latent blocks w, w+4, ... of the V latent
    {
      float al[QB][16];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) al[qb][jj] = alpha[qb * 32 + acc_row(jj, hf)];
      // Slots past the context hold whatever the pool held before: P is zero there, but 0 * NaN is not,
      // so the V operand is masked.  vmask[kp] = bit e set when position kp*16 + 8*hf + e is cached.
      // Loads are unconditional (for a page that is not cached they return zeros and are fully masked) so that
      // all of a block's operands are in flight together.
      uint32_t vmask[KP];
#pragma unroll
      for (int kp = 0; kp < KP; ++kp) {
        int nv = valid - kp * 16 - 8 * hf;
        nv = nv < 0 ? 0 : (nv > 8 ? 8 : nv);
        vmask[kp] = page_ptr[kp >> 2] != nullptr ? (1u << nv) - 1u : 0u;
      }
      // The V operands of up to four latent blocks (all positions of the tile) are requested before any is
      // used: the loads are the only HBM traffic of this phase and need that much in flight to stream.  The
      // first group was requested ahead.
#pragma unroll
      for (int n0 = 0; n0 < NBW; n0 += NG) {
        u32x4 vraw[NG][KP];
#pragma unroll
        for (int i = 0; i < NG; ++i) {
          const int nb = w + 4 * (n0 + i);
          const int nbc = nb * 32 < r_v ? nb : w;  // clamp: blocks past r_v are loaded but never used
#pragma unroll
          for (int kp = 0; kp < KP; ++kp) {
            if (n0 == 0) {
              vraw[i][kp] = vraw0[i][kp];
            } else {
              vraw[i][kp] = v_operand(page_ptr[kp >> 2], nbc * 4 + (kp & 3), lane);
            }
          }
        }
#pragma unroll
        for (int i = 0; i < NG; ++i) {
          const int nbw = n0 + i;
          const int nb = w + 4 * nbw;
          if (nb * 32 < r_v) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
              for (int jj = 0; jj < 16; ++jj) o[qb][nbw][jj] *= al[qb][jj];
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) {
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                const uint32_t two = (vmask[kp] >> (2 * c)) & 3u;
                vraw[i][kp][c] &= (two & 1u ? 0x0000ffffu : 0u) | (two & 2u ? 0xffff0000u : 0u);
              }
              const bf16x8 vb = __builtin_bit_cast(bf16x8, vraw[i][kp]);
#pragma unroll
              for (int qb = 0; qb < QB; ++qb) {
                const bf16x8 pa = load_frag(pbuf + ((size_t)(qb * KP + kp) * 64 + lane) * 8);
                o[qb][nbw] = mfma32(pa, vb, o[qb][nbw]);
              }
            }
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    lds_barrier();
#pragma unroll
    for (int pg = 0; pg < PAGES; ++pg) page_ptr[pg] = next_ptr[pg];
  }

  // ---- partials of this split
  const size_t pbase = (size_t)seq * p.n_splits + split;
  __syncthreads();
  const int te = my_tid();
  if (te < p.h_q) {
    p.part_ml[(pbase * p.h_q + te) * 2 + 0] = m_run[te];
    p.part_ml[(pbase * p.h_q + te) * 2 + 1] = l_run[te];
  }
  // The split's latent-space output is stored normalised by its own sum (so that it is bounded by the value
  // latents and fits fp16, half the bytes of fp32); always written (zeros for a split past the context) so that
  // the merge can read without guards.  The workgroup's rows [h_q][r_v] are one contiguous range of the
  // workspace: when they fit into the (now dead) K tile they are staged there and written as whole 16-byte
  // chunks, a full row per wave and store, instead of as two-byte elements.
  const int pitch = r_v * 2 + 16;  // bytes; the +16 puts the two half-wave rows of an accumulator on different banks
  const bool staged = (size_t)QB * 32 * pitch <= (size_t)T * r_k * 2;
  unsigned char* stage = smem;
  uint16_t* dst_rows = p.part_o + pbase * p.h_q * r_v;
  float inv_l[QB][16];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int jj = 0; jj < 16; ++jj) {
      const float l = l_run[qb * 32 + acc_row(jj, hf)];
      inv_l[qb][jj] = l > 0.f ? __builtin_amdgcn_rcpf(l) : 0.f;
    }
  if (staged) {  // one branch around the whole write-out: the element loops below are straight-line code
    unsigned char* lane_base = stage + (size_t)(4 * hf) * pitch + l32 * 2 + w * 64;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int nbw = 0; nbw < NBW; ++nbw) {
        if ((w + 4 * nbw) * 32 < r_v) {
#pragma unroll
          for (int jj = 0; jj < 16; ++jj)
            *reinterpret_cast<uint16_t*>(lane_base + (qb * 32 + 8 * (jj >> 2) + (jj & 3)) * pitch + nbw * 256) =
                f16_bits(o[qb][nbw][jj] * inv_l[qb][jj]);
        }
      }
    lds_barrier();
    const int cpr = r_v >> 3;  // 16-byte chunks per row
    const int n_chunks = p.h_q * cpr;
    for (int c = te; c < n_chunks; c += 256) {
      const int h = c / cpr, cc = c - h * cpr;
      const u32x4 v = *reinterpret_cast<const u32x4*>(stage + (size_t)h * pitch + cc * 16);
      *reinterpret_cast<u32x4*>(dst_rows + (size_t)c * 8) = v;
    }
  } else {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int nbw = 0; nbw < NBW; ++nbw) {
        const int nb = w + 4 * nbw;
        if (nb * 32 < r_v) {
#pragma unroll
          for (int jj = 0; jj < 16; ++jj) {
            const int h = qb * 32 + acc_row(jj, hf);
            if (h < p.h_q) dst_rows[(size_t)h * r_v + nb * 32 + l32] = f16_bits(o[qb][nbw][jj] * inv_l[qb][jj]);
          }
        }
      }
  }
}

// ------------------------------------------------------------------------------------------------ merge
// One workgroup per (sequence, query head): softmax-merge the splits' (m, l, o_lat), then the value
// up-projection o = o_lat B_v^g with the 256 threads laid out as head_dim columns x latent slices.
constexpr int kMaxSplits = 512;

template <int HD>
__global__ __launch_bounds__(256) void decode_merge_kernel(DecodeParams p) {
  constexpr int NS = 256 / HD;  // latent slices reduced through LDS
  __shared__ float olat[kWideMaxRank];
  __shared__ float wgt[kMaxSplits];
  __shared__ float red[NS][HD];
  const int tid = threadIdx.x, lane = tid & 63;
  const int seq = blockIdx.x / p.h_q, h = blockIdx.x % p.h_q, g = h / p.G;
  const int r_v = p.r_v, ns = p.n_splits;
  if (tid < 64) {  // first wave: weights of the splits
    const float* ml = p.part_ml + ((size_t)seq * ns * p.h_q + h) * 2;
    const size_t st = (size_t)p.h_q * 2;
    float M = kNegInf;
    for (int s = lane; s < ns; s += 64) M = fmaxf(M, ml[s * st]);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
    float L = 0.f;
    for (int s = lane; s < ns; s += 64) {
      const float ms = ml[s * st];
      const float e = (ms == kNegInf ? 0.f : exp2f(ms - M)) * ml[s * st + 1];  // partials are stored normalised
      L += e;
      wgt[s] = e;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) L += __shfl_xor(L, off);
    const float invL = L > 0.f ? 1.f / L : 0.f;
    for (int s = lane; s < ns; s += 64) wgt[s] *= invL;
  }
  __syncthreads();
  {
    const uint16_t* po = p.part_o + ((size_t)seq * ns * p.h_q + h) * r_v;
    const size_t st = (size_t)p.h_q * r_v;
    for (int j = tid; j < r_v; j += 256) {
      float a = 0.f;
      int s = 0;
      for (; s + 8 <= ns; s += 8) {
        uint16_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = po[(size_t)(s + u) * st + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) a += wgt[s + u] * (float)__builtin_bit_cast(_Float16, v[u]);
      }
      for (; s < ns; ++s) a += wgt[s] * (float)__builtin_bit_cast(_Float16, po[(size_t)s * st + j]);
      olat[j] = a;
    }
  }
  __syncthreads();
  if (p.latent_out) {  // o_lat / l itself is the result: the caller applies B_v (or a matrix that absorbed it)
    for (int j = tid; j < r_v; j += 256) p.out[((size_t)seq * p.h_q + h) * r_v + j] = bf16_bits(olat[j]);
    return;
  }
  const int c = tid % HD, sl = tid / HD;
  const int cg = g * HD + c;
  const int per = ((r_v / 8 + NS - 1) / NS) * 8;  // latent indices per slice (multiple of 8)
  const int j_begin = sl * per, j_end = (j_begin + per) < r_v ? (j_begin + per) : r_v;
  float acc = 0.f;
  int j = j_begin;
  for (; j + 32 <= j_end; j += 32) {
    bf16x8 bv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) bv[u] = load_frag(p.bv + b_tile_index(r_v, j + 8 * u, cg));
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc += olat[j + 8 * u + e] * (float)bv[u][e];
  }
  for (; j < j_end; j += 8) {
    const bf16x8 bv = load_frag(p.bv + b_tile_index(r_v, j, cg));
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += olat[j + e] * (float)bv[e];
  }
  red[sl][c] = acc;
  __syncthreads();
  if (tid < HD) {
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i) v += red[i][tid];
    p.out[((size_t)seq * p.h_q + h) * HD + tid] = bf16_bits(v);
  }
}

// ------------------------------------------------------------------------------------------------ merge, common shapes
// One workgroup of sixteen waves per (sequence, KV head): the G query heads of the group share the factor block
// B_v^g, which is read once, as matrix-core operands, and requested before anything else; the split partials are
// requested next (four fp16 columns per thread, 32 splits in flight), the split weights are worked out
// while they travel.  The up-projection runs on the matrix cores with o_lat split into a bf16 head and a bf16
// remainder (two products), so that it keeps the accuracy of an fp32 o_lat.  Shapes: G <= 8, at most 64 splits,
// r_v <= 512.
// HS = 2: the group's heads are dealt to two workgroups of eight waves (small batches: twice as many workgroups,
// each with half the partials to fetch; the factor block is then read by both).
constexpr int kMgMaxG = 8, kMgMaxSplits = 64, kMgMaxRank = 512, kMgBatch = 32;

template <int HD, int HS>
__global__ __launch_bounds__(1024 / HS) void decode_merge_group_kernel(DecodeParams p) {
  constexpr int NCB = HD / 32, NKQ = (16 / HS) / NCB, MAXKS = (kMgMaxRank / 16 + NKQ - 1) / NKQ;
  constexpr int MAXG = kMgMaxG / HS;
  __shared__ float wgt[MAXG][kMgMaxSplits];
  __shared__ __align__(16) uint16_t o_hi[MAXG][kMgMaxRank];
  __shared__ __align__(16) uint16_t o_lo[MAXG][kMgMaxRank];
  __shared__ float red[NKQ][HD][MAXG];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int sg = blockIdx.x / HS, seq = sg / p.h_kv, g = sg % p.h_kv;
  const int G = p.G / HS, r_v = p.r_v, ns = p.n_splits, nks = r_v >> 4;  // G: heads of this workgroup
  const int h0 = g * p.G + (blockIdx.x % HS) * G;                        // its first query head

  // ---- factor operands of this wave: column block cb of the head, k-steps [ks0, ks1)
  const int cb = w % NCB, kq = w / NCB;
  const int ks_per = (nks + NKQ - 1) / NKQ;
  const int ks0 = kq * ks_per, ks1 = ks0 + ks_per < nks ? ks0 + ks_per : nks;
  bf16x8 bvf[MAXKS];
  if (!p.latent_out) {
    const uint16_t* bp = p.bv + ((size_t)(g * NCB + cb) * nks * 64 + lane) * 8;
#pragma unroll
    for (int u = 0; u < MAXKS; ++u) {
      const int ks = ks0 + u < nks ? ks0 + u : nks - 1;
      bvf[u] = load_frag(bp + (size_t)ks * 512);
    }
  }

  // ---- first batch of partials: thread t owns o_lat[head t / (r_v/4)][4 * (t % (r_v/4)) .. +3]
  const int qpr = r_v >> 2;  // column groups per head
  const bool owner = tid < G * qpr;
  const int oh = owner ? tid / qpr : 0, oj = owner ? (tid % qpr) * 4 : 0;
  const uint16_t* po = p.part_o + (((size_t)seq * ns) * p.h_q + (size_t)h0 + oh) * r_v + oj;
  const size_t pst = (size_t)p.h_q * r_v;
  u32x2 pre[kMgBatch];
  auto load_batch = [&](int s0) {
#pragma unroll
    for (int u = 0; u < kMgBatch; ++u) {
      const int sidx = s0 + u < ns ? s0 + u : ns - 1;  // clamped: the tail is loaded again and weighted zero
      pre[u] = *reinterpret_cast<const u32x2*>(po + (size_t)sidx * pst);
    }
  };
  if (owner) load_batch(0);

  // ---- split weights: wave h < G handles head h, one split per lane
  if (w < G) {
    const int h = h0 + w;
    const float* ml = p.part_ml + (((size_t)seq * ns) * p.h_q + h) * 2;
    const size_t st = (size_t)p.h_q * 2;
    const float ms = lane < ns ? ml[lane * st] : kNegInf;
    const float ls = lane < ns ? ml[lane * st + 1] : 0.f;
    float M = ms;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float e = (ms == kNegInf ? 0.f : exp2f(ms - M)) * ls;  // partials are stored normalised
    float L = e;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) L += __shfl_xor(L, off);
    if (lane < ns) wgt[w][lane] = L > 0.f ? e / L : 0.f;
  }
  __syncthreads();

  // ---- o_lat = sum over splits of weight * partial
  if (owner) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < ns; s0 += kMgBatch) {
      if (s0 != 0) load_batch(s0);
#pragma unroll
      for (int u = 0; u < kMgBatch; ++u) {
        const float wv = s0 + u < ns ? wgt[oh][s0 + u] : 0.f;
        typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
        const f16x4 hv = __builtin_bit_cast(f16x4, pre[u]);
        const f32x4 fv = {(float)hv[0], (float)hv[1], (float)hv[2], (float)hv[3]};
        a += wv * fv;
      }
    }
    if (p.latent_out) {
      uint16_t* dst = p.out + ((size_t)seq * p.h_q + (size_t)h0 + oh) * r_v + oj;
      u32x2 pk = {(uint32_t)bf16_bits(a[0]) | ((uint32_t)bf16_bits(a[1]) << 16),
                  (uint32_t)bf16_bits(a[2]) | ((uint32_t)bf16_bits(a[3]) << 16)};
      *reinterpret_cast<u32x2*>(dst) = pk;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint16_t hi = bf16_bits(a[i]);
        o_hi[oh][oj + i] = hi;
        o_lo[oh][oj + i] = bf16_bits(a[i] - bf16_to_float(hi));
      }
    }
  }
  if (p.latent_out) return;
  __syncthreads();

  // ---- out^T[c][h] = sum_j B_v[j][c] o_lat[h][j]: A operand = factor tile (m = column), B operand = o_lat^T
  f32x16 acc;
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.f;
#pragma unroll
  for (int u = 0; u < MAXKS; ++u) {
    if (ks0 + u < ks1) {
      const int j0 = (ks0 + u) * 16 + 8 * hf;
      bf16x8 fh = zero_frag(), fl = zero_frag();
      if (l32 < G) {
        fh = load_frag(&o_hi[l32][j0]);
        fl = load_frag(&o_lo[l32][j0]);
      }
      acc = mfma32(bvf[u], fh, acc);
      acc = mfma32(bvf[u], fl, acc);
    }
  }
  if (l32 < G) {
#pragma unroll
    for (int j = 0; j < 16; ++j) red[kq][cb * 32 + acc_row(j, hf)][l32] = acc[j];
  }
  __syncthreads();
  if (tid < HD * G) {
    const int c = tid % HD, h = tid / HD;
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < NKQ; ++i) v += red[i][c][h];
    p.out[((size_t)seq * p.h_q + (size_t)h0 + h) * HD + c] = bf16_bits(v);
  }
}

// ------------------------------------------------------------------------------------------------ absorbed split
// Decode without positional rotation (Section 4.1, Eq. 7): the key factor is folded into the query, scores are
// taken in latent space, s[h][j] = q_lat[h] . c_K[j], and nothing is rebuilt.  32 flop per byte of latent: the
// kernel is a stream over the cache.  One workgroup per (sequence, context split), two per CU.  Every wave owns
// 16 of a tile's 64 positions for all heads (16x16x32 matrix-core products); a K operand block (16 positions x 32
// latent indices) is therefore used by exactly one wave and needs no staging in LDS: it goes from the cache
// straight into registers as the B operand, read out of the page's own tiling.  What sits in LDS is the absorbed
// query (A operands, tiled in operand order).  Softmax: row statistics inside the wave by DPP, one exchange of
// (max, sum) between the four waves through LDS, running statistics in LDS.  P C_v, the partials and the merge
// are those of the rotary path.  All loads are plain buffer loads of fixed count (also past the last tile, from a
// page nobody reads), so the compiler's partial waits are exact; 204 registers, no scratch.
constexpr int kAbsMaxRankK = 512;  // sixteen K operands per wave and tile, one register ring

__host__ __device__ inline size_t absorbed_lds_bytes(int r_k, int r_v) {
  const size_t qb = (size_t)32 * r_k * 2, st = (size_t)32 * (r_v * 2 + 16);
  return (qb > st ? qb : st) + (size_t)32 * kPage * 2 + 128 + (size_t)(2 * 32 * 4 + 32 + 32 + 32) * 4;
}

template <int NBW>
__global__ __launch_bounds__(256, 2) void decode_absorbed_kernel(DecodeParams p) {
  constexpr int T = kPage, KP = T / 16, NK32 = kAbsMaxRankK / 32;
  static_assert(NBW * KP == NK32, "K and V operands of a tile share one register ring");
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31, n16 = lane & 15, kg = lane >> 4;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int seq = blockIdx.x / p.n_splits, split = blockIdx.x % p.n_splits;
  const int r_k = p.r_k, r_v = p.r_v, nks = r_k >> 4, nk32 = r_k >> 5;
  const size_t qbytes = (size_t)32 * r_k * 2, stbytes = (size_t)32 * (r_v * 2 + 16);
  uint16_t* qlds = reinterpret_cast<uint16_t*>(smem);                           // [2 head blocks][nk32][64 lanes][8]
  uint16_t* pbuf = reinterpret_cast<uint16_t*>(smem + (qbytes > stbytes ? qbytes : stbytes));  // P operands (+ scrap)
  float* xm = reinterpret_cast<float*>(pbuf + 32 * T + 64);                     // [32 heads][4 waves] wave-local maxima
  float* xs = xm + 32 * 4;
  float* alpha = xs + 32 * 4;
  float* l_fin = alpha + 32;   // running sums (final after the last tile)
  float* m_fin = l_fin + 32;   // running maxima

  const int tile_begin = split * p.tiles_per_split;
  int ctx = __builtin_amdgcn_readfirstlane(p.ctx_len[seq]);
  ctx = ctx < 0 ? 0 : (ctx > p.max_ctx ? p.max_ctx : ctx);
  int tile_end = tile_begin + p.tiles_per_split;
  const int n_tiles = (ctx + T - 1) / T;
  if (tile_end > n_tiles) tile_end = n_tiles;

  // Set-up order: the page ids, the absorbed query and the first tile's K operands are three round trips to
  // memory; they are requested back to back (ids, query chunks into registers, then -- as soon as the ids are
  // back -- the K operands) and the query goes to LDS while the K operands travel.
  auto fetch_id = [&](int tile_) { return p.block_table[(size_t)seq * p.max_pages + (tile_ < p.max_pages ? tile_ : p.max_pages - 1)]; };
  const int id0 = fetch_id(tile_begin), id1 = fetch_id(tile_begin + 1);
  int id_nn = fetch_id(tile_begin + 2);
  // absorbed query: chunk c (8 latent indices) of head h goes to lane (h % 16) + 16 (c % 4) of operand
  // (h / 16, c / 4); heads past h_q are zero.  Unconditional loads of a fixed count (clamped, masked afterwards).
  constexpr int QCH = 32 * (kAbsMaxRankK / 8) / 256;
  const int cpr = r_k >> 3;
  u32x4 qv[QCH];
  {
    const uint16_t* qsrc = p.q + (size_t)seq * p.h_q * r_k;
#pragma unroll
    for (int u = 0; u < QCH; ++u) {
      const int c = tid + 256 * u < 32 * cpr ? tid + 256 * u : 32 * cpr - 1;
      const int h = c / cpr, cc = c - h * cpr;
      qv[u] = *reinterpret_cast<const u32x4*>(qsrc + (size_t)(h < p.h_q ? h : p.h_q - 1) * r_k + cc * 8);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  if (tid < 32) {
    alpha[tid] = 0.f;
    l_fin[tid] = 0.f;
    m_fin[tid] = kNegInf;
  }
  // Page ids are fetched a tile before they are needed and turned into wave-uniform pointers then; nullptr = not
  // cached or past the split's last tile: the loads are still issued (their count stays fixed) through a
  // descriptor of size zero, so they fetch nothing and return zeros, and everything read is masked as well.
  auto to_page = [&](int id_raw, int tile_) -> const uint16_t* {
    const int id = __builtin_amdgcn_readfirstlane(id_raw);
    return tile_ < tile_end && id >= 0 && id < p.n_pages ? p.cache + (size_t)id * p.page_elems : nullptr;
  };
  // K operand (positions 16 w .. 16 w + 15 of the page, latent indices 32 ks .. 32 ks + 31) straight from the page
  // tiling: lane (n, kg) takes the 16 bytes of position n, indices 8 kg .. 8 kg + 7.
  const uint32_t k_lane = (uint32_t)((((w >> 1) * nks + (kg >> 1)) * 64 + (w & 1) * 16 + n16 + 32 * (kg & 1)) * 16);
  auto k_frag = [&](const uint16_t* page, int ks) {
    const __amdgpu_buffer_rsrc_t pr = make_rsrc(uniform_ptr(page != nullptr ? page : p.cache), page != nullptr ? (uint32_t)kPage * r_k * 2u : 0u);
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(pr, k_lane, (ks < nk32 ? ks : nk32 - 1) * 2048, 2));
  };
  auto v_frag = [&](const uint16_t* page, int idx) {  // V operand idx = 4 * (block slot i) + kp of this wave
    const __amdgpu_buffer_rsrc_t vr = make_rsrc(uniform_ptr(page != nullptr ? page : p.cache) + (size_t)kPage * r_k, page != nullptr ? (uint32_t)kPage * r_v * 2u : 0u);
    const int nb = w + 4 * (idx >> 2);
    const int nbc = nb * 32 < r_v ? nb : w;  // clamp: blocks past r_v are loaded but never used
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(vr, lane * 16, (nbc * 4 + (idx & 3)) * 1024, 2));
  };

  f32x16 o[NBW];
#pragma unroll
  for (int b = 0; b < NBW; ++b)
#pragma unroll
    for (int j = 0; j < 16; ++j) o[b][j] = 0.f;

  const uint16_t* page_cur = to_page(id0, tile_begin);
  const uint16_t* page_nxt = to_page(id1, tile_begin + 1);
  // One ring of sixteen operand registers per wave carries the whole stream: slot j holds K operand j of a tile until
  // the scores have used it, then V operand j of the same tile until P C_v has used it, then K operand j of the
  // next tile.  Every slot is re-requested the moment it is consumed, so a workgroup always has one tile's K or V
  // latents (64 KiB) on their way.
  u32x4 ring[NK32];
#pragma unroll
  for (int u = 0; u < NK32; ++u) ring[u] = k_frag(page_cur, u);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < QCH; ++u) {
    const int c = tid + 256 * u;
    if (c < 32 * cpr) {
      const int h = c / cpr, cc = c - h * cpr;
      const u32x4 z = {0u, 0u, 0u, 0u};
      *reinterpret_cast<u32x4*>(qlds + ((size_t)((h >> 4) * nk32 + (cc >> 2)) * 64 + (h & 15) + 16 * (cc & 3)) * 8) = h < p.h_q ? qv[u] : z;
    }
  }
  __syncthreads();  // absorbed query in place
  const uint16_t* qa_lane = qlds + (size_t)lane * 8;

  for (int tile = tile_begin; tile < tile_end; ++tile) {
    const int valid = (ctx - tile * T) < T ? (ctx - tile * T) : T;
    // ---- scores; every K operand consumed is replaced by the request for the V operand of the same slot
    f32x4 sacc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int ks = 0; ks < NK32; ++ks) {
      // straight-line: a step past the rank re-reads the last query block and is switched off by zeroing that operand
      const int kc = ks < nk32 ? ks : nk32 - 1;
      const uint32_t keep = ks < nk32 ? 0xffffffffu : 0u;
      u32x4 a0 = *reinterpret_cast<const u32x4*>(qa_lane + (size_t)kc * 512), a1 = *reinterpret_cast<const u32x4*>(qa_lane + (size_t)(nk32 + kc) * 512);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        a0[c] &= keep;
        a1[c] &= keep;
      }
      const bf16x8 kf = __builtin_bit_cast(bf16x8, ring[ks]);
      sacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0), kf, sacc[0], 0, 0, 0);
      sacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1), kf, sacc[1], 0, 0, 0);
      ring[ks] = v_frag(page_cur, ks);
      __builtin_amdgcn_sched_barrier(0);  // keeps the query operand reads of later steps from being hoisted (and spilled)
    }
    // ---- wave-local softmax statistics (rows of 16 lanes share a head), exchanged once between the waves
    float pv[2][4], m_loc[2][4], s_loc[2][4];
    const bool in_ctx = page_cur != nullptr && 16 * w + n16 < valid;
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        pv[hb][j] = in_ctx ? sacc[hb][j] * p.q_scale : kNegInf;
        float m = pv[hb][j];
        m = fmaxf(m, half_wave_peer<0>(m));
        m = fmaxf(m, half_wave_peer<1>(m));
        m = fmaxf(m, half_wave_peer<2>(m));
        m = fmaxf(m, half_wave_peer<3>(m));
        m_loc[hb][j] = m;
        const float e = __builtin_amdgcn_exp2f(pv[hb][j] - fmaxf(m, -1e30f));  // all masked: exp2(-inf) = 0
        pv[hb][j] = e;
        float su = e;
        su += half_wave_peer<0>(su);
        su += half_wave_peer<1>(su);
        su += half_wave_peer<2>(su);
        su += half_wave_peer<3>(su);
        s_loc[hb][j] = su;
      }
    lds_barrier();  // the previous tile's readers of pbuf, alpha and the exchange arrays are done
    if (n16 == 0) {
#pragma unroll
      for (int hb = 0; hb < 2; ++hb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int h = hb * 16 + 4 * kg + j;
          xm[h * 4 + w] = m_loc[hb][j];
          xs[h * 4 + w] = s_loc[hb][j];
        }
    }
    lds_barrier();
    float lnew[2][4], mnew[2][4];
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int h = hb * 16 + 4 * kg + j;
        const f32x4 wm = *reinterpret_cast<const f32x4*>(xm + h * 4);
        const f32x4 wsu = *reinterpret_cast<const f32x4*>(xs + h * 4);
        const float m_old = m_fin[h];
        const float m_new = fmaxf(fmaxf(m_old, fmaxf(wm[0], wm[1])), fmaxf(wm[2], wm[3]));
        const float m_ref = fmaxf(m_new, -1e30f);
        if (w == 0 && n16 == 0) {  // one lane per head keeps the running state (read by everyone before the barrier below)
          float lsum = 0.f;
#pragma unroll
          for (int u = 0; u < 4; ++u) lsum += wsu[u] * __builtin_amdgcn_exp2f(wm[u] - m_ref);
          const float a = __builtin_amdgcn_exp2f(m_old - m_ref);
          alpha[h] = a;
          lnew[hb][j] = l_fin[h] * a + lsum;
        }
        mnew[hb][j] = m_new;
        pbuf[((size_t)w * 64 + h + 32 * (n16 >> 3)) * 8 + (n16 & 7)] = bf16_bits(pv[hb][j] * __builtin_amdgcn_exp2f(m_loc[hb][j] - m_ref));
      }
    lds_barrier();  // every lane has read the old running maxima: they can be replaced
    if (w == 0 && n16 == 0) {
#pragma unroll
      for (int hb = 0; hb < 2; ++hb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          m_fin[hb * 16 + 4 * kg + j] = mnew[hb][j];
          l_fin[hb * 16 + 4 * kg + j] = lnew[hb][j];
        }
    }
    // ---- o_lat = alpha * o_lat + P C_v : wave w owns latent blocks w, w + 4, ...
    {
      const bool ragged = page_cur == nullptr || valid < T;  // wave-uniform: only then the V operand needs masking
#pragma unroll
      for (int i = 0; i < NBW; ++i) {
        if ((w + 4 * i) * 32 < r_v) {
#pragma unroll
          for (int jj = 0; jj < 16; ++jj) o[i][jj] *= alpha[acc_row(jj, hf)];
          if (!ragged) {
#pragma unroll
            for (int kp = 0; kp < KP; ++kp)
              o[i] = mfma32(load_frag(pbuf + ((size_t)kp * 64 + lane) * 8), __builtin_bit_cast(bf16x8, ring[i * KP + kp]), o[i]);
          } else {
#pragma unroll
            for (int kp = 0; kp < KP; ++kp) {
              int nv = valid - kp * 16 - 8 * hf;
              nv = nv < 0 ? 0 : (nv > 8 ? 8 : nv);
              const uint32_t vmask = page_cur != nullptr ? (1u << nv) - 1u : 0u;
              u32x4 vv = ring[i * KP + kp];
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                const uint32_t two = (vmask >> (2 * c)) & 3u;
                vv[c] &= (two & 1u ? 0x0000ffffu : 0u) | (two & 2u ? 0xffff0000u : 0u);
              }
              o[i] = mfma32(load_frag(pbuf + ((size_t)kp * 64 + lane) * 8), __builtin_bit_cast(bf16x8, vv), o[i]);
            }
          }
        }
        // the slots of this block now take the next tile's K operands (past the last tile: a page nobody reads)
#pragma unroll
        for (int kp = 0; kp < KP; ++kp) ring[i * KP + kp] = k_frag(page_nxt, i * KP + kp);
      }
    }
    page_cur = page_nxt;
    page_nxt = to_page(id_nn, tile + 2);
    id_nn = fetch_id(tile + 3);
  }

  // ---- partials of this split (same format as the rotary path)
  const size_t pbase = (size_t)seq * p.n_splits + split;
  __syncthreads();  // every wave is done with the query operands: their memory becomes the staging area
  if (tid < p.h_q) {
    p.part_ml[(pbase * p.h_q + tid) * 2 + 0] = m_fin[tid];
    p.part_ml[(pbase * p.h_q + tid) * 2 + 1] = l_fin[tid];
  }
  __syncthreads();
  float inv_l[16];
#pragma unroll
  for (int jj = 0; jj < 16; ++jj) {
    const float l = l_fin[acc_row(jj, hf)];
    inv_l[jj] = l > 0.f ? __builtin_amdgcn_rcpf(l) : 0.f;
  }
  const int pitch = r_v * 2 + 16;
  unsigned char* lane_base = smem + (size_t)(4 * hf) * pitch + l32 * 2 + w * 64;
#pragma unroll
  for (int i = 0; i < NBW; ++i) {
    if ((w + 4 * i) * 32 < r_v) {
#pragma unroll
      for (int jj = 0; jj < 16; ++jj)
        *reinterpret_cast<uint16_t*>(lane_base + (8 * (jj >> 2) + (jj & 3)) * pitch + i * 256) = f16_bits(o[i][jj] * inv_l[jj]);
    }
  }
  lds_barrier();
  uint16_t* dst_rows = p.part_o + pbase * p.h_q * r_v;
  const int cpv = r_v >> 3, n_chunks = p.h_q * cpv;
  for (int c = tid; c < n_chunks; c += 256) {
    const int h = c / cpv, cc = c - h * cpv;
    *reinterpret_cast<u32x4*>(dst_rows + (size_t)c * 8) = *reinterpret_cast<const u32x4*>(smem + (size_t)h * pitch + cc * 16);
  }
}

// ------------------------------------------------------------------------------------------------ host
static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Context splits: about one tile-walk per workgroup slot of the device, never more than kMaxSplits per sequence.
// A context of zero positions still gets one split (it writes empty partials, which the merge turns into zeros).
static void plan_splits(DecodePlan& pl, int b, int max_ctx, int slots) {
  int n_tiles = (max_ctx + pl.tile - 1) / pl.tile;
  if (n_tiles < 1) n_tiles = 1;
  long tps = (long)b * n_tiles / slots;
  if (tps < 1) tps = 1;
  if (tps > n_tiles) tps = n_tiles;
  if ((n_tiles + tps - 1) / tps > kMaxSplits) tps = (n_tiles + kMaxSplits - 1) / kMaxSplits;
  pl.tiles_per_split = (int)tps;
  pl.n_splits = (int)((n_tiles + tps - 1) / tps);
}

static void plan_workspace(DecodePlan& pl, const lorc_layer_desc& d, int b) {
  size_t off = 0;
  pl.off_ml = off;
  off = align256(off + (size_t)b * pl.n_splits * d.n_q_heads * 2 * 4);
  pl.off_o = off;
  off = align256(off + (size_t)b * pl.n_splits * d.n_q_heads * d.rank_v * 2);
  pl.total_bytes = off;
}

DecodePlan make_decode_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus) {
  if (stationary_shape_ok(d)) return make_stationary_plan(d, b, max_ctx, n_cus);
  const int qb_ = (d.n_q_heads + 31) / 32;
  // More than 32 query heads: the streaming kernel needs two score blocks per wave and spills; scores + values + merge
  // as three launches is 1.1x (rank 256) to 1.6x (rank 1024) faster at 64 heads, b 32, context 8192.
  if (qb_ > 1 && wide_shape_ok(d)) return make_wide_plan(d, b, max_ctx, n_cus, false);
  if (d.rank_k > kStreamMaxRank || d.rank_v > kStreamMaxRank ||
      decode_lds_bytes(64, qb_, d.n_q_heads / d.n_kv_heads, d.rank_k, d.head_dim / 2) > 160 * 1024) {
    // no single-pass kernel holds this shape: the three-launch path, or nothing (total_bytes = 0: unsupported)
    if (wide_shape_ok(d)) return make_wide_plan(d, b, max_ctx, n_cus, false);
    return DecodePlan{};
  }
  DecodePlan pl{};
  pl.stationary = 0;
  // Two shapes: a 128-position tile with one workgroup per CU (each B_k operand is reused over 128 positions), or
  // 64-position tiles with two co-resident workgroups (the second hides the first one's loads and VALU phases)
  // when two latent tiles fit LDS together and the per-wave state fits 256 registers.
  const int G = d.n_q_heads / d.n_kv_heads;
  const bool two_wg = d.rank_k <= 512 && d.rank_v <= 512 && d.n_q_heads <= 32 && G <= 8 &&
                      2 * ((decode_lds_bytes(64, 1, G, d.rank_k, d.head_dim / 2) + 1023) & ~(size_t)1023) <= 160 * 1024;
  // the 128-position tile only where its LDS image fits (64 query heads at rank 512 do not: they take the
  // 64-position tile with one workgroup per CU)
  const int qb = (d.n_q_heads + 31) / 32;
  const bool fits128 = decode_lds_bytes(128, qb, G, d.rank_k, d.head_dim / 2) <= 160 * 1024;
  pl.tile = (d.rank_k <= 512 && !two_wg && fits128) ? 128 : 64;
  pl.occupancy = two_wg ? 2 : 1;
  plan_splits(pl, b, max_ctx, (n_cus > 0 ? n_cus : 256) * pl.occupancy);
  plan_workspace(pl, d, b);
  return pl;
}

template <int HD, int NPB, int QB, int NBW, int JR, int OCC>
static int launch_split(const DecodeParams& p, hipStream_t s, bool attr_only) {
  auto kern = decode_split_kernel<HD, NPB, QB, NBW, JR, OCC>;
  if (attr_only)
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) == hipSuccess
               ? LORC_OK : LORC_EHIP;
  const size_t lds = decode_lds_bytes(32 * NPB, QB, p.G, p.r_k, HD / 2);
  if (lds > 160 * 1024) return LORC_EUNSUPPORTED;
  return launch_kernel(kern, dim3(p.b * p.n_splits), dim3(256), lds, s, p);
}

// Picks the instantiation for a shape and launches it; with attr_all it walks every instantiation instead and
// sets its LDS attribute (nothing is launched).
template <int HD, int NPB>
static int dispatch_split(const DecodeParams& p, const DecodePlan& plan, hipStream_t s, bool attr_all = false) {
  const int qb = (p.h_q + 31) / 32;
  const int nbw = (p.r_v / 32 + 3) / 4;  // V latent blocks per wave
  int rc = LORC_OK;
  if (attr_all || (NPB == 2 && plan.occupancy == 2 && p.G <= 8 && qb == 1 && nbw <= 4)) {
    rc = launch_split<HD, 2, 1, 4, 4, 2>(p, s, attr_all);
    if (!attr_all || rc) return rc;
  }
  if (attr_all || p.G <= 8) {
    if (attr_all || (qb == 1 && nbw <= 4)) { rc = launch_split<HD, NPB, 1, 4, 4, 1>(p, s, attr_all); if (!attr_all || rc) return rc; }
    if (attr_all || qb == 1) { rc = launch_split<HD, NPB, 1, 8, 4, 1>(p, s, attr_all); if (!attr_all || rc) return rc; }
    if (attr_all || nbw <= 4) { rc = launch_split<HD, NPB, 2, 4, 4, 1>(p, s, attr_all); if (!attr_all || rc) return rc; }
    rc = launch_split<HD, NPB, 2, 8, 4, 1>(p, s, attr_all);
    if (!attr_all || rc) return rc;
  }
  // large query groups (G > 8): one generic instantiation per query-block count
  if (attr_all || qb == 1) { rc = launch_split<HD, NPB, 1, 8, 16, 1>(p, s, attr_all); if (!attr_all || rc) return rc; }
  return launch_split<HD, NPB, 2, 8, 16, 1>(p, s, attr_all);
}

static bool merge_group_ok(const DecodeParams& p) {
  return p.G <= kMgMaxG && p.n_splits <= kMgMaxSplits && p.r_v <= kMgMaxRank;
}

// The merge launch that follows every split kernel.
static int launch_merge(const DecodeParams& p, hipStream_t s) {
  const bool halves = p.G % 2 == 0 && p.b * p.h_kv <= 256;  // two workgroups per group while that still adds CUs
  if (!merge_group_ok(p)) {
    if (p.head_dim == 128) return launch_kernel(decode_merge_kernel<128>, dim3(p.b * p.h_q), dim3(256), 0, s, p);
    return launch_kernel(decode_merge_kernel<64>, dim3(p.b * p.h_q), dim3(256), 0, s, p);
  }
  if (halves) {
    if (p.head_dim == 128) return launch_kernel(decode_merge_group_kernel<128, 2>, dim3(p.b * p.h_kv * 2), dim3(512), 0, s, p);
    return launch_kernel(decode_merge_group_kernel<64, 2>, dim3(p.b * p.h_kv * 2), dim3(512), 0, s, p);
  }
  if (p.head_dim == 128) return launch_kernel(decode_merge_group_kernel<128, 1>, dim3(p.b * p.h_kv), dim3(1024), 0, s, p);
  return launch_kernel(decode_merge_group_kernel<64, 1>, dim3(p.b * p.h_kv), dim3(1024), 0, s, p);
}

DecodePlan make_absorbed_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus) {
  if (d.n_q_heads > 32 || d.rank_k > kAbsMaxRankK || d.rank_v > 512) {
    // beyond the single-pass kernel (one register ring per wave): scores, values in column chunks, merge
    if (!wide_absorbed_shape_ok(d)) return DecodePlan{};
    DecodePlan pl = make_wide_plan(d, b, max_ctx, n_cus, false);
    pl.wide = 3;
    return pl;
  }
  DecodePlan pl{};
  pl.stationary = 0;
  pl.tile = kPage;
  pl.occupancy = 2;
  plan_splits(pl, b, max_ctx, 2 * (n_cus > 0 ? n_cus : 256));  // two workgroups per CU
  plan_workspace(pl, d, b);
  return pl;
}

int set_kernel_attributes_decode() {
  const DecodeParams none{};
  const DecodePlan plan{};
  if (int rc = dispatch_split<128, 4>(none, plan, nullptr, true)) return rc;
  if (int rc = dispatch_split<128, 2>(none, plan, nullptr, true)) return rc;
  if (int rc = dispatch_split<64, 4>(none, plan, nullptr, true)) return rc;
  if (int rc = dispatch_split<64, 2>(none, plan, nullptr, true)) return rc;
  if (int rc = set_kernel_attributes_decode_stationary()) return rc;
  if (int rc = set_kernel_attributes_decode_wide()) return rc;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(decode_absorbed_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             160 * 1024) == hipSuccess ? LORC_OK : LORC_EHIP;
}

static int record(hipEvent_t ev, hipStream_t s) {
  return ev == nullptr || hipEventRecord(ev, s) == hipSuccess ? LORC_OK : LORC_EHIP;
}

int launch_decode_absorbed(const DecodeParams& p, const DecodePlan& plan, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end) {
  if (plan.total_bytes == 0) return LORC_EUNSUPPORTED;
  if (plan.wide) {
    if (int rc = record(ev_begin, s)) return rc;
    if (int rc = launch_decode_wide(p, plan, s)) return rc;
    if (int rc = record(ev_end, s)) return rc;
    if (p.head_dim == 128) return launch_kernel(decode_merge_kernel<128>, dim3(p.b * p.h_q), dim3(256), 0, s, p);
    return launch_kernel(decode_merge_kernel<64>, dim3(p.b * p.h_q), dim3(256), 0, s, p);
  }
  if (p.h_q > 32 || p.r_k > kAbsMaxRankK || p.r_v > 512) return LORC_EUNSUPPORTED;
  const size_t lds = absorbed_lds_bytes(p.r_k, p.r_v);
  if (lds > 160 * 1024) return LORC_EUNSUPPORTED;
  if (int rc = record(ev_begin, s)) return rc;
  if (int rc = launch_kernel(decode_absorbed_kernel<4>, dim3(p.b * p.n_splits), dim3(256), lds, s, p)) return rc;  // up to 16 V latent blocks, four per wave
  if (int rc = record(ev_end, s)) return rc;
  return launch_merge(p, s);
}

int launch_decode(const DecodeParams& p, const DecodePlan& plan, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end) {
  // shapes no instantiation covers are refused before anything (the begin event included) is put on the stream
  const int npb = plan.tile / 32, qb = (p.h_q + 31) / 32;
  if (plan.total_bytes == 0) return LORC_EUNSUPPORTED;
  if (!plan.stationary && !plan.wide && decode_lds_bytes(32 * npb, qb, p.G, p.r_k, p.head_dim / 2) > 160 * 1024) return LORC_EUNSUPPORTED;
  if (plan.wide == 1 && p.latent_out == 0 && p.r_v > kWideMaxRank) return LORC_EUNSUPPORTED;
  if (int rc = record(ev_begin, s)) return rc;
  int rc;
  if (plan.wide) {
    rc = launch_decode_wide(p, plan, s);
    if (rc != LORC_OK) return rc;
    if (int rc2 = record(ev_end, s)) return rc2;
    // the generic merge: softmax-merge of the splits; wide layers then apply B_v, uncompressed layers have none
    // (their partial rows are head_dim wide and are written out as they are)
    if (plan.wide == 2) {
      DecodeParams pm = p;
      pm.r_v = p.head_dim;
      pm.latent_out = 1;
      return launch_kernel(decode_merge_kernel<128>, dim3(pm.b * pm.h_q), dim3(256), 0, s, pm);
    }
    return launch_merge(p, s);  // the group merge where its limits hold, the generic one otherwise
  }
  if (plan.stationary) rc = launch_decode_stationary_split(p, plan, s);
  else if (p.head_dim == 128) rc = plan.tile == 128 ? dispatch_split<128, 4>(p, plan, s) : dispatch_split<128, 2>(p, plan, s);
  else rc = plan.tile == 128 ? dispatch_split<64, 4>(p, plan, s) : dispatch_split<64, 2>(p, plan, s);
  if (rc != LORC_OK) return rc;
  if (int rc2 = record(ev_end, s)) return rc2;
  return launch_merge(p, s);
}

}  // namespace lorc
