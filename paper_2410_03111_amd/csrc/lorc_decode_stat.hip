// Decode attention over the latent cache with the key factor held stationary in registers (Eq. 1 on cached
// latents; GQA of Section 4.3; RoPE applied at read time to the rebuilt keys, as the cache holds un-rotated latents).
//
// The rebuild K^T = B_k^T C_k^T is a [n x r_k] x [r_k x positions] product whose left operand never changes.  One
// workgroup (four waves, one per SIMD, 512 registers each) owns two KV heads: every wave keeps the 64 columns of
// B_k it is responsible for (a 32-column block and its RoPE partner block) in registers for the whole kernel, 256
// registers at rank 512, and walks the context of one (sequence, context split).  The only operand that moves is
// the latent tile: it is copied global -> LDS once per workgroup and read from there by the four waves, so a rebuilt
// position costs one 1 KiB LDS read per two matrix-core ops and no L2 traffic at all for the factor.  The h_kv / 2
// workgroups that share a (sequence, split) are dealt to the same XCD, so that the latent tile they all read comes
// out of that XCD's L2 after the first of them has fetched it.
//
// Per 64-position tile: rebuild the wave's 64 x 64 block of K^T (position block 0, then 1), rotate it in
// registers, score it against the group's query heads (fp16 operands), leave the two half-head partial scores in
// LDS; then one softmax pass over the workgroup's 2 G heads x 64 positions, and o_lat += P C_v on 16x16x32
// matrix-core ops with the V latents read from their LDS copy.  Split partials and the merge are those of
// lorc_decode.hip.
//
// Latent copies are direct global -> LDS loads issued from inline assembly, on purpose: the compiler would make
// every LDS read that follows such a load in program order wait for it, which forbids refilling one part of the K
// tile while another is being read.  Their completion is tracked by hand (fixed number of loads per wave between
// any two waits, s_waitcnt vmcnt(N) immediates).  The K tile is a ring of four chunks, each refilled for the next
// tile as soon as all waves have consumed it, so every chunk has a whole tile time to arrive.
#include <type_traits>
#include <utility>

#include "lorc_device.h"
#include "lorc_kernels.h"
#include "lorc_rebuild.h"

namespace lorc {

namespace {
constexpr float kNegInfS = -__builtin_huge_valf();
constexpr float kLazy = 8.0f;  // log2 of the largest exponential a tile may produce before the reference maximum moves

typedef __attribute__((ext_vector_type(4))) float f32x4s;

// D[16x16] += A[16x32] B[32x16].  Lane l supplies A[m = l%16][k = 8*(l/16) .. +7] and B[k = 8*(l/16) .. +7][n = l%16];
// it receives D[m = 4*(l/16) + j][n = l%16] in register j.
__device__ __forceinline__ f32x4s mfma16(bf16x8 a, bf16x8 b, f32x4s c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Buffer descriptor as four scalar words (base, size in bytes; raw 32-bit elements, no swizzle).
__device__ __forceinline__ u32x4 dma_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  u32x4 r;
  r[0] = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)a);
  r[1] = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(a >> 32)) & 0xffffu;
  r[2] = (uint32_t)__builtin_amdgcn_readfirstlane(bytes);
  r[3] = 0x00020000u;
  return r;
}

// One 1 KiB copy global -> LDS: lane l moves the 16 bytes at rsrc.base + soff + 16 l to LDS byte lds_off + 16 l.
// Counts as one vector-memory load of the issuing wave (vmcnt).  A read beyond the descriptor's size fetches nothing.
__device__ __forceinline__ void dma_1k(u32x4 rsrc, uint32_t lds_off, uint32_t lane16, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_off), "v"(lane16), "s"(rsrc), "s"(soff)
               : "memory");
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order, every index a compile-time constant.
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Wait until at most N of this wave's vector-memory loads are outstanding and all of its LDS operations are done,
// then meet the other waves.  No fence: loads younger than the N-th youngest stay in flight.
template <int N>
__device__ __forceinline__ void dma_barrier() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));  // vmcnt(N) lgkmcnt(0)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
}  // namespace

constexpr int kStatTile = 64;          // positions per tile = one cache page
constexpr int kStatMaxHeads = 16;      // query heads per workgroup: 2 KV heads x G <= 8
constexpr int kStatMaxTiles = 512;     // tiles one workgroup walks at most (page ids of the split live in LDS)
constexpr int kStatVLoads = 16;        // 1 KiB V copies per wave and tile (r_v <= 512)
constexpr int kStatNks = 32;           // k-steps the K tile is padded to in the one instantiation that is launched (ranks 400 .. 512)

__host__ __device__ inline size_t stat_lds_bytes(int nks_pad, int r_v, int tiles_per_split) {
  size_t b = (size_t)2 * nks_pad * 1024;                  // K tile, padded to nks_pad k-steps per position block
  b += (size_t)r_v * 128;                                 // V tile (page order)
  b += 1024;                                              // sink for copies that must not land anywhere
  b += (size_t)2 * kStatMaxHeads * kStatTile * 4;         // partial scores of the two head halves
  b += (size_t)2 * 1024;                                  // P operands
  b += (size_t)kStatMaxHeads * 128 * 2;                   // rotated, scaled queries (fp16)
  b += (size_t)3 * 64 * 8;                                // rotation bases: position block 0, position block 1 by tile parity
  b += (size_t)3 * kStatMaxHeads * 4;                     // alpha, running max, running sum
  b += (size_t)64 * 8;                                    // rotation frequencies in turns per position
  b += (size_t)tiles_per_split * 4;                       // page ids of the split
  return (b + 15) & ~(size_t)15;
}

// Where the latent copies of a tile sit in its rebuild stream (compile-time table).  The stream has NG = 4 H k-steps;
// chunk c of the K tile holds k-steps [c H, (c + 1) H).  A copy may only be issued once every wave is through the
// data it overwrites: chunks 0 / 1 / 2 of the next tile after the barriers kB2 / kB3 / kB4, chunk 3 and the V tile
// after kB0 (their copies wrap around into the next tile's stream).  Copies are spread, at most a few per k-step:
// each costs issue time next to the matrix-core stream, and a burst fills the memory pipeline's queue.
template <int NKS>
struct CopySched {
  static constexpr int H = NKS / 2, NG = 4 * H, D = 3, KI = NKS / 8, NV = kStatVLoads, MAXI = 4;
  static constexpr int kB0 = NG - D, kB1 = H - D, kB2 = 2 * H - D, kB3 = 3 * H - D, kB4 = 3 * H + H / 2;
  int n[NG];            // copies issued in k-step gi (after the step's barrier, if it has one)
  int kind[NG][MAXI];   // 0 .. 3: chunk of the K tile, 4: V tile
  int idx[NG][MAXI];    // which of the wave's copies of that kind
  constexpr void put(int step, int k, int j) {
    kind[step][n[step]] = k;
    idx[step][n[step]] = j;
    ++n[step];
  }
  constexpr void place(int k, int count, int first) {  // one copy every 2 H / 16 k-steps from `first` on
    for (int j = 0; j < count; ++j) put((first + (j * 2 * H) / 16) % NG, k, j);
  }
  constexpr CopySched() : n{}, kind{}, idx{} {
    place(4, NV, kB0);
    place(3, KI, kB0 + 1);
    place(0, KI, kB2 + 1);
    place(1, KI, kB3 + 1);
    for (int j = 0; j < KI; ++j) put(kB4 + j, 2, j);
  }
  // Copies issued after the last one of kind k and before the barrier of k-step gb (which precedes that step's own
  // copies), walking back around the stream: the vmcnt that guarantees kind k has landed.
  constexpr int younger(int k, int gb) const {
    int count = 0;
    for (int back = 1; back <= NG; ++back) {
      const int s = ((gb - back) % NG + NG) % NG;
      for (int i = n[s] - 1; i >= 0; --i) {
        if (kind[s][i] == k) return count;
        ++count;
      }
    }
    return count;
  }
};

// NKS: k-steps (of 16 latent indices) the K tile is padded to; ranks up to 16 * NKS.  Padding k-steps multiply zero
// factor operands with a zeroed part of the tile.
template <int NKS>
__global__ __launch_bounds__(256, 1) void decode_stationary_kernel(DecodeParams p) {
  constexpr int HD = 128, HALF = 64, T = kStatTile;
  static_assert(NKS % 8 == 0 && NKS <= 32, "chunks of the K ring");
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

  // workgroup -> (sequence, split, head pair): the head pairs of one (sequence, split) are 8 workgroup ids apart,
  // i.e. on one XCD, and next to each other in dispatch order
  const int NQ = p.h_kv >> 1;
  const int grp = blockIdx.x / (8 * NQ), rem = blockIdx.x % (8 * NQ);
  const int hp = rem >> 3, unit = grp * 8 + (rem & 7);
  if (unit >= p.b * p.n_splits) return;
  const int seq = unit / p.n_splits, split = unit % p.n_splits;
  const int G = p.G, r_k = p.r_k, r_v = p.r_v, nks = r_k >> 4;
  const int n_heads = 2 * G;               // query heads of this workgroup
  const int h0 = hp * n_heads;             // its first query head

  // Lane / thread index rebuilt where it is used (two VALU ops), so that nothing derived from it stays in a
  // register across the rebuild stream.
  auto my_lane = [&]() {
    int l = lane_id();
    asm volatile("" : "+v"(l));
    return l;
  };
  auto my_tid = [&]() { return my_lane() + (w << 6); };

  unsigned char* kbuf = smem;
  unsigned char* vbuf = kbuf + (size_t)2 * NKS * 1024;
  unsigned char* sink = vbuf + (size_t)r_v * 128;
  float* sbuf = reinterpret_cast<float*>(sink + 1024);
  uint16_t* pbuf = reinterpret_cast<uint16_t*>(sbuf + 2 * kStatMaxHeads * T);
  _Float16* qrot = reinterpret_cast<_Float16*>(pbuf + 1024);
  float2* cs_base = reinterpret_cast<float2*>(qrot + kStatMaxHeads * HD);
  float* alpha = reinterpret_cast<float*>(cs_base + 3 * HALF);
  float* m_fin = alpha + kStatMaxHeads;
  float* l_fin = m_fin + kStatMaxHeads;
  double* theta_rev_tab = reinterpret_cast<double*>(l_fin + kStatMaxHeads);  // turns per position of frequency i
  int* ids = reinterpret_cast<int*>(theta_rev_tab + HALF);
  const uint32_t kbuf_off = (uint32_t)(uintptr_t)kbuf, vbuf_off = (uint32_t)(uintptr_t)vbuf, sink_off = (uint32_t)(uintptr_t)sink;

  // ---- what the set-up needs from memory
  int ctx = p.ctx_len[seq];
  ctx = ctx < 0 ? 0 : (ctx > p.max_ctx ? p.max_ctx : ctx);
  const int tile_begin = split * p.tiles_per_split;
  int tile_end = tile_begin + p.tiles_per_split;
  const int n_tiles = (ctx + T - 1) / T;
  if (tile_end > n_tiles) tile_end = n_tiles;
  const int nt = tile_end > tile_begin ? tile_end - tile_begin : 0;
  const int q_pos = p.q_pos[seq];
  const double theta = p.rope_tab[tid & (HALF - 1)];

  const int g = 2 * hp + (w >> 1), wh = w & 1;  // this wave's KV head and half of its head dimension
  const int fbase = 32 * wh;
  bf16x8 bk[2][NKS];  // stationary factor operands, loaded below while the first latent chunks travel
  // page ids of the split (validated here: -1 = not cached)
  for (int i = tid; i < nt; i += 256) {
    const int id = p.block_table[(size_t)seq * p.max_pages + tile_begin + i];
    ids[i] = id >= 0 && id < p.n_pages ? id : -1;
  }
  // the K tile's padding, the V tile (read under a zero P before its first copy lands) and the P operands start as zeros
  {
    const u32x4 z = {0u, 0u, 0u, 0u};
    if (nks < NKS)
      for (int i = tid; i < (2 * NKS * 1024) / 16; i += 256) reinterpret_cast<u32x4*>(kbuf)[i] = z;
    for (int i = tid; i < (r_v * 128) / 16; i += 256) reinterpret_cast<u32x4*>(vbuf)[i] = z;
    if (tid < 128) reinterpret_cast<u32x4*>(pbuf)[tid] = z;
    if (tid < 3 * HALF / 2) reinterpret_cast<u32x4*>(cs_base)[tid] = z;
    if (tid < kStatMaxHeads) {
      alpha[tid] = 1.f;
      m_fin[tid] = kNegInfS;
      l_fin[tid] = 0.f;
    }
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();  // page ids and zeroed tiles in place: the copies may start

  // ---- latent copies.  Wave w moves blocks w, w + 4, ... of whatever is copied.
  constexpr CopySched<NKS> sched{};
  constexpr int H = sched.H, NG = sched.NG, D = sched.D;
  constexpr int kB0 = sched.kB0, kB1 = sched.kB1, kB2 = sched.kB2, kB3 = sched.kB3, kB4 = sched.kB4;
  // descriptor of one part of a cached page (id < 0: not cached, or no such tile: a descriptor of size zero, whose
  // copies fetch nothing)
  auto page_rsrc = [&](int id, uint32_t part_off, uint32_t part_bytes) {
    const bool ok = id >= 0 && id < p.n_pages;
    const uint16_t* base = p.cache + (ok ? (size_t)id * p.page_elems : 0);
    return dma_rsrc(reinterpret_cast<const unsigned char*>(base) + (ok ? part_off : 0u), ok ? part_bytes : 0u);
  };
  auto k_rsrc = [&](int id) { return page_rsrc(id, 0u, (uint32_t)T * r_k * 2u); };
  auto v_rsrc = [&](int id) { return page_rsrc(id, (uint32_t)T * r_k * 2u, (uint32_t)T * r_v * 2u); };
  auto tile_id = [&](int t_local) {  // page id of tile t_local of the split, -1 outside [0, nt)
    const bool in_split = t_local >= 0 && t_local < nt;
    const int id = __builtin_amdgcn_readfirstlane(ids[in_split ? t_local : 0]);
    return in_split ? id : -1;
  };
  // copy j (of KI) of chunk c of a K tile: position block c / 2, k-step (c % 2) H + w + 4 j; k-steps past the rank
  // go to the sink
  // the one lane-derived value that stays in a register for the whole kernel: every copy needs it (32 per tile)
  const uint32_t lane16 = (uint32_t)lane * 16u;
  auto issue_k_copy = [&](const u32x4& kr, int c, int j) {
    const int pb = c >> 1, ks = (c & 1) * H + w + 4 * j;
    const bool real = ks < nks;
    dma_1k(kr, real ? kbuf_off + (uint32_t)(pb * NKS + ks) * 1024u : sink_off, lane16, real ? (uint32_t)(pb * nks + ks) * 1024u : 0u);
  };
  // copy j of a V tile: block w + 4 j (1 KiB: 16 positions x 32 latent indices)
  auto issue_v_copy = [&](const u32x4& vr, int j) {
    const int blk = w + 4 * j;
    const bool real = blk * 8 < r_v;
    dma_1k(vr, real ? vbuf_off + (uint32_t)blk * 1024u : sink_off, lane16, real ? (uint32_t)blk * 1024u : 0u);
  };
  // The copies the schedule places in k-step gi.  kr_cur / kr_next: K parts of the current and the next tile's page,
  // v_prev / v_cur: V parts of the previous and the current tile's page.  Chunks 0 .. 2 are the next tile's; chunk 3
  // and the V tile are released at kB0, their copies wrap around into the next tile's stream.
  auto issue_step = [&](auto gi_c, const u32x4& kr_cur, const u32x4& kr_next, const u32x4& v_prev, const u32x4& v_cur) {
    constexpr int gi = decltype(gi_c)::value;
    static_for<sched.MAXI>([&](auto i_c) {
      constexpr int i = decltype(i_c)::value;
      if constexpr (i < sched.n[gi]) {
        constexpr int kind = sched.kind[gi][i], j = sched.idx[gi][i];
        if constexpr (kind < 3) issue_k_copy(kr_next, kind, j);
        else if constexpr (kind == 3) issue_k_copy(gi >= kB0 ? kr_next : kr_cur, 3, j);
        else issue_v_copy(gi >= kB0 ? v_cur : v_prev, j);
      }
    });
  };

  f32x4s o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = f32x4s{0.f, 0.f, 0.f, 0.f};

  const uint16_t* kl = reinterpret_cast<const uint16_t*>(kbuf) + (size_t)lane * 8;

  // Rotation of a rebuilt key: position p = block base + lane, frequency i: angle p theta_i.  In turns it is
  // frac(base theta_i / 2 pi) + lane (theta_i / 2 pi); the first term is reduced in fp64 once per tile and
  // frequency, the sum (below 6 turns) is exact to 5e-7 in fp32, and the hardware sine / cosine take turns.
  const float l32f = (float)l32;
  f32x16 zero16;
#pragma unroll
  for (int j = 0; j < 16; ++j) zero16[j] = 0.f;

  // Rotation of rows [J0, J1) of position block PB of the wave's K^T block into fp16 score operands.  The rows'
  // bases (frac(base theta / 2 pi), theta / 2 pi) come from LDS; they are fetched one k-step before they are used.
  auto rot_fetch = [&](float2* bt, const float2* csb, auto j0_c, auto j1_c) {
    constexpr int J0 = decltype(j0_c)::value, J1 = decltype(j1_c)::value;
    static_for<J1 - J0>([&](auto d_c) {
      constexpr int d = decltype(d_c)::value;
      bt[d] = csb[fbase + acc_row(J0 + d, hf)];
    });
  };
  auto rotate_rows = [&](const f32x16 (&acc)[2][2], f16x8 (&kf)[4], const float2* bt, auto pb_c, auto j0_c, auto j1_c) {
    constexpr int PB = decltype(pb_c)::value, J0 = decltype(j0_c)::value, J1 = decltype(j1_c)::value;
    static_for<J1 - J0>([&](auto d_c) {
      constexpr int d = decltype(d_c)::value, jj = J0 + d;
      // angle of (block base + lane) x frequency, in turns: base fraction + lane x turns per position
      const float turns = __builtin_fmaf(l32f, bt[d].y, bt[d].x);
      const float cA = __builtin_amdgcn_cosf(turns), sA = __builtin_amdgcn_sinf(turns);
      const float x = acc[0][PB][jj], y = acc[1][PB][jj];
      kf[jj >> 3][jj & 7] = static_cast<_Float16>(x * cA - y * sA);
      kf[2 + (jj >> 3)][jj & 7] = static_cast<_Float16>(y * cA + x * sA);
    });
  };
  // Scores of a position block against the group's heads, in steps that the stream puts one k-step apart (a step
  // only consumes what an earlier one requested or issued): the query operands are read raw, masked where they are
  // used (rows of the A operand = heads; rows past G are zero), the four products form one dependent chain.
  struct ScoreOps {
    u32x2 lo[4], hi[4];
  };
  auto score_load = [&](ScoreOps& q) {
    const _Float16* qh = qrot + (size_t)((w >> 1) * G + (l32 < G ? l32 : 0)) * HD + 32 * wh + 4 * hf;
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const _Float16* src = qh + HALF * (s4 >> 1) + 16 * (s4 & 1);
      q.lo[s4] = *reinterpret_cast<const u32x2*>(src);
      q.hi[s4] = *reinterpret_cast<const u32x2*>(src + 8);
    }
  };
  auto score_mfma = [&](const ScoreOps& q, const f16x8 (&kf)[4], f32x16& sa, auto s4_c) {
    constexpr int s4 = decltype(s4_c)::value;
    const bool qreal = l32 < G;
    const u32x4 v = {qreal ? q.lo[s4][0] : 0u, qreal ? q.lo[s4][1] : 0u, qreal ? q.hi[s4][0] : 0u, qreal ? q.hi[s4][1] : 0u};
    sa = mfma32_f16(__builtin_bit_cast(f16x8, v), kf[s4], s4 == 0 ? zero16 : sa);
  };
  // rows 4 hf + j (j < 4) of the score block are the group's heads; this wave holds half of the head-dim sum
  auto score_store = [&](const f32x16& sa, auto pb_c) {
    constexpr int PB = decltype(pb_c)::value;
    // no branches in the stream: a row that is not a head of the group is stored into the copy sink instead
    float* sb = sbuf + (size_t)(wh * kStatMaxHeads + (w >> 1) * G) * T + PB * 32 + l32;
    float* scrap = reinterpret_cast<float*>(sink) + my_lane();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float* dst = 4 * hf + j < G ? sb + (4 * hf + j) * T : scrap;
      *dst = sa[j];
    }
  };

  // ---- softmax of one tile over the workgroup's heads, in four stages that the rebuild stream spreads over
  // consecutive k-steps (each stage only consumes what the one before requested): 16 lanes per head, four
  // positions per lane; threads past the workgroup's last head repeat it (same values to the same words).  The reference maximum of a head only moves when a tile's maximum exceeds it by more than
  // kLazy (exponentials then stay below 2^kLazy): most tiles leave o_lat unscaled, alpha = 1.
  struct Softmax {
    f32x4s a0, a1;
    float m_old, l_old, s[4], mx, pv[4], sum, m_new, a;
  };
  auto softmax_a = [&](Softmax& sm) {
    const int tx = my_tid();
    const int hl = (tx >> 4) < n_heads ? (tx >> 4) : n_heads - 1, p0 = 4 * (tx & 15);
    sm.a0 = *reinterpret_cast<const f32x4s*>(sbuf + (size_t)hl * T + p0);
    sm.a1 = *reinterpret_cast<const f32x4s*>(sbuf + (size_t)(kStatMaxHeads + hl) * T + p0);
    sm.m_old = m_fin[hl];
    sm.l_old = l_fin[hl];
  };
  // stages b1 .. b3: tile maximum per head; c1 .. c3: exponentials, their sum, the rescale factor.  The cross-lane
  // steps are dependent chains: two per stage, so that the stream's matrix-core ops issue between them.
  auto softmax_b1 = [&](Softmax& sm, int valid_, bool page_ok_) {
    const int p0 = 4 * (my_lane() & 15);
    float mx = kNegInfS;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sm.s[i] = page_ok_ ? sm.a0[i] + sm.a1[i] : 0.f;  // a page that is not cached counts as zero latents
      if (p0 + i >= valid_) sm.s[i] = kNegInfS;
      mx = fmaxf(mx, sm.s[i]);
    }
    sm.mx = mx;
  };
  auto softmax_b2 = [&](Softmax& sm) {
    sm.mx = fmaxf(sm.mx, half_wave_peer<0>(sm.mx));
    sm.mx = fmaxf(sm.mx, half_wave_peer<1>(sm.mx));
  };
  auto softmax_b3 = [&](Softmax& sm) {
    sm.mx = fmaxf(sm.mx, half_wave_peer<2>(sm.mx));
    sm.mx = fmaxf(sm.mx, half_wave_peer<3>(sm.mx));
  };
  auto softmax_c1 = [&](Softmax& sm) {
    const bool move = sm.mx > sm.m_old + kLazy || (sm.m_old == kNegInfS && sm.mx > kNegInfS);
    sm.m_new = move ? sm.mx : sm.m_old;
    const float m_ref = fmaxf(sm.m_new, -1e30f);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sm.pv[i] = __builtin_amdgcn_exp2f(sm.s[i] - m_ref);
      sum += sm.pv[i];
    }
    sm.sum = sum;
    sm.a = __builtin_amdgcn_exp2f((move ? sm.m_old : m_ref) - m_ref);  // 1 unless the reference moved
  };
  auto softmax_c2 = [&](Softmax& sm) {
    sm.sum += half_wave_peer<0>(sm.sum);
    sm.sum += half_wave_peer<1>(sm.sum);
  };
  auto softmax_c3 = [&](Softmax& sm) {
    sm.sum += half_wave_peer<2>(sm.sum);
    sm.sum += half_wave_peer<3>(sm.sum);
  };
  auto softmax_d = [&](const Softmax& sm, bool page_ok_) {
    const int tx = my_tid();
    const int hl = (tx >> 4) < n_heads ? (tx >> 4) : n_heads - 1, i16 = tx & 15;
    // all 16 lanes of a head hold the same state and store the same words (no branch in the stream)
    alpha[hl] = sm.a;
    m_fin[hl] = sm.m_new;
    l_fin[hl] = sm.l_old * sm.a + sm.sum;
    // P operand of the 16x16x32 product: position 32 ph + 8 kg + e of head hl sits in lane hl + 16 kg, element e.
    // A page that is not cached counts in the sums (zero keys) but adds nothing to o_lat (zero values): its P is
    // filed as zero, and whatever finite data the V tile holds is multiplied by it.
    const u32x2 pk = {page_ok_ ? (uint32_t)bf16_bits(sm.pv[0]) | ((uint32_t)bf16_bits(sm.pv[1]) << 16) : 0u,
                      page_ok_ ? (uint32_t)bf16_bits(sm.pv[2]) | ((uint32_t)bf16_bits(sm.pv[3]) << 16) : 0u};
    *reinterpret_cast<u32x2*>(pbuf + ((size_t)((i16 >> 3) * 64 + hl + 16 * ((i16 & 7) >> 1)) * 8 + 4 * (i16 & 1))) = pk;
  };

  // ---- o_lat = alpha o_lat + P C_v of one tile: wave w owns the 16-wide latent blocks w, w + 4, ...
  struct PV {
    f32x4s al;
    bf16x8 pa0, pa1;
    u32x4 v0[8], v1[8];
  };
  auto pv_prep = [&](PV& pv) {
    const int ln = my_lane();
    pv.al = *reinterpret_cast<const f32x4s*>(alpha + 4 * (ln >> 4));
    pv.pa0 = load_frag(pbuf + (size_t)ln * 8);
    pv.pa1 = load_frag(pbuf + (size_t)(64 + ln) * 8);
  };
  auto pv_rescale = [&](const PV& pv) {
    if (__builtin_amdgcn_ballot_w64(pv.al[0] != 1.0f || pv.al[1] != 1.0f || pv.al[2] != 1.0f || pv.al[3] != 1.0f) != 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] *= pv.al;
    }
  };
  // V operand of block I (positions 32 ph + 8 kg .. + 7, latent 16 jb + n16) out of the page tiling of the V tile
  auto pv_load = [&](PV& pv, auto i_c) {
    constexpr int I = decltype(i_c)::value;
    const int jbr = w + 4 * I, jb = jbr * 16 < r_v ? jbr : w;  // a block past r_v re-reads the wave's first one, unused
    const int ln = my_lane();
    const int n16 = ln & 15, kg = ln >> 4;
    const unsigned char* vp = vbuf + (size_t)((((jb >> 1) * 4 + (kg >> 1)) * 64 + 16 * (jb & 1) + n16 + 32 * (kg & 1)) * 16);
    pv.v0[I] = *reinterpret_cast<const u32x4*>(vp);
    pv.v1[I] = *reinterpret_cast<const u32x4*>(vp + 2 * 1024);
  };
  // inside the stream: whole tiles only (a ragged tile is the last of its split and is finished after the loop), a
  // block past r_v multiplies the re-read data into an accumulator that is never written out
  auto pv_mfma_plain = [&](const PV& pv, auto i_c) {
    constexpr int I = decltype(i_c)::value;
    o[I] = mfma16(pv.pa0, __builtin_bit_cast(bf16x8, pv.v0[I]), o[I]);
    o[I] = mfma16(pv.pa1, __builtin_bit_cast(bf16x8, pv.v1[I]), o[I]);
  };
  auto pv_mfma = [&](PV& pv, auto i_c, int valid_, bool page_ok_) {
    constexpr int I = decltype(i_c)::value;
    const int jb = w + 4 * I;
    if (jb * 16 < r_v) {
      if (!page_ok_ || valid_ < T) {  // wave-uniform: slots past the context (or a page that is not cached) hold anything
        const int kg = my_lane() >> 4;
#pragma unroll
        for (int ph = 0; ph < 2; ++ph) {
          int nv = valid_ - 32 * ph - 8 * kg;
          nv = nv < 0 ? 0 : (nv > 8 ? 8 : nv);
          const uint32_t vmask = page_ok_ ? (1u << nv) - 1u : 0u;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t two = (vmask >> (2 * c)) & 3u;
            const uint32_t keep = (two & 1u ? 0x0000ffffu : 0u) | (two & 2u ? 0xffff0000u : 0u);
            if (ph == 0) pv.v0[I][c] &= keep;
            else pv.v1[I][c] &= keep;
          }
        }
      }
      o[I] = mfma16(pv.pa0, __builtin_bit_cast(bf16x8, pv.v0[I]), o[I]);
      o[I] = mfma16(pv.pa1, __builtin_bit_cast(bf16x8, pv.v1[I]), o[I]);
    }
  };

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I16 = std::integral_constant<int, 16>;
  // Schedule of a tile's stream (k-step indices; the copies have their own table).  Besides its own rebuild, the
  // stream of tile t carries the rest of tile t - 1 (rotation and scores of its second position block, its softmax,
  // its P C_v product) and the rotation and scores of tile t's first position block, each placed where its inputs
  // are certainly there.  Barriers: kB1 / kB2 / kB3 = chunk 1 / 2 / 3 of the tile has landed (D steps before its first
  // k-step, where its first operand is requested), kB4 = chunk 2 is free, kB0 = the next tile's chunk 0 has landed
  // and every wave is through this tile's reads of chunk 3 and of the V tile.
  constexpr int kRotPer = (16 + H - 1) / H;             // rows rotated per k-step: 16 rows inside one chunk's time
  constexpr int kBase = 1;                               // rotation bases of the tile
  constexpr int kRotSteps = (16 + kRotPer - 1) / kRotPer;  // k-steps one block's rotation takes
  constexpr int kIdRead = 2, kIdUse = 4;                   // page id of the tile after the next: LDS read, then its use
  // the previous tile's scores of position block 1: operands at H, products at sc1(1) .. sc1(4), results filed at sc1(6)
  auto sc1 = [](int off) constexpr { return H + off < kB2 - 1 ? H + off : kB2 - 1; };
  auto sc0 = [](int off) constexpr { return 3 * H + off < NG - 1 ? 3 * H + off : NG - 1; };
  auto sm_at = [](int stage) constexpr { return kB2 + (stage * (H - 1)) / 7; };  // the eight softmax stages, between kB2 and kB3
  constexpr int kPvPrep = kB3, kPvFirst = kB3 + 1, kPvSpan = kB0 - 1 - kPvFirst;  // block I: operands at kPvFirst + I kPvSpan / 8, product one step later
  static_assert(H >= kRotSteps && kPvSpan >= 1 && NG % (D + 1) == 0 && kBase < kB2 && kIdUse < NG, "stream schedule");

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[a][b][j] = 0.f;
  int valid_prev = 0;          // the tile before the first one: no positions, everything it contributes is zero
  bool page_ok_prev = false;
  float2* cs0 = cs_base;                  // bases of position block 0 of the current tile
  float2* cs1 = cs_base + HALF;           // bases of position block 1: two copies, by tile parity
  bf16x8 c[D + 1];                        // latent operands read ahead; carried from one tile's stream into the next
  float2 bt[2][kRotPer];                  // rotation bases fetched a k-step ahead, two sets in turn; carried likewise

  // ---- what a tile before the first one would have left in flight: the first tile's K chunks, in the order and
  // at the places of the schedule (the waits of the first stream count copies exactly like those of any other)
  int id_prev = -1, id_cur = -1, id_next = tile_id(0);
  {
    const u32x4 none = k_rsrc(-1), kr0 = k_rsrc(id_next);
    static_for<kB0 - kB2>([&](auto d_c) { issue_step(std::integral_constant<int, kB2 + decltype(d_c)::value>{}, none, kr0, none, none); });
    // While the first chunks travel: the factor operands, the queries, the frequency table.  Their loads are
    // younger than the copies, so the wait below covers both, once.
  // stationary factor operands: column blocks cb0 (dims 32 wh .. of head g) and cb1 (its RoPE partners, + 64)
  {
    const __amdgpu_buffer_rsrc_t bk_rsrc = make_rsrc(p.bk, (uint32_t)p.h_kv * HD * r_k * 2u);
    const uint32_t s0 = (uint32_t)((g * 4 + wh) * nks) * 1024u, s1 = (uint32_t)((g * 4 + wh + 2) * nks) * 1024u;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      if (ks < nks) {
        bk[0][ks] = buf_frag(bk_rsrc, (uint32_t)lane * 16u, s0 + (uint32_t)ks * 1024u);
        bk[1][ks] = buf_frag(bk_rsrc, (uint32_t)lane * 16u, s1 + (uint32_t)ks * 1024u);
      } else {
        bk[0][ks] = zero_frag();
        bk[1][ks] = zero_frag();
      }
    }
  }
  // queries of the workgroup's heads: rotated at q_pos, scaled (softmax scale x log2 e), fp16, kept in LDS
  {
    const double turns = (double)q_pos * theta * 0.15915494309189533576888;
    const float fr = (float)(turns - rint(turns));
    const float cs = __builtin_amdgcn_cosf(fr), sn = __builtin_amdgcn_sinf(fr);
    const uint16_t* qsrc = p.q + ((size_t)seq * p.h_q + h0) * HD;
    const int i = tid & (HALF - 1);
#pragma unroll
    for (int u = 0; u < kStatMaxHeads * HALF / 256; ++u) {
      const int hl = (tid >> 6) + 4 * u;
      if (hl < n_heads) {
        const float lo = bf16_to_float(qsrc[hl * HD + i]) * p.q_scale, hi = bf16_to_float(qsrc[hl * HD + i + HALF]) * p.q_scale;
        qrot[hl * HD + i] = static_cast<_Float16>(lo * cs - hi * sn);
        qrot[hl * HD + i + HALF] = static_cast<_Float16>(hi * cs + lo * sn);
      }
    }
  }
  if (tid < HALF) theta_rev_tab[tid] = theta * 0.15915494309189533576888;
    // Every load of the set-up has to be back here: a wait for one of them placed inside the tile loop would be a
    // wait for the latent copies issued after it (one in-order counter), on every tile.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    static_for<NG - kB0>([&](auto d_c) {
      constexpr int gi = kB0 + decltype(d_c)::value;
      issue_step(std::integral_constant<int, gi>{}, none, kr0, none, none);
      c[(gi + D - NG) % (D + 1)] = load_frag(kl + (size_t)(gi + D - NG) * 512);
    });
  }
  id_cur = id_next;
  id_next = tile_id(1);
  rot_fetch(bt[0], cs1 + HALF, I0{}, std::integral_constant<int, kRotPer>{});

  for (int t = 0; t < nt; ++t) {
    const int pos0 = (tile_begin + t) * T;
    const int valid = (ctx - pos0) < T ? (ctx - pos0) : T;
    const bool page_ok = id_cur >= 0;
    const u32x4 kr_cur = k_rsrc(id_cur), kr_next = k_rsrc(id_next), v_prev = v_rsrc(id_prev), v_cur = v_rsrc(id_cur);
    const float2* cs1_prev = cs1 + ((t + 1) & 1) * HALF;
    const float2* cs1_cur = cs1 + (t & 1) * HALF;
    int id_after_raw = -1, id_after = -1;

    f16x8 kf[4];
    ScoreOps qf;
    f32x16 sa;
    Softmax sm;
    PV pv;
    static_for<NG>([&](auto gi_c) {
      constexpr int gi = decltype(gi_c)::value, nx = gi + D;
      // -- barriers and latent copies
      if constexpr (gi == kB0) dma_barrier<sched.younger(0, kB0)>();
      if constexpr (gi == kB1) dma_barrier<sched.younger(1, kB1)>();
      if constexpr (gi == kB2) dma_barrier<sched.younger(2, kB2)>();   // also: the previous tile's scores are complete
      if constexpr (gi == kB3) dma_barrier<(sched.younger(3, kB3) < sched.younger(4, kB3) ? sched.younger(3, kB3) : sched.younger(4, kB3))>();  // also: its P is visible
      if constexpr (gi == kB4) lds_barrier();
      issue_step(gi_c, kr_cur, kr_next, v_prev, v_cur);
      // -- LDS read-ahead (past the end of the stream: the next tile's first k-steps) and the two matrix-core ops
      {
        constexpr int nxw = nx % NG, pbn = nxw / (2 * H), ksn = nxw % (2 * H);
        c[nx % (D + 1)] = load_frag(kl + (size_t)(pbn * NKS + ksn) * 512);
      }
      constexpr int pb = gi / (2 * H), ks = gi % (2 * H);
      acc[0][pb] = mfma32(bk[0][ks], c[gi % (D + 1)], ks == 0 ? zero16 : acc[0][pb]);
      acc[1][pb] = mfma32(bk[1][ks], c[gi % (D + 1)], ks == 0 ? zero16 : acc[1][pb]);
      // -- rotation bases of this tile's two position blocks: frac(base theta / 2 pi) and theta / 2 pi per frequency
      if constexpr (gi == kBase) {
        // every thread takes part (two threads per entry store the same words): no branch in the stream
        const int tt = my_tid() & (2 * HALF - 1);
        const double tr = theta_rev_tab[tt & (HALF - 1)], turns = (double)(pos0 + 32 * (tt >> 6)) * tr;
        float2* dst = tt < HALF ? cs0 + tt : cs1 + (t & 1) * HALF + (tt - HALF);
        *dst = make_float2((float)(turns - rint(turns)), (float)tr);
      }
      // -- page id of the tile after the next
      if constexpr (gi == kIdRead) id_after_raw = ids[t + 2 < nt ? t + 2 : 0];
      if constexpr (gi == kIdUse) id_after = t + 2 < nt ? __builtin_amdgcn_readfirstlane(id_after_raw) : -1;
      // -- the previous tile's second position block: rotation (bases fetched a step ahead), scores
      if constexpr (gi < kRotSteps) {
        constexpr int j0 = gi * kRotPer, j1 = (j0 + kRotPer < 16 ? j0 + kRotPer : 16), j2 = (j1 + kRotPer < 16 ? j1 + kRotPer : 16);
        if constexpr (j1 < 16) rot_fetch(bt[(gi + 1) & 1], cs1_prev, std::integral_constant<int, j1>{}, std::integral_constant<int, j2>{});
        rotate_rows(acc, kf, bt[gi & 1], I1{}, std::integral_constant<int, j0>{}, std::integral_constant<int, j1>{});
      }
      if constexpr (gi == sc1(0)) score_load(qf);
      static_for<4>([&](auto s4_c) {
        if constexpr (gi == sc1(1 + decltype(s4_c)::value)) score_mfma(qf, kf, sa, s4_c);
      });
      if constexpr (gi == sc1(6)) score_store(sa, I1{});
      // -- the previous tile's softmax
      if constexpr (gi == sm_at(0)) softmax_a(sm);
      if constexpr (gi == sm_at(1)) softmax_b1(sm, valid_prev, page_ok_prev);
      if constexpr (gi == sm_at(2)) softmax_b2(sm);
      if constexpr (gi == sm_at(3)) softmax_b3(sm);
      if constexpr (gi == sm_at(4)) softmax_c1(sm);
      if constexpr (gi == sm_at(5)) softmax_c2(sm);
      if constexpr (gi == sm_at(6)) softmax_c3(sm);
      if constexpr (gi == sm_at(7)) softmax_d(sm, page_ok_prev);
      // -- this tile's first position block: rotation, scores
      if constexpr (gi == 2 * H - 1) rot_fetch(bt[0], cs0, I0{}, std::integral_constant<int, kRotPer>{});
      if constexpr (gi >= 2 * H && gi - 2 * H < kRotSteps) {
        constexpr int r = gi - 2 * H, j0 = r * kRotPer, j1 = (j0 + kRotPer < 16 ? j0 + kRotPer : 16), j2 = (j1 + kRotPer < 16 ? j1 + kRotPer : 16);
        if constexpr (j1 < 16) rot_fetch(bt[(r + 1) & 1], cs0, std::integral_constant<int, j1>{}, std::integral_constant<int, j2>{});
        rotate_rows(acc, kf, bt[r & 1], I0{}, std::integral_constant<int, j0>{}, std::integral_constant<int, j1>{});
      }
      if constexpr (gi == sc0(0)) score_load(qf);
      static_for<4>([&](auto s4_c) {
        if constexpr (gi == sc0(1 + decltype(s4_c)::value)) score_mfma(qf, kf, sa, s4_c);
      });
      if constexpr (gi == sc0(6)) score_store(sa, I0{});
      // -- the bases of the next stream's first rotation step (this tile's second position block)
      if constexpr (gi == NG - 1) rot_fetch(bt[0], cs1_cur, I0{}, std::integral_constant<int, kRotPer>{});
      // -- the previous tile's P C_v
      if constexpr (gi == kPvPrep) pv_prep(pv);
      if constexpr (gi == kPvFirst) pv_rescale(pv);
      static_for<8>([&](auto i_c) {
        constexpr int I = decltype(i_c)::value, at = kPvFirst + I * kPvSpan / 8;
        if constexpr (gi == at + 1) pv_mfma_plain(pv, i_c);
      });
      static_for<8>([&](auto i_c) {
        constexpr int I = decltype(i_c)::value, at = kPvFirst + I * kPvSpan / 8;
        if constexpr (gi == at) pv_load(pv, i_c);
      });
      __builtin_amdgcn_sched_barrier(0);
    });
    valid_prev = valid;
    page_ok_prev = page_ok;
    id_prev = id_cur;
    id_cur = id_next;
    id_next = id_after;
  }

  // ---- the last tile's second half: the rest of its V tile, rotation and scores of position block 1, softmax,
  // P C_v (with the masks a ragged tile needs: only the last tile of a context can be one)
  if (nt > 0) {
    {
      const u32x4 vr = v_rsrc(id_prev);
      static_for<kB0>([&](auto gi_c) {  // the copies of the V tile that the schedule leaves to the next stream
        constexpr int gi = decltype(gi_c)::value;
        static_for<sched.MAXI>([&](auto i_c) {
          constexpr int i = decltype(i_c)::value;
          if constexpr (i < sched.n[gi]) {
            if constexpr (sched.kind[gi][i] == 4) issue_v_copy(vr, sched.idx[gi][i]);
          }
        });
      });
    }
    f16x8 kf[4];
    ScoreOps qf;
    f32x16 sa;
    float2 bt16[16];
    rot_fetch(bt16, cs1 + ((nt - 1) & 1) * HALF, I0{}, I16{});
    rotate_rows(acc, kf, bt16, I1{}, I0{}, I16{});
    score_load(qf);
    static_for<4>([&](auto s4_c) { score_mfma(qf, kf, sa, s4_c); });
    score_store(sa, I1{});
    lds_barrier();
    Softmax sm;
    PV pv;
    softmax_a(sm);
    softmax_b1(sm, valid_prev, page_ok_prev);
    softmax_b2(sm);
    softmax_b3(sm);
    softmax_c1(sm);
    softmax_c2(sm);
    softmax_c3(sm);
    softmax_d(sm, page_ok_prev);
    dma_barrier<0>();  // P and alpha visible; the V tile (and every other copy) has landed
    pv_prep(pv);
    pv_rescale(pv);
    static_for<8>([&](auto i_c) { pv_load(pv, i_c); });
    static_for<8>([&](auto i_c) { pv_mfma(pv, i_c, valid_prev, page_ok_prev); });
  }

  // ---- partials of this split (format of lorc_decode.hip): every copy still in flight has to land first, the
  // staging area reuses the K tile
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  const size_t pbase = (size_t)seq * p.n_splits + split;
  if (tid < n_heads) {
    p.part_ml[(pbase * p.h_q + h0 + tid) * 2 + 0] = m_fin[tid];
    p.part_ml[(pbase * p.h_q + h0 + tid) * 2 + 1] = l_fin[tid];
  }
  const int pitch = r_v * 2 + 16;  // bytes per staged row
  {
    const int n16 = lane & 15, kg = lane >> 4;
    float inv_l[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float l = l_fin[4 * kg + j];
      inv_l[j] = l > 0.f ? __builtin_amdgcn_rcpf(l) : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int jb = w + 4 * i;
      if (jb * 16 < r_v) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          *reinterpret_cast<uint16_t*>(smem + (size_t)(4 * kg + j) * pitch + (jb * 16 + n16) * 2) = f16_bits(o[i][j] * inv_l[j]);
      }
    }
  }
  lds_barrier();
  uint16_t* dst_rows = p.part_o + (pbase * p.h_q + h0) * r_v;
  const int cpr = r_v >> 3, n_chunks = n_heads * cpr;  // 16-byte chunks
  for (int c = tid; c < n_chunks; c += 256) {
    const int h = c / cpr, cc = c - h * cpr;
    *reinterpret_cast<u32x4*>(dst_rows + (size_t)c * 8) = *reinterpret_cast<const u32x4*>(smem + (size_t)h * pitch + cc * 16);
  }
}

// ------------------------------------------------------------------------------------------------ host
// Shapes the kernel is built for, and (last condition) those where it measures faster than the streaming kernel of
// lorc_decode.hip: its per-tile cost outside the matrix cores does not shrink with the rank, so below rank 384 the
// streaming kernel with two workgroups per CU wins (8B shape, batch 32, context 8192: rank 256: 229 against 256 us,
// rank 384: 313 against 334, rank 512: 355 against 355; 70B shape, batch 64, context 32768: 3.35 against 2.68 ms).
bool stationary_shape_ok(const lorc_layer_desc& d) {
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.head_dim == 128 && d.n_kv_heads % 2 == 0 && G <= 8 && d.rank_k <= 512 && d.rank_v <= 512 && d.rank_k > 384;
}

DecodePlan make_stationary_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus) {
  DecodePlan pl{};
  pl.tile = kStatTile;
  pl.occupancy = 1;
  pl.stationary = 1;
  int n_tiles = (max_ctx + kStatTile - 1) / kStatTile;
  if (n_tiles < 1) n_tiles = 1;
  const int cus = n_cus > 0 ? n_cus : 256;
  const long wgs_per_split = (long)b * (d.n_kv_heads / 2);
  // Context splits: the count that minimises (rounds of workgroups over the device) x (tiles per workgroup + the
  // fixed cost of a workgroup, about two tiles' worth: factor load, first tile, write-out).
  int min_splits = (n_tiles + kStatMaxTiles - 1) / kStatMaxTiles;
  int best = min_splits;
  double best_cost = 0;
  for (int ns = min_splits; ns <= n_tiles && ns <= 64; ++ns) {
    const int tps = (n_tiles + ns - 1) / ns;
    const int ns_eff = (n_tiles + tps - 1) / tps;
    const long rounds = (wgs_per_split * ns_eff + cus - 1) / cus;
    const double cost = (double)rounds * (tps + 2.0);
    if (ns == min_splits || cost < best_cost * 0.999) {
      best = ns_eff;
      best_cost = cost;
    }
  }
  pl.tiles_per_split = (n_tiles + best - 1) / best;
  pl.n_splits = (n_tiles + pl.tiles_per_split - 1) / pl.tiles_per_split;
  size_t off = 0;
  pl.off_ml = off;
  off = ((off + (size_t)b * pl.n_splits * d.n_q_heads * 2 * 4) + 255) & ~(size_t)255;
  pl.off_o = off;
  off = ((off + (size_t)b * pl.n_splits * d.n_q_heads * d.rank_v * 2) + 255) & ~(size_t)255;
  pl.total_bytes = off;
  return pl;
}

int set_kernel_attributes_decode_stationary() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(decode_stationary_kernel<kStatNks>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             160 * 1024) == hipSuccess ? LORC_OK : LORC_EHIP;
}

int launch_decode_stationary_split(const DecodeParams& p, const DecodePlan& plan, hipStream_t s) {
  const size_t lds = stat_lds_bytes(kStatNks, p.r_v, plan.tiles_per_split);
  if (lds > 160 * 1024 || plan.tiles_per_split > kStatMaxTiles || 2 * p.G > kStatMaxHeads || p.r_k > 16 * kStatNks) return LORC_EUNSUPPORTED;
  const int units = p.b * p.n_splits, nq = p.h_kv / 2;
  const dim3 grid(((units + 7) / 8) * 8 * nq), block(256);
  return launch_kernel(decode_stationary_kernel<kStatNks>, grid, block, lds, s, p);
}

}  // namespace lorc
