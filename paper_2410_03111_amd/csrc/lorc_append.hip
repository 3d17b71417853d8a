// Factor packing and the cache write (down-projection GEMM + paged scatter).
//
// lorc_append: C^T[j, t] = sum_k At[j, k] X[t, k]  (the compressed key/value x A of Section 4.1), bf16
// operands, fp32 accumulation on the 32x32x16 matrix-core op, RNE to bf16, scattered into the tiled pages.
#include "lorc_device.h"
#include "lorc_kernels.h"
#include "lorc_rebuild.h"

namespace lorc {

// ------------------------------------------------------------------------------------------------ packing
__global__ void pack_factors_kernel(const uint16_t* __restrict__ A_k, const uint16_t* __restrict__ A_v,
                                    const uint16_t* __restrict__ B_k, const uint16_t* __restrict__ B_v,
                                    uint16_t* __restrict__ packed, int D, int r_k, int r_v, int n, int head_dim,
                                    float rope_base) {
  if (blockIdx.x == 0) {  // rotation tables: theta_i, and (cos, sin)(l * theta_i) in the arithmetic of the kernels
    const int half = head_dim / 2;
    double* theta = reinterpret_cast<double*>(packed + packed_off_rope(D, r_k, r_v, n));
    float2* lane_cs = reinterpret_cast<float2*>(theta + 64);
    for (int i = threadIdx.x; i < half; i += blockDim.x) theta[i] = rope_theta(i, head_dim, rope_base);
    for (int idx = threadIdx.x; idx < 32 * half; idx += blockDim.x) {
      const float th = (float)rope_theta(idx % half, head_dim, rope_base);
      float sn, cs;
      sincosf((float)(idx / half) * th, &sn, &cs);
      lane_cs[idx] = make_float2(cs, sn);
    }
  }
  const size_t n_at = packed_at_elems(D, r_k, r_v);
  const size_t n_bk = packed_b_elems(r_k, n);
  const size_t n_bv = packed_b_elems(r_v, n);
  const size_t total = n_at + n_bk + n_bv;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    if (i < n_at) {  // i = j * D + k  (output order: coalesced writes)
      const int j = (int)(i / D), k = (int)(i % D);
      const uint16_t v = j < r_k ? A_k[(size_t)k * r_k + j] : A_v[(size_t)k * r_v + (j - r_k)];
      packed[i] = v;
      packed[total + at_tile_index(D, j, k)] = v;
    } else if (B_k == nullptr) {  // uncompressed layer: no read-side factors
    } else if (i < n_at + n_bk) {  // source order: i' = j * n + c
      const size_t s = i - n_at;
      const int j = (int)(s / n), c = (int)(s % n);
      packed[n_at + b_tile_index(r_k, j, c)] = B_k[s];
    } else {
      const size_t s = i - n_at - n_bk;
      const int j = (int)(s / n), c = (int)(s % n);
      packed[n_at + n_bk + b_tile_index(r_v, j, c)] = B_v[s];
    }
  }
}

// ------------------------------------------------------------------------------------------------ append
// Mid-size batches.  Block tile: BM latent rows x BN tokens (128 x 128 or 64 x 64), k-tile 64; 4 waves as 2x2.
// LDS rows are 64 bf16 = 8 chunks of 16 B; chunk c of row r is stored at c ^ (r & 7) so that the 32 rows a
// fragment load touches spread over all banks.  With so few workgroups the walk over the model dimension is a
// chain of memory latencies, so every thread keeps PF k-tiles of both operands in flight in registers (buffer
// loads: rows past the end of either operand read as zero).
constexpr int kApBK = 64;

__device__ __forceinline__ int swz(int row, int chunk) { return (row * 8 + (chunk ^ (row & 7))) * 8; }

template <int BM, int PF>
__global__ __launch_bounds__(256) void append_kernel(AppendParams p) {
  constexpr int BN = BM, NB = BM / 64, LD = BM / 32;  // accumulator blocks per wave and side; 16-byte loads per thread, operand and k-tile
  static_assert(PF % 2 == 0, "the LDS buffer of a k-tile is chosen by its stage's parity");
  __shared__ __align__(16) uint16_t sA[2][BM * kApBK];
  __shared__ __align__(16) uint16_t sB[2][BN * kApBK];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, wm = w >> 1, wn = w & 1;
  const int hf = lane >> 5, l32 = lane & 31;
  const int j0 = blockIdx.y * BM, t0 = blockIdx.x * BN;
  const int rt = p.r_k + p.r_v;
  const int D = p.D, nkt = D / kApBK;

  f32x16 acc[NB][NB];
#pragma unroll
  for (int a = 0; a < NB; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[a][b][j] = 0.f;

  auto rows_rsrc = [&](const uint16_t* base, long long rows) {  // raw buffer over `rows` rows of D elements
    const long long bytes = rows * (long long)D * 2;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, bytes > 0x7fffffffLL ? 0x7fffffff : (int)bytes, 0x00020000);
  };
  const __amdgpu_buffer_rsrc_t at_rsrc = rows_rsrc(p.at + (size_t)j0 * D, rt - j0);
  const __amdgpu_buffer_rsrc_t x_rsrc = rows_rsrc(p.x + (size_t)t0 * D, p.T - t0);
  uint32_t off[LD];
#pragma unroll
  for (int i = 0; i < LD; ++i) {
    const int c = tid + 256 * i, row = c >> 3, ch = c & 7;
    off[i] = (uint32_t)((row * D + ch * 8) * 2);
  }
  u32x4 ra[PF][LD], rb[PF][LD];
  auto request = [&](int st, int kt) {  // k-tile kt (the last one again past the end: never used, keeps the count fixed)
    const uint32_t koff = (uint32_t)((kt < nkt ? kt : nkt - 1) * (kApBK * 2));
#pragma unroll
    for (int i = 0; i < LD; ++i) {
      ra[st][i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(at_rsrc, (int)(off[i] + koff), 0, 0));
      rb[st][i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, (int)(off[i] + koff), 0, 0));
    }
  };
  auto to_lds = [&](int st) {  // stage st's registers into the LDS buffer of its parity
#pragma unroll
    for (int i = 0; i < LD; ++i) {
      const int c = tid + 256 * i, row = c >> 3, ch = c & 7;
      *reinterpret_cast<u32x4*>(sA[st & 1] + swz(row, ch)) = ra[st][i];
      *reinterpret_cast<u32x4*>(sB[st & 1] + swz(row, ch)) = rb[st][i];
    }
  };
  auto multiply = [&](int buf) {
#pragma unroll
    for (int ks = 0; ks < kApBK / 16; ++ks) {
      bf16x8 a[NB], b[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        a[i] = load_frag(sA[buf] + swz(wm * (BM / 2) + i * 32 + l32, ks * 2 + hf));
        b[i] = load_frag(sB[buf] + swz(wn * (BN / 2) + i * 32 + l32, ks * 2 + hf));
      }
#pragma unroll
      for (int mi = 0; mi < NB; ++mi)
#pragma unroll
        for (int ni = 0; ni < NB; ++ni) acc[mi][ni] = mfma32(a[mi], b[ni], acc[mi][ni]);
    }
  };
  // k-tile kt lives in stage kt % PF; while it is multiplied out of one LDS buffer, tile kt + 1 is written into
  // the other and tile kt + PF is requested into the registers tile kt left: one barrier per k-tile.
#pragma unroll
  for (int st = 0; st < PF; ++st) request(st, st);
  to_lds(0);
  __syncthreads();
  int kt0 = 0;
  for (; kt0 + PF <= nkt; kt0 += PF) {
#pragma unroll
    for (int st = 0; st < PF; ++st) {
      request(st, kt0 + st + PF);
      to_lds((st + 1) % PF);  // past the last k-tile: a copy of the last one, never multiplied
      multiply(st & 1);
      __syncthreads();
    }
  }
#pragma unroll
  for (int st = 0; st < PF; ++st) {
    if (kt0 + st < nkt) {  // same for the whole workgroup
      if (st + 1 < PF) to_lds(st + 1);
      multiply(st & 1);
      __syncthreads();
    }
  }

  // Epilogue: lane holds token column l32 of each block and 16 latent rows; 4 consecutive rows per group.
#pragma unroll
  for (int ni = 0; ni < NB; ++ni) {
    const int t = t0 + wn * (BN / 2) + ni * 32 + l32;
    if (t >= p.T) continue;
    const int seq = p.slot_seq[t], pos = p.slot_pos[t];
    if (seq < 0 || seq >= p.n_seqs || pos < 0 || pos >= p.max_pages * kPage) continue;
    const int page = p.block_table[(size_t)seq * p.max_pages + pos / kPage];
    if (page < 0 || page >= p.n_pages) continue;
    const int slot = pos % kPage;
    uint16_t* base = p.cache + (size_t)page * p.page_elems;
#pragma unroll
    for (int mi = 0; mi < NB; ++mi) {
      const int jb = j0 + wm * (BM / 2) + mi * 32;
      if (jb >= rt) continue;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int j = jb + 8 * q4 + 4 * hf;
        uint16_t v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = bf16_bits(acc[mi][ni][4 * q4 + i]);
        if (j < p.r_k) {
          u32x2 pk = {(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16)};
          *reinterpret_cast<u32x2*>(base + k_index(p.r_k, slot, j)) = pk;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) base[v_index(p.r_k, slot, j - p.r_k + i)] = v[i];
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------ append, large T
// Prefill down-projection: 256 latent rows x 256 tokens per workgroup, four waves of 128 x 128 (16 accumulator
// blocks each: eight LDS operand reads per sixteen MFMAs).  Both operands go through a five-slot LDS ring (k-tile
// 64, 32 KiB per slot = all 160 KiB of the CU) filled by direct global -> LDS loads; the only other loads in the
// loop are LDS reads, so the in-order memory counter measures exactly the ring.
// Row blocks of the V latent are computed with the operands swapped (tokens along accumulator rows), which puts
// four consecutive cache slots of one latent index in one lane: 8-byte stores into the V tiling.
constexpr int kGmBM = 256, kGmBN = 256, kGmBK = 64, kGmSlots = 5;
constexpr int kGmSlotElems = 256 * kGmBK;  // one operand tile: 256 rows x 64 = 32 KiB
constexpr int kGmLdsBytes = kGmSlots * kGmSlotElems * 2;

// Slot ring: operand tiles are filled in the order X0 A0 X1 A1 ... into slots 0 1 2 3 4 0 1 ...; k-tile kt uses
// fills 2kt (tokens) and 2kt+1 (weights).  The refills are spread over the k-steps, four loads per wave and
// k-step: once k-tile kt has been handed over, its two slots take the weights of k-tile kt+2 (half in the last
// k-step of kt, half in the first of kt+1) and the tokens of k-tile kt+3 (second and third k-step of kt+1).
// Rows are 128 B = one cache line per row and k-tile (8 chunks of 16 B, chunk c of row r at c ^ (r & 7)): every
// line fetched is fully used, and operand reads stay conflict-free with per-lane bases.
template <bool SWAP>
__device__ __forceinline__ void gemm_mainloop(f32x16 (&acc)[4][4], uint16_t* lds, __amdgpu_buffer_rsrc_t at, __amdgpu_buffer_rsrc_t x,
                                              const uint32_t (&aoff)[8], const uint32_t (&xoff)[8], int nkt, int w, int wm,
                                              int wn, int hf, int l32) {
  int ra[4], rb[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int phys = (2 * ks + hf) ^ (l32 & 7);
    ra[ks] = ((wm * 128 + l32) * 8 + phys) * 8;
    rb[ks] = ((wn * 128 + l32) * 8 + phys) * 8;
  }
  auto fill_part = [&](int f, int half) {  // half of fill number f: operand f & 1 (0 = X, 1 = At) of k-tile f >> 1
    const int kt = f >> 1, k = kt < nkt ? kt : nkt - 1;  // clamped refills keep the loads in flight constant
    uint16_t* base = lds + (size_t)(f % kGmSlots) * kGmSlotElems;
#pragma unroll
    for (int i = 4 * half; i < 4 * half + 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds((f & 1) ? at : x, (__attribute__((address_space(3))) void*)(base + (size_t)(i * 4 + w) * 512), 16,
                                               (f & 1) ? aoff[i] : xoff[i], k * (kGmBK * 2), 0, 0);
  };
  auto fill = [&](int f) { fill_part(f, 0); fill_part(f, 1); };
  // Operand fragments are double-buffered in registers: the LDS reads of k-step s+1 are issued among the MFMAs
  // of k-step s, so no MFMA waits on an LDS round trip.  The barrier that hands over the next k-tile therefore
  // sits inside the last k-step of the current one.
  bf16x8 fa[2][4], fb[2][4];
  auto frags = [&](int buf, int kt, int ks) {
    const uint16_t* sa = lds + (size_t)((2 * kt + 1) % kGmSlots) * kGmSlotElems;
    const uint16_t* sb = lds + (size_t)((2 * kt) % kGmSlots) * kGmSlotElems;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fa[buf][i] = load_frag(sa + ra[ks] + i * 32 * 8 * 8);
      fb[buf][i] = load_frag(sb + rb[ks] + i * 32 * 8 * 8);
    }
  };
  auto mfmas = [&](int buf) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
        acc[mi][ni] = SWAP ? mfma32(fb[buf][ni], fa[buf][mi], acc[mi][ni]) : mfma32(fa[buf][mi], fb[buf][ni], acc[mi][ni]);
  };
  // The refills are spread evenly over the k-steps, four loads per k-step and wave: a burst of sixteen at the
  // hand-over asks for more than the L2 -> CU path sustains, the queue backs up and the wave -- in-order, one per
  // SIMD -- stalls in the issue of a load with its MFMAs behind it.
  fill(0);
  fill(1);
  fill(2);
  fill_part(3, 0);
  __builtin_amdgcn_s_waitcnt(0x0F7C);  // vmcnt(12): fills 0 and 1 landed
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  frags(0, 0, 0);
  for (int kt = 0; kt < nkt; ++kt) {
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      frags((ks + 1) & 1, kt, ks + 1);
      // ks 0: second half of the weights of k-tile kt+1;  ks 1, 2: the tokens of k-tile kt+2
      if (ks == 0) fill_part(2 * kt + 3, 1);
      else fill_part(2 * kt + 4, ks - 1);
      mfmas(ks & 1);
      // the ring writes may alias the fragment reads as far as the compiler knows, so the reads go first
#pragma unroll
      // an MFMA leads: the wait in front of it then covers only the previous k-step's reads, long since back
      for (int g = 0; g < 8; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);  // two MFMAs
        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // one global -> LDS load
      }
    }
    // Last k-step.  Its fragments are in registers, so once every wave is here k-tile kt's two slots are free;
    // fills 2kt+2 and 2kt+3 (k-tile kt+1) must have landed, fill 2kt+4 (8 loads per wave, issued in this
    // k-tile's second and third k-step) may still be in flight.
    __builtin_amdgcn_s_waitcnt(0x0078);  // vmcnt(8) lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();  // bare: a fence would make the compiler drain every LDS-bound load in flight
    asm volatile("" ::: "memory");
    frags(0, kt + 1, 0);
    fill_part(2 * kt + 5, 0);  // first half of the weights of k-tile kt+2, into the slot of k-tile kt's tokens
    mfmas(1);
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);
    }
  }
  __builtin_amdgcn_s_waitcnt(0);  // drain the clamped tail loads before LDS is reused
  __syncthreads();
}

__global__ __launch_bounds__(256, 1) void append_gemm_kernel(AppendParams p) {
  extern __shared__ __align__(16) unsigned char smem_gemm[];
  uint16_t* const lds = reinterpret_cast<uint16_t*>(smem_gemm);
  // after the main loop the ring's memory holds, per token of the tile, the element offset of its page in the
  // pool (or -1) and its slot
  long long* const tok_page = reinterpret_cast<long long*>(smem_gemm);
  int* const tok_slot = reinterpret_cast<int*>(tok_page + kGmBN);
  long long* const grp_page = reinterpret_cast<long long*>(tok_slot + kGmBN);  // per aligned group of 4 tokens
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6), wm = w >> 1, wn = w & 1;
  // Workgroups are dealt round-robin over the 8 XCDs (each with its own L2).  The row blocks that share a token
  // tile get consecutive turns on ONE XCD, so that the tile comes from HBM once and is an L2 hit for the others.
  const int ny = (p.r_k + p.r_v + kGmBM - 1) / kGmBM;
  const int n_virtual = (((p.T + kGmBN - 1) / kGmBN + 7) / 8) * 8 * ny;
  // Persistent: the grid is one workgroup per CU (a multiple of 8, so that a workgroup stays on its XCD's turn
  // sequence) and every workgroup walks its tiles; a tile's stores drain while the next tile's ring fills.
  for (int vb = blockIdx.x; vb < n_virtual; vb += gridDim.x) {
  const int xcd = vb & 7, turn = vb >> 3;
  const int bx = (turn / ny) * 8 + xcd, by = turn % ny;
  if (bx * kGmBN >= p.T) continue;
  const int j0 = by * kGmBM, t0 = bx * kGmBN;
  const int rt = p.r_k + p.r_v, D = p.D;
  const int nkt = D / kGmBK;

  // The workgroup's 256 latent rows; at the matrix edge the window is slid back so that every row is real,
  // and rows outside a wave's own share are skipped by the epilogue.
  const int j0_eff = j0 + kGmBM <= rt ? j0 : (rt - kGmBM > 0 ? rt - kGmBM : 0);
  const int jw_eff = j0_eff + wm * 128;
  // This lane's eight source chunks per operand, as byte offsets from the tile's first row (rows past the matrices
  // are clamped, never stored).  The copies are buffer loads -- a descriptor of the tile's rows, a 32-bit lane
  // offset, the k-tile as scalar offset: next to a saturated MFMA stream they issue in a few cycles, where a
  // load with 64-bit lane addresses holds the wave, and its MFMAs, for about thirty.
  uint32_t aoff[8], xoff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int L = (i * 4 + w) * 64 + lane, row = L >> 3, c = (L & 7) ^ (row & 7);
    const int ja = j0_eff + row < rt ? row : rt - 1 - j0_eff;
    const int tb = t0 + row < p.T ? row : p.T - 1 - t0;
    aoff[i] = (uint32_t)((ja * D + c * 8) * 2);
    xoff[i] = (uint32_t)((tb * D + c * 8) * 2);
  }
  auto rows_rsrc = [&](const uint16_t* base, long long rows) {  // raw buffer over `rows` rows of D elements
    const long long bytes = rows * D * 2;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, bytes > 0x7fffffffLL ? 0x7fffffff : (int)bytes, 0x00020000);
  };
  const __amdgpu_buffer_rsrc_t at_rsrc = rows_rsrc(p.at + (size_t)j0_eff * D, rt - j0_eff);
  const __amdgpu_buffer_rsrc_t x_rsrc = rows_rsrc(p.x + (size_t)t0 * D, p.T - t0);
  // this thread's token of the tile: where it goes (looked up now, its latency hides behind the main loop)
  long long my_page_off = -1;
  int my_slot = 0;
  if (t0 + tid < p.T) {
    const int seq = p.slot_seq[t0 + tid], pos = p.slot_pos[t0 + tid];
    if (seq >= 0 && seq < p.n_seqs && pos >= 0 && pos < p.max_pages * kPage) {
      const int page = p.block_table[(size_t)seq * p.max_pages + pos / kPage];
      if (page >= 0 && page < p.n_pages) {
        my_page_off = (long long)page * (long long)p.page_elems;
        my_slot = pos % kPage;
      }
    }
  }
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[a][b][j] = 0.f;
  const bool all_v = jw_eff >= p.r_k;  // every block of this wave lies in the V latent: swapped operands
  if (all_v) gemm_mainloop<true>(acc, lds, at_rsrc, x_rsrc, aoff, xoff, nkt, w, wm, wn, hf, l32);
  else gemm_mainloop<false>(acc, lds, at_rsrc, x_rsrc, aoff, xoff, nkt, w, wm, wn, hf, l32);
  tok_page[tid] = my_page_off;
  tok_slot[tid] = my_slot;
  __syncthreads();
  if (tid < kGmBN / 4) {  // aligned groups of four tokens that sit in four consecutive slots of one page
    const long long pg0 = tok_page[4 * tid];
    const int s0 = tok_slot[4 * tid];
    bool run = pg0 >= 0 && (s0 & 3) == 0;
#pragma unroll
    for (int i = 1; i < 4; ++i) run = run && tok_page[4 * tid + i] == pg0 && tok_slot[4 * tid + i] == s0 + i;
    grp_page[tid] = run ? pg0 : -1;
  }
  __syncthreads();

  // ---------------- epilogue
  // Index arithmetic is hoisted: a destination is (page, slot)-dependent part + (latent block)-dependent part, the
  // first computed once per token (group), the second wave-uniform.
  auto pack4 = [&](const f32x16& a, int q4) {
    uint16_t v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = bf16_bits(a[4 * q4 + i]);
    return u32x2{(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16)};
  };
  if (!all_v) {
    // accumulator rows = latent index, lane = token: 4 consecutive latent indices per register group
    const int nks = p.r_k >> 4;
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int tl = wn * 128 + ni * 32 + l32;
      const long long page_off = tok_page[tl];
      if (page_off < 0) continue;
      const int slot = tok_slot[tl];
      uint16_t* base = p.cache + page_off;
      // K tiling: k_index(slot, jb + 8 q4 + 4 hf) = [slot part] + 4 hf + 32 jb + 256 q4   (jb a multiple of 32)
      uint16_t* kdst = base + ((size_t)(slot >> 5) * nks * 512 + (slot & 31) * 8 + 4 * hf);
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
        const int jb = jw_eff + mi * 32;
        if (jb < j0 || jb >= rt) continue;  // rows of the slid-back window that belong to the previous workgroup
        if (jb + 32 <= p.r_k) {             // wave-uniform: the whole block is K latent
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) *reinterpret_cast<u32x2*>(kdst + (size_t)jb * 32 + q4 * 256) = pack4(acc[mi][ni], q4);
        } else {
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int j = jb + 8 * q4 + 4 * hf;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const uint16_t v = bf16_bits(acc[mi][ni][4 * q4 + i]);
              if (j + i < p.r_k) base[k_index(p.r_k, slot, j + i)] = v;
              else base[v_index(p.r_k, slot, j + i - p.r_k)] = v;
            }
          }
        }
      }
    }
  } else {
    // swapped: accumulator rows = token, lane = latent index; 4 consecutive tokens per register group
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int tl = wn * 128 + ni * 32 + 8 * q4 + 4 * hf;
        const long long pg0 = grp_page[tl >> 2];
        const int s0 = tok_slot[tl];
        if (pg0 >= 0) {  // four consecutive slots of one page: contiguous in the V tiling
          // v_index(s0, jv) = 64 r_k + [slot part] + 8 (jv % 32) + 2048 (jv / 32),  jv = jb - r_k + l32
          uint16_t* vdst = p.cache + pg0 + ((size_t)kPage * p.r_k + (size_t)(s0 >> 4) * 512 + ((s0 & 15) >> 3) * 256 + (s0 & 7) + l32 * 8);
#pragma unroll
          for (int mi = 0; mi < 4; ++mi) {
            const int jb = jw_eff + mi * 32;
            if (jb < j0 || jb >= rt) continue;
            *reinterpret_cast<u32x2*>(vdst + (size_t)((jb - p.r_k) >> 5) * 2048) = pack4(acc[mi][ni], q4);
          }
        } else {
#pragma unroll
          for (int mi = 0; mi < 4; ++mi) {
            const int jb = jw_eff + mi * 32;
            if (jb < j0 || jb >= rt) continue;
            const int jv = jb + l32 - p.r_k;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const long long pg = tok_page[tl + i];
              if (pg >= 0) p.cache[pg + v_index(p.r_k, tok_slot[tl + i], jv)] = bf16_bits(acc[mi][ni][4 * q4 + i]);
            }
          }
        }
      }
    }
  }
  __syncthreads();  // the token arrays in the ring's memory have been read by everyone: the next tile may fill it
  }
}

// ------------------------------------------------------------------------------------------- append, small T
// Decode-time append: a handful of tokens against the whole down-projection.  The work is one pass over the
// weights (8 MiB for the 8B shape); a CU pulls a few tens of GB/s at best, so the pass must be spread over all of
// them: one workgroup per FOUR latent rows (256 workgroups for 1024 rows), no matrix cores.  Each thread owns an
// 8-wide slice of the model dimension per trip, multiplies it against up to 16 tokens with packed bf16 dot
// products (fp32 accumulation), and the 4 x 16 partial sums of the 256 threads meet in LDS.
constexpr int kSkRows = 4, kSkTok = 16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
// Pair c of an 8-element operand.  Taken with a vector shuffle: re-interpreting one 32-bit element of an integer
// vector as a bf16 pair was observed to be mis-compiled (every pair read element 0) by this toolchain.
__device__ __forceinline__ bf16x2 bf16_pair(bf16x8 v, int c) {
  switch (c) {
    case 0: return __builtin_shufflevector(v, v, 0, 1);
    case 1: return __builtin_shufflevector(v, v, 2, 3);
    case 2: return __builtin_shufflevector(v, v, 4, 5);
    default: return __builtin_shufflevector(v, v, 6, 7);
  }
}

__global__ __launch_bounds__(256) void append_skinny_kernel(AppendParams p) {
  constexpr int NO = kSkRows * kSkTok, RS = NO + 1;  // outputs per workgroup; padded row stride (bank-conflict free)
  __shared__ float red[128 * RS];                    // [thread pair][output]
  const int tid = threadIdx.x;
  const int j0 = blockIdx.x * kSkRows;
  const int D = p.D;
  for (int t0 = 0; t0 < p.T; t0 += kSkTok) {
    const int nt = p.T - t0 < kSkTok ? p.T - t0 : kSkTok;
    // Where output (row o / 16, token t0 + o % 16) goes: looked up by thread o now, so that the chain of
    // dependent loads overlaps the pass over the weights.
    long long dst_page = -1;
    int dst_slot = 0;
    if (tid < kSkRows * kSkTok && (tid % kSkTok) < nt) {
      const int t = t0 + tid % kSkTok;
      const int seq = p.slot_seq[t], pos = p.slot_pos[t];
      if (seq >= 0 && seq < p.n_seqs && pos >= 0 && pos < p.max_pages * kPage) {
        const int page = p.block_table[(size_t)seq * p.max_pages + pos / kPage];
        if (page >= 0 && page < p.n_pages) {
          dst_page = (long long)page * (long long)p.page_elems;
          dst_slot = pos % kPage;
        }
      }
    }
    float acc[kSkRows][kSkTok];
#pragma unroll
    for (int r = 0; r < kSkRows; ++r)
#pragma unroll
      for (int t = 0; t < kSkTok; ++t) acc[r][t] = 0.f;
    // two 8-wide slices per trip: 40 independent 16-byte loads in flight per thread
    for (int k0 = tid * 8; k0 < D; k0 += 2 * 256 * 8) {
      const int k1 = k0 + 256 * 8 < D ? k0 + 256 * 8 : k0;  // second slice (repeated and weighted zero past the end)
      const bool two = k0 + 256 * 8 < D;
      bf16x8 wv[2][kSkRows], xv[2][kSkTok];
#pragma unroll
      for (int r = 0; r < kSkRows; ++r) {
        wv[0][r] = load_frag(p.at + (size_t)(j0 + r) * D + k0);
        wv[1][r] = load_frag(p.at + (size_t)(j0 + r) * D + k1);
      }
#pragma unroll
      for (int t = 0; t < kSkTok; ++t) {  // tokens past the batch re-read the last one; their sums are never stored
        const uint16_t* xr = p.x + (size_t)(t0 + (t < nt ? t : nt - 1)) * D;
        xv[0][t] = load_frag(xr + k0);
        xv[1][t] = load_frag(xr + k1);
      }
      if (!two) {
#pragma unroll
        for (int r = 0; r < kSkRows; ++r) wv[1][r] = zero_frag();
      }
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int r = 0; r < kSkRows; ++r)
#pragma unroll
          for (int t = 0; t < kSkTok; ++t)
#pragma unroll
            for (int c = 0; c < 4; ++c)
              acc[r][t] = __builtin_amdgcn_fdot2_f32_bf16(bf16_pair(wv[h][r], c), bf16_pair(xv[h][t], c), acc[r][t], false);
    }
    __syncthreads();  // the previous token pass is done with red
    // neighbouring threads are added in registers (one DPP step), the even one files the pair's sums
#pragma unroll
    for (int r = 0; r < kSkRows; ++r)
#pragma unroll
      for (int t = 0; t < kSkTok; ++t) {
        const float v = acc[r][t] + half_wave_peer<0>(acc[r][t]);
        if ((tid & 1) == 0) red[(tid >> 1) * RS + r * kSkTok + t] = v;
      }
    __syncthreads();
    float part = 0.f;
    {
      const int o = tid & 63, q = tid >> 6;  // output o, quarter q of the pairs
#pragma unroll 16
      for (int i = 0; i < 32; ++i) part += red[(q * 32 + i) * RS + o];
    }
    __syncthreads();  // everyone has read its partial sums: the front of red is reused for the four quarters
    red[tid] = part;
    __syncthreads();
    if (tid < kSkRows * kSkTok && dst_page >= 0) {
      const float v = red[tid] + red[64 + tid] + red[128 + tid] + red[192 + tid];  // kSkRows * kSkTok == 64 outputs
      const int j = j0 + tid / kSkTok;
      uint16_t* base = p.cache + dst_page;
      base[j < p.r_k ? k_index(p.r_k, dst_slot, j) : v_index(p.r_k, dst_slot, j - p.r_k)] = bf16_bits(v);
    }
  }
}

// ------------------------------------------------------------------------------------------------ probe
__global__ void stream_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink) {
  uint32_t acc = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;  // practically never true: keeps the loads alive without a store
}

// Matrix-core rate probe: every wave issues `iters` x 8 independent 32x32x16 bf16 MFMAs on operands held in registers
// (no memory traffic in the loop).  What it sustains is what the board's power management leaves of the nominal
// peak for this operand data: 0 = pseudo-random sign and mantissa, 1 = zeros, 2 = ones.
__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(float* sink, int iters, int operands) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    u32x4 va, vb;
    uint32_t sa = (uint32_t)threadIdx.x * 9781u + (uint32_t)i * 7u + 1u, sb = (uint32_t)threadIdx.x * 6271u + (uint32_t)i * 13u + 5u + blockIdx.x;
#pragma unroll
    for (int c = 0; c < 4; ++c) {  // xorshift; |x| in [2^-5, 2^-4)
      sa ^= sa << 13; sa ^= sa >> 17; sa ^= sa << 5;
      sb ^= sb << 13; sb ^= sb >> 17; sb ^= sb << 5;
      va[c] = operands == 0 ? ((sa & 0x807f807fu) | 0x3d003d00u) : (operands == 2 ? 0x3f803f80u : 0u);
      vb[c] = operands == 0 ? ((sb & 0x807f807fu) | 0x3d003d00u) : (operands == 2 ? 0x3f803f80u : 0u);
    }
    a[i] = __builtin_bit_cast(bf16x8, va);
    b[i] = __builtin_bit_cast(bf16x8, vb);
  }
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  for (int it = 0; it < iters; ++it)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = mfma32(a[i & 3], b[(i >> 1) & 3], acc[i]);
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) r += acc[i][j];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}

int launch_mfma_probe(float* sink, int workgroups, int iters, int operands, hipStream_t s) {
  return launch_kernel(mfma_rate_kernel, dim3(workgroups), dim3(256), 0, s, sink, iters, operands);
}

int launch_pack(const lorc_layer_desc& d, const void* A_k, const void* A_v, const void* B_k, const void* B_v,
                void* packed, hipStream_t s) {
  const int n = d.n_kv_heads * d.head_dim;
  return launch_kernel(pack_factors_kernel, dim3(2048), dim3(256), 0, s, (const uint16_t*)A_k, (const uint16_t*)A_v,
                       (const uint16_t*)B_k, (const uint16_t*)B_v, (uint16_t*)packed, d.d_model, d.rank_k, d.rank_v, n,
                       d.head_dim, d.rope_base);
}

int set_kernel_attributes_append() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(append_gemm_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             160 * 1024) == hipSuccess ? LORC_OK : LORC_EHIP;
}

// Which kernel takes which batch (measured, 8B shape, us per call):  T = 64: dot-product kernel 21, 64-tile GEMM 23;
// T = 128: 38 / 23;  T = 256 .. 1024: 64-tile GEMM 21 .. 27;  T = 2048: 64-tile 39 .. 45, 128-tile 45 .. 55;
// T = 4096: 64-tile 73 .. 81, 128-tile 49, 256-tile 75;  T = 8192: 128-tile 97, 256-tile 86;  T = 16384: 185 / 114.
// Below a few thousand tokens every GEMM is bound by its serial walk over the model dimension with few workgroups
// (splitting it would need scratch memory, which this entry point does not take).
constexpr int kSkinnyMaxT = 64, kGemmMinT = 8192, kSmallTileMaxWgs = 512;

int launch_append(const AppendParams& p, int n_cus, hipStream_t s) {
  if (p.T <= kSkinnyMaxT) return launch_kernel(append_skinny_kernel, dim3((p.r_k + p.r_v) / kSkRows), dim3(256), 0, s, p);
  if (p.T >= kGemmMinT && p.D % kGmBK == 0 && p.D / kGmBK >= 2) {
    const size_t lds = kGmLdsBytes;
    const int nx = (p.T + kGmBN - 1) / kGmBN, ny = (p.r_k + p.r_v + kGmBM - 1) / kGmBM;
    const int n_virtual = ((nx + 7) / 8) * 8 * ny, slots = (n_cus / 8) * 8;
    dim3 grid(n_virtual < slots ? n_virtual : slots);
    return launch_kernel(append_gemm_kernel, grid, dim3(256), lds, s, p);
  }
  // the small tile while all its workgroups are resident at once (two per CU)
  const int rt = p.r_k + p.r_v;
  const long wg64 = (long)((p.T + 63) / 64) * ((rt + 63) / 64);
  if (wg64 <= kSmallTileMaxWgs) {
    dim3 grid((p.T + 63) / 64, (rt + 63) / 64);
    return launch_kernel(append_kernel<64, 8>, grid, dim3(256), 0, s, p);
  }
  dim3 grid((p.T + 127) / 128, (rt + 127) / 128);
  return launch_kernel(append_kernel<128, 4>, grid, dim3(256), 0, s, p);
}

int launch_stream_probe(const void* src, size_t bytes, void* sink, hipStream_t s) {
  return launch_kernel(stream_read_kernel, dim3(256 * 8), dim3(256), 0, s, (const u32x4*)src, bytes / 16, (uint32_t*)sink);
}

}  // namespace lorc

