// Internal: geometry checks and the index functions of the paged latent cache and of the packed factors.
// Shared by the host translation unit and the HIP kernels of this library (and by nothing else).
#ifndef LORC_LAYOUT_H_
#define LORC_LAYOUT_H_

#include <stddef.h>
#include <stdint.h>

#include "lorc.h"

#if defined(__HIPCC__)
#define LORC_HD __host__ __device__ __forceinline__
#else
#define LORC_HD inline
#endif

namespace lorc {

constexpr int kPage = LORC_PAGE_TOKENS;  // positions per cache page
constexpr int kMaxRank = 8192;           // largest latent width a layer may declare (each kernel path has its own limit)
constexpr int kStreamMaxRank = 1024;     // largest latent width the single-pass decode kernels keep resident in LDS
constexpr int kWideMaxRank = 2048;       // largest latent width of the three-launch decode path (merge kernel's LDS row)

inline int check_desc(const lorc_layer_desc& d) {
  if (d.d_model <= 0 || d.n_q_heads <= 0 || d.n_kv_heads <= 0 || d.rank_k <= 0 || d.rank_v <= 0) return LORC_EINVAL;
  if (d.n_q_heads % d.n_kv_heads != 0) return LORC_EINVAL;
  if (!(d.rope_base > 1.0f) || !(d.softmax_scale >= 0.0f)) return LORC_EINVAL;
  const long n = (long)d.n_kv_heads * d.head_dim;
  if (d.rank_k > n || d.rank_v > n) return LORC_EINVAL;
  if (d.head_dim != 64 && d.head_dim != 128) return LORC_EUNSUPPORTED;
  if (d.page_size != kPage) return LORC_EUNSUPPORTED;
  if (d.rank_k % 32 != 0 || d.rank_v % 32 != 0 || d.rank_k > kMaxRank || d.rank_v > kMaxRank) return LORC_EUNSUPPORTED;
  if (d.d_model % 64 != 0 || n % 64 != 0) return LORC_EUNSUPPORTED;
  if (d.n_q_heads / d.n_kv_heads > 32 || d.n_q_heads > 64) return LORC_EUNSUPPORTED;
  return LORC_OK;
}

// ---- latent cache page: [K part: 64 x r_k][V part: 64 x r_v], element = bf16 --------------------------
LORC_HD size_t page_elems(int r_k, int r_v) { return (size_t)kPage * (size_t)(r_k + r_v); }

// K part is tiled [slot/32][j/16][64 lanes][8]: lane = slot%32 + 32*((j%16)/8) holds 8 consecutive latent
// indices of one position -- the B operand (k = latent index, n = position) of a 32x32x16 matrix-core op.
LORC_HD int64_t k_index(int r_k, int slot, int j) {
  return ((int64_t)((slot >> 5) * (r_k >> 4) + (j >> 4)) * 64 + (slot & 31) + 32 * ((j & 15) >> 3)) * 8 + (j & 7);
}

// V part is tiled [j/32][slot/16][64 lanes][8]: lane = j%32 + 32*((slot%16)/8) holds 8 consecutive
// positions of one latent index -- the B operand (k = position, n = latent index).
LORC_HD int64_t v_index(int r_k, int slot, int j) {
  return (int64_t)kPage * r_k +
         ((int64_t)((j >> 5) * 4 + (slot >> 4)) * 64 + (j & 31) + 32 * ((slot & 15) >> 3)) * 8 + (slot & 7);
}

// ---- packed factors: [At: (r_k + r_v) x D][Bk tiles][Bv tiles][At tiles][rotation tables], element = bf16 ----
// At row j (< r_k: column j of A_k, else column j - r_k of A_v) is contiguous over the model dimension.
// B tiles are [c/32][j/16][64 lanes][8]: lane = c%32 + 32*((j%16)/8) holds 8 consecutive latent indices of
// output column c -- the A operand (m = column, k = latent index).
LORC_HD size_t packed_at_elems(int D, int r_k, int r_v) { return (size_t)(r_k + r_v) * (size_t)D; }
LORC_HD size_t packed_b_elems(int r, int n) { return (size_t)r * (size_t)n; }
LORC_HD int64_t b_tile_index(int r, int j, int c) {
  return ((int64_t)((c >> 5) * (r >> 4) + (j >> 4)) * 64 + (c & 31) + 32 * ((j & 15) >> 3)) * 8 + (j & 7);
}
LORC_HD size_t packed_off_bk(int D, int r_k, int r_v) { return packed_at_elems(D, r_k, r_v); }
LORC_HD size_t packed_off_bv(int D, int r_k, int r_v, int n) { return packed_off_bk(D, r_k, r_v) + packed_b_elems(r_k, n); }
// A second copy of At, tiled [j/32][k/16][64 lanes][8] (lane = j%32 + 32*((k%16)/8), 8 consecutive k): the
// operand (rows = latent index, contraction over the model dimension) the large-T append streams to registers.
LORC_HD size_t packed_off_at_tiled(int D, int r_k, int r_v, int n) { return packed_off_bv(D, r_k, r_v, n) + packed_b_elems(r_v, n); }
LORC_HD int64_t at_tile_index(int D, int j, int k) {
  return ((int64_t)((j >> 5) * (D >> 4) + (k >> 4)) * 64 + (j & 31) + 32 * ((k & 15) >> 3)) * 8 + (k & 7);
}
// Rotation tables of the layer (they depend on head_dim and the RoPE base only): 64 doubles theta_i, then
// 32 x 64 float pairs (cos, sin)(l * theta_i) for the position offsets l < 32 inside an operand block.
constexpr size_t kRopeTabBytes = 64 * 8 + 32 * 64 * 8;
LORC_HD size_t packed_off_rope(int D, int r_k, int r_v, int n) {
  return packed_off_at_tiled(D, r_k, r_v, n) + packed_at_elems(D, r_k, r_v);
}
LORC_HD size_t packed_total_elems(int D, int r_k, int r_v, int n) {
  return packed_off_rope(D, r_k, r_v, n) + kRopeTabBytes / 2;
}

}  // namespace lorc
#endif  // LORC_LAYOUT_H_
