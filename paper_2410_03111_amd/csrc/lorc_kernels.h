// Internal: parameter blocks and launchers of the HIP kernels (defined in the .hip files, called by the C ABI).
#ifndef LORC_KERNELS_H_
#define LORC_KERNELS_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <utility>

#include "lorc.h"

namespace lorc {

// One kernel launch that reports its own status.  (hipGetLastError() after a <<<>>> launch would also return, and
// clear, an error left behind by an unrelated earlier call of the process.)
template <typename... KArgs, size_t... I>
inline hipError_t launch_kernel_impl(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s,
                                     std::tuple<KArgs...>& held, std::index_sequence<I...>) {
  void* ptrs[] = {static_cast<void*>(&std::get<I>(held))...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kern), grid, block, ptrs, lds, s);
}
template <typename... KArgs, typename... Args>
inline int launch_kernel(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t s, Args&&... args) {
  static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count of the kernel");
  std::tuple<KArgs...> held(static_cast<KArgs>(std::forward<Args>(args))...);
  return launch_kernel_impl(kern, grid, block, lds, s, held, std::index_sequence_for<KArgs...>{}) == hipSuccess
             ? LORC_OK : LORC_EHIP;
}

struct AppendParams {
  const uint16_t* x;        // [T x D]
  const uint16_t* at;       // packed At [(r_k + r_v) x D]
  const uint16_t* at_tiled; // the same matrix in 32 x 16 operand tiles
  const int32_t* slot_seq;  // [T]
  const int32_t* slot_pos;  // [T]
  const int32_t* block_table;
  uint16_t* cache;
  int T, D, r_k, r_v, n_seqs, max_pages, n_pages;
  size_t page_elems;
};

// Split plan of one decode call; computed on the host from (desc, b, max_ctx) only, so that the workspace
// size and the launch agree.
struct DecodePlan {
  int tile;             // positions per tile (64 or 128)
  int occupancy;        // workgroups meant to share a CU (1 or 2)
  int stationary;       // 1: the split kernel with the key factor held in registers (lorc_decode_stat.hip)
  int wide;             // three-launch path (lorc_decode_wide.hip): 1 ranks above 1024, 2 uncompressed layer, 3 absorbed query
  int score_stride;     // wide: positions per score row (max_ctx rounded up to whole tiles)
  int v_chunks;         // wide: column chunks of the value kernel (512 latent columns each; uncompressed: KV heads)
  size_t off_scores;    // wide: fp32 scores [b][h_q][score_stride]
  int n_splits;         // context splits per sequence
  int tiles_per_split;  // tiles each split walks
  size_t off_ml, off_o, total_bytes;  // workspace carve-up (bytes)
};

struct DecodeParams {
  const uint16_t* q;        // [b x h_q x d]
  const int32_t* q_pos;     // [b]
  const int32_t* ctx_len;   // [b]
  const uint16_t* bk;       // packed B_k tiles
  const uint16_t* bv;       // packed B_v tiles
  const uint16_t* cache;
  const int32_t* block_table;
  uint16_t* out;            // [b x h_q x d], or [b x h_q x r_v] when latent_out is set
  int latent_out;           // 1: the merge writes the normalised latent-space output and skips the up-projection
  const double* rope_tab;   // packed: theta_i, i < head_dim / 2
  const float2* lane_cs;    // packed: (cos, sin)(l * theta_i), l < 32, [l][head_dim / 2]
  float* part_ml;           // workspace: [b][split][h_q][2]
  uint16_t* part_o;         // workspace: [b][split][h_q][r_v] fp16, each split's o_lat normalised by its own sum
  float* scores;            // workspace of the three-launch path: [b][h_q][score_stride], scaled by softmax scale x log2 e
  int score_stride, v_chunks;
  int b, h_q, h_kv, G, head_dim, r_k, r_v, n_tasks, max_ctx, max_pages, n_pages, n_splits, tiles_per_split;
  size_t page_elems;
  float rope_base, q_scale;  // q_scale = softmax scale * log2(e)
};

struct PrefillPlan {
  int tiles_per_seq;  // 64-position pages per sequence slot of the scratch
  int lp;             // padded sequence length of the scratch (tiles_per_seq * 64)
  size_t off_rope, off_krot, off_vt, total_bytes;
};

struct PrefillParams {
  const uint16_t* q;          // [total x h_q x d] bf16
  const int32_t* cu_seqlens;  // [b + 1]
  const uint16_t* bk;
  const uint16_t* bv;
  const uint16_t* cache;
  const int32_t* block_table;
  uint16_t* out;              // [total x h_q x d] bf16
  const double* rope_tab;     // packed: theta_i
  uint16_t* krot;             // workspace: rotated keys, fp16 [b][lp][n]
  uint16_t* vt;               // workspace: values transposed, fp16 [b][n][lp], positions permuted in groups of 16
  int b, h_q, h_kv, G, head_dim, r_k, r_v, max_pages, n_pages, tiles_per_seq, lp;
  size_t page_elems;
  float rope_base, q_scale;
};

// Every launcher returns LORC_OK or the lorc_status of the first launch (or event record) that failed.
PrefillPlan make_prefill_plan(const lorc_layer_desc& d, int b, int max_seqlen);
int launch_prefill(const PrefillParams& p, hipStream_t s, bool plain = false);

DecodePlan make_decode_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus);

int launch_pack(const lorc_layer_desc& d, const void* A_k, const void* A_v, const void* B_k, const void* B_v,
                void* packed, hipStream_t s);
int launch_append(const AppendParams& p, int n_cus, hipStream_t s);
int launch_decode(const DecodeParams& p, const DecodePlan& plan, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end);
DecodePlan make_absorbed_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus);
int launch_decode_absorbed(const DecodeParams& p, const DecodePlan& plan, hipStream_t s, hipEvent_t ev_begin, hipEvent_t ev_end);
int launch_stream_probe(const void* src, size_t bytes, void* sink, hipStream_t s);
int launch_mfma_probe(float* sink, int workgroups, int iters, int operands, hipStream_t s);

// Kernels that use more than 64 KiB of LDS need a function attribute, set once per device (the call is not
// capturable into a HIP graph).  Each translation unit sets it for its own kernels.
int set_kernel_attributes_append();
int set_kernel_attributes_decode();
int set_kernel_attributes_prefill();
int set_kernel_attributes_decode_stationary();

// Split kernel that keeps the key factor in registers (head_dim 128, an even number of KV heads, G <= 8, ranks
// <= 512); its plan and launch.  The merge launch that follows is the common one.
bool stationary_shape_ok(const lorc_layer_desc& d);
DecodePlan make_stationary_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus);
int launch_decode_stationary_split(const DecodeParams& p, const DecodePlan& plan, hipStream_t s);

// Three-launch decode (scores, values in column chunks, merge) for ranks above 1024 and for uncompressed layers.
bool wide_shape_ok(const lorc_layer_desc& d);
bool plain_shape_ok(const lorc_layer_desc& d);
bool wide_absorbed_shape_ok(const lorc_layer_desc& d);
DecodePlan make_wide_plan(const lorc_layer_desc& d, int b, int max_ctx, int n_cus, bool plain);
int launch_decode_wide(const DecodeParams& p, const DecodePlan& plan, hipStream_t s);
int set_kernel_attributes_decode_wide();

}  // namespace lorc
#endif  // LORC_KERNELS_H_
