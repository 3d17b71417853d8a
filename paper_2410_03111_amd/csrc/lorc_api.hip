// C ABI of the device entry points: argument validation on the host, then kernel launches on the caller's
// stream.  Nothing here allocates or synchronises.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>

#include "lorc.h"
#include "lorc_kernels.h"
#include "lorc_layout.h"

using namespace lorc;

namespace {
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// The only state the library keeps: per device, whether the large-LDS function attributes have been set and how
// many compute units it has.  Filled by the first entry point called with that device current (normally
// lorc_pack_factors); the attribute call cannot be captured into a HIP graph, every later call can.
constexpr int kMaxDevices = 64;
std::atomic<int> g_device_cus[kMaxDevices];  // 0 = not initialised yet

// Split partials of lorc_decode_attention_static: device memory that belongs to the library's code object, one
// copy per GPU.  Host code never uses the array's name as an address; it asks the runtime for the device address
// once per device (below) and passes that pointer on.
constexpr size_t kStaticScratchBytes = LORC_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device; valid once g_device_cus is set

int device_ready(int* n_cus) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORC_EHIP;
  int v = g_device_cus[dev].load(std::memory_order_acquire);
  if (v == 0) {
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return LORC_EHIP;
    if (int rc = set_kernel_attributes_append()) return rc;
    if (int rc = set_kernel_attributes_decode()) return rc;
    if (int rc = set_kernel_attributes_prefill()) return rc;
    void* sp = nullptr;
    if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || sp == nullptr) return LORC_EHIP;
    g_scratch_ptr[dev] = sp;
    g_device_cus[dev].store(v, std::memory_order_release);
  }
  if (n_cus) *n_cus = v;
  return LORC_OK;
}

// Compute-unit count for the workspace-size helpers, which must agree with the launch: the current device's if it
// can be asked, else the MI355X's.
int cu_count_or_default() {
  int dev = 0, v = 0;
  if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices) {
    v = g_device_cus[dev].load(std::memory_order_acquire);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) return v;
  }
  (void)hipGetLastError();  // no device: not an error of this call
  return 256;
}

float softmax_scale_log2(const lorc_layer_desc& d) {
  const float scale = d.softmax_scale > 0.f ? d.softmax_scale : 1.0f / std::sqrt((float)d.head_dim);
  return scale * 1.4426950408889634f;
}

// Argument checks shared by the decode entry points (rotary, latent-space output, absorbed query): everything that
// can be refused without asking the device.
int decode_args(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos, bool needs_q_pos, const int32_t* ctx_len,
                int32_t b, int32_t max_ctx, const void* packed, const void* cache, const int32_t* block_table,
                int32_t max_pages, int32_t n_pages, const void* out, const void* workspace) {
  if (!desc || !q || (needs_q_pos && !q_pos) || !ctx_len || !packed || !cache || !block_table || !out || !workspace) return LORC_EINVAL;
  if (int rc = check_desc(*desc)) return rc;
  if (b <= 0 || max_ctx < 0 || max_pages <= 0 || n_pages <= 0) return LORC_EINVAL;
  if ((long)max_pages * kPage < max_ctx) return LORC_EINVAL;
  if (!aligned16(q) || !aligned16(packed) || !aligned16(cache) || !aligned16(out)) return LORC_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return LORC_EINVAL;
  return LORC_OK;
}

// Workspace check and the parameter block of the decode kernels.
int decode_params(DecodeParams& p, const lorc_layer_desc* desc, const void* q, const int32_t* q_pos, bool needs_q_pos,
                  const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed, const void* cache,
                  const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out, void* workspace,
                  size_t workspace_bytes, const DecodePlan& plan, int latent_out) {
  if (plan.total_bytes == 0) return LORC_EUNSUPPORTED;  // no kernel path takes this shape
  if (workspace_bytes < plan.total_bytes) return LORC_EWORKSPACE;
  const int n = desc->n_kv_heads * desc->head_dim;
  const uint16_t* pk = static_cast<const uint16_t*>(packed);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  p.q = static_cast<const uint16_t*>(q);
  p.q_pos = q_pos;
  p.ctx_len = ctx_len;
  p.bk = pk + packed_off_bk(desc->d_model, desc->rank_k, desc->rank_v);
  p.bv = pk + packed_off_bv(desc->d_model, desc->rank_k, desc->rank_v, n);
  p.cache = static_cast<const uint16_t*>(cache);
  p.block_table = block_table;
  p.out = static_cast<uint16_t*>(out);
  p.latent_out = latent_out;
  p.rope_tab = reinterpret_cast<const double*>(pk + packed_off_rope(desc->d_model, desc->rank_k, desc->rank_v, n));
  p.lane_cs = reinterpret_cast<const float2*>(p.rope_tab + 64);
  p.part_ml = reinterpret_cast<float*>(ws + plan.off_ml);
  p.part_o = reinterpret_cast<uint16_t*>(ws + plan.off_o);
  p.scores = reinterpret_cast<float*>(ws + plan.off_scores);
  p.score_stride = plan.score_stride;
  p.v_chunks = plan.v_chunks;
  p.b = b;
  p.h_q = desc->n_q_heads;
  p.h_kv = desc->n_kv_heads;
  p.G = desc->n_q_heads / desc->n_kv_heads;
  p.head_dim = desc->head_dim;
  p.r_k = desc->rank_k;
  p.r_v = desc->rank_v;
  p.n_tasks = n / 64;
  p.max_ctx = max_ctx;
  p.max_pages = max_pages;
  p.n_pages = n_pages;
  p.n_splits = plan.n_splits;
  p.tiles_per_split = plan.tiles_per_split;
  p.page_elems = page_elems(desc->rank_k, desc->rank_v);
  p.rope_base = desc->rope_base;
  p.q_scale = softmax_scale_log2(*desc);
  return LORC_OK;
}

int decode_rotary(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos, const int32_t* ctx_len, int32_t b,
                  int32_t max_ctx, const void* packed, const void* cache, const int32_t* block_table, int32_t max_pages,
                  int32_t n_pages, void* out, void* workspace, size_t workspace_bytes, void* stream, void* ev_begin,
                  void* ev_end, int latent_out, bool plain = false) {
  if (int rc = decode_args(desc, q, q_pos, true, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages, out, workspace))
    return rc;
  if (plain && !plain_shape_ok(*desc)) return LORC_EUNSUPPORTED;
  int n_cus = 0;
  if (int rc = device_ready(&n_cus)) return rc;
  const DecodePlan plan = plain ? make_wide_plan(*desc, b, max_ctx, n_cus, true) : make_decode_plan(*desc, b, max_ctx, n_cus);
  DecodeParams p;
  if (int rc = decode_params(p, desc, q, q_pos, true, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages,
                             out, workspace, workspace_bytes, plan, latent_out))
    return rc;
  return launch_decode(p, plan, static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(ev_begin),
                       static_cast<hipEvent_t>(ev_end));
}
}  // namespace

extern "C" {

size_t lorc_packed_bytes(const lorc_layer_desc* desc) {
  if (!desc || check_desc(*desc) != LORC_OK) return 0;
  return packed_total_elems(desc->d_model, desc->rank_k, desc->rank_v, desc->n_kv_heads * desc->head_dim) * 2;
}

int lorc_pack_factors(const lorc_layer_desc* desc, const void* A_k, const void* A_v, const void* B_k,
                      const void* B_v, void* packed, void* stream) {
  if (!desc || !A_k || !A_v || !packed) return LORC_EINVAL;
  if (int rc = check_desc(*desc)) return rc;
  // an uncompressed layer (rank = n on both sides) has identity read-side factors, which are never stored
  const int n_cols = desc->n_kv_heads * desc->head_dim;
  const bool no_b = !B_k && !B_v;
  if ((!B_k || !B_v) && !(no_b && desc->rank_k == n_cols && desc->rank_v == n_cols)) return LORC_EINVAL;
  if (!aligned16(packed)) return LORC_EINVAL;
  if (int rc = device_ready(nullptr)) return rc;
  return launch_pack(*desc, A_k, A_v, B_k, B_v, packed, static_cast<hipStream_t>(stream));
}

int lorc_append_latent(const lorc_layer_desc* desc, const void* x, int32_t T, const void* packed,
                       const int32_t* slot_seq, const int32_t* slot_pos, const int32_t* block_table,
                       int32_t n_seqs, int32_t max_pages, int32_t n_pages, void* cache, void* stream) {
  if (!desc || !x || !packed || !slot_seq || !slot_pos || !block_table || !cache) return LORC_EINVAL;
  if (int rc = check_desc(*desc)) return rc;
  if (T < 0 || n_seqs <= 0 || max_pages <= 0 || n_pages <= 0) return LORC_EINVAL;
  if (!aligned16(x) || !aligned16(packed) || !aligned16(cache)) return LORC_EINVAL;
  if (T == 0) return LORC_OK;
  int n_cus = 0;
  if (int rc = device_ready(&n_cus)) return rc;
  AppendParams p;
  p.x = static_cast<const uint16_t*>(x);
  p.at = static_cast<const uint16_t*>(packed);
  p.at_tiled = p.at + packed_off_at_tiled(desc->d_model, desc->rank_k, desc->rank_v, desc->n_kv_heads * desc->head_dim);
  p.slot_seq = slot_seq;
  p.slot_pos = slot_pos;
  p.block_table = block_table;
  p.cache = static_cast<uint16_t*>(cache);
  p.T = T;
  p.D = desc->d_model;
  p.r_k = desc->rank_k;
  p.r_v = desc->rank_v;
  p.n_seqs = n_seqs;
  p.max_pages = max_pages;
  p.n_pages = n_pages;
  p.page_elems = page_elems(desc->rank_k, desc->rank_v);
  return launch_append(p, n_cus, static_cast<hipStream_t>(stream));
}

size_t lorc_decode_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx) {
  if (!desc || check_desc(*desc) != LORC_OK || b <= 0 || max_ctx < 0) return 0;
  return make_decode_plan(*desc, b, max_ctx, cu_count_or_default()).total_bytes;
}

const char* lorc_decode_plan_info(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx, int32_t* n_splits,
                                  int32_t* tiles_per_split) {
  if (!desc || check_desc(*desc) != LORC_OK || b <= 0 || max_ctx < 0) return nullptr;
  const DecodePlan plan = make_decode_plan(*desc, b, max_ctx, cu_count_or_default());
  if (plan.total_bytes == 0) return nullptr;
  if (n_splits) *n_splits = plan.n_splits;
  if (tiles_per_split) *tiles_per_split = plan.tiles_per_split;
  return plan.wide ? "wide_scores_kernel" : (plan.stationary ? "decode_stationary_kernel" : "decode_split_kernel");
}

size_t lorc_decode_plain_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx) {
  if (!desc || check_desc(*desc) != LORC_OK || !plain_shape_ok(*desc) || b <= 0 || max_ctx < 0) return 0;
  return make_wide_plan(*desc, b, max_ctx, cu_count_or_default(), true).total_bytes;
}

int lorc_decode_attention_plain(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                const void* cache, const int32_t* block_table, int32_t max_pages, int32_t n_pages,
                                void* out, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_rotary(desc, q, q_pos, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages, out, workspace,
                       workspace_bytes, stream, nullptr, nullptr, 0, true);
}

int lorc_decode_attention(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                          const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                          const void* cache, const int32_t* block_table, int32_t max_pages, int32_t n_pages,
                          void* out, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_rotary(desc, q, q_pos, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages, out, workspace,
                       workspace_bytes, stream, nullptr, nullptr, 0);
}

int lorc_decode_attention_timed(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                const void* cache, const int32_t* block_table, int32_t max_pages,
                                int32_t n_pages, void* out, void* workspace, size_t workspace_bytes,
                                void* stream, void* ev_split_begin, void* ev_split_end) {
  return decode_rotary(desc, q, q_pos, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages, out, workspace,
                       workspace_bytes, stream, ev_split_begin, ev_split_end, 0);
}

int lorc_decode_attention_latent(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                 const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                 const void* cache, const int32_t* block_table, int32_t max_pages,
                                 int32_t n_pages, void* out_latent, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  return decode_rotary(desc, q, q_pos, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages, out_latent,
                       workspace, workspace_bytes, stream, nullptr, nullptr, 1);
}

int lorc_decode_attention_static(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                 const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                 const void* cache, const int32_t* block_table, int32_t max_pages, int32_t n_pages,
                                 void* out, void* stream) {
  if (!desc) return LORC_EINVAL;
  if (int rc = check_desc(*desc)) return rc;
  if (int rc = device_ready(nullptr)) return rc;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LORC_EHIP;
  // a problem whose partials do not fit the array is refused by the workspace check (LORC_EWORKSPACE)
  return decode_rotary(desc, q, q_pos, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages, out,
                       g_scratch_ptr[dev], kStaticScratchBytes, stream, nullptr, nullptr, 0);
}

// ---- decode without positional rotation, absorbed query (Section 4.1, Eq. 7)
size_t lorc_decode_absorbed_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx) {
  if (!desc || check_desc(*desc) != LORC_OK || b <= 0 || max_ctx < 0) return 0;
  return make_absorbed_plan(*desc, b, max_ctx, cu_count_or_default()).total_bytes;
}

int lorc_decode_attention_absorbed_timed(const lorc_layer_desc* desc, const void* q_lat, const int32_t* ctx_len, int32_t b,
                                         int32_t max_ctx, const void* packed, const void* cache,
                                         const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                                         void* workspace, size_t workspace_bytes, void* stream, void* ev_split_begin,
                                         void* ev_split_end) {
  if (int rc = decode_args(desc, q_lat, nullptr, false, ctx_len, b, max_ctx, packed, cache, block_table, max_pages, n_pages, out,
                           workspace))
    return rc;
  int n_cus = 0;
  if (int rc = device_ready(&n_cus)) return rc;
  const DecodePlan plan = make_absorbed_plan(*desc, b, max_ctx, n_cus);
  DecodeParams p;
  if (int rc = decode_params(p, desc, q_lat, nullptr, false, ctx_len, b, max_ctx, packed, cache, block_table, max_pages,
                             n_pages, out, workspace, workspace_bytes, plan, 0))
    return rc;
  return launch_decode_absorbed(p, plan, static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(ev_split_begin),
                                static_cast<hipEvent_t>(ev_split_end));
}

int lorc_decode_attention_absorbed(const lorc_layer_desc* desc, const void* q_lat, const int32_t* ctx_len, int32_t b,
                                   int32_t max_ctx, const void* packed, const void* cache, const int32_t* block_table,
                                   int32_t max_pages, int32_t n_pages, void* out, void* workspace, size_t workspace_bytes,
                                   void* stream) {
  return lorc_decode_attention_absorbed_timed(desc, q_lat, ctx_len, b, max_ctx, packed, cache, block_table, max_pages,
                                              n_pages, out, workspace, workspace_bytes, stream, nullptr, nullptr);
}

size_t lorc_prefill_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_seqlen) {
  if (!desc || check_desc(*desc) != LORC_OK || b <= 0 || max_seqlen < 0) return 0;
  return make_prefill_plan(*desc, b, max_seqlen).total_bytes;
}

namespace {
int prefill_common(const lorc_layer_desc* desc, const void* q, const int32_t* cu_seqlens, int32_t b,
                   int32_t total_tokens, int32_t max_seqlen, const void* packed, const void* cache,
                   const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                   void* workspace, size_t workspace_bytes, void* stream, bool plain) {
  if (!desc || !q || !cu_seqlens || !packed || !cache || !block_table || !out || !workspace) return LORC_EINVAL;
  if (int rc = check_desc(*desc)) return rc;
  if (b <= 0 || total_tokens < 0 || max_seqlen < 0 || max_seqlen > total_tokens || max_pages <= 0 || n_pages <= 0)
    return LORC_EINVAL;
  if ((long)max_pages * kPage < max_seqlen) return LORC_EINVAL;
  if (!aligned16(q) || !aligned16(packed) || !aligned16(cache) || !aligned16(out)) return LORC_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return LORC_EINVAL;
  if (plain && !plain_shape_ok(*desc)) return LORC_EUNSUPPORTED;
  if (total_tokens == 0) return LORC_OK;
  const PrefillPlan plan = make_prefill_plan(*desc, b, max_seqlen);
  const int n = desc->n_kv_heads * desc->head_dim;
  // the attention kernel addresses one sequence's rebuilt keys with 32-bit byte offsets
  if ((size_t)plan.lp * n * 2 > 0x7fffffffu) return LORC_EUNSUPPORTED;
  if (workspace_bytes < plan.total_bytes) return LORC_EWORKSPACE;
  if (int rc = device_ready(nullptr)) return rc;
  const uint16_t* pk = static_cast<const uint16_t*>(packed);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  PrefillParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.cu_seqlens = cu_seqlens;
  p.bk = pk + packed_off_bk(desc->d_model, desc->rank_k, desc->rank_v);
  p.bv = pk + packed_off_bv(desc->d_model, desc->rank_k, desc->rank_v, n);
  p.cache = static_cast<const uint16_t*>(cache);
  p.block_table = block_table;
  p.out = static_cast<uint16_t*>(out);
  p.rope_tab = reinterpret_cast<const double*>(pk + packed_off_rope(desc->d_model, desc->rank_k, desc->rank_v, n));
  p.krot = reinterpret_cast<uint16_t*>(ws + plan.off_krot);
  p.vt = reinterpret_cast<uint16_t*>(ws + plan.off_vt);
  p.b = b;
  p.h_q = desc->n_q_heads;
  p.h_kv = desc->n_kv_heads;
  p.G = desc->n_q_heads / desc->n_kv_heads;
  p.head_dim = desc->head_dim;
  p.r_k = desc->rank_k;
  p.r_v = desc->rank_v;
  p.max_pages = max_pages;
  p.n_pages = n_pages;
  p.tiles_per_seq = plan.tiles_per_seq;
  p.lp = plan.lp;
  p.page_elems = page_elems(desc->rank_k, desc->rank_v);
  p.rope_base = desc->rope_base;
  p.q_scale = softmax_scale_log2(*desc);
  return launch_prefill(p, static_cast<hipStream_t>(stream), plain);
}
}  // namespace

int lorc_prefill_attention(const lorc_layer_desc* desc, const void* q, const int32_t* cu_seqlens, int32_t b,
                           int32_t total_tokens, int32_t max_seqlen, const void* packed, const void* cache,
                           const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                           void* workspace, size_t workspace_bytes, void* stream) {
  return prefill_common(desc, q, cu_seqlens, b, total_tokens, max_seqlen, packed, cache, block_table, max_pages, n_pages, out,
                        workspace, workspace_bytes, stream, false);
}

int lorc_prefill_attention_plain(const lorc_layer_desc* desc, const void* q, const int32_t* cu_seqlens, int32_t b,
                                 int32_t total_tokens, int32_t max_seqlen, const void* packed, const void* cache,
                                 const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  return prefill_common(desc, q, cu_seqlens, b, total_tokens, max_seqlen, packed, cache, block_table, max_pages, n_pages, out,
                        workspace, workspace_bytes, stream, true);
}

int lorc_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes == 0 || (bytes & 15) || !aligned16(src)) return LORC_EINVAL;
  return launch_stream_probe(src, bytes, sink, static_cast<hipStream_t>(stream));
}

int lorc_mfma_rate_probe(float* sink, size_t sink_floats, int32_t workgroups, int32_t iters, int32_t operands, void* stream) {
  if (!sink || workgroups <= 0 || workgroups > 65536 || iters <= 0 || iters > (1 << 24) || operands < 0 || operands > 2) return LORC_EINVAL;
  if (sink_floats < (size_t)workgroups * 256) return LORC_EINVAL;
  return launch_mfma_probe(sink, workgroups, iters, operands, static_cast<hipStream_t>(stream));
}

}  // extern "C"
