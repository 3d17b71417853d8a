/*
 * lorc.h -- C ABI of the MI355X (gfx950) library for attention over a KV cache stored as rank-r latents.
 *
 * Method: LoRC (arXiv 2410.03111).  Offline, the key/value projection weights W_k, W_v [D x n], n = h_kv*d,
 * are factored by truncated SVD (Section 4.1, Algorithm 1):  W ~ A B,  A = U_r Sigma_r [D x r],
 * B = V_r^T [r x n].  At run time the latent c = x A of every token is cached instead of its key/value
 * (Section 4.1: the cache shrinks from h*d to d_c per token); a decode step reads the latents back, rebuilds
 * K = C_k B_k per KV head, rotates it (the cache holds un-rotated latents; Appendix "Adjusted Position
 * Embedding"), shares it across the G = h_q/h_kv query heads of its group (Section 4.3), evaluates
 * softmax(q k^T / sqrt(d)) (Eq. 1) and applies the value up-projection B_v after the weighted sum.
 *
 * Conventions
 *   - All device entry points are asynchronous on the HIP stream passed as `void* stream` (a hipStream_t;
 *     NULL = the default stream).  They never allocate, free or synchronise.  Every device pointer is owned
 *     by the caller and must stay valid until the stream has run.
 *   - State: none between calls, except one flag per device.  The first device entry point called with a
 *     device current (normally lorc_pack_factors, the one-time call per layer) raises the LDS limit of the
 *     library's kernels on that device (hipFuncSetAttribute) and remembers that it did.  That first call
 *     cannot be recorded into a HIP graph; every later call on the device only launches kernels and
 *     records the optional events, and can be captured.
 *   - "bf16" = bfloat16 bit patterns (uint16_t).  Arithmetic accumulates in fp32; latents, factors,
 *     queries and outputs are stored as bf16 (round to nearest even).
 *   - Supported magnitudes: rebuilt keys, scaled queries, per-split partial outputs and the prefill's
 *     rebuilt K/V pass through fp16 (largest finite value 65504) inside the kernels.  Inputs whose
 *     rebuilt keys or values exceed about 6e4 in magnitude give inf/NaN outputs; latents of the size that
 *     normalised hidden states produce (O(1) .. O(100)) are far inside the range.
 *   - Return value: LORC_OK (0) or a negative lorc_status; lorc_strerror() gives the text.  Shapes are
 *     validated on the host before anything is launched; LORC_EHIP is the status of this call's own launch.
 *   - Query head h reads KV head h / G.  RoPE pairs coordinate i with i + d/2, theta_i = base^(-2i/d).
 *
 * Latent cache (device, caller-allocated):  a pool of pages, each holding LORC_PAGE_TOKENS = 64
 * consecutive positions of one sequence for one layer; page p starts at byte p * lorc_page_bytes().
 * Sequence s, position t lives in page block_table[s * max_pages + t / 64], slot t % 64.
 * Inside a page the K latents come first, then the V latents, each tiled so that a 64-lane wavefront
 * loads one matrix-core operand as 1 KiB of consecutive memory (element = bf16, index in elements):
 *     K latent j of slot t:  ((t/32 * (r_k/16) + j/16) * 64 + (t%32) + 32*((j%16)/8)) * 8 + j%8
 *     V latent j of slot t:  64*r_k + (((j/32) * 4 + t/16) * 64 + (j%32) + 32*((t%16)/8)) * 8 + t%8
 * (K tiles are contracted over the latent index when K is rebuilt, V tiles over the position when the
 * softmax weights are applied, hence the two different tilings.)  lorc_cache_index_k/v() evaluate these.
 */
#ifndef LORC_H_
#define LORC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LORC_PAGE_TOKENS 64

typedef enum {
  LORC_OK = 0,
  LORC_EINVAL = -1,       /* NULL pointer, non-positive size, inconsistent shape                        */
  LORC_EUNSUPPORTED = -2, /* head_dim / rank / page size that no kernel is built for                    */
  LORC_ENOCONV = -3,      /* the SVD iteration did not converge                                          */
  LORC_EWORKSPACE = -4,   /* workspace_bytes smaller than lorc_*_workspace_bytes()                       */
  LORC_EHIP = -5          /* the HIP runtime reported an error at launch                                 */
} lorc_status;

/* Geometry of one attention layer (Table 3 of the paper lists the shapes of the evaluated models). */
typedef struct {
  int32_t d_model;       /* D                                                                            */
  int32_t n_q_heads;     /* h_q, multiple of n_kv_heads                                                  */
  int32_t n_kv_heads;    /* h_kv; n = n_kv_heads * head_dim must be a multiple of 64                     */
  int32_t head_dim;      /* d: 64 or 128                                                                 */
  int32_t rank_k;        /* r_k = d_c of the key latent:  multiple of 32, 32 <= r_k <= min(n, 8192)      */
  int32_t rank_v;        /* r_v = d_c of the value latent: multiple of 32, 32 <= r_v <= min(n, 8192)     */
  float rope_base;       /* e.g. 10000 or 500000                                                         */
  float softmax_scale;   /* 0 selects 1/sqrt(head_dim) (Eq. 1)                                           */
  int32_t page_size;     /* must equal LORC_PAGE_TOKENS                                                  */
} lorc_layer_desc;

const char* lorc_strerror(int code);

/* ---------------------------------------------------------------------------------------------- offline
 * Truncated SVD of one weight matrix (Section 4.1; Algorithm 1, key/value compression steps).  HOST
 * pointers, synchronous, fp64, multi-threaded.
 *   W      [rows x cols] row-major, rows >= cols (rows = D, cols = n)
 *   A      [rows x rank] row-major = U_r Sigma_r      (down-projection, applied when a token is cached)
 *   B      [rank x cols] row-major = V_r^T            (up-projection, orthonormal rows, applied at read)
 *   sigma  [cols] all singular values, descending     (may be NULL)
 *   rel_frob_err  ||W - A B||_F / ||W||_F (Appendix B) (may be NULL)
 * Signs are normalised so that the entry of largest magnitude in every row of B is positive.
 * Errors: LORC_EINVAL (NULL, rank outside [1, cols], rows < cols), LORC_ENOCONV.
 */
int lorc_factorize(const double* W, int32_t rows, int32_t cols, int32_t rank, double* A, double* B,
                   double* sigma, double* rel_frob_err);

/* Progressive per-layer ranks (Section 4.2: Eq. 10, Eq. 12, Eq. (dc); Algorithm 1, first two loops).  HOST.
 *   sigma_k, sigma_v [n_layers x n_sigma] singular values per layer (as returned by lorc_factorize)
 *   d_max, d_min     largest / smallest allowed compressed dimension
 *   align            ranks are rounded to the nearest multiple of align (ties up) and clamped to [d_min,d_max]
 *   log_threshold    layers whose log cumulative condition number exceeds it are left uncompressed
 *                    (rank = n_sigma); pass a non-finite or <= 0 value to disable
 *   ranks            [n_layers] output
 */
int lorc_rank_schedule(const double* sigma_k, const double* sigma_v, int32_t n_layers, int32_t n_sigma,
                       int32_t d_max, int32_t d_min, int32_t align, double log_threshold, int32_t* ranks);

/* Error diagnostics (Section 5, Theorems 1 and 3).  HOST.  For an L-layer chain x_i = phi(W_i x_{i-1}) with an
 * L_phi-Lipschitz phi and layer i truncated to rank k_i,
 *   terms[i] = sigma^{(i)}_{k_i+1} * L_phi^(L-1-i) * prod_{j>i} sigma^{(j)}_1,   bound = sum_i terms[i]
 * (the bound on the output error for layer inputs of norm at most 1; one layer: Theorem 1's constant).
 *   sigma   [n_layers x n_sigma] singular values per layer, decreasing (as returned by lorc_factorize)
 *   ranks   [n_layers], 0 <= rank <= n_sigma (rank = n_sigma: the layer contributes nothing)
 *   terms   [n_layers] output, may be NULL;  bound: scalar output
 * The per-layer relative Frobenius error of Appendix B is lorc_factorize's rel_frob_err. */
int lorc_error_bound(const double* sigma, const int32_t* ranks, int32_t n_layers, int32_t n_sigma, double lipschitz,
                     double* terms, double* bound);

/* ---------------------------------------------------------------------------------------------- packing
 * One-time re-tiling of a layer's bf16 factors into the operand order the kernels read (DEVICE pointers):
 *   A_k [D x r_k], A_v [D x r_v], B_k [r_k x n], B_v [r_v x n]  row-major bf16 (the caller rounds the
 *   fp64 factors of lorc_factorize to bf16 and uploads them)
 *   packed: lorc_packed_bytes(desc) bytes, 256-byte aligned; opaque to the caller, valid for this desc only.
 * Uncompressed layer (one that Algorithm 1's threshold on the cumulative condition number leaves alone,
 * Section 6.2): desc has rank_k = rank_v = n, A_k = W_k and A_v = W_v [D x n], and B_k = B_v = NULL -- the
 * read-side factors are the identity and are neither stored nor multiplied.  lorc_append_latent then caches the
 * un-rotated keys and the values themselves in the page tiling above, and lorc_decode_attention_plain reads them.
 * NULL for only one of B_k, B_v, or with ranks below n, is LORC_EINVAL.
 */
size_t lorc_packed_bytes(const lorc_layer_desc* desc);
int lorc_pack_factors(const lorc_layer_desc* desc, const void* A_k, const void* A_v, const void* B_k,
                      const void* B_v, void* packed, void* stream);

/* ---------------------------------------------------------------------------------------------- cache
 * Bytes per page, and the element (bf16) index inside a page of latent j of slot t (host helpers; see the
 * formulas at the top of this file).  Return 0 / -1 for an invalid desc or out-of-range argument. */
size_t lorc_page_bytes(const lorc_layer_desc* desc);
int64_t lorc_cache_index_k(const lorc_layer_desc* desc, int32_t slot, int32_t j);
int64_t lorc_cache_index_v(const lorc_layer_desc* desc, int32_t slot, int32_t j);

/* Cache write (Section 4.1: the compressed key/value  x A  is what is stored).  DEVICE pointers.
 *   x           [T x D] bf16 row-major hidden states of the T new tokens
 *   packed      from lorc_pack_factors
 *   slot_seq    [T] int32 sequence index of each token;  slot_pos [T] int32 position inside that sequence
 *   block_table [n_seqs x max_pages] int32 page ids;  n_pages = pages in the pool (ids are validated on
 *               the device: a token whose page id or position is out of range is skipped, nothing is
 *               written for it)
 *   cache       page pool, n_pages * lorc_page_bytes(desc) bytes
 * Writes exactly the (r_k + r_v) bf16 latents of each token; every other byte of the pool is untouched.
 */
int lorc_append_latent(const lorc_layer_desc* desc, const void* x, int32_t T, const void* packed,
                       const int32_t* slot_seq, const int32_t* slot_pos, const int32_t* block_table,
                       int32_t n_seqs, int32_t max_pages, int32_t n_pages, void* cache, void* stream);

/* Decode attention (Eq. 1 over the cached latents; Section 4.3; Appendix on RoPE).  DEVICE pointers.
 *   q        [b x h_q x d] bf16, un-rotated;  q_pos [b] int32 position of the query token
 *   ctx_len  [b] int32: sequence s attends to its cached positions 0 .. ctx_len[s]-1 (the caller appends
 *            the new token first, so normally q_pos = ctx_len-1);  0 gives an all-zero output row
 *   max_ctx  host copy of max(ctx_len), used to size the launch (ctx_len[s] > max_ctx is clamped; 0 is legal)
 *   block_table, max_pages, n_pages  as for lorc_append_latent; page ids are validated on the device: a page
 *            inside ctx_len whose id is negative or >= n_pages is not read, its positions count as zero
 *            latents (key 0, value 0)
 *   out      [b x h_q x d] bf16
 *   workspace  lorc_decode_workspace_bytes(desc, b, max_ctx) bytes, 256-byte aligned (split partials)
 */
size_t lorc_decode_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx);
/* The launch that lorc_decode_attention would make for (desc, b, max_ctx) on the current device: returns the name
 * of the split kernel (a static string, the symbol a profiler shows; NULL for an invalid or unsupported desc) and,
 * where the pointers are not NULL, the number of context splits per sequence and of 64-position tiles per split.
 * HOST call; touches no device memory.  For benchmarks and profiles that must name the kernel they time. */
const char* lorc_decode_plan_info(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx, int32_t* n_splits,
                                  int32_t* tiles_per_split);
int lorc_decode_attention(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                          const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                          const void* cache, const int32_t* block_table, int32_t max_pages, int32_t n_pages,
                          void* out, void* workspace, size_t workspace_bytes, void* stream);

/* Which shapes lorc_decode_attention takes.  Single-pass kernels: head_dim 64 or 128, ranks <= 1024, G <= 32,
 * h_q <= 64.  Ranks up to 2048 (Table 2's LLaMA-2-13B row: 40 MHA heads, n = 5120 -> 2048) run as three launches
 * (scores with the rank walked in parts, softmax weights x value latents in column chunks, merge): head_dim 128,
 * G <= 8, h_q <= 64; the workspace then also holds the fp32 scores [b x h_q x max_ctx].  Anything else:
 * lorc_decode_workspace_bytes returns 0 and the call LORC_EUNSUPPORTED.
 *
 * Decode attention over an uncompressed layer (packed with B_k = B_v = NULL; rank_k = rank_v = n; head_dim 128,
 * h_q <= 64): same arguments, conventions and result as lorc_decode_attention, without the rebuild and without the
 * value up-projection -- the pages hold keys (rotated as they are read) and values. */
size_t lorc_decode_plain_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx);
int lorc_decode_attention_plain(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                const void* cache, const int32_t* block_table, int32_t max_pages, int32_t n_pages,
                                void* out, void* workspace, size_t workspace_bytes, void* stream);

/* lorc_decode_attention for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, serving loops and harnesses that forbid hipMalloc): same arguments, result and kernels, but the split
 * partials live in a fixed array of LORC_STATIC_WORKSPACE_BYTES inside the library's device code, one copy per GPU,
 * held until the process ends.  The call allocates nothing.
 *   - LORC_EWORKSPACE when lorc_decode_workspace_bytes(desc, b, max_ctx) exceeds LORC_STATIC_WORKSPACE_BYTES.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels overlap in time (different streams
 *     without an ordering between them) race; calls on one stream, or ordered by events, are safe.  Nothing in the
 *     array has to be cleared between calls: every split writes all of its partials before the merge reads them.
 *   - The device address of the array is looked up once per device by the first device entry point called with
 *     that device current (see "State" above). */
#define LORC_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
int lorc_decode_attention_static(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                 const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                 const void* cache, const int32_t* block_table, int32_t max_pages, int32_t n_pages,
                                 void* out, void* stream);

/* Measurement aid: lorc_decode_attention that also records two caller-created HIP events (hipEvent_t passed
 * as void*, either may be NULL) on `stream` immediately before and after the split kernel, the launch that
 * streams the latent cache and dominates the call. */
int lorc_decode_attention_timed(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                const void* cache, const int32_t* block_table, int32_t max_pages,
                                int32_t n_pages, void* out, void* workspace, size_t workspace_bytes,
                                void* stream, void* ev_split_begin, void* ev_split_end);

/* Decode attention that stops in latent space (Section 4.1, Eq. 9: the value up-projection can be absorbed into
 * the output weights, W_o' = U^T W_o in the paper's notation).  Same arguments and workspace as
 * lorc_decode_attention, but the result is the normalised weighted sum of the cached value latents,
 *   out_latent [b x h_q x r_v] bf16,  out_latent[s][h] = sum_j p_j^h c_v[j]   (softmax weights p of Eq. 1),
 * so that  out_latent[s][h] B_v^{g(h)}  equals the output of lorc_decode_attention up to rounding.  The caller
 * multiplies by B_v, or by a matrix that has B_v folded in. */
int lorc_decode_attention_latent(const lorc_layer_desc* desc, const void* q, const int32_t* q_pos,
                                 const int32_t* ctx_len, int32_t b, int32_t max_ctx, const void* packed,
                                 const void* cache, const int32_t* block_table, int32_t max_pages,
                                 int32_t n_pages, void* out_latent, void* workspace, size_t workspace_bytes,
                                 void* stream);

/* Decode attention for a model WITHOUT positional rotation between query and key, with the key factor folded
 * into the query (Section 4.1, Eq. 7: q . (c B_k^g) = (B_k^g q) . c): scores are taken directly on the cached K
 * latents, nothing is rebuilt, and the step is a single stream over the cache.  DEVICE pointers.
 *   q_lat       [b x h_q x r_k] bf16, q_lat[s][h] = B_k^{g(h)} q[s][h] (the caller folds B_k into its query
 *               projection); the softmax scale of desc is applied here, desc.rope_base is ignored
 *   ctx_len, max_ctx, packed, cache, block_table, max_pages, n_pages, out: as lorc_decode_attention
 *   workspace   lorc_decode_absorbed_workspace_bytes(desc, b, max_ctx) bytes, 256-byte aligned
 * h_q <= 32 and ranks <= 512 run as one streaming kernel + merge; h_q <= 64 and ranks up to 8192 (keys) / 2048 (values)
 * as three launches (scores, softmax weights x value latents in column chunks, merge), the workspace then also holding
 * the fp32 scores; anything else LORC_EUNSUPPORTED (workspace size 0).  The _timed variant records the two HIP events
 * (may be NULL) around the streaming kernel(s), on `stream`. */
size_t lorc_decode_absorbed_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_ctx);
int lorc_decode_attention_absorbed(const lorc_layer_desc* desc, const void* q_lat, const int32_t* ctx_len, int32_t b,
                                   int32_t max_ctx, const void* packed, const void* cache,
                                   const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                                   void* workspace, size_t workspace_bytes, void* stream);
int lorc_decode_attention_absorbed_timed(const lorc_layer_desc* desc, const void* q_lat, const int32_t* ctx_len,
                                         int32_t b, int32_t max_ctx, const void* packed, const void* cache,
                                         const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                                         void* workspace, size_t workspace_bytes, void* stream,
                                         void* ev_split_begin, void* ev_split_end);

/* Causal prefill attention over the cached latents (Eq. 1 with mask j <= i).  DEVICE pointers.
 *   q           [total_tokens x h_q x d] bf16, sequences packed back to back, un-rotated
 *   cu_seqlens  [b+1] int32 prefix sums of the sequence lengths (token i of sequence s is at position i;
 *               lorc_append_latent must have cached the whole prompt first)
 *   total_tokens, max_seqlen  host copies of cu_seqlens[b] and of the longest sequence
 *   out         [total_tokens x h_q x d] bf16
 *   workspace   lorc_prefill_workspace_bytes(desc, b, max_seqlen) bytes, 256-byte aligned (rebuilt K/V, fp16)
 * One sequence's rebuilt keys (max_seqlen rounded up to pages x h_kv x d x 2 bytes) must stay below 2 GiB:
 * LORC_EUNSUPPORTED otherwise. */
size_t lorc_prefill_workspace_bytes(const lorc_layer_desc* desc, int32_t b, int32_t max_seqlen);
int lorc_prefill_attention(const lorc_layer_desc* desc, const void* q, const int32_t* cu_seqlens, int32_t b,
                           int32_t total_tokens, int32_t max_seqlen, const void* packed, const void* cache,
                           const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Causal prefill attention over an uncompressed layer (packed with B_k = B_v = NULL; rank_k = rank_v = n; head_dim
 * 128): same arguments, workspace size (lorc_prefill_workspace_bytes) and result as lorc_prefill_attention; the
 * keys and values are gathered from the pages (keys rotated on the way) instead of being rebuilt. */
int lorc_prefill_attention_plain(const lorc_layer_desc* desc, const void* q, const int32_t* cu_seqlens, int32_t b,
                                 int32_t total_tokens, int32_t max_seqlen, const void* packed, const void* cache,
                                 const int32_t* block_table, int32_t max_pages, int32_t n_pages, void* out,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aid: streams `bytes` (multiple of 16) from src with 16-byte loads and folds them into
 * sink[0] (4 bytes); gives the practical HBM read ceiling that the decode roofline is compared with. */
int lorc_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream);

/* Measurement aid: `workgroups` workgroups of four waves, each wave issuing iters x 8 independent 32x32x16 bf16
 * matrix-core products on operands held in registers (no memory traffic in the loop): 4 * workgroups * iters * 8 *
 * 32768 flop per launch.  Timed by the caller, it gives the matrix-core rate the board sustains for that operand
 * data, which the MFMA rooflines are compared with.  operands: 0 = pseudo-random signs and mantissas, 1 = zeros,
 * 2 = ones.  sink (device, sink_floats >= 256 * workgroups floats) receives, per thread, the sum of its 128
 * accumulators: 0 for zeros, 2048 * iters for ones.  LORC_EINVAL for arguments outside these ranges
 * (workgroups 1..65536, iters 1..2^24). */
int lorc_mfma_rate_probe(float* sink, size_t sink_floats, int32_t workgroups, int32_t iters, int32_t operands, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LORC_H_ */
