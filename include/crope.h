/*
 * crope.h — C ABI of the per-chunk attention step of causal autoregressive video-DiT
 * inference with Causal-RoPE, for AMD MI355X (gfx950).
 *
 * The operations follow the optimized sequence-parallel self-attention call of the
 * paper (Algorithm 3): step 2/3 (global token offset, causal 3D RoPE computed locally
 * from the global start frame), step 5 (KV-cache update) and step 6 (attention of the
 * chunk's queries over the whole cache).  The local projection (step 1) is available fused
 * with steps 2, 3 and 5 as crope_qkv_project_norm_rotate_append.  The collectives (steps 4, 7)
 * are outside this library.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers to caller-owned memory unless a parameter is
 *     documented as host memory.  The library never allocates, frees or keeps a pointer
 *     after the call's work has been enqueued.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued and the call returns; there is no implicit synchronisation.  Calls issued
 *     back to back on one stream execute in order (append, then attention).
 *   - Return value: CROPE_OK (0) or a negative error code.  On error nothing has been
 *     launched and crope_last_error() returns a thread-local, human-readable message.
 *   - The library keeps no state between calls except that error string: how a call divides
 *     its work depends on its arguments only.
 *   - Activations are bf16, laid out [token][head][128] with the 128 head channels
 *     contiguous; token and head strides are given in elements.
 */
#ifndef CROPE_H
#define CROPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CROPE_OK = 0,
  CROPE_EINVAL = -1,     /* null pointer, non-positive size, bad enum value            */
  CROPE_ESHAPE = -2,     /* head_dim != 128, odd axis width, widths not summing to 128 */
  CROPE_EALIGN = -3,     /* base pointer or stride not 16-byte aligned                 */
  CROPE_ERANGE = -4,     /* position beyond table extent, rows beyond cache capacity   */
  CROPE_EWORKSPACE = -5, /* workspace missing or too small                             */
  CROPE_EHIP = -6        /* the HIP runtime reported a launch error                    */
};

/* Immutable description of the rotary tables (host memory, passed by pointer).
 * Within a head, channel pairs (2j, 2j+1) are rotated; the first dim_t/2 pairs take the
 * temporal angle, the next dim_h/2 the height angle, the last dim_w/2 the width angle
 * (Algorithm 2: concatenation of the time, height and width frequency slices). */
typedef struct {
  int32_t head_dim;            /* must be 128                                          */
  int32_t dim_t, dim_h, dim_w; /* channels per axis: even, sum == head_dim (44/42/42)  */
  double theta;                /* rotary base, 10000                                   */
  int32_t max_t, max_h, max_w; /* table extents: valid positions are 0..max-1          */
} crope_table_desc;

/* Strides of a [token][head][128] bf16 tensor, in elements; channel stride is 1. */
typedef struct {
  int64_t token;
  int64_t head;
} crope_strides;

/* A run of consecutive cache rows (tokens) visible to attention. */
typedef struct {
  int64_t start;
  int64_t len;
} crope_kv_segment;

/* Size in bytes of the table buffer for `desc` (0 if desc is invalid).  Layout: three
 * contiguous fp32 arrays, time [max_t][dim_t/2][2], height [max_h][dim_h/2][2], width
 * [max_w][dim_w/2][2]; innermost pair is (cos, sin) of pos * theta^(-2j/dim_axis). */
size_t crope_table_bytes(const crope_table_desc* desc);

/* Precompute the rotary tables once, into contiguous device memory, so that no host
 * work or cache lookup remains on the per-chunk path (Section 3.4.1 item 2; the per-axis
 * tables are Algorithm 2's freqs[0..2]).  Angles are formed in fp64 on the device and
 * rounded once to fp32.
 *   d_table  device, `bytes` >= crope_table_bytes(desc), 16-byte aligned; overwritten. */
int crope_build_table(const crope_table_desc* desc, float* d_table, size_t bytes,
                      void* stream);

/* Fused qk-RMSNorm + causal 3D RoPE + KV-cache update for one call's local token rows
 * (Algorithm 3 steps 2, 3 and 5; position rule of Section 3.3.3).
 *
 * Row i of the inputs is token i_global = token_offset + i of the current chunk, whose
 * position is t_global = start_frame + i_global / (grid_h*grid_w), h = (i_global mod
 * grid_h*grid_w) / grid_w, w = i_global mod grid_w.  q and k are RMS-normalised (fp32
 * statistics over `norm_group` channels, times a learned gain), rotated, rounded once to
 * bf16; rotated q goes to q_out, rotated k and the untouched v are ASSIGNED to cache rows
 * [dst_token, dst_token + n_tokens) (rewriting rows is how repeated denoising passes and
 * a rolling window work; the caller picks dst_token).
 *
 *   desc, d_table   as built by crope_build_table
 *   q, k, v         device bf16 [n_tokens][n_heads][128], strides `in` (shared by all three)
 *   gain_q, gain_k  device fp32 [n_heads*128]
 *   eps             RMSNorm epsilon
 *   norm_group      n_heads*128 (statistics over the token's whole projection vector)
 *                   or 128 (per head)
 *   grid_h, grid_w  latent token grid of one frame; must be <= max_h, max_w, and
 *                   grid_h * grid_w below 2^31 (CROPE_ERANGE)
 *   start_frame     s, global index of the chunk's first frame
 *   token_offset    Delta = rank * (chunk tokens / ranks); 0 on one GPU;
 *                   token_offset + n_tokens must stay below 2^31 (CROPE_ERANGE)
 *   q_out           device bf16 [n_tokens][n_heads][128], strides q_out_strides
 *   k_cache,v_cache device bf16 [cache_capacity_tokens][n_heads][128], strides cache_strides
 * Errors: CROPE_ERANGE if any row's t_global >= max_t or dst_token + n_tokens exceeds the
 * capacity; CROPE_EALIGN unless every base pointer and stride*2 bytes is a multiple of 16.
 * n_tokens == 0 is a no-op that returns CROPE_OK; at most 262140 tokens and 64 heads per
 * call (CROPE_ERANGE / CROPE_ESHAPE beyond).  Input and output buffers must not overlap,
 * except that q_out may alias q. */
int crope_qk_norm_rotate_append(
    const crope_table_desc* desc, const float* d_table,
    const void* q, const void* k, const void* v, crope_strides in,
    const float* gain_q, const float* gain_k, float eps, int32_t norm_group,
    int32_t n_tokens, int32_t n_heads, int32_t grid_h, int32_t grid_w,
    int32_t start_frame, int32_t token_offset,
    void* q_out, crope_strides q_out_strides,
    void* k_cache, void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens, int64_t dst_token, void* stream);

/* crope_qk_norm_rotate_append whose rotated q is additionally multiplied by q_scale before its
 * single rounding to bf16 (k, v and every other argument and error as above; q_scale must be
 * positive and finite).  With q_scale = crope_folded_q_scale(softmax scale) = scale * log2(e)
 * the attention calls below can be given scale = CROPE_SCALE_FOLDED: the products q.k are then
 * the softmax exponents themselves and the attention kernel has no per-score multiply left
 * (Algorithm 3 steps 3 and 6 share the factor; nothing is rounded twice). */
int crope_qk_norm_rotate_append_qscaled(
    const crope_table_desc* desc, const float* d_table,
    const void* q, const void* k, const void* v, crope_strides in,
    const float* gain_q, const float* gain_k, float eps, int32_t norm_group,
    int32_t n_tokens, int32_t n_heads, int32_t grid_h, int32_t grid_w,
    int32_t start_frame, int32_t token_offset, float q_scale,
    void* q_out, crope_strides q_out_strides,
    void* k_cache, void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens, int64_t dst_token, void* stream);

/* softmax_scale * log2(e), the q_scale that goes with CROPE_SCALE_FOLDED. */
float crope_folded_q_scale(float softmax_scale);

/* Value of `scale` in the attention calls that says: q was written with
 * q_scale = crope_folded_q_scale(softmax scale). */
#define CROPE_SCALE_FOLDED 0.0f

/* Bytes of scratch chunk_attention needs for this problem size (may be 0). */
size_t chunk_attention_workspace_bytes(int32_t n_q, int32_t n_heads, int64_t n_keys);

/* Attention of the chunk's rotated queries over every visible cache row (Algorithm 3
 * step 6): per head and query, softmax(scale * q.K^T) V over the union of `segs`.  There
 * is no element mask: causality comes from what the cache holds (the chunk is the causal
 * block, so its queries see all cached keys and all keys of their own chunk).  bf16 MFMA
 * with fp32 accumulation and fp32 online softmax; probabilities are rounded to bf16 for
 * the second product.
 *
 *   q              device bf16 [n_q][n_heads][128] (already rotated), strides q_strides
 *   k_cache,v_cache device bf16 caches, strides cache_strides
 *   segs           HOST array of n_segs (1..4) row ranges; 2 when a ring cache wraps.
 *                  Ranges must lie inside [0, cache_capacity_tokens) and have len > 0.
 *   scale          softmax scale (1/sqrt(128) for the model this follows), positive and finite;
 *                  or CROPE_SCALE_FOLDED when q already carries scale * log2(e)
 *                  (crope_qk_norm_rotate_append_qscaled), which is the faster path
 *   out            device bf16 [n_q][n_heads][128], strides out_strides
 *   lse_or_null    device fp32 [n_heads][n_q], natural-log sum-exp of the scaled scores
 *   workspace      device scratch of >= chunk_attention_workspace_bytes(...) bytes, 16-byte
 *                  aligned; may be NULL when that size is 0.  Contents are undefined after.
 * n_q == 0 is a no-op.  Limits (CROPE_ERANGE beyond): cache capacity < 2^31 rows, cache token
 * stride <= 2^24 elements, at most 2^30 visible keys.  Head strides below 128 are CROPE_EINVAL. */
int chunk_attention(
    const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
    const void* k_cache, const void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens,
    const crope_kv_segment* segs, int32_t n_segs, float scale,
    void* out, crope_strides out_strides, float* lse_or_null,
    void* workspace, size_t workspace_bytes, void* stream);

/* How chunk_attention divides its work (host memory).  A field that is 0 is chosen by the
 * library from the problem size. */
typedef struct {
  int32_t waves;  /* waves per work-group, 32 queries each: 4 or 8                         */
  int32_t splits; /* 1..16 ranges of the visible keys handled by separate work-groups and
                     merged by a second kernel; lowered until no range is empty            */
} crope_attention_plan;

/* Resolve a plan: on entry the non-zero fields of *plan are kept, on return every field holds
 * the value chunk_attention_planned would use for this problem size (all zeros on entry gives
 * the plan chunk_attention itself uses).  CROPE_EINVAL for a null pointer, non-positive sizes
 * or field values outside the ranges above. */
int chunk_attention_choose_plan(int32_t n_q, int32_t n_heads, int64_t n_keys,
                                crope_attention_plan* plan);

/* Bytes of scratch chunk_attention_planned needs with `plan` (NULL = automatic); 0 also for
 * an invalid plan. */
size_t chunk_attention_planned_workspace_bytes(int32_t n_q, int32_t n_heads, int64_t n_keys,
                                               const crope_attention_plan* plan);

/* chunk_attention (Algorithm 3 step 6) with the work division given by the caller instead of
 * chosen by the library; for tuning and for tests that must reach every kernel shape.  The
 * result differs between plans by rounding only (a split changes the summation order).
 *   plan       host; NULL or all zeros = exactly chunk_attention
 *   workspace  >= chunk_attention_planned_workspace_bytes(n_q, n_heads, total keys, plan)
 * Everything else, and every error, as for chunk_attention; CROPE_EINVAL for a field outside
 * its range. */
int chunk_attention_planned(
    const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
    const void* k_cache, const void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens,
    const crope_kv_segment* segs, int32_t n_segs, float scale,
    const crope_attention_plan* plan,
    void* out, crope_strides out_strides, float* lse_or_null,
    void* workspace, size_t workspace_bytes, void* stream);

/* chunk_attention for callers that cannot allocate device memory or carry a workspace around
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * scratch for the partial results of a split key range is a buffer of
 * CROPE_STATIC_SCRATCH_BYTES built into the library, one copy per GPU, held from the moment the
 * library is loaded on that GPU until the process ends.  The call allocates and frees nothing.
 * Same arguments, same kernels, same work division and bit-identical results as
 * chunk_attention, minus workspace / workspace_bytes.
 *   - CROPE_EWORKSPACE, before anything is launched, if the problem would need more scratch
 *     than the buffer holds (chunk_attention_workspace_bytes(...) > CROPE_STATIC_SCRATCH_BYTES);
 *     the 40-head 585-query x 32760-key rank share needs 58 MiB.
 *   - The first call on a GPU looks the buffer's device address up (a runtime query, no
 *     allocation) and keeps it for later calls; call with that GPU current.  Make that first
 *     call outside any graph capture.
 *   - Every call on a GPU shares that GPU's buffer.  Nothing in it needs clearing between
 *     calls (each partial result is written before it is read), but two calls whose work
 *     overlaps in time on one GPU (different streams) race on it: serialise them. */
#define CROPE_STATIC_SCRATCH_BYTES (64u << 20)
size_t chunk_attention_static_capacity(void);   /* == CROPE_STATIC_SCRATCH_BYTES */
int chunk_attention_static(
    const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
    const void* k_cache, const void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens,
    const crope_kv_segment* segs, int32_t n_segs, float scale,
    void* out, crope_strides out_strides, float* lse_or_null, void* stream);

/* chunk_attention with a per-query prefix limit: query i attends only to the first
 * q_limit[i] rows of the visible set (rows counted in the order of `segs`).  With keys laid
 * out in generation order this is the block-causal rule of the generator itself (Section
 * 3.2: a token attends only to earlier tokens, at the granularity of the generation block of
 * Section 3.3.2) applied inside ONE call: limit = end of the query's own block reproduces,
 * in a single pass over a whole sequence, what chunk-by-chunk generation with the cache
 * computes; limit = i + 1 is token-causal attention.
 *   q_limit   device int32 [n_q]; values are clamped to [1, total visible rows]
 * No workspace is needed.  Everything else is as for chunk_attention. */
int chunk_attention_limited(
    const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
    const void* k_cache, const void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens,
    const crope_kv_segment* segs, int32_t n_segs, float scale,
    const int32_t* q_limit,
    void* out, crope_strides out_strides, float* lse_or_null, void* stream);

/* Bytes of scratch crope_qkv_project_norm_rotate_append needs (0 for norm_group == 128; for the
 * row-wide norm about 512 bytes per token and head). */
size_t crope_qkv_project_workspace_bytes(int32_t n_tokens, int32_t n_heads, int32_t norm_group);

/* Local QKV projection fused with crope_qk_norm_rotate_append (Algorithm 3 steps 1, 2, 3 and
 * 5 in one call; the projection + RoPE operator fusion of Section 3.4.1 item 3).
 *
 * y[i][o] = sum_c x[i][c] * w_qkv[o][c] + bias[o] (bf16 products, fp32 accumulation); columns
 * [0, HD) of y are q, [HD, 2HD) k, [2HD, 3HD) v, HD = n_heads*128, head h = columns
 * h*128..h*128+127 of each.  q and k are then normalised, rotated and stored, and v stored,
 * exactly as crope_qk_norm_rotate_append does, but from the fp32 accumulators: y is never
 * rounded to bf16.  With norm_group == 128 every output is rounded once.  With norm_group ==
 * n_heads*128 the 1/rms factor of a token is only known once all heads are done, so
 * z = rotate(gain*y) is first stored as two bf16 numbers (bf16(z) in the destination row, the
 * bf16 of the remainder in the workspace) and a second pass stores the bf16 rounding of their
 * sum times 1/rms: one rounding of the fp32 value up to 2^-17 relative.
 *
 * Which path is faster (one MI355X, bf16): this call ties with a vendor GEMM followed by
 * crope_qk_norm_rotate_append at 12 heads x 4680 tokens with norm_group == 128 (80 against
 * 79 us) and is the slower one there with the row-wide norm (100 us: the second pass and the
 * workspace round trip), at 40 heads x 585 tokens (125 against 88 us) and at 18720 tokens; it
 * is the faster one where the GEMM is small (5 heads x 4680 tokens: 31 against 45 us; 12 heads
 * x 1728 tokens: 32 against 41 us).  Callers who want the fastest path at the large shapes
 * should use the two-kernel sequence.
 *
 *   x              device bf16 [n_tokens][c_in], row stride x_token_stride elements
 *   w_qkv          device bf16 [3*n_heads*128][c_in], contiguous ([out][in] like a linear layer)
 *   bias_or_null   device fp32 [3*n_heads*128]
 *   c_in           reduction length, a positive multiple of 64
 *   workspace      device, >= crope_qkv_project_workspace_bytes(...) bytes, 16-byte aligned; may
 *                  be NULL when that size is 0.  Contents are undefined afterwards.
 * Everything else, and every error, as for crope_qk_norm_rotate_append; additionally
 * CROPE_ESHAPE if c_in is not a positive multiple of 64, CROPE_ERANGE if c_in exceeds 2^20 or
 * x_token_stride exceeds 2^22, CROPE_EWORKSPACE if the workspace is missing or too small.  x and w_qkv must
 * not overlap any output. */
int crope_qkv_project_norm_rotate_append(
    const crope_table_desc* desc, const float* d_table,
    const void* x, int64_t x_token_stride, const void* w_qkv, const float* bias_or_null,
    int32_t c_in,
    const float* gain_q, const float* gain_k, float eps, int32_t norm_group,
    int32_t n_tokens, int32_t n_heads, int32_t grid_h, int32_t grid_w,
    int32_t start_frame, int32_t token_offset,
    void* q_out, crope_strides q_out_strides,
    void* k_cache, void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens, int64_t dst_token,
    void* workspace, size_t workspace_bytes, void* stream);

/* Thread-local message describing the last error returned on this thread ("" if none). */
const char* crope_last_error(void);

/* Library version string, e.g. "crope 0.1 (gfx950)". */
const char* crope_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CROPE_H */
