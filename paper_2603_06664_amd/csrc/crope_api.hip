// Host side of the C ABI: argument validation and kernel launches.  No allocation, no
// synchronisation, no state except a thread-local error string.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <climits>
#include "crope_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool stride_ok(int64_t s) { return s > 0 && (s % 8) == 0; }  // bf16: 8 elements = 16 bytes

int check_desc(const crope_table_desc* d) {
  if (!d) return fail(CROPE_EINVAL, "table descriptor is null");
  if (d->head_dim != crope::kHeadDim)
    return fail(CROPE_ESHAPE, "head_dim must be 128, got %d", d->head_dim);
  if (d->dim_t < 0 || d->dim_h < 0 || d->dim_w < 0 || (d->dim_t | d->dim_h | d->dim_w) & 1)
    return fail(CROPE_ESHAPE, "axis widths must be even and non-negative (%d,%d,%d)", d->dim_t,
                d->dim_h, d->dim_w);
  if (d->dim_t + d->dim_h + d->dim_w != d->head_dim)
    return fail(CROPE_ESHAPE, "axis widths %d+%d+%d do not sum to head_dim %d", d->dim_t,
                d->dim_h, d->dim_w, d->head_dim);
  if (d->max_t <= 0 || d->max_h <= 0 || d->max_w <= 0)
    return fail(CROPE_EINVAL, "table extents must be positive (%d,%d,%d)", d->max_t, d->max_h,
                d->max_w);
  if (d->max_t > (1 << 20) || d->max_h > (1 << 20) || d->max_w > (1 << 20))
    return fail(CROPE_ERANGE, "table extents above 2^20 positions are not supported");
  if (!(d->theta > 0.0)) return fail(CROPE_EINVAL, "theta must be positive");
  return CROPE_OK;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(CROPE_EHIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char* crope_last_error(void) { return g_err; }
const char* crope_version(void) { return "crope 0.1 (gfx950)"; }

size_t crope_table_bytes(const crope_table_desc* desc) {
  if (check_desc(desc) != CROPE_OK) return 0;
  return (size_t)crope::table_layout(*desc).total_floats * sizeof(float);
}

int crope_build_table(const crope_table_desc* desc, float* d_table, size_t bytes, void* stream) {
  if (int rc = check_desc(desc)) return rc;
  if (!d_table) return fail(CROPE_EINVAL, "d_table is null");
  if (!aligned16(d_table)) return fail(CROPE_EALIGN, "d_table is not 16-byte aligned");
  const size_t need = (size_t)crope::table_layout(*desc).total_floats * sizeof(float);
  if (bytes < need)
    return fail(CROPE_EWORKSPACE, "table buffer has %zu bytes, needs %zu", bytes, need);
  hipError_t e = crope::launch_build_table(*desc, d_table, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "crope_build_table launch");
  g_err[0] = 0;
  return CROPE_OK;
}

}  // extern "C"
#pragma GCC visibility pop

namespace {
int append_impl(
    const crope_table_desc* desc, const float* d_table, const void* q, const void* k,
    const void* v, crope_strides in, const float* gain_q, const float* gain_k, float eps,
    int32_t norm_group, int32_t n_tokens, int32_t n_heads, int32_t grid_h, int32_t grid_w,
    int32_t start_frame, int32_t token_offset, float q_scale, void* q_out, crope_strides q_out_strides,
    void* k_cache, void* v_cache, crope_strides cache_strides, int64_t cache_capacity_tokens,
    int64_t dst_token, void* stream) {
  if (int rc = check_desc(desc)) return rc;
  if (!(q_scale > 0.0f) || !(q_scale < 1e30f)) return fail(CROPE_EINVAL, "q_scale must be positive and finite");
  if (!d_table || !q || !k || !v || !gain_q || !gain_k || !q_out || !k_cache || !v_cache)
    return fail(CROPE_EINVAL, "null pointer argument");
  if (n_tokens < 0) return fail(CROPE_EINVAL, "n_tokens is negative");
  if (n_tokens > 4 * 65535) return fail(CROPE_ERANGE, "more than 262140 tokens in one call");
  if (n_heads <= 0) return fail(CROPE_EINVAL, "n_heads must be positive");
  if (n_heads > crope::rope_max_heads())
    return fail(CROPE_ESHAPE, "n_heads %d exceeds the supported maximum %d", n_heads,
                crope::rope_max_heads());
  if (grid_h <= 0 || grid_w <= 0) return fail(CROPE_EINVAL, "grid sizes must be positive");
  if ((int64_t)grid_h * grid_w > INT32_MAX)
    return fail(CROPE_ERANGE, "grid_h * grid_w exceeds 2^31-1 tokens per frame");
  if (start_frame < 0 || token_offset < 0)
    return fail(CROPE_EINVAL, "start_frame and token_offset must be non-negative");
  if ((int64_t)token_offset + n_tokens > INT32_MAX)
    return fail(CROPE_ERANGE, "token_offset + n_tokens exceeds 2^31-1");
  if (!(eps >= 0.0f)) return fail(CROPE_EINVAL, "eps must be non-negative");
  const int64_t hd = (int64_t)n_heads * crope::kHeadDim;
  if (norm_group != hd && norm_group != crope::kHeadDim)
    return fail(CROPE_EINVAL, "norm_group must be n_heads*128 (%lld) or 128, got %d",
                (long long)hd, norm_group);
  if (!aligned16(d_table) || !aligned16(q) || !aligned16(k) || !aligned16(v) ||
      !aligned16(gain_q) || !aligned16(gain_k) || !aligned16(q_out) || !aligned16(k_cache) ||
      !aligned16(v_cache))
    return fail(CROPE_EALIGN, "every base pointer must be 16-byte aligned");
  if (!stride_ok(in.token) || !stride_ok(in.head) || !stride_ok(q_out_strides.token) ||
      !stride_ok(q_out_strides.head) || !stride_ok(cache_strides.token) ||
      !stride_ok(cache_strides.head))
    return fail(CROPE_EALIGN, "strides must be positive multiples of 8 elements");
  if (in.head < crope::kHeadDim || q_out_strides.head < crope::kHeadDim ||
      cache_strides.head < crope::kHeadDim)
    return fail(CROPE_EINVAL, "head stride smaller than head_dim");
  // the kernel addresses a row's chunks with 32-bit byte offsets: 63 * stride * 2 + 256 < 2^32
  if (in.head > (1 << 24) || q_out_strides.head > (1 << 24) || cache_strides.head > (1 << 24))
    return fail(CROPE_ERANGE, "head stride above 2^24 elements");
  if (grid_h > desc->max_h || grid_w > desc->max_w)
    return fail(CROPE_ERANGE, "grid %dx%d exceeds table extents %dx%d", grid_h, grid_w,
                desc->max_h, desc->max_w);
  if (cache_capacity_tokens <= 0) return fail(CROPE_EINVAL, "cache capacity must be positive");
  if (dst_token < 0 || dst_token + n_tokens > cache_capacity_tokens)
    return fail(CROPE_ERANGE, "cache rows [%lld, %lld) exceed capacity %lld", (long long)dst_token,
                (long long)(dst_token + n_tokens), (long long)cache_capacity_tokens);
  if (n_tokens == 0) { g_err[0] = 0; return CROPE_OK; }
  const int64_t hw = (int64_t)grid_h * grid_w;
  const int64_t last_frame = start_frame + ((int64_t)token_offset + n_tokens - 1) / hw;
  if (last_frame >= desc->max_t)
    return fail(CROPE_ERANGE, "global frame %lld reaches beyond the time table (max_t %d)",
                (long long)last_frame, desc->max_t);

  crope::RopeArgs a;
  a.table = d_table; a.tl = crope::table_layout(*desc);
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.in_tok = in.token; a.in_head = in.head;
  a.gain_q = gain_q; a.gain_k = gain_k; a.eps = eps;
  a.per_head_norm = (norm_group == crope::kHeadDim && n_heads > 1) ? 1 : 0;
  a.q_scale = q_scale;
  a.n_tokens = n_tokens; a.n_heads = n_heads; a.grid_h = grid_h; a.grid_w = grid_w;
  a.start_frame = start_frame; a.token_offset = token_offset;
  a.div_hw = crope::make_fastdiv((uint32_t)hw); a.div_w = crope::make_fastdiv((uint32_t)grid_w);
  a.q_out = (uint16_t*)q_out; a.qo_tok = q_out_strides.token; a.qo_head = q_out_strides.head;
  a.k_cache = (uint16_t*)k_cache; a.v_cache = (uint16_t*)v_cache;
  a.c_tok = cache_strides.token; a.c_head = cache_strides.head;
  a.dst_token = dst_token;
  hipError_t e = crope::launch_rope(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "crope_qk_norm_rotate_append launch");
  g_err[0] = 0;
  return CROPE_OK;
}
}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int crope_qk_norm_rotate_append(
    const crope_table_desc* desc, const float* d_table, const void* q, const void* k,
    const void* v, crope_strides in, const float* gain_q, const float* gain_k, float eps,
    int32_t norm_group, int32_t n_tokens, int32_t n_heads, int32_t grid_h, int32_t grid_w,
    int32_t start_frame, int32_t token_offset, void* q_out, crope_strides q_out_strides,
    void* k_cache, void* v_cache, crope_strides cache_strides, int64_t cache_capacity_tokens,
    int64_t dst_token, void* stream) {
  return append_impl(desc, d_table, q, k, v, in, gain_q, gain_k, eps, norm_group, n_tokens, n_heads, grid_h,
                     grid_w, start_frame, token_offset, 1.0f, q_out, q_out_strides, k_cache, v_cache,
                     cache_strides, cache_capacity_tokens, dst_token, stream);
}

int crope_qk_norm_rotate_append_qscaled(
    const crope_table_desc* desc, const float* d_table, const void* q, const void* k,
    const void* v, crope_strides in, const float* gain_q, const float* gain_k, float eps,
    int32_t norm_group, int32_t n_tokens, int32_t n_heads, int32_t grid_h, int32_t grid_w,
    int32_t start_frame, int32_t token_offset, float q_scale, void* q_out, crope_strides q_out_strides,
    void* k_cache, void* v_cache, crope_strides cache_strides, int64_t cache_capacity_tokens,
    int64_t dst_token, void* stream) {
  return append_impl(desc, d_table, q, k, v, in, gain_q, gain_k, eps, norm_group, n_tokens, n_heads, grid_h,
                     grid_w, start_frame, token_offset, q_scale, q_out, q_out_strides, k_cache, v_cache,
                     cache_strides, cache_capacity_tokens, dst_token, stream);
}

float crope_folded_q_scale(float softmax_scale) { return softmax_scale * 1.44269504088896340736f; }

size_t chunk_attention_workspace_bytes(int32_t n_q, int32_t n_heads, int64_t n_keys) {
  if (n_q <= 0 || n_heads <= 0 || n_keys <= 0) return 0;
  return crope::attention_workspace_bytes(n_q, n_heads, n_keys, crope::AttnPlan{0, 0});
}

}  // extern "C"
#pragma GCC visibility pop

namespace {
// 0 = ok and *want filled (zeros when plan is null)
int check_plan(const crope_attention_plan* plan, crope::AttnPlan* want) {
  *want = crope::AttnPlan{0, 0};
  if (!plan) return CROPE_OK;
  if (plan->waves != 0 && plan->waves != 4 && plan->waves != 8)
    return fail(CROPE_EINVAL, "plan.waves must be 0, 4 or 8, got %d", plan->waves);
  if (plan->splits < 0 || plan->splits > 16)
    return fail(CROPE_EINVAL, "plan.splits must be 0..16, got %d", plan->splits);
  *want = crope::AttnPlan{plan->waves, plan->splits};
  return CROPE_OK;
}

int attention_impl(const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
                   const void* k_cache, const void* v_cache, crope_strides cache_strides,
                   int64_t cache_capacity_tokens, const crope_kv_segment* segs, int32_t n_segs,
                   float scale, const int32_t* q_limit, bool limited, const crope_attention_plan* plan,
                   void* out, crope_strides out_strides,
                   float* lse_or_null, void* workspace, size_t workspace_bytes, void* stream) {
  crope::AttnPlan want;
  if (int rc = check_plan(plan, &want)) return rc;
  if (limited && !q_limit) return fail(CROPE_EINVAL, "q_limit is null");
  if (limited && ((uintptr_t)q_limit & 3)) return fail(CROPE_EALIGN, "q_limit is not 4-byte aligned");
  if (!q || !k_cache || !v_cache || !out || !segs)
    return fail(CROPE_EINVAL, "null pointer argument");
  if (n_q < 0) return fail(CROPE_EINVAL, "n_q is negative");
  if (n_heads <= 0 || n_heads > 65535) return fail(CROPE_EINVAL, "n_heads out of range");
  if (n_segs < 1 || n_segs > crope::kMaxSegments)
    return fail(CROPE_EINVAL, "n_segs must be 1..%d, got %d", crope::kMaxSegments, n_segs);
  // scale == CROPE_SCALE_FOLDED (0): the queries already carry scale*log2(e)
  if (!(scale >= 0.0f) || !(scale < 1e30f)) return fail(CROPE_EINVAL, "scale must be positive and finite, or CROPE_SCALE_FOLDED");
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
      (workspace && !aligned16(workspace)) || (lse_or_null && ((uintptr_t)lse_or_null & 3)))
    return fail(CROPE_EALIGN, "every base pointer must be 16-byte aligned (lse: 4)");
  if (!stride_ok(q_strides.token) || !stride_ok(q_strides.head) ||
      !stride_ok(cache_strides.token) || !stride_ok(cache_strides.head) ||
      !stride_ok(out_strides.token) || !stride_ok(out_strides.head))
    return fail(CROPE_EALIGN, "strides must be positive multiples of 8 elements");
  if (q_strides.head < crope::kHeadDim || out_strides.head < crope::kHeadDim ||
      cache_strides.head < crope::kHeadDim)
    return fail(CROPE_EINVAL, "head stride smaller than head_dim");
  if (cache_capacity_tokens <= 0) return fail(CROPE_EINVAL, "cache capacity must be positive");
  if (cache_capacity_tokens > INT32_MAX) return fail(CROPE_ERANGE, "cache capacity above 2^31-1 rows");
  if (cache_strides.token > (1 << 24)) return fail(CROPE_ERANGE, "cache token stride above 2^24 elements");
  crope::AttnArgs a;
  a.segs.n = n_segs;
  int64_t n_keys = 0;
  for (int i = 0; i < crope::kMaxSegments; ++i) { a.segs.end[i] = INT32_MAX; a.segs.base[i] = 0; }
  for (int i = 0; i < n_segs; ++i) {
    if (segs[i].len <= 0) return fail(CROPE_EINVAL, "segment %d has non-positive length", i);
    if (segs[i].start < 0 || segs[i].start + segs[i].len > cache_capacity_tokens)
      return fail(CROPE_ERANGE, "segment %d [%lld, %lld) lies outside the cache (capacity %lld)", i,
                  (long long)segs[i].start, (long long)(segs[i].start + segs[i].len),
                  (long long)cache_capacity_tokens);
    if (n_keys + segs[i].len > ((int64_t)1 << 30)) return fail(CROPE_ERANGE, "more than 2^30 visible keys");
    a.segs.base[i] = (int32_t)(segs[i].start - n_keys);
    n_keys += segs[i].len;
    a.segs.end[i] = (int32_t)n_keys;
  }
  for (int i = n_segs; i < crope::kMaxSegments; ++i) a.segs.base[i] = a.segs.base[n_segs - 1];
  const size_t need = limited ? 0 : crope::attention_workspace_bytes(n_q > 0 ? n_q : 1, n_heads, n_keys, want);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(CROPE_EWORKSPACE, "workspace has %zu bytes, needs %zu", workspace ? workspace_bytes : 0,
                need);
  if (n_q == 0) { g_err[0] = 0; return CROPE_OK; }
  a.q = (const uint16_t*)q; a.q_tok = q_strides.token; a.q_head = q_strides.head;
  a.n_q = n_q; a.n_heads = n_heads;
  a.q_limit = limited ? q_limit : nullptr;
  a.k_cache = (const uint16_t*)k_cache; a.v_cache = (const uint16_t*)v_cache;
  a.c_tok = cache_strides.token; a.c_head = cache_strides.head;
  a.n_keys = n_keys; a.folded = scale == 0.0f ? 1 : 0; a.scale = a.folded ? 1.0f : scale;
  a.out = (uint16_t*)out; a.o_tok = out_strides.token; a.o_head = out_strides.head;
  a.lse = lse_or_null; a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  hipError_t e = crope::launch_attention(a, want, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "chunk_attention launch");
  g_err[0] = 0;
  return CROPE_OK;
}
}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int chunk_attention(const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
                    const void* k_cache, const void* v_cache, crope_strides cache_strides,
                    int64_t cache_capacity_tokens, const crope_kv_segment* segs, int32_t n_segs,
                    float scale, void* out, crope_strides out_strides, float* lse_or_null,
                    void* workspace, size_t workspace_bytes, void* stream) {
  return attention_impl(q, q_strides, n_q, n_heads, k_cache, v_cache, cache_strides, cache_capacity_tokens,
                        segs, n_segs, scale, nullptr, false, nullptr, out, out_strides, lse_or_null, workspace,
                        workspace_bytes, stream);
}

int chunk_attention_choose_plan(int32_t n_q, int32_t n_heads, int64_t n_keys, crope_attention_plan* plan) {
  if (!plan) return fail(CROPE_EINVAL, "plan is null");
  if (n_q <= 0 || n_heads <= 0 || n_keys <= 0) return fail(CROPE_EINVAL, "sizes must be positive");
  crope::AttnPlan want;
  if (int rc = check_plan(plan, &want)) return rc;
  const crope::AttnPlan p = crope::attention_plan(n_q, n_heads, n_keys, want);
  plan->waves = p.waves;
  plan->splits = p.splits;
  g_err[0] = 0;
  return CROPE_OK;
}

size_t chunk_attention_planned_workspace_bytes(int32_t n_q, int32_t n_heads, int64_t n_keys,
                                               const crope_attention_plan* plan) {
  if (n_q <= 0 || n_heads <= 0 || n_keys <= 0) return 0;
  crope::AttnPlan want;
  if (check_plan(plan, &want) != CROPE_OK) return 0;
  return crope::attention_workspace_bytes(n_q, n_heads, n_keys, want);
}

int chunk_attention_planned(const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
                            const void* k_cache, const void* v_cache, crope_strides cache_strides,
                            int64_t cache_capacity_tokens, const crope_kv_segment* segs, int32_t n_segs,
                            float scale, const crope_attention_plan* plan, void* out,
                            crope_strides out_strides, float* lse_or_null, void* workspace,
                            size_t workspace_bytes, void* stream) {
  return attention_impl(q, q_strides, n_q, n_heads, k_cache, v_cache, cache_strides, cache_capacity_tokens,
                        segs, n_segs, scale, nullptr, false, plan, out, out_strides, lse_or_null, workspace,
                        workspace_bytes, stream);
}

}  // extern "C"
#pragma GCC visibility pop

namespace {
// Scratch of chunk_attention_static: the partial results of a split key range.  Every GPU the
// library runs on holds its own copy of this array, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)CROPE_STATIC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, once resolved

// Device address of the current GPU's copy of `scratch` (the array's name itself is only a
// host-side handle, never a pointer a kernel may use).  Resolved once per device.
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(CROPE_ERANGE, "device index %d out of range", dev);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p) return fail(CROPE_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // every thread resolves the same address
  }
  *out = p;
  return CROPE_OK;
}
}  // namespace

#pragma GCC visibility push(default)
extern "C" {

size_t chunk_attention_static_capacity(void) { return kStaticScratchBytes; }

int chunk_attention_static(const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
                           const void* k_cache, const void* v_cache, crope_strides cache_strides,
                           int64_t cache_capacity_tokens, const crope_kv_segment* segs, int32_t n_segs,
                           float scale, void* out, crope_strides out_strides, float* lse_or_null,
                           void* stream) {
  // the size check comes first: a problem too large for the static buffer touches no GPU state
  if (n_q > 0 && n_heads > 0 && segs && n_segs >= 1 && n_segs <= crope::kMaxSegments) {
    int64_t n_keys = 0;
    for (int i = 0; i < n_segs; ++i) n_keys += segs[i].len > 0 ? segs[i].len : 0;
    if (n_keys > 0 && n_keys <= ((int64_t)1 << 30)) {
      const size_t need = crope::attention_workspace_bytes(n_q, n_heads, n_keys, crope::AttnPlan{0, 0});
      if (need > kStaticScratchBytes)
        return fail(CROPE_EWORKSPACE,
                    "chunk_attention_static: this problem needs %zu bytes of scratch, the built-in "
                    "buffer holds %zu; use chunk_attention with a caller-provided workspace",
                    need, kStaticScratchBytes);
    }
  }
  void* ws = nullptr;
  if (int rc = static_scratch(&ws)) return rc;
  return attention_impl(q, q_strides, n_q, n_heads, k_cache, v_cache, cache_strides, cache_capacity_tokens,
                        segs, n_segs, scale, nullptr, false, nullptr, out, out_strides, lse_or_null, ws,
                        kStaticScratchBytes, stream);
}

int chunk_attention_limited(const void* q, crope_strides q_strides, int32_t n_q, int32_t n_heads,
                            const void* k_cache, const void* v_cache, crope_strides cache_strides,
                            int64_t cache_capacity_tokens, const crope_kv_segment* segs, int32_t n_segs,
                            float scale, const int32_t* q_limit, void* out, crope_strides out_strides,
                            float* lse_or_null, void* stream) {
  return attention_impl(q, q_strides, n_q, n_heads, k_cache, v_cache, cache_strides, cache_capacity_tokens,
                        segs, n_segs, scale, q_limit, true, nullptr, out, out_strides, lse_or_null, nullptr, 0,
                        stream);
}

size_t crope_qkv_project_workspace_bytes(int32_t n_tokens, int32_t n_heads, int32_t norm_group) {
  if (n_tokens <= 0 || n_heads <= 0) return 0;
  return crope::project_workspace_bytes(n_tokens, n_heads, norm_group == crope::kHeadDim);
}

int crope_qkv_project_norm_rotate_append(
    const crope_table_desc* desc, const float* d_table, const void* x, int64_t x_token_stride,
    const void* w_qkv, const float* bias_or_null, int32_t c_in, const float* gain_q,
    const float* gain_k, float eps, int32_t norm_group, int32_t n_tokens, int32_t n_heads,
    int32_t grid_h, int32_t grid_w, int32_t start_frame, int32_t token_offset, void* q_out,
    crope_strides q_out_strides, void* k_cache, void* v_cache, crope_strides cache_strides,
    int64_t cache_capacity_tokens, int64_t dst_token, void* workspace, size_t workspace_bytes,
    void* stream) {
  if (int rc = check_desc(desc)) return rc;
  if (!d_table || !x || !w_qkv || !gain_q || !gain_k || !q_out || !k_cache || !v_cache)
    return fail(CROPE_EINVAL, "null pointer argument");
  if (n_tokens < 0) return fail(CROPE_EINVAL, "n_tokens is negative");
  if (n_tokens > 4 * 65535) return fail(CROPE_ERANGE, "more than 262140 tokens in one call");
  if (n_heads <= 0) return fail(CROPE_EINVAL, "n_heads must be positive");
  if (n_heads > crope::rope_max_heads())
    return fail(CROPE_ESHAPE, "n_heads %d exceeds the supported maximum %d", n_heads,
                crope::rope_max_heads());
  if (c_in <= 0 || c_in % 64 != 0)
    return fail(CROPE_ESHAPE, "c_in must be a positive multiple of 64, got %d", c_in);
  if (c_in > (1 << 20)) return fail(CROPE_ERANGE, "c_in above 2^20");
  if (grid_h <= 0 || grid_w <= 0) return fail(CROPE_EINVAL, "grid sizes must be positive");
  if ((int64_t)grid_h * grid_w > INT32_MAX)
    return fail(CROPE_ERANGE, "grid_h * grid_w exceeds 2^31-1 tokens per frame");
  if (start_frame < 0 || token_offset < 0)
    return fail(CROPE_EINVAL, "start_frame and token_offset must be non-negative");
  if ((int64_t)token_offset + n_tokens > INT32_MAX)
    return fail(CROPE_ERANGE, "token_offset + n_tokens exceeds 2^31-1");
  if (!(eps >= 0.0f)) return fail(CROPE_EINVAL, "eps must be non-negative");
  const int64_t hd = (int64_t)n_heads * crope::kHeadDim;
  if (norm_group != hd && norm_group != crope::kHeadDim)
    return fail(CROPE_EINVAL, "norm_group must be n_heads*128 (%lld) or 128, got %d",
                (long long)hd, norm_group);
  if (!aligned16(d_table) || !aligned16(x) || !aligned16(w_qkv) || !aligned16(gain_q) ||
      !aligned16(gain_k) || !aligned16(q_out) || !aligned16(k_cache) || !aligned16(v_cache) ||
      (bias_or_null && !aligned16(bias_or_null)) || (workspace && !aligned16(workspace)))
    return fail(CROPE_EALIGN, "every base pointer must be 16-byte aligned");
  if (!stride_ok(x_token_stride) || !stride_ok(q_out_strides.token) || !stride_ok(q_out_strides.head) ||
      !stride_ok(cache_strides.token) || !stride_ok(cache_strides.head))
    return fail(CROPE_EALIGN, "strides must be positive multiples of 8 elements");
  if (x_token_stride < c_in) return fail(CROPE_EINVAL, "x_token_stride smaller than c_in");
  // the kernel forms (row in tile) * stride * 2 bytes in 32 bits, rows up to 255
  if (x_token_stride > (1 << 22)) return fail(CROPE_ERANGE, "x_token_stride above 2^22 elements");
  if (q_out_strides.head < crope::kHeadDim || cache_strides.head < crope::kHeadDim)
    return fail(CROPE_EINVAL, "head stride smaller than head_dim");
  if (grid_h > desc->max_h || grid_w > desc->max_w)
    return fail(CROPE_ERANGE, "grid %dx%d exceeds table extents %dx%d", grid_h, grid_w,
                desc->max_h, desc->max_w);
  if (cache_capacity_tokens <= 0) return fail(CROPE_EINVAL, "cache capacity must be positive");
  if (dst_token < 0 || dst_token + n_tokens > cache_capacity_tokens)
    return fail(CROPE_ERANGE, "cache rows [%lld, %lld) exceed capacity %lld", (long long)dst_token,
                (long long)(dst_token + n_tokens), (long long)cache_capacity_tokens);
  if (n_tokens == 0) { g_err[0] = 0; return CROPE_OK; }
  const int64_t hw = (int64_t)grid_h * grid_w;
  const int64_t last_frame = start_frame + ((int64_t)token_offset + n_tokens - 1) / hw;
  if (last_frame >= desc->max_t)
    return fail(CROPE_ERANGE, "global frame %lld reaches beyond the time table (max_t %d)",
                (long long)last_frame, desc->max_t);
  const bool per_head = norm_group == crope::kHeadDim;
  const size_t need = crope::project_workspace_bytes(n_tokens, n_heads, per_head);
  if (need > 0 && (!workspace || workspace_bytes < need))
    return fail(CROPE_EWORKSPACE, "workspace has %zu bytes, needs %zu", workspace ? workspace_bytes : 0,
                need);

  crope::ProjArgs a;
  a.table = d_table; a.tl = crope::table_layout(*desc);
  a.x = (const uint16_t*)x; a.x_tok = x_token_stride;
  a.w = (const uint16_t*)w_qkv; a.c_in = c_in; a.bias = bias_or_null;
  a.gain_q = gain_q; a.gain_k = gain_k; a.eps = eps;
  a.per_head_norm = per_head ? 1 : 0;
  a.n_tokens = n_tokens; a.n_heads = n_heads; a.grid_h = grid_h; a.grid_w = grid_w;
  a.start_frame = start_frame; a.token_offset = token_offset;
  a.q_out = (uint16_t*)q_out; a.qo_tok = q_out_strides.token; a.qo_head = q_out_strides.head;
  a.k_cache = (uint16_t*)k_cache; a.v_cache = (uint16_t*)v_cache;
  a.c_tok = cache_strides.token; a.c_head = cache_strides.head;
  a.dst_token = dst_token;
  a.sumsq = (float*)workspace;
  a.resid = nullptr;
  hipError_t e = crope::launch_project(a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "crope_qkv_project_norm_rotate_append launch");
  g_err[0] = 0;
  return CROPE_OK;
}

}  // extern "C"
#pragma GCC visibility pop
