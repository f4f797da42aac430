// Internal launch interface between the host-side ABI (crope_api.hip) and the kernels.
// Not installed; include/crope.h is the public boundary.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/crope.h"
#include "fastdiv.h"

namespace crope {

constexpr int kHeadDim = 128;
constexpr int kMaxSegments = 4;

struct TableLayout {
  int pairs_t, pairs_h, pairs_w;      // dim_axis / 2
  int max_t, max_h, max_w;
  // offsets in floats from the table base
  int64_t off_t, off_h, off_w, total_floats;
};

inline TableLayout table_layout(const crope_table_desc& d) {
  TableLayout L;
  L.pairs_t = d.dim_t / 2; L.pairs_h = d.dim_h / 2; L.pairs_w = d.dim_w / 2;
  L.max_t = d.max_t; L.max_h = d.max_h; L.max_w = d.max_w;
  L.off_t = 0;
  L.off_h = L.off_t + (int64_t)d.max_t * L.pairs_t * 2;
  L.off_w = L.off_h + (int64_t)d.max_h * L.pairs_h * 2;
  L.total_floats = L.off_w + (int64_t)d.max_w * L.pairs_w * 2;
  return L;
}

struct RopeArgs {
  const float* table; TableLayout tl;
  const uint16_t *q, *k, *v;
  int64_t in_tok, in_head;
  const float *gain_q, *gain_k;
  float eps; int per_head_norm;
  float q_scale;   // factor on the rotated q (1 for the plain call)
  int n_tokens, n_heads, grid_h, grid_w, start_frame, token_offset;
  FastDiv div_hw, div_w;   // division by grid_h*grid_w and by grid_w
  uint16_t* q_out; int64_t qo_tok, qo_head;
  uint16_t *k_cache, *v_cache; int64_t c_tok, c_head;
  int64_t dst_token;
};

// Visible key index vk (0 .. n_keys-1) -> cache row: row = vk + base[i] for the first i with
// vk < end[i].  `end` are cumulative segment ends (unused entries hold INT32_MAX).
struct Segments {
  int n;
  int32_t end[kMaxSegments];
  int32_t base[kMaxSegments];   // cache rows are below 2^31
};

struct AttnArgs {
  const uint16_t* q; int64_t q_tok, q_head;
  int n_q, n_heads;
  const int32_t* q_limit;   // optional: query i sees only the first q_limit[i] visible keys
  const uint16_t *k_cache, *v_cache; int64_t c_tok, c_head;
  Segments segs; int64_t n_keys;
  float scale;
  int folded;   // the queries already carry scale*log2(e): the kernels neither multiply nor need `scale`
  uint16_t* out; int64_t o_tok, o_head;
  float* lse;
  void* workspace; size_t workspace_bytes;
};

struct ProjArgs {
  const float* table; TableLayout tl;
  const uint16_t* x; int64_t x_tok;   // [n_tokens][c_in], token stride in elements
  const uint16_t* w; int c_in;        // [3*H*128][c_in], rows contiguous
  const float* bias;                  // [3*H*128] or null
  const float *gain_q, *gain_k;
  float eps; int per_head_norm;
  int n_tokens, n_heads, grid_h, grid_w, start_frame, token_offset;
  uint16_t* q_out; int64_t qo_tok, qo_head;
  uint16_t *k_cache, *v_cache; int64_t c_tok, c_head;
  int64_t dst_token;
  float* sumsq;                       // [2][n_tokens][H] (row-wide norm only)
  uint16_t* resid;                    // [2][n_tokens][H][128] bf16 low parts (row-wide norm only)
};

hipError_t launch_build_table(const crope_table_desc& d, float* table, hipStream_t st);
hipError_t launch_rope(const RopeArgs& a, hipStream_t st);
int rope_max_heads();
// waves per work-group (4 or 8) and key splits (1..16); 0 = let the library choose
struct AttnPlan { int waves; int splits; };
AttnPlan attention_plan(int n_q, int n_heads, int64_t n_keys, AttnPlan want);
hipError_t launch_attention(const AttnArgs& a, AttnPlan want, hipStream_t st);
size_t attention_workspace_bytes(int n_q, int n_heads, int64_t n_keys, AttnPlan want);
hipError_t launch_project(const ProjArgs& a, hipStream_t st);
size_t project_workspace_bytes(int n_tokens, int n_heads, bool per_head_norm);

}  // namespace crope
