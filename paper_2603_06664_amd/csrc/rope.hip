// Rotary table build and the fused qk-RMSNorm + causal 3D RoPE + KV-cache update kernel.
//
// The fused kernel is bandwidth-bound: per token it reads q, k, v (3 * H*128 bf16) and
// writes rotated q, rotated k, v (another 3 * H*128 bf16).  One 64-lane wave owns one token
// of one of the three tensors;
// every lane moves 16-byte pieces (8 channels of one head), so a wave's requests cover
// whole contiguous 1 KB spans.  Statistics are fp32, reduced across the wave with
// cross-lane shuffles; nothing is staged through LDS.  Calls with few tokens of many heads use
// a variant with four waves per token row (rope_split_kernel below).
#include "crope_internal.h"

namespace crope {
namespace {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);  // v_cvt_pk_bf16_f32, round-nearest-even
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// ---------------------------------------------------------------- table build
// One thread per (axis, position, pair).  The angle pos * theta^(-2j/dim) is formed in
// fp64 (an fp32 product would already be off by ~1e-4 rad at pos ~ 1000) and rounded once.
__global__ void build_table_kernel(float* __restrict__ table, TableLayout tl, int dim_t, int dim_h,
                                   int dim_w, double theta) {
  const int64_t n_t = (int64_t)tl.max_t * tl.pairs_t;
  const int64_t n_h = (int64_t)tl.max_h * tl.pairs_h;
  const int64_t n_w = (int64_t)tl.max_w * tl.pairs_w;
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_t + n_h + n_w) return;
  int pairs, dim;
  int64_t off;
  if (idx < n_t) { pairs = tl.pairs_t; dim = dim_t; off = tl.off_t; }
  else if (idx < n_t + n_h) { idx -= n_t; pairs = tl.pairs_h; dim = dim_h; off = tl.off_h; }
  else { idx -= n_t + n_h; pairs = tl.pairs_w; dim = dim_w; off = tl.off_w; }
  const int pos = (int)(idx / pairs);
  const int j = (int)(idx % pairs);
  const double omega = pow(theta, -2.0 * (double)j / (double)dim);
  const double phi = (double)pos * omega;
  double s, c;
  sincos(phi, &s, &c);
  float2 cs = make_float2((float)c, (float)s);
  reinterpret_cast<float2*>(table + off)[idx] = cs;
}

// ---------------------------------------------------------------- fused kernel
constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}
__device__ __forceinline__ float group16_sum(float x) {
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}

// ITERS = ceil(n_heads / 4): lane l owns 16-byte chunk c = l + 64*it of the token's H*16
// chunks; chunk c is head c/16, channels 8*(c%16)..+7, and c%16 == l%16 for every it, so a
// lane's four rotation angles are the same for all of its chunks.
//
// blockIdx.x selects the tensor a work-group handles (0: q, 1: k, 2: v; fastest-varying, so
// the three streams of a token block are dispatched together).  Splitting the
// three tensors over different waves triples the number of independent load/store streams in
// flight and lets one wave's stores overlap another's loads; v is a plain copy.
template <int ITERS>
__global__ __launch_bounds__(64 * kWavesPerBlock) void rope_kernel(RopeArgs a) {
  const int lane = threadIdx.x & 63;
  const int tok = blockIdx.y * kWavesPerBlock + (threadIdx.x >> 6);
  if (tok >= a.n_tokens) return;
  const int n_chunks = a.n_heads * 16;
  const int role = blockIdx.x;
  const uint16_t* src = role == 0 ? a.q : role == 1 ? a.k : a.v;
  const int64_t in_base = (int64_t)tok * a.in_tok;
  const int64_t c_base = (a.dst_token + tok) * a.c_tok;

  // issue all loads first
  uint4 rx[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int c = lane + 64 * it;
    if (c < n_chunks)
      rx[it] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(
                                             src + in_base + (int64_t)(c >> 4) * a.in_head + (c & 15) * 8)));
    else
      rx[it] = make_uint4(0, 0, 0, 0);
  }

  if (role == 2) {   // v goes to the cache untouched
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int c = lane + 64 * it;
      if (c < n_chunks)
        *reinterpret_cast<uint4*>(a.v_cache + c_base + (int64_t)(c >> 4) * a.c_head + (c & 15) * 8) = rx[it];
    }
    return;
  }

  // global position of this token (index decode with the global time index)
  const int hw = a.grid_h * a.grid_w;
  const int ig = a.token_offset + tok;
  const int f = ig / hw;
  const int r = ig - f * hw;
  const int ph = r / a.grid_w;
  const int pw = r - ph * a.grid_w;
  const int pt = a.start_frame + f;

  // the lane's four (cos, sin) pairs: pair index j = 4*(lane%16) + p
  float cs[4], sn[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int j = 4 * (lane & 15) + p;
    const float* tsrc;
    if (j < a.tl.pairs_t) tsrc = a.table + a.tl.off_t + ((int64_t)pt * a.tl.pairs_t + j) * 2;
    else if (j < a.tl.pairs_t + a.tl.pairs_h)
      tsrc = a.table + a.tl.off_h + ((int64_t)ph * a.tl.pairs_h + (j - a.tl.pairs_t)) * 2;
    else
      tsrc = a.table + a.tl.off_w + ((int64_t)pw * a.tl.pairs_w + (j - a.tl.pairs_t - a.tl.pairs_h)) * 2;
    const float2 t = *reinterpret_cast<const float2*>(tsrc);
    cs[p] = t.x; sn[p] = t.y;
  }

  // sums of squares
  float ss[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const uint32_t* u = reinterpret_cast<const uint32_t*>(&rx[it]);
    float sq = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x0 = bf16_lo(u[e]), x1 = bf16_hi(u[e]);
      sq = fmaf(x0, x0, sq); sq = fmaf(x1, x1, sq);
    }
    ss[it] = sq;
  }
  float r_scale[ITERS];
  if (a.per_head_norm) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it)
      r_scale[it] = 1.0f / sqrtf(group16_sum(ss[it]) * (1.0f / kHeadDim) + a.eps);
  } else {
    float t = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) t += ss[it];
    t = wave_sum(t);
    const float sc = 1.0f / sqrtf(t * (1.0f / (float)(a.n_heads * kHeadDim)) + a.eps);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) r_scale[it] = sc;
  }

  // normalise, apply gain, rotate, round once to bf16, store
  const float* gain = role == 0 ? a.gain_q : a.gain_k;
  uint16_t* dst = role == 0 ? a.q_out + (int64_t)tok * a.qo_tok : a.k_cache + c_base;
  const int64_t dst_head = role == 0 ? a.qo_head : a.c_head;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int c = lane + 64 * it;
    if (c >= n_chunks) continue;
    const int head = c >> 4, d0 = (c & 15) * 8;
    const float4 g0 = *reinterpret_cast<const float4*>(gain + head * kHeadDim + d0);
    const float4 g1 = *reinterpret_cast<const float4*>(gain + head * kHeadDim + d0 + 4);
    const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    const uint32_t* u = reinterpret_cast<const uint32_t*>(&rx[it]);
    uint32_t o[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const float xa = bf16_lo(u[p]) * r_scale[it] * gg[2 * p];
      const float xb = bf16_hi(u[p]) * r_scale[it] * gg[2 * p + 1];
      o[p] = pack_bf16x2(xa * cs[p] - xb * sn[p], xa * sn[p] + xb * cs[p]);
    }
    *reinterpret_cast<uint4*>(dst + (int64_t)head * dst_head + d0) = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

// Few tokens with many heads (a sequence-parallel rank's share of a wide model): one wave per
// (tensor, token) leaves most of the chip idle and makes every wave's load -> compute -> store
// chain long.  Here the four waves of a work-group share one token row, each taking a
// contiguous quarter of its heads (whole heads, so the lane -> channel mapping and with it the
// lane's four rotation angles are as above); the row-wide sum of squares goes through LDS.
template <int ITERS>   // ITERS = ceil(heads per wave / 4)
__global__ __launch_bounds__(64 * kWavesPerBlock) void rope_split_kernel(RopeArgs a, int heads_per_wave) {
  __shared__ float part[kWavesPerBlock];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int tok = blockIdx.y;
  const int role = blockIdx.x;
  const int c_begin = wave * heads_per_wave * 16;
  const int c_end = min(a.n_heads, (wave + 1) * heads_per_wave) * 16;   // may be <= c_begin: idle wave
  const uint16_t* src = role == 0 ? a.q : role == 1 ? a.k : a.v;
  const int64_t in_base = (int64_t)tok * a.in_tok;
  const int64_t c_base = (a.dst_token + tok) * a.c_tok;

  uint4 rx[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int c = c_begin + lane + 64 * it;
    if (c < c_end)
      rx[it] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(
                                             src + in_base + (int64_t)(c >> 4) * a.in_head + (c & 15) * 8)));
    else
      rx[it] = make_uint4(0, 0, 0, 0);
  }
  if (role == 2) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int c = c_begin + lane + 64 * it;
      if (c < c_end)
        *reinterpret_cast<uint4*>(a.v_cache + c_base + (int64_t)(c >> 4) * a.c_head + (c & 15) * 8) = rx[it];
    }
    return;   // the whole work-group has role 2: nobody waits at the barrier below
  }
  const int hw = a.grid_h * a.grid_w;
  const int ig = a.token_offset + tok;
  const int f = ig / hw;
  const int r = ig - f * hw;
  const int ph = r / a.grid_w;
  const int pw = r - ph * a.grid_w;
  const int pt = a.start_frame + f;
  float cs[4], sn[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int j = 4 * (lane & 15) + p;
    const float* tsrc;
    if (j < a.tl.pairs_t) tsrc = a.table + a.tl.off_t + ((int64_t)pt * a.tl.pairs_t + j) * 2;
    else if (j < a.tl.pairs_t + a.tl.pairs_h)
      tsrc = a.table + a.tl.off_h + ((int64_t)ph * a.tl.pairs_h + (j - a.tl.pairs_t)) * 2;
    else
      tsrc = a.table + a.tl.off_w + ((int64_t)pw * a.tl.pairs_w + (j - a.tl.pairs_t - a.tl.pairs_h)) * 2;
    const float2 t = *reinterpret_cast<const float2*>(tsrc);
    cs[p] = t.x; sn[p] = t.y;
  }
  float ss[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const uint32_t* u = reinterpret_cast<const uint32_t*>(&rx[it]);
    float sq = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x0 = bf16_lo(u[e]), x1 = bf16_hi(u[e]);
      sq = fmaf(x0, x0, sq); sq = fmaf(x1, x1, sq);
    }
    ss[it] = sq;
  }
  float r_scale[ITERS];
  if (a.per_head_norm) {
#pragma unroll
    for (int it = 0; it < ITERS; ++it)
      r_scale[it] = 1.0f / sqrtf(group16_sum(ss[it]) * (1.0f / kHeadDim) + a.eps);
  } else {
    float t = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) t += ss[it];
    t = wave_sum(t);
    if (lane == 0) part[wave] = t;
    __syncthreads();
    t = (part[0] + part[1]) + (part[2] + part[3]);   // fixed order
    const float sc = 1.0f / sqrtf(t * (1.0f / (float)(a.n_heads * kHeadDim)) + a.eps);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) r_scale[it] = sc;
  }
  const float* gain = role == 0 ? a.gain_q : a.gain_k;
  uint16_t* dst = role == 0 ? a.q_out + (int64_t)tok * a.qo_tok : a.k_cache + c_base;
  const int64_t dst_head = role == 0 ? a.qo_head : a.c_head;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int c = c_begin + lane + 64 * it;
    if (c >= c_end) continue;
    const int head = c >> 4, d0 = (c & 15) * 8;
    const float4 g0 = *reinterpret_cast<const float4*>(gain + head * kHeadDim + d0);
    const float4 g1 = *reinterpret_cast<const float4*>(gain + head * kHeadDim + d0 + 4);
    const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    const uint32_t* u = reinterpret_cast<const uint32_t*>(&rx[it]);
    uint32_t o[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const float xa = bf16_lo(u[p]) * r_scale[it] * gg[2 * p];
      const float xb = bf16_hi(u[p]) * r_scale[it] * gg[2 * p + 1];
      o[p] = pack_bf16x2(xa * cs[p] - xb * sn[p], xa * sn[p] + xb * cs[p]);
    }
    *reinterpret_cast<uint4*>(dst + (int64_t)head * dst_head + d0) = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

template <int ITERS>
hipError_t launch_rope_split_t(const RopeArgs& a, int heads_per_wave, hipStream_t st) {
  hipLaunchKernelGGL(rope_split_kernel<ITERS>, dim3(3, a.n_tokens), dim3(64 * kWavesPerBlock), 0, st, a,
                     heads_per_wave);
  return hipGetLastError();
}

template <int ITERS>
hipError_t launch_rope_t(const RopeArgs& a, hipStream_t st) {
  const int blocks = (a.n_tokens + kWavesPerBlock - 1) / kWavesPerBlock;
  hipLaunchKernelGGL(rope_kernel<ITERS>, dim3(3, blocks), dim3(64 * kWavesPerBlock), 0, st, a);
  return hipGetLastError();
}

}  // namespace

int rope_max_heads() { return 64; }

hipError_t launch_build_table(const crope_table_desc& d, float* table, hipStream_t st) {
  const TableLayout tl = table_layout(d);
  const int64_t n = tl.total_floats / 2;
  const int threads = 256;
  const int blocks = (int)((n + threads - 1) / threads);
  hipLaunchKernelGGL(build_table_kernel, dim3(blocks), dim3(threads), 0, st, table, tl, d.dim_t,
                     d.dim_h, d.dim_w, d.theta);
  return hipGetLastError();
}

hipError_t launch_rope(const RopeArgs& a, hipStream_t st) {
  // few token rows of a wide model: four waves per row (grid.y = tokens <= 65535)
  if (a.n_heads >= 16 && a.n_tokens <= 2048) {
    const int hpw = (a.n_heads + kWavesPerBlock - 1) / kWavesPerBlock;   // 4 .. 16 heads per wave
    const int it = (hpw + 3) / 4;
    if (it <= 1) return launch_rope_split_t<1>(a, hpw, st);
    if (it <= 2) return launch_rope_split_t<2>(a, hpw, st);
    if (it <= 3) return launch_rope_split_t<3>(a, hpw, st);
    return launch_rope_split_t<4>(a, hpw, st);
  }
  const int iters = (a.n_heads + 3) / 4;
  if (iters <= 1) return launch_rope_t<1>(a, st);
  if (iters <= 2) return launch_rope_t<2>(a, st);
  if (iters <= 3) return launch_rope_t<3>(a, st);
  if (iters <= 4) return launch_rope_t<4>(a, st);
  if (iters <= 6) return launch_rope_t<6>(a, st);
  if (iters <= 8) return launch_rope_t<8>(a, st);
  if (iters <= 10) return launch_rope_t<10>(a, st);
  if (iters <= 12) return launch_rope_t<12>(a, st);
  return launch_rope_t<16>(a, st);
}

}  // namespace crope
