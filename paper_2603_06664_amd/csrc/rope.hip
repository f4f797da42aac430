// Rotary table build and the fused qk-RMSNorm + causal 3D RoPE + KV-cache update kernel.
//
// The fused kernel is bandwidth-bound: per token it reads q, k, v (3 * H*128 bf16) and
// writes rotated q, rotated k, v (another 3 * H*128 bf16).  One 64-lane wave owns one to three
// token rows of one of the three tensors; every lane moves 16-byte pieces (8 channels of one
// head), so a wave's requests cover whole contiguous 1 KB spans, and all of a wave's loads are
// issued before anything else.  Statistics are fp32, reduced across the wave with DPP adds and
// the row-swapping permutes (no LDS traffic); the gains are staged once per work-group in LDS;
// everything that depends on the token only is computed on the scalar unit.  Calls with few
// tokens of many heads use four waves per token row.
#include "crope_internal.h"

namespace crope {
namespace {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

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
constexpr int kMaxHeads = 64;

// Cross-lane sums without LDS traffic: DPP adds inside a row of 16 lanes (after the four steps
// every lane of the row holds the row's total), then the row-swapping permutes between rows.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float group16_sum(float x) {
  x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]: lane ^ 1
  x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]: lane ^ 2
  x = dpp_add<0x141>(x);   // row_half_mirror: lane -> 7 - lane inside each 8
  x = dpp_add<0x140>(x);   // row_mirror: lane -> 15 - lane inside the row
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
  x = group16_sum(x);
  u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(r[0]) + __uint_as_float(r[1]);   // rows 0+1 and 2+3
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One wave owns the 16-byte chunks c_begin + lane + 64*it (it < ITERS, c < c_end) of a token
// row; chunk c is head c/16, channels 8*(c%16)..+7, and c%16 == lane%16 for every it, so a
// lane's four rotation angles are the same for all of its chunks.
//
// blockIdx.x selects the tensor a work-group handles (0: q, 1: k, 2: v; fastest-varying, so
// the three streams of a token block are dispatched together); v is a plain copy.
//
// SPLIT = false: a wave owns whole rows, TPW consecutive tokens of them.  All its loads are
//   issued before anything else; the gains are fetched once and serve every token.
// SPLIT = true (few tokens of many heads, a sequence-parallel rank's share of a wide model):
//   the four waves of a work-group share ONE token row, a contiguous quarter of its heads
//   each; the row-wide sum of squares crosses the waves through LDS in a fixed order.
//
// Everything that depends only on the token (row addresses, the index decode, table rows) is
// wave-uniform and computed on the scalar unit; per lane there are only 32-bit offsets.
// NT: streaming store (written through instead of left dirty in the L2, which would have to be
// flushed when the kernel ends)
template <bool NT>
__device__ __forceinline__ void store16(uint8_t* p, uint4 v) {
  if (NT) __builtin_nontemporal_store(__builtin_bit_cast(u32x4_t, v), reinterpret_cast<u32x4_t*>(p));
  else *reinterpret_cast<uint4*>(p) = v;
}

template <int ITERS, int TPW, bool SPLIT, bool PER_HEAD, bool NT_ST>
__global__ __launch_bounds__(64 * kWavesPerBlock) __attribute__((amdgpu_waves_per_eu(!SPLIT && ITERS * TPW <= 6 ? 7 : 1, 8)))
void rope_kernel(RopeArgs a, int heads_per_wave) {
  __shared__ float part[kWavesPerBlock];
  extern __shared__ __attribute__((aligned(16))) float gain_lds[];   // n_heads * 128 floats
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int role = blockIdx.x;
  const int by = blockIdx.y;
  int tok0, c_begin, c_end, nt;
  if (SPLIT) {
    tok0 = by;
    c_begin = wave * heads_per_wave * 16;
    c_end = min(a.n_heads, (wave + 1) * heads_per_wave) * 16;   // may be <= c_begin: idle wave
    nt = 1;
  } else {
    tok0 = (by * kWavesPerBlock + wave) * TPW;
    c_begin = 0;
    c_end = a.n_heads * 16;
    nt = max(0, min(TPW, a.n_tokens - tok0));   // 0: a wave past the end, which only takes part in the barrier
  }
  const uint8_t* src = reinterpret_cast<const uint8_t*>(role == 0 ? a.q : role == 1 ? a.k : a.v) +
                       (int64_t)tok0 * a.in_tok * 2;
  uint8_t* dst = role == 0 ? reinterpret_cast<uint8_t*>(a.q_out) + (int64_t)tok0 * a.qo_tok * 2
                           : reinterpret_cast<uint8_t*>(role == 1 ? a.k_cache : a.v_cache) +
                                 (a.dst_token + tok0) * a.c_tok * 2;
  const int64_t src_tok_bytes = a.in_tok * 2;
  const int64_t dst_tok_bytes = (role == 0 ? a.qo_tok : a.c_tok) * 2;
  const uint32_t src_head_bytes = (uint32_t)a.in_head * 2, dst_head_bytes = (uint32_t)(role == 0 ? a.qo_head : a.c_head) * 2;

  bool valid[ITERS];
  uint32_t in_off[ITERS], out_off[ITERS];
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int c = c_begin + lane + 64 * it;
    valid[it] = c < c_end;
    in_off[it] = (uint32_t)(c >> 4) * src_head_bytes + (uint32_t)(c & 15) * 16u;
    out_off[it] = (uint32_t)(c >> 4) * dst_head_bytes + (uint32_t)(c & 15) * 16u;
  }

  // every load of the wave's rows first (non-temporal: the inputs are read once and should not
  // displace what the caches hold for the kernels that follow)
  uint4 rx[TPW][ITERS];
#pragma unroll
  for (int t = 0; t < TPW; ++t)
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      if (t < nt && valid[it])
        rx[t][it] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(
                                                  src + t * src_tok_bytes + in_off[it])));
      else
        rx[t][it] = make_uint4(0, 0, 0, 0);
    }

  if (role == 2) {   // v goes to the cache untouched
#pragma unroll
    for (int t = 0; t < TPW; ++t)
#pragma unroll
      for (int it = 0; it < ITERS; ++it)
        if (t < nt && valid[it]) store16<NT_ST>(dst + t * dst_tok_bytes + out_off[it], rx[t][it]);
    return;   // SPLIT: the whole work-group has role 2, nobody waits at the barrier below
  }

  // gains: staged once per work-group in LDS (every wave of it handles the same tensor), read
  // back per chunk when needed, so that they occupy no registers while the loads are in flight
  {
    const float4* gsrc = reinterpret_cast<const float4*>(role == 0 ? a.gain_q : a.gain_k);
    const int n4 = a.n_heads * (kHeadDim / 4);
    for (int i = threadIdx.x; i < n4; i += 64 * kWavesPerBlock) reinterpret_cast<float4*>(gain_lds)[i] = gsrc[i];
    __syncthreads();
  }

  // the lane's four pairs j = 4*(lane%16) + p: which axis table each one reads
  const int j0 = 4 * (lane & 15);
  bool on_t[4], on_h[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    on_t[p] = j0 + p < a.tl.pairs_t;
    on_h[p] = !on_t[p] && j0 + p < a.tl.pairs_t + a.tl.pairs_h;
  }
  const float2* tab2 = reinterpret_cast<const float2*>(a.table);
  const float inv_group = 1.0f / (float)(PER_HEAD ? kHeadDim : a.n_heads * kHeadDim);
  const float out_scale = role == 0 ? a.q_scale : 1.0f;   // folded into 1/rms: no extra arithmetic per element

#pragma unroll
  for (int t = 0; t < TPW; ++t) {
    if (t >= nt) break;   // wave-uniform
    // global position of this token (index decode with the global time index), scalar unit
    const uint32_t ig = (uint32_t)(a.token_offset + tok0 + t);
    const uint32_t f = fastdiv(ig, a.div_hw);
    const uint32_t r = ig - f * a.div_hw.d;
    const uint32_t ph = fastdiv(r, a.div_w);
    const uint32_t pw = r - ph * a.div_w.d;
    const uint32_t pt = (uint32_t)a.start_frame + f;
    // table entry of pair j on each axis, as if j ran through that axis' row (scalar bases)
    const int bt = (int)(a.tl.off_t / 2) + (int)pt * a.tl.pairs_t;
    const int bh = (int)(a.tl.off_h / 2) + (int)ph * a.tl.pairs_h - a.tl.pairs_t;
    const int bw = (int)(a.tl.off_w / 2) + (int)pw * a.tl.pairs_w - a.tl.pairs_t - a.tl.pairs_h;
    float cs[4], sn[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const float2 e = tab2[(uint32_t)(j0 + p + (on_t[p] ? bt : on_h[p] ? bh : bw))];
      cs[p] = e.x; sn[p] = e.y;
    }

    // sums of squares
    float ss[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const uint32_t* u = reinterpret_cast<const uint32_t*>(&rx[t][it]);
      float sq = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {   // two bf16 squares per instruction, fp32 accumulation
        const bf16x2_t h = __builtin_bit_cast(bf16x2_t, u[e]);
        sq = __builtin_amdgcn_fdot2_f32_bf16(h, h, sq, false);
      }
      ss[it] = sq;
    }
    // 1/rms, folded into the rotation: out = (g*x) * (r*cos, r*sin)
    float row_scale = 0.f;
    if (!PER_HEAD) {
      float tot = 0.f;
#pragma unroll
      for (int it = 0; it < ITERS; ++it) tot += ss[it];
      tot = wave_sum(tot);
      if (SPLIT) {
        if (lane == 0) part[wave] = tot;
        __syncthreads();
        tot = (part[0] + part[1]) + (part[2] + part[3]);   // fixed order
      }
      row_scale = __builtin_amdgcn_rsqf(tot * inv_group + a.eps) * out_scale;
#pragma unroll
      for (int p = 0; p < 4; ++p) { cs[p] *= row_scale; sn[p] *= row_scale; }
    }

    // normalise, apply gain, rotate, round once to bf16, store
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      if (!valid[it]) continue;
      float c_it[4], s_it[4];
      if (PER_HEAD) {
        const float hs = __builtin_amdgcn_rsqf(group16_sum(ss[it]) * inv_group + a.eps) * out_scale;
#pragma unroll
        for (int p = 0; p < 4; ++p) { c_it[p] = cs[p] * hs; s_it[p] = sn[p] * hs; }
      } else {
#pragma unroll
        for (int p = 0; p < 4; ++p) { c_it[p] = cs[p]; s_it[p] = sn[p]; }
      }
      const uint32_t* u = reinterpret_cast<const uint32_t*>(&rx[t][it]);
      const int c = c_begin + lane + 64 * it;
      const float4 g0 = *reinterpret_cast<const float4*>(gain_lds + c * 8);
      const float4 g1 = *reinterpret_cast<const float4*>(gain_lds + c * 8 + 4);
      const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      uint32_t o[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const float xa = bf16_lo(u[p]) * gg[2 * p];
        const float xb = bf16_hi(u[p]) * gg[2 * p + 1];
        o[p] = pack_bf16x2(xa * c_it[p] - xb * s_it[p], xa * s_it[p] + xb * c_it[p]);
      }
      store16<NT_ST>(dst + t * dst_tok_bytes + out_off[it], make_uint4(o[0], o[1], o[2], o[3]));
    }
  }
}

// Outputs up to this size are stored with streaming stores: for a launch of this size the L2
// flush at the end of the kernel costs more than writing through as the kernel runs (C4 shape:
// 15.4 -> 15.0 us; 32-36 MB launches: 8.6 -> 7.1 us).  Larger outputs fit the last-level cache
// better when left to the normal write-back path (960x1664 chunk, 172 MB: 54.7 vs 57.3 us).
constexpr int64_t kStreamStoreMaxBytes = 128 << 20;

template <int ITERS, int TPW, bool SPLIT>
hipError_t launch_rope_t(const RopeArgs& a, int heads_per_wave, hipStream_t st) {
  const size_t lds_bytes = (size_t)a.n_heads * kHeadDim * sizeof(float);
  const int rows = SPLIT ? a.n_tokens : (a.n_tokens + kWavesPerBlock * TPW - 1) / (kWavesPerBlock * TPW);
  const dim3 grid(3, rows), block(64 * kWavesPerBlock);
  const bool nt = (int64_t)a.n_tokens * a.n_heads * kHeadDim * 2 * 3 <= kStreamStoreMaxBytes;
  if (a.per_head_norm) {
    if (nt) hipLaunchKernelGGL((rope_kernel<ITERS, TPW, SPLIT, true, true>), grid, block, lds_bytes, st, a, heads_per_wave);
    else hipLaunchKernelGGL((rope_kernel<ITERS, TPW, SPLIT, true, false>), grid, block, lds_bytes, st, a, heads_per_wave);
  } else {
    if (nt) hipLaunchKernelGGL((rope_kernel<ITERS, TPW, SPLIT, false, true>), grid, block, lds_bytes, st, a, heads_per_wave);
    else hipLaunchKernelGGL((rope_kernel<ITERS, TPW, SPLIT, false, false>), grid, block, lds_bytes, st, a, heads_per_wave);
  }
  return hipGetLastError();
}

template <int TPW>
hipError_t launch_rope_rows(const RopeArgs& a, hipStream_t st) {
  const int iters = (a.n_heads + 3) / 4;
  if (iters <= 1) return launch_rope_t<1, TPW, false>(a, 0, st);
  if (iters <= 2) return launch_rope_t<2, TPW, false>(a, 0, st);
  if (iters <= 3) return launch_rope_t<3, TPW, false>(a, 0, st);
  if (iters <= 4) return launch_rope_t<4, TPW, false>(a, 0, st);
  if (TPW > 1) return hipErrorInvalidValue;   // not instantiated: launch_rope sends wider rows here with TPW = 1
  if (iters <= 6) return launch_rope_t<6, 1, false>(a, 0, st);
  if (iters <= 8) return launch_rope_t<8, 1, false>(a, 0, st);
  if (iters <= 10) return launch_rope_t<10, 1, false>(a, 0, st);
  if (iters <= 12) return launch_rope_t<12, 1, false>(a, 0, st);
  return launch_rope_t<16, 1, false>(a, 0, st);
}

}  // namespace

int rope_max_heads() { return kMaxHeads; }

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
    if (it <= 1) return launch_rope_t<1, 1, true>(a, hpw, st);
    if (it <= 2) return launch_rope_t<2, 1, true>(a, hpw, st);
    if (it <= 3) return launch_rope_t<3, 1, true>(a, hpw, st);
    return launch_rope_t<4, 1, true>(a, hpw, st);
  }
  // Tokens per wave.  A launch is fastest when all of its waves are resident at once (the whole
  // read stream is requested up front and the stores follow as one phase), so rows of up to 16
  // heads are grouped 2 or 3 to a wave as soon as that brings the wave count under six per
  // SIMD; launches too large for that anyway stream with one token per wave.
  if (a.n_heads <= 16) {
    const int64_t resident = 1024 * 6;
    if (3 * (int64_t)a.n_tokens > resident) {
      if (3 * (int64_t)((a.n_tokens + 1) / 2) <= resident) return launch_rope_rows<2>(a, st);
      if (3 * (int64_t)((a.n_tokens + 2) / 3) <= resident) return launch_rope_rows<3>(a, st);
    }
  }
  return launch_rope_rows<1>(a, st);
}

}  // namespace crope
