// Chunk attention: softmax(scale * q.K^T) V of one chunk's queries over the visible cache
// rows, flash style (online softmax, no score matrix in memory), bf16 MFMA on gfx950.
//
// Operand roles are chosen so that the softmax is lane-local.  Each wave owns 32 queries
// and computes S^T = K . Q^T with v_mfma_f32_32x32x16_bf16: keys are the MFMA rows, queries
// the columns, so accumulator lane l holds 16 keys of ONE query (column l%32) and the row
// max / row sum need a single exchange between lane l and lane l^32.  The same registers,
// rounded to bf16, are then the B operand (P^T) of O^T += V^T . P^T; the key order inside a
// 16-key MFMA step is whatever the accumulator layout gives, and the V^T fragment is
// fetched in that same order with the transposing LDS read (ds_read_b64_tr_b16) from the
// row-major V tile.
//
// A work-group is 4 waves (128 queries of one head); two work-groups share a CU so that one
// wave's softmax (VALU) overlaps the other's MFMAs.  K and V tiles of 64 keys are copied
// HBM -> LDS without passing through registers (global_load_lds, 16 B per lane), double
// buffered, XOR-swizzled by choosing which global chunk each lane fetches.
#include "crope_internal.h"

namespace crope {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ int64_t key_row(const Segments& s, int vk) {
  // visible key index -> cache row, branch-free over at most four segments
  int64_t base = s.base[3];
  base = vk < s.end[2] ? s.base[2] : base;
  base = vk < s.end[1] ? s.base[1] : base;
  base = vk < s.end[0] ? s.base[0] : base;
  return base + vk;
}

// max over both halves of the wave (lane l and lane l^32), result in every lane
__device__ __forceinline__ float max_across_halves(float x) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr int BM = 128;                 // queries per work-group: 4 waves x 32
constexpr int BN = 64;                  // keys per tile
constexpr int kRowBytes = kHeadDim * 2; // 256 B per key row in LDS (swizzled, unpadded)
constexpr int kTileBytes = BN * kRowBytes;   // 16 KB
constexpr int kBufBytes = 2 * kTileBytes;    // K tile + V tile
constexpr float kLog2e = 1.44269504088896340736f;
// A query's reference maximum is only raised when a tile's maximum exceeds it by more than
// this many powers of two; until then probabilities may exceed 1 (at most 2^8), which fp32
// accumulators and bf16's exponent range absorb, and the O rescale is skipped.
constexpr float kRescaleLog2 = 8.0f;

struct SplitInfo {
  int n_splits;
  int tiles_per_split;
};

// LDS layout of one K tile: row r (key), 16-byte chunk c (8 channels) at r*256 + ((c ^ (r&15))*16).
// LDS layout of one V tile: row r, 32-byte pair slot p (16 channels) at r*256 + ((p ^ (r&3))*32).
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void attention_kernel(AttnArgs a, SplitInfo sp) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds[2 * kBufBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int n = lane & 31;   // query column inside the wave's 32
  const int g = lane >> 5;   // which half of each 8-key group this lane holds
  const int head = blockIdx.y;
  const int split = blockIdx.z;
  const int q0 = blockIdx.x * BM + wave * 32;

  const int n_tiles_total = (int)((a.n_keys + BN - 1) / BN);
  const int tile_begin = split * sp.tiles_per_split;
  const int tile_end = min(n_tiles_total, tile_begin + sp.tiles_per_split);

  // ---- loader constants: lane i of load instruction t moves one 16-byte chunk of tile row
  // 16*wave + 4*t + i/16 into LDS position (that row, chunk i%16)
  const int l_row = lane >> 4, l_chunk = lane & 15;
  int k_src_chunk[4], v_src_chunk[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int row = 16 * wave + 4 * t + l_row;
    k_src_chunk[t] = (l_chunk ^ (row & 15)) * 8;                               // elements
    v_src_chunk[t] = ((((l_chunk >> 1) ^ (row & 3)) << 1) | (l_chunk & 1)) * 8;
  }
  const uint16_t* kc_head = a.k_cache + (int64_t)head * a.c_head;
  const uint16_t* vc_head = a.v_cache + (int64_t)head * a.c_head;

  auto issue_tile_loads = [&](int kt, int buf) {
    uint8_t* kdst = lds + buf * kBufBytes + (16 * wave) * kRowBytes;
    uint8_t* vdst = kdst + kTileBytes;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      int vk = kt * BN + 16 * wave + 4 * t + l_row;
      vk = min(vk, (int)a.n_keys - 1);   // tail rows re-read the last key; their scores are masked
      const int64_t off = key_row(a.segs, vk) * a.c_tok;
      __builtin_amdgcn_global_load_lds(GLB_PTR(kc_head + off + k_src_chunk[t]),
                                       LDS_PTR(kdst + t * 4 * kRowBytes), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(GLB_PTR(vc_head + off + v_src_chunk[t]),
                                       LDS_PTR(vdst + t * 4 * kRowBytes), 16, 0, 0);
    }
  };

  // ---- Q^T fragments (B operand): lane holds query n, channels 16*ks + 8g .. +7
  bf16x8_t qf[8];
  {
    int qrow = q0 + n;
    if (qrow >= a.n_q) qrow = a.n_q - 1;
    const uint16_t* qp = a.q + (int64_t)qrow * a.q_tok + (int64_t)head * a.q_head + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qf[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qp + 16 * ks));
  }

  // ---- fragment read offsets (bytes inside a buffer)
  // K: row kb*32 + n, logical chunk 2*ks + g  ->  (2*ks) ^ (g ^ (n&15)) after the swizzle
  int k_off[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k_off[ks] = n * kRowBytes + (((2 * ks + g) ^ (n & 15)) << 4);
  // V (transposing read): 16-lane group G = lane/16 covers channel half mh = G&1 of key half g;
  // lane i of the group points at row 4g + i/4 (+ step offset), channels 16*(db + 4*mh) + 4*(i%4)
  int v_off[4];
  {
    const int i16 = lane & 15, mh = (lane >> 4) & 1;
    const int kk = i16 >> 2, cc = i16 & 3;
#pragma unroll
    for (int db = 0; db < 4; ++db)
      v_off[db] = kTileBytes + (4 * g + kk) * kRowBytes + (((db ^ kk) + 4 * mh) << 5) + cc * 8;
  }

  f32x16_t o_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;
  const float c = a.scale * kLog2e;   // exp(x*scale) = exp2(x*c)
  const float tau = kRescaleLog2 / c; // in raw score units
  float m_ref = -INFINITY;            // reference maximum of raw scores of query n
  float mc = 0.f;                     // m_ref * c
  float l_run = 0.f;                  // this lane's share of the denominator

  if (tile_begin < tile_end) issue_tile_loads(tile_begin, 0);

  for (int kt = tile_begin; kt < tile_end; ++kt) {
    const int buf = (kt - tile_begin) & 1;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();   // tile kt has landed for every wave; everyone is done with buffer buf^1
    if (kt + 1 < tile_end) issue_tile_loads(kt + 1, buf ^ 1);
    const uint8_t* base = lds + buf * kBufBytes;

    // ---- S^T = K . Q^T : two independent 32-key accumulators, interleaved
    f32x16_t s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_acc[kb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8_t kf = __builtin_bit_cast(
            bf16x8_t, *reinterpret_cast<const uint4*>(base + k_off[ks] + kb * 32 * kRowBytes));
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s_acc[kb], 0, 0, 0);
      }
    }
    // accumulator element i of block kb: key kt*BN + kb*32 + 8*(i/4) + 4*g + (i%4), query n
    if (kt == n_tiles_total - 1) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int vk = kt * BN + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
          if (vk >= (int)a.n_keys) s_acc[kb][i] = -INFINITY;
        }
    }
    // ---- online softmax for query n
    float mx = fmaxf(s_acc[0][0], s_acc[1][0]);
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, fmaxf(s_acc[0][i], s_acc[1][i]));
    mx = max_across_halves(mx);
    const bool raise = mx > m_ref + tau;   // always true on the first tile (m_ref = -inf)
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
      const float m_new = raise ? mx : m_ref;
      const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c);   // 1 where unchanged, 0 at start
      m_ref = m_new;
      mc = m_new * c;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;
    }
    uint32_t pf[2][8];
    const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][i], c, -mc));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][i + 1], c, -mc));
        const uint32_t u = pack_bf16x2(p0, p1);
        pf[kb][i >> 1] = u;
        // denominator from the rounded values the MFMA sees
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, u), ones, l_run, false);
      }

    // ---- O^T += V^T . P^T : 4 steps of 16 keys x 4 channel blocks
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int kb = j >> 1, jj = j & 1;
      const uint4 pu = make_uint4(pf[kb][4 * jj], pf[kb][4 * jj + 1], pf[kb][4 * jj + 2], pf[kb][4 * jj + 3]);
      const bf16x8_t pb = __builtin_bit_cast(bf16x8_t, pu);
      const int step_off = (kb * 32 + 16 * jj) * kRowBytes;
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4_t*)(base + v_off[db] + step_off));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4_t*)(base + v_off[db] + step_off + 8 * kRowBytes));
        const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
        const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb, o_acc[db], 0, 0, 0);
      }
    }
  }

  // ---- epilogue.  O^T block db, element i: channel 16*db + 64*(i/8) + 8*((i/4)&1) + 4*g + (i%4)
  const float l_tot = sum_across_halves(l_run);
  const int qrow = q0 + n;
  if (qrow >= a.n_q) return;
  if (sp.n_splits == 1) {
    const float inv_l = 1.0f / l_tot;
    uint16_t* op = a.out + (int64_t)qrow * a.o_tok + (int64_t)head * a.o_head;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 16 * db + 64 * (i4 >> 1) + 8 * (i4 & 1) + 4 * g;
        uint2 w;
        w.x = pack_bf16x2(o_acc[db][4 * i4 + 0] * inv_l, o_acc[db][4 * i4 + 1] * inv_l);
        w.y = pack_bf16x2(o_acc[db][4 * i4 + 2] * inv_l, o_acc[db][4 * i4 + 3] * inv_l);
        *reinterpret_cast<uint2*>(op + d) = w;
      }
    if (a.lse && g == 0) a.lse[(int64_t)head * a.n_q + qrow] = m_ref * a.scale + logf(l_tot);
  } else {
    // partial result: unnormalised O (fp32), reference maximum and denominator
    float* ws = reinterpret_cast<float*>(a.workspace);
    const int64_t row = ((int64_t)split * a.n_heads + head) * a.n_q + qrow;
    float* op = ws + row * kHeadDim;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 16 * db + 64 * (i4 >> 1) + 8 * (i4 & 1) + 4 * g;
        *reinterpret_cast<float4*>(op + d) = make_float4(o_acc[db][4 * i4 + 0], o_acc[db][4 * i4 + 1],
                                                          o_acc[db][4 * i4 + 2], o_acc[db][4 * i4 + 3]);
      }
    if (g == 0) {
      float* ml = ws + (int64_t)sp.n_splits * a.n_heads * a.n_q * kHeadDim + row * 2;
      ml[0] = m_ref;
      ml[1] = l_tot;
    }
  }
}

// Merge the per-split partial results: one thread per (query, head, 4 channels).
__global__ __launch_bounds__(256) void combine_kernel(AttnArgs a, SplitInfo sp) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)a.n_heads * a.n_q * (kHeadDim / 4);
  if (idx >= total) return;
  const int d4 = (int)(idx % (kHeadDim / 4));
  const int64_t hq = idx / (kHeadDim / 4);   // head * n_q + q
  const int head = (int)(hq / a.n_q);
  const int q = (int)(hq % a.n_q);
  const float* ws = reinterpret_cast<const float*>(a.workspace);
  const int64_t rows = (int64_t)a.n_heads * a.n_q;
  const float* ml = ws + (int64_t)sp.n_splits * rows * kHeadDim;
  const float c = a.scale * kLog2e;
  float m = -INFINITY;
  for (int s = 0; s < sp.n_splits; ++s) m = fmaxf(m, ml[(s * rows + hq) * 2]);
  float l = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < sp.n_splits; ++s) {
    const float ms = ml[(s * rows + hq) * 2], ls = ml[(s * rows + hq) * 2 + 1];
    const float w = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((ms - m) * c);
    l += w * ls;
    const float4 o = *reinterpret_cast<const float4*>(ws + (s * rows + hq) * kHeadDim + d4 * 4);
    acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
  }
  const float inv = 1.0f / l;
  uint2 wv;
  wv.x = pack_bf16x2(acc.x * inv, acc.y * inv);
  wv.y = pack_bf16x2(acc.z * inv, acc.w * inv);
  *reinterpret_cast<uint2*>(a.out + (int64_t)q * a.o_tok + (int64_t)head * a.o_head + d4 * 4) = wv;
  if (a.lse && d4 == 0) a.lse[hq] = m * a.scale + logf(l);
}

constexpr int kSlots = 512;   // 256 CUs x 2 resident work-groups
constexpr int kMaxSplits = 16;

// Split the key range so that (query tiles x heads x splits) fills whole rounds of the
// chip's work-group slots; every split costs a partial-result round trip, so a split must
// pay for itself.
int choose_splits(int n_q, int n_heads, int64_t n_keys) {
  const int64_t units = (int64_t)((n_q + BM - 1) / BM) * n_heads;
  const int n_tiles = (int)((n_keys + BN - 1) / BN);
  int best = 1;
  double best_cost = 1e30;
  for (int s = 1; s <= kMaxSplits && s <= n_tiles; ++s) {
    const int tiles_per = (n_tiles + s - 1) / s;
    if ((int64_t)(s - 1) * tiles_per >= n_tiles) continue;   // would leave an empty split
    const double rounds = (double)((units * s + kSlots - 1) / kSlots);
    double cost = rounds * tiles_per;                         // key tiles on the critical path
    if (s > 1) cost += 2.0 + 0.03 * n_tiles * s / 16.0;       // partial write + combine pass
    if (cost < best_cost - 1e-9) { best_cost = cost; best = s; }
  }
  return best;
}

}  // namespace

size_t attention_workspace_bytes(int n_q, int n_heads, int64_t n_keys) {
  const int s = choose_splits(n_q, n_heads, n_keys);
  if (s == 1) return 0;
  return (size_t)s * n_heads * n_q * (kHeadDim + 2) * sizeof(float);
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  SplitInfo sp;
  sp.n_splits = choose_splits(a.n_q, a.n_heads, a.n_keys);
  const int n_tiles = (int)((a.n_keys + BN - 1) / BN);
  sp.tiles_per_split = (n_tiles + sp.n_splits - 1) / sp.n_splits;
  dim3 grid((a.n_q + BM - 1) / BM, a.n_heads, sp.n_splits);
  hipLaunchKernelGGL(attention_kernel, grid, dim3(256), 0, st, a, sp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || sp.n_splits == 1) return e;
  const int64_t total = (int64_t)a.n_heads * a.n_q * (kHeadDim / 4);
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, sp);
  return hipGetLastError();
}

}  // namespace crope
