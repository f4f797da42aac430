// Chunk attention: softmax(scale * q.K^T) V of one chunk's queries over the visible cache
// rows, flash style (online softmax, no score matrix in memory), bf16 MFMA on gfx950.
//
// Operand roles are chosen so that the softmax is lane-local.  Each wave owns 32 queries
// and computes S^T = K . Q^T with v_mfma_f32_32x32x16_bf16: keys are the MFMA rows, queries
// the columns, so accumulator lane l holds 16 keys of ONE query (column l%32) and the row
// max / row sum need a single exchange between lane l and lane l^32.  The same registers,
// rounded to bf16, are then the B operand (P^T) of O^T += V^T . P^T; the key order inside a
// 16-key MFMA step is whatever the accumulator layout gives, and the V^T fragment is
// gathered in that same order.
#include "crope_internal.h"

namespace crope {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ int64_t key_row(const Segments& s, int64_t vk) {
  // visible key index -> cache row
#pragma unroll
  for (int i = 0; i < kMaxSegments; ++i) {
    if (i < s.n) {
      if (vk < s.len[i]) return s.start[i] + vk;
      vk -= s.len[i];
    }
  }
  return -1;
}

constexpr int BM = 128;           // queries per work-group: 4 waves x 32
constexpr int BN = 64;            // keys per tile
constexpr int KS = kHeadDim + 8;  // K tile row pitch in LDS (elements): 272 B spreads rows over banks
constexpr int VS = BN + 8;        // V^T tile row pitch (elements)

__global__ __launch_bounds__(256) void attention_kernel_v0(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[BN * KS];
  __shared__ __attribute__((aligned(16))) uint16_t Vt[kHeadDim * VS];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int n = lane & 31;  // query column inside the wave's 32
  const int g = lane >> 5;  // which half of each 8-key group this lane holds
  const int head = blockIdx.y;
  const int q0 = blockIdx.x * BM + wave * 32;

  // Q^T fragments (B operand): lane holds query n, channels 16*ks + 8g .. +7
  bf16x8_t qf[8];
  {
    int qrow = q0 + n;
    if (qrow >= a.n_q) qrow = a.n_q - 1;
    const uint16_t* qp = a.q + (int64_t)qrow * a.q_tok + (int64_t)head * a.q_head + 8 * g;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qf[ks] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qp + 16 * ks));
  }

  f32x16_t o_acc[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;
  float m_run = -INFINITY;  // running max of raw (unscaled) scores of query n
  float l_run = 0.f;        // this lane's share of the running denominator
  const float c = a.scale * 1.44269504088896340736f;  // exp(x*scale) = exp2(x*c)

  const int n_tiles = (int)((a.n_keys + BN - 1) / BN);
  for (int kt = 0; kt < n_tiles; ++kt) {
    __syncthreads();  // previous tile fully consumed
    // ---- stage K (row-major) and V (transposed) tiles in LDS
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int chunk = tid + 256 * r;
      const int row = chunk >> 4, col = chunk & 15;
      const int64_t vk = (int64_t)kt * BN + row;
      uint4 kk = make_uint4(0, 0, 0, 0), vv = kk;
      if (vk < a.n_keys) {
        const int64_t off = key_row(a.segs, vk) * a.c_tok + (int64_t)head * a.c_head + col * 8;
        kk = *reinterpret_cast<const uint4*>(a.k_cache + off);
        vv = *reinterpret_cast<const uint4*>(a.v_cache + off);
      }
      *reinterpret_cast<uint4*>(&Ks[row * KS + col * 8]) = kk;
      const uint16_t* ve = reinterpret_cast<const uint16_t*>(&vv);
#pragma unroll
      for (int e = 0; e < 8; ++e) Vt[(col * 8 + e) * VS + row] = ve[e];
    }
    __syncthreads();

    // ---- S^T = K . Q^T : two 32-key blocks
    f32x16_t s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s_acc[kb][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const bf16x8_t kf = __builtin_bit_cast(
            bf16x8_t, *reinterpret_cast<const uint4*>(&Ks[(kb * 32 + n) * KS + ks * 16 + 8 * g]));
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s_acc[kb], 0, 0, 0);
      }
    }
    // accumulator element i of block kb: key kt*BN + kb*32 + 8*(i/4) + 4*g + (i%4), query n
    if (kt == n_tiles - 1) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int64_t vk = (int64_t)kt * BN + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
          if (vk >= a.n_keys) s_acc[kb][i] = -INFINITY;
        }
    }
    // ---- online softmax for query n
    float mx = s_acc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s_acc[kb][i]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
    const float mc = m_new * c;
    m_run = m_new;
    uint32_t pf[2][8];
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][i], c, -mc));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][i + 1], c, -mc));
        const uint32_t u = pack_bf16x2(p0, p1);
        pf[kb][i >> 1] = u;
        psum += bf16_lo(u) + bf16_hi(u);  // denominator from the rounded values the MFMA sees
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;

    // ---- O^T += V^T . P^T : 4 channel blocks x 4 steps of 16 keys
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int kb = j >> 1, jj = j & 1;
      const uint4 pu = make_uint4(pf[kb][4 * jj], pf[kb][4 * jj + 1], pf[kb][4 * jj + 2], pf[kb][4 * jj + 3]);
      const bf16x8_t pb = __builtin_bit_cast(bf16x8_t, pu);
      const int k0 = kb * 32 + 16 * jj + 4 * g;
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const int d = db * 32 + n;
        const uint2 lo = *reinterpret_cast<const uint2*>(&Vt[d * VS + k0]);
        const uint2 hi = *reinterpret_cast<const uint2*>(&Vt[d * VS + k0 + 8]);
        const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, make_uint4(lo.x, lo.y, hi.x, hi.y));
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb, o_acc[db], 0, 0, 0);
      }
    }
  }

  // ---- epilogue
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv_l = 1.0f / l_tot;
  const int qrow = q0 + n;
  if (qrow < a.n_q) {
    uint16_t* op = a.out + (int64_t)qrow * a.o_tok + (int64_t)head * a.o_head;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = db * 32 + 8 * i4 + 4 * g;
        uint2 w;
        w.x = pack_bf16x2(o_acc[db][4 * i4 + 0] * inv_l, o_acc[db][4 * i4 + 1] * inv_l);
        w.y = pack_bf16x2(o_acc[db][4 * i4 + 2] * inv_l, o_acc[db][4 * i4 + 3] * inv_l);
        *reinterpret_cast<uint2*>(op + d) = w;
      }
    if (a.lse && g == 0) a.lse[(int64_t)head * a.n_q + qrow] = m_run * a.scale + logf(l_tot);
  }
}

}  // namespace

size_t attention_workspace_bytes(int, int, int64_t) { return 0; }

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  dim3 grid((a.n_q + BM - 1) / BM, a.n_heads);
  hipLaunchKernelGGL(attention_kernel_v0, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace crope
