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
// A work-group is 4 or 8 waves (128 or 256 queries of one head), always two waves per SIMD:
// a wave issues in order, so whenever its next instruction waits (for an MFMA result, an LDS
// fragment, the barrier) its matrix and vector slots go unused unless a second wave is there
// to fill them.  K and V tiles of 64 keys are copied HBM -> LDS without passing through
// registers (global_load_lds, 16 B per lane), double buffered, XOR-swizzled by choosing
// which global chunk each lane fetches.
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

// max over both halves of the wave (lane l and lane l^32), result in every lane
__device__ __forceinline__ float max_across_halves(float x) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float x) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr int BN = 64;                  // keys per tile
constexpr int kRowBytes = kHeadDim * 2; // 256 B per key row in LDS (swizzled, unpadded)
constexpr int kTileBytes = BN * kRowBytes;   // 16 KB
constexpr float kLog2e = 1.44269504088896340736f;
constexpr float kLn2 = 0.69314718055994530942f;
// A query's reference maximum is only raised when a block's maximum exceeds it by more than
// this many powers of two; until then probabilities may exceed 1, which fp32 accumulators and
// bf16's exponent range absorb, and the O rescale is skipped.  Whether to look at all is decided
// from a lane's 16-key share of the block's denominator: above kTrigger some probability is
// above 2^5, below it none is above 2^9.
constexpr float kRescaleLog2 = 8.0f;
constexpr float kTrigger = 512.0f;

struct SplitInfo {
  int n_splits;
  int tiles_per_split;
  int q_tiles;        // ceil(n_q / (32 * waves per work-group))
  int total_units;    // q_tiles * n_heads * n_splits
  int units_per_xcd;  // ceil(total_units / 8)
};
constexpr int kXcds = 8;

// LDS layout of one K tile: row r (key), 16-byte chunk c (8 channels) at r*256 + ((c ^ (r&15))*16).
// LDS layout of one V tile: row r, 32-byte pair slot p (16 channels) at r*256 + ((p ^ (r&3))*32).
//
// Software pipeline over 32-key blocks b (two per tile).  Sub-iteration b holds three
// independent instruction streams in ONE basic block, interleaved by the scheduler
// directives at its end:
//   MFMA:  S_{b+1} = K_{b+1} . Q^T          and   O^T += V_{b-1}^T . P_{b-1}^T
//   VALU:  P_b = exp2(S_b * c - m_ref * c), row sums, and the block maximum of S_b
// so K is needed one block ahead of V: tile T+1's K and tile T's V are live together, and
// the four 16 KB LDS buffers hold K_{T+1}, K_{T+2} (arriving), V_T, V_{T+1} (arriving).
// The probabilities are formed against the reference maximum as it stood BEFORE the block;
// only afterwards is the block maximum compared with it, and in the rare case that it
// exceeds the reference by more than 2^8 the block's probabilities are recomputed and the
// running sums rescaled.  The score blocks alternate between two register sets.
struct PipeState {
  f32x16_t o_acc[4];
  f32x16_t s_a, s_b;   // raw scores: one block being exponentiated, the next being accumulated
  uint32_t p_prev[8];  // bf16 probabilities of the block whose P.V is due
  float m_ref, mc, l_run;
  f32x16_t seed;       // FOLDED: minus the reference in every element, the S accumulators' start value
};

struct FragOffsets {
  int k_off[8];
  int v_off[4];
};

// key0_next: global index of the first key of the block scored by this call (S_{b+1});
// lim: this lane's query sees keys [0, lim) (the number of visible keys, or less under a
// per-query limit).
// FOLDED: the queries already carry the factor scale*log2(e) (folded into their single bf16
// rounding by the kernel that wrote them), so the MFMA result is the exponent itself once the
// accumulators are seeded with minus the reference: no per-score arithmetic in front of the
// exp.  Otherwise scores are raw and each costs one fma (times scale*log2 e, minus reference).
// FORCE: this is the first block of the key range; its maximum becomes the reference whatever
// its value.
template <bool DO_S, bool DO_PV, bool DO_SOFTMAX, bool MASK_S, bool FOLDED, bool FORCE = false>
__device__ __forceinline__ void sub_iteration(PipeState& st, const f32x16_t& s_in, f32x16_t& s_out,
                                              const bf16x8_t (&qf)[8],
                                              const uint8_t* k_half,   // K rows of block b+1
                                              const uint8_t* v_half,   // V rows of block b-1
                                              const FragOffsets& fo, int key0_next, int lim, int g,
                                              float c, float tau) {
  f32x16_t s_new;
#pragma unroll
  for (int i = 0; i < 16; ++i) {   // keys past the end are masked by seeding their scores with -inf
    const float seed = FOLDED ? st.seed[i] : 0.f;
    s_new[i] = (MASK_S && key0_next + 8 * (i >> 2) + 4 * g + (i & 3) >= lim) ? -INFINITY : seed;
  }
  uint32_t p_new[8];
  const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
  bf16x8_t pb[2];
  if (DO_PV) {
    pb[0] = __builtin_bit_cast(bf16x8_t, make_uint4(st.p_prev[0], st.p_prev[1], st.p_prev[2], st.p_prev[3]));
    pb[1] = __builtin_bit_cast(bf16x8_t, make_uint4(st.p_prev[4], st.p_prev[5], st.p_prev[6], st.p_prev[7]));
  }
  float l_blk = 0.f;   // this lane's share of the block's denominator
  // Program order = the order in which the scheduler hands out fragment reads: V first (its
  // MFMAs run first), then K (the S chain closes the block), then the softmax stream.
  if (DO_PV) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int jj = i >> 2, db = i & 3;
      const uint8_t* vp = v_half + fo.v_off[db] + jj * 16 * kRowBytes;
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(vp));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4_t*)(vp + 8 * kRowBytes));
      const uint2 lo2 = __builtin_bit_cast(uint2, lo), hi2 = __builtin_bit_cast(uint2, hi);
      const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, make_uint4(lo2.x, lo2.y, hi2.x, hi2.y));
      st.o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[jj], st.o_acc[db], 0, 0, 0);
    }
  }
  if (DO_S) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bf16x8_t kf = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(k_half + fo.k_off[i]));
      s_new = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[i], s_new, 0, 0, 0);
    }
  }
  if (DO_SOFTMAX) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float s0 = s_in[2 * i], s1 = s_in[2 * i + 1];
      const uint32_t u = FOLDED ? pack_bf16x2(__builtin_amdgcn_exp2f(s0), __builtin_amdgcn_exp2f(s1))
                                : pack_bf16x2(__builtin_amdgcn_exp2f(fmaf(s0, c, -st.mc)),
                                              __builtin_amdgcn_exp2f(fmaf(s1, c, -st.mc)));
      p_new[i] = u;
      // denominator from the rounded values the MFMA will see
      l_blk = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, u), ones, l_blk, false);
    }
  }
  // Issue order inside the block: a few fragment reads first, then every MFMA is followed by
  // VALU / transcendental instructions of the softmax stream and the next fragment reads.
  if (DO_S && DO_PV && DO_SOFTMAX) {
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);    // V fragments of the first four MFMAs
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, FOLDED ? 1 : 2, 0);   // VALU
      __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);   // TRANS
      if (i < 8) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // DS reads, four MFMAs ahead
    }
  }
  if (DO_SOFTMAX) {
    // keep the softmax stream inside this scheduling region (it would otherwise be sunk to
    // its first use in the next sub-iteration)
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(p_new[i]));
    asm volatile("" : "+v"(l_blk));
    // ---- rare: a probability of this block is large (above 2^5 at least, 2^9 at most), i.e. a
    // score outgrew the reference; seen from the block's denominator, so that the common case
    // pays no per-score maximum.  (!(x <= t) is also true for an overflowed, non-finite sum.)
    const bool big = !(l_blk <= kTrigger);
    if (FORCE || __builtin_amdgcn_ballot_w64(big) != 0) {
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < 8; ++i) mx = fmaxf(fmaxf(mx, s_in[2 * i]), s_in[2 * i + 1]);
      mx = max_across_halves(mx);
      if (FOLDED) {
        // s_in holds exponents relative to the reference: move the reference up by `shift`
        const bool raise = FORCE || mx > kRescaleLog2;
        const float shift = raise ? mx : 0.f;
        if (!FORCE) {   // at the first block O and the denominator are still zero
          const float alpha = __builtin_amdgcn_exp2f(-shift);   // 1 where unchanged
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) st.o_acc[db][i] *= alpha;
          st.l_run *= alpha;
        }
        st.m_ref += shift;
#pragma unroll
        for (int i = 0; i < 16; ++i) st.seed[i] = -st.m_ref;
        if (DO_S) {   // the block in flight was seeded with the old reference
#pragma unroll
          for (int i = 0; i < 16; ++i) s_new[i] -= shift;
        }
        l_blk = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t u = pack_bf16x2(__builtin_amdgcn_exp2f(s_in[2 * i] - shift),
                                         __builtin_amdgcn_exp2f(s_in[2 * i + 1] - shift));
          p_new[i] = u;
          l_blk = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, u), ones, l_blk, false);
        }
      } else {
        const bool raise = FORCE || mx > st.m_ref + tau;
        const float m_new = raise ? mx : st.m_ref;
        if (!FORCE) {
          const float alpha = __builtin_amdgcn_exp2f((st.m_ref - m_new) * c);   // 1 where unchanged
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) st.o_acc[db][i] *= alpha;
          st.l_run *= alpha;
        }
        st.m_ref = m_new;
        st.mc = m_new * c;
        l_blk = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t u = pack_bf16x2(__builtin_amdgcn_exp2f(fmaf(s_in[2 * i], c, -st.mc)),
                                         __builtin_amdgcn_exp2f(fmaf(s_in[2 * i + 1], c, -st.mc)));
          p_new[i] = u;
          l_blk = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, u), ones, l_blk, false);
        }
      }
    }
    st.l_run += l_blk;
#pragma unroll
    for (int i = 0; i < 8; ++i) st.p_prev[i] = p_new[i];
  }
  if (DO_S) s_out = s_new;
}

// HBM -> LDS tile copy by a work-group of NW waves.  Load instruction t of wave w moves tile
// rows 4*NW*t + 4*w .. +3: lane i carries one 16-byte chunk of row 4*NW*t + 4*w + i/16 into LDS
// position (that row, chunk i%16); which global chunk it fetches implements the swizzle,
// which depends on the row only through 4*w + i/16, so one per-lane byte offset serves every
// t.  A tile whose 64 keys are consecutive cache rows (the common case) is addressed as a
// wave-uniform base plus that offset: no vector address arithmetic in the steady state.
struct Loader {     // scalars only, so that it is promoted to registers at once
  const uint8_t *k_head, *v_head;    // cache base of this head (bytes)
  int seg_end0, seg_end1, seg_end2;  // visible key index -> cache row: vk + base of its segment
  int seg_base3, d2, d1, d0;         // base3, base2-base3, base1-base2, base0-base1
  int64_t row_bytes;                 // c_tok * 2
  int row0;       // 4*wave + lane/16
  int lds_row0;   // 4*wave
  int key_first;  // first visible key of this work-group's split
  int n_keys;
  uint32_t k_chunk_bytes, v_chunk_bytes;   // swizzled chunk offset inside the lane's row
  uint32_t k_lane_off, v_lane_off;         // row0 * row_bytes + chunk offset
};

// 16 bytes per lane, HBM -> LDS without passing through registers: lane i's data lands at
// LDS address lds_dst + 16*i.  The LDS base travels in M0, which the compiler loads itself
// (an input operand bound to that register); the s_nop covers the wait state the hardware
// wants between a write of M0 and a copy that uses it.  Written as inline assembly, not
// with the compiler's builtin: while a builtin copy is in flight the compiler's wait-count
// insertion turns every later "wait for this LDS read" into "wait for ALL LDS reads", which
// exposes the full LDS latency at each MFMA that consumes a fragment.  The copies are
// waited for explicitly (s_waitcnt vmcnt) before the barrier that publishes a tile.
#define LDS_ADDR(p) ((uint32_t)(uintptr_t)((__attribute__((address_space(3))) void*)(p)))
__device__ __forceinline__ void copy16_uniform(const uint8_t* base /* wave-uniform */, uint32_t lane_off,
                                               uint8_t* lds_dst /* wave-uniform */) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(LDS_ADDR(lds_dst));
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(lane_off), "s"(base), "{m0}"(m0) : "memory");
}
__device__ __forceinline__ void copy16_per_lane(const uint8_t* src, uint8_t* lds_dst /* wave-uniform */) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(LDS_ADDR(lds_dst));
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(src), "{m0}"(m0) : "memory");
}

__device__ __forceinline__ int seg_row(const Loader& L, int vk) {
  // arithmetic select (no value select the compiler could turn into a table lookup)
  return vk + L.seg_base3 + (vk < L.seg_end2 ? L.d2 : 0) + (vk < L.seg_end1 ? L.d1 : 0) +
         (vk < L.seg_end0 ? L.d0 : 0);
}

template <bool IS_V, int NW>
__device__ __forceinline__ void load_tile(const Loader& L, int tile, uint8_t* dst_tile) {
  uint8_t* dst = dst_tile + L.lds_row0 * kRowBytes;
  const int k_first = L.key_first + tile * BN;   // wave-uniform
  const int k_last = k_first + BN - 1;
  const uint8_t* head = IS_V ? L.v_head : L.k_head;
  const int r_first = seg_row(L, k_first);
  // no segment ends inside (k_first, k_last]: both keys lie in one segment, whose rows are consecutive
  const bool one_segment = !((k_first < L.seg_end0 && k_last >= L.seg_end0) ||
                             (k_first < L.seg_end1 && k_last >= L.seg_end1) ||
                             (k_first < L.seg_end2 && k_last >= L.seg_end2));
  if (k_last < L.n_keys && one_segment) {
    // 64 consecutive cache rows: uniform base + constant per-lane offset
    const uint8_t* base = head + (int64_t)r_first * L.row_bytes;
    const uint32_t lane_off = IS_V ? L.v_lane_off : L.k_lane_off;
#pragma unroll
    for (int t = 0; t < 16 / NW; ++t)
      copy16_uniform(base + (int64_t)(4 * NW * t) * L.row_bytes, lane_off, dst + t * 4 * NW * kRowBytes);
  } else {
    // tile straddles a segment boundary or the end of the keys: per-lane row lookup; rows
    // past the end re-read the last key (their scores are masked)
#pragma unroll
    for (int t = 0; t < 16 / NW; ++t) {
      const int vk = min(k_first + L.row0 + 4 * NW * t, L.n_keys - 1);
      const uint8_t* src = head + (int64_t)seg_row(L, vk) * L.row_bytes +
                           (IS_V ? L.v_chunk_bytes : L.k_chunk_bytes);
      copy16_per_lane(src, dst + t * 4 * NW * kRowBytes);
    }
  }
}

// Iteration T: wait for K of tile T+1 and V of tile T, start the copies of K_{T+2} and V_{T+1}
// into the two buffers nobody reads any more, then run the two 32-key sub-iterations.
// On entry st.s_b holds S of block 2T+1 and st.p_prev holds P of block 2T.
template <int NW, bool MASK_S, bool FOLDED>
__device__ __forceinline__ void tile_iteration(PipeState& st, const Loader& L, const bf16x8_t (&qf)[8],
                                               const FragOffsets& fo, int T, int n_t, uint8_t* k_load,
                                               uint8_t* v_load, const uint8_t* k_read, const uint8_t* v_read,
                                               int lim, int g, float c, float tau) {
  constexpr int kHalf = 32 * kRowBytes;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();   // K_{T+1}, V_T have landed; every wave is done with K_T and V_{T-1}
  if (T + 2 < n_t) load_tile<false, NW>(L, T + 2, k_load);
  load_tile<true, NW>(L, T + 1, v_load);
  sub_iteration<true, true, true, MASK_S, FOLDED>(st, st.s_b, st.s_a, qf, k_read, v_read, fo,
                                          L.key_first + (2 * T + 2) * 32, lim, g, c, tau);
  sub_iteration<true, true, true, MASK_S, FOLDED>(st, st.s_a, st.s_b, qf, k_read + kHalf, v_read + kHalf, fo,
                                          L.key_first + (2 * T + 3) * 32, lim, g, c, tau);
}

// NW = waves per work-group (4 or 8), each owning 32 queries.  NW = 4: two work-groups per
// CU.  NW = 8: one work-group per CU, so each K/V tile is copied into LDS once per CU
// instead of twice, at a coarser query-tile granularity.
// LIMITED: every query carries its own count of leading visible keys (a block-causal or
// causal prefix mask); every score block is then masked per lane and the key loop stops at the
// largest limit of the work-group.
template <int NW, bool LIMITED, bool FOLDED>
__global__ __attribute__((amdgpu_flat_work_group_size(64 * NW, 64 * NW), amdgpu_waves_per_eu(2, 2)))
void attention_kernel(AttnArgs a, SplitInfo sp) {
  constexpr int BM = 32 * NW;   // queries per work-group
  // Four separate LDS objects (not one array): the compiler can then prove that the
  // fragment reads of one buffer do not alias the in-flight HBM->LDS copies into another,
  // and does not make the reads wait for the prefetch.
  __shared__ __attribute__((aligned(1024))) uint8_t k_lds0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t k_lds1[kTileBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t v_lds0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) uint8_t v_lds1[kTileBytes];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int n = lane & 31;   // query column inside the wave's 32
  const int g = lane >> 5;   // which half of each 8-key group this lane holds
  // Work-groups are dealt round-robin over the 8 XCDs (each with its own L2).  Give every XCD
  // a contiguous run of the (head, split, query tile) list, so the work-groups that stream
  // the same K/V rows at the same time share one L2.
  const int unit = (int)(blockIdx.x % kXcds) * sp.units_per_xcd + (int)(blockIdx.x / kXcds);
  if (unit >= sp.total_units) return;   // whole work-group leaves before any barrier
  // under per-query limits later query tiles usually see more keys: start the long ones first
  const int q_tile = LIMITED ? sp.q_tiles - 1 - unit % sp.q_tiles : unit % sp.q_tiles;
  const int hs = unit / sp.q_tiles;
  const int split = hs % sp.n_splits;
  const int head = hs / sp.n_splits;
  const int q0 = q_tile * BM + wave * 32;
  int n_keys = (int)a.n_keys;
  int lim = n_keys;   // keys visible to this lane's query
  int n_unmasked = 0;  // LIMITED: key tiles wholly below the smallest limit of this wave's queries
  if (LIMITED) {
    const int qrow = min(q0 + n, a.n_q - 1);
    lim = min(n_keys, max(1, a.q_limit[qrow]));
    int wmax = lim, wmin = lim;
#pragma unroll
    for (int m = 16; m >= 1; m >>= 1) {
      wmax = max(wmax, __shfl_xor(wmax, m, 64));
      wmin = min(wmin, __shfl_xor(wmin, m, 64));
    }
    n_unmasked = __builtin_amdgcn_readfirstlane(wmin) / BN;
    // largest limit of the work-group, through the (still unused) first K buffer
    int* scratch = reinterpret_cast<int*>(k_lds0);
    if (lane == 0) scratch[wave] = wmax;
    __syncthreads();
    int gmax = 1;
#pragma unroll
    for (int w = 0; w < NW; ++w) gmax = max(gmax, scratch[w]);
    __syncthreads();   // everyone has read before the first tile copy overwrites the buffer
    n_keys = __builtin_amdgcn_readfirstlane(gmax);   // nothing beyond is visible to this work-group
  }

  const int n_tiles_total = (n_keys + BN - 1) / BN;
  const int tile_begin = split * sp.tiles_per_split;
  const int n_t = min(n_tiles_total, tile_begin + sp.tiles_per_split) - tile_begin;   // >= 1

  Loader L;
  {
    const int l_row = lane >> 4, l_chunk = lane & 15;
    const int row = 4 * wave + l_row;   // the lane's row inside every 4*NW-row group
    L.row_bytes = a.c_tok * 2;
    L.k_chunk_bytes = (l_chunk ^ (row & 15)) * 16;
    L.v_chunk_bytes = ((((l_chunk >> 1) ^ (row & 3)) << 1) | (l_chunk & 1)) * 16;
    L.k_lane_off = (uint32_t)(row * L.row_bytes) + L.k_chunk_bytes;
    L.v_lane_off = (uint32_t)(row * L.row_bytes) + L.v_chunk_bytes;
    L.k_head = reinterpret_cast<const uint8_t*>(a.k_cache + (int64_t)head * a.c_head);
    L.v_head = reinterpret_cast<const uint8_t*>(a.v_cache + (int64_t)head * a.c_head);
    // through readfirstlane: plain scalar values, not addresses the compiler may select between
    L.seg_end0 = __builtin_amdgcn_readfirstlane(a.segs.end[0]);
    L.seg_end1 = __builtin_amdgcn_readfirstlane(a.segs.end[1]);
    L.seg_end2 = __builtin_amdgcn_readfirstlane(a.segs.end[2]);
    L.seg_base3 = __builtin_amdgcn_readfirstlane(a.segs.base[3]);
    L.d2 = __builtin_amdgcn_readfirstlane(a.segs.base[2] - a.segs.base[3]);
    L.d1 = __builtin_amdgcn_readfirstlane(a.segs.base[1] - a.segs.base[2]);
    L.d0 = __builtin_amdgcn_readfirstlane(a.segs.base[0] - a.segs.base[1]);
    L.row0 = row;
    L.lds_row0 = 4 * wave;
    L.key_first = tile_begin * BN;
    L.n_keys = n_keys;
  }

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

  // ---- fragment read offsets (bytes inside a 32-key half tile)
  // K: row n, logical chunk 2*ks + g  ->  (2*ks) ^ (g ^ (n&15)) after the swizzle
  FragOffsets fo;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) fo.k_off[ks] = n * kRowBytes + (((2 * ks + g) ^ (n & 15)) << 4);
  // V (transposing read): 16-lane group G = lane/16 covers channel half mh = G&1 of key half g;
  // lane i of the group points at row 4g + i/4 (+ step offset), channels 16*(db + 4*mh) + 4*(i%4)
  {
    const int i16 = lane & 15, mh = (lane >> 4) & 1;
    const int kk = i16 >> 2, cc = i16 & 3;
#pragma unroll
    for (int db = 0; db < 4; ++db)
      fo.v_off[db] = (4 * g + kk) * kRowBytes + (((db ^ kk) + 4 * mh) << 5) + cc * 8;
  }

  PipeState st;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o_acc[db][i] = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) st.p_prev[i] = 0u;
  const float c = a.scale * kLog2e;   // exp(x*scale) = exp2(x*c)
  const float tau = kRescaleLog2 / c; // in raw score units
  // reference maximum of query n's scores: raw score units (FOLDED: exponent units; the first
  // block's maximum is added to this 0)
  st.m_ref = FOLDED ? 0.f : -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; ++i) st.seed[i] = 0.f;
  st.mc = 0.f;                        // m_ref * c
  st.l_run = 0.f;                     // this lane's share of the denominator
  const int key_base = tile_begin * BN;
  constexpr int kHalf = 32 * kRowBytes;

  // ---- prologue: S_0 -> s_a and S_1 -> s_b from tile 0, then P_0
  load_tile<false, NW>(L, 0, k_lds0);
  load_tile<true, NW>(L, 0, v_lds0);
  if (n_t > 1) load_tile<false, NW>(L, 1, k_lds1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (q0 >= a.n_q) {
    // A wave whose 32 rows all lie past the last query (ragged last query tile) does no
    // arithmetic: it only takes its share of the tile copies and passes the same barriers as
    // the others (one per tile iteration, one before the drain).
    for (int T = 0; T + 1 < n_t; ++T) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (T + 2 < n_t) load_tile<false, NW>(L, T + 2, (T & 1) ? k_lds1 : k_lds0);
      load_tile<true, NW>(L, T + 1, (T & 1) ? v_lds0 : v_lds1);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    return;
  }
  sub_iteration<true, false, false, true, FOLDED>(st, st.s_a, st.s_a, qf, k_lds0, nullptr, fo, key_base, lim, g, c,
                                                  tau);
  sub_iteration<true, false, false, true, FOLDED>(st, st.s_b, st.s_b, qf, k_lds0 + kHalf, nullptr, fo, key_base + 32,
                                                  lim, g, c, tau);
  sub_iteration<false, false, true, false, FOLDED, true>(st, st.s_a, st.s_a, qf, nullptr, nullptr, fo, 0, lim, g, c,
                                                         tau);
  if (FOLDED) {   // S_1 was accumulated before there was a reference
#pragma unroll
    for (int i = 0; i < 16; ++i) st.s_b[i] -= st.m_ref;
  }

  // ---- steady state: iteration T scores tile T+1 (K) and accumulates tile T (V)
  int T = 0;
  if (LIMITED) {   // tiles below every limit of this wave: the unmasked code (same barriers per iteration)
    for (; T + 3 < n_t && T + 2 < n_unmasked; T += 2) {
      tile_iteration<NW, false, FOLDED>(st, L, qf, fo, T, n_t, k_lds0, v_lds1, k_lds1, v_lds0, lim, g, c, tau);
      tile_iteration<NW, false, FOLDED>(st, L, qf, fo, T + 1, n_t, k_lds1, v_lds0, k_lds0, v_lds1, lim, g, c, tau);
    }
  }
  for (; T + 3 < n_t; T += 2) {
    tile_iteration<NW, LIMITED, FOLDED>(st, L, qf, fo, T, n_t, k_lds0, v_lds1, k_lds1, v_lds0, lim, g, c, tau);       // even T
    tile_iteration<NW, LIMITED, FOLDED>(st, L, qf, fo, T + 1, n_t, k_lds1, v_lds0, k_lds0, v_lds1, lim, g, c, tau);   // odd T
  }
  if (T + 2 < n_t) {
    tile_iteration<NW, LIMITED, FOLDED>(st, L, qf, fo, T, n_t, k_lds0, v_lds1, k_lds1, v_lds0, lim, g, c, tau);
    ++T;
  }
  // ---- T == n_t - 2 scores the last tile, which may reach beyond the visible keys
  if (T + 1 < n_t) {
    if (T & 1) tile_iteration<NW, true, FOLDED>(st, L, qf, fo, T, n_t, k_lds1, v_lds0, k_lds0, v_lds1, lim, g, c, tau);
    else tile_iteration<NW, true, FOLDED>(st, L, qf, fo, T, n_t, k_lds0, v_lds1, k_lds1, v_lds0, lim, g, c, tau);
    ++T;
  }
  // ---- drain: T == n_t - 1; last tile's V, last block's softmax
  {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const uint8_t* vb = (T & 1) ? v_lds1 : v_lds0;
    sub_iteration<false, true, true, false, FOLDED>(st, st.s_b, st.s_b, qf, nullptr, vb, fo, 0, lim, g, c, tau);
    sub_iteration<false, true, false, false, FOLDED>(st, st.s_a, st.s_a, qf, nullptr, vb + kHalf, fo, 0, lim, g, c, tau);
  }
  f32x16_t* o_acc = st.o_acc;
  const float m_ref = st.m_ref, l_run = st.l_run;

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
    if (a.lse && g == 0)
      a.lse[(int64_t)head * a.n_q + qrow] = FOLDED ? (m_ref + log2f(l_tot)) * kLn2 : m_ref * a.scale + logf(l_tot);
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
  const float c = a.folded ? 1.0f : a.scale * kLog2e;   // the partial maxima are exponents already when folded
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
  if (a.lse && d4 == 0) a.lse[hq] = a.folded ? (m + log2f(l)) * kLn2 : m * a.scale + logf(l);
}

constexpr int kCus = 256;
constexpr int kMaxSplits = 16;

// Pick the work-group shape and the number of key splits.  Cost = key tiles on the critical
// path of the busiest CU slot, in units of one 4-wave work-group tile; an 8-wave work-group
// shares its K/V copies between twice the queries and runs its tile ~4 % faster (measured).  Every
// split costs a partial-result round trip, so a split must pay for itself.  Non-zero fields of
// `want` pin that choice; a pinned split count is lowered until no split is empty.
AttnPlan choose_plan(int n_q, int n_heads, int64_t n_keys, AttnPlan want) {
  const int n_tiles = (int)((n_keys + BN - 1) / BN);
  if (want.splits > 0) {
    int s = want.splits < n_tiles ? want.splits : n_tiles;
    while (s > 1 && (int64_t)(s - 1) * ((n_tiles + s - 1) / s) >= n_tiles) --s;
    want.splits = s;
  }
  AttnPlan best{want.waves ? want.waves : 4, want.splits ? want.splits : 1};
  double best_cost = 1e30;
  for (int nw = 4; nw <= 8; nw += 4) {
    if (want.waves && nw != want.waves) continue;
    const int bm = 32 * nw;
    const int slots = kCus * (8 / nw);
    const int64_t units = (int64_t)((n_q + bm - 1) / bm) * n_heads;
    for (int s = 1; s <= kMaxSplits && s <= n_tiles; ++s) {
      const int tiles_per = (n_tiles + s - 1) / s;
      if ((int64_t)(s - 1) * tiles_per >= n_tiles) continue;   // would leave an empty split
      if (want.splits && s != want.splits) continue;
      const double rounds = (double)((units * s + slots - 1) / slots);
      double cost = rounds * tiles_per * (nw == 8 ? 0.96 : 1.0);
      if (s > 1) {
        // fp32 partials are written and read back once: (128+2)*4 B per query, head and
        // split, at ~4 TB/s, in units of one key tile (~2 us); a split must win clearly
        cost += 2.0 + (double)s * n_q * n_heads * 1040.0 / 8.4e6;
        cost *= 1.05;
      }
      if (cost < best_cost - 1e-9) { best_cost = cost; best = AttnPlan{nw, s}; }
    }
  }
  return best;
}

template <int NW, bool LIMITED, bool FOLDED>
hipError_t launch_attention_t(const AttnArgs& a, SplitInfo sp, hipStream_t st) {
  sp.q_tiles = (a.n_q + 32 * NW - 1) / (32 * NW);
  const int64_t total_units = (int64_t)sp.q_tiles * a.n_heads * sp.n_splits;
  if (total_units > (1 << 30)) return hipErrorInvalidValue;
  sp.total_units = (int)total_units;
  sp.units_per_xcd = (sp.total_units + kXcds - 1) / kXcds;
  hipLaunchKernelGGL((attention_kernel<NW, LIMITED, FOLDED>), dim3(kXcds * sp.units_per_xcd), dim3(64 * NW), 0, st, a, sp);
  return hipGetLastError();
}

}  // namespace

AttnPlan attention_plan(int n_q, int n_heads, int64_t n_keys, AttnPlan want) {
  return choose_plan(n_q, n_heads, n_keys, want);
}

size_t attention_workspace_bytes(int n_q, int n_heads, int64_t n_keys, AttnPlan want) {
  const int s = choose_plan(n_q, n_heads, n_keys, want).splits;
  if (s == 1) return 0;
  return (size_t)s * n_heads * n_q * (kHeadDim + 2) * sizeof(float);
}

hipError_t launch_attention(const AttnArgs& a, AttnPlan want, hipStream_t st) {
  AttnPlan plan = choose_plan(a.n_q, a.n_heads, a.n_keys, want);
  if (a.q_limit) plan.splits = 1;   // the per-query limits already shorten the key loops
  SplitInfo sp;
  sp.n_splits = plan.splits;
  const int n_tiles = (int)((a.n_keys + BN - 1) / BN);
  sp.tiles_per_split = (n_tiles + sp.n_splits - 1) / sp.n_splits;
  hipError_t e;
  if (a.folded) {
    if (a.q_limit) e = plan.waves == 8 ? launch_attention_t<8, true, true>(a, sp, st) : launch_attention_t<4, true, true>(a, sp, st);
    else e = plan.waves == 8 ? launch_attention_t<8, false, true>(a, sp, st) : launch_attention_t<4, false, true>(a, sp, st);
  } else {
    if (a.q_limit) e = plan.waves == 8 ? launch_attention_t<8, true, false>(a, sp, st) : launch_attention_t<4, true, false>(a, sp, st);
    else e = plan.waves == 8 ? launch_attention_t<8, false, false>(a, sp, st) : launch_attention_t<4, false, false>(a, sp, st);
  }
  if (e != hipSuccess || sp.n_splits == 1) return e;
  const int64_t total = (int64_t)a.n_heads * a.n_q * (kHeadDim / 4);
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, sp);
  return hipGetLastError();
}

}  // namespace crope
