// Local QKV projection with qk-RMSNorm, causal 3D RoPE and the KV-cache update applied in
// the GEMM's epilogue (Algorithm 3 steps 1, 2, 3 and 5 in one pass; the operator fusion of
// Section 3.4.1 item 3), bf16 MFMA on gfx950.
//
// y[token][o] = sum_c x[token][c] * w[o][c] + bias[o];  o in [0, HD) is q, [HD, 2HD) k,
// [2HD, 3HD) v.  Both operands have the reduction index contiguous, so both are MFMA
// fragments as they lie in memory.  The product is formed transposed, C^T = W . x^T
// (channels = MFMA rows, tokens = columns): an accumulator lane then holds 4 consecutive
// channels of ONE token, i.e. two whole rotation pairs, and the epilogue needs no cross-lane
// traffic for the rotation; the bf16 tile is then transposed through LDS and leaves in whole
// 256-byte (token, head) rows.
//
// A work-group (8 waves, 2 x 4) owns 128 output channels (one head of q, k or v) x 256
// tokens; a wave owns 64 x 64 (four 32x32 accumulators).  The reduction runs in steps of
// 64 through three LDS stages filled by global_load_lds (16 B per lane, no registers), one
// barrier per step.  LDS rows are 128 B; 16-byte chunk c of row r sits at slot
// c ^ ((r >> 1) & 7), which makes the fragment reads (32 rows x 16 B per half wave)
// conflict-free.
//
// RMSNorm over one head is local to the tile and fully fused.  RMSNorm over the token's
// whole H*128 vector needs every head's sum of squares: the rotation commutes with the
// per-token scalar, so the epilogue stores z = rotate(gain * y) and the per-head sums of
// squares, and a second, bandwidth-bound pass multiplies q and k rows by 1/rms.  z is kept
// as TWO bf16 numbers, hi = bf16(z) in the destination row and lo = bf16(z - hi) in the
// workspace (16 mantissa bits together), so that the second pass rounds (hi + lo) / rms to
// bf16 once: the stored result is the single rounding of the fp32 value up to 2^-17 relative.
#include "crope_internal.h"

namespace crope {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

#define LDS_ADDR(p) ((uint32_t)(uintptr_t)((__attribute__((address_space(3))) void*)(p)))

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float sum_across_halves(float x) {
  const u32x2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr int kTileCh = 128;    // output channels per work-group: one head
constexpr int kTileTok = 256;   // tokens per work-group
constexpr int kStepK = 64;      // reduction elements per LDS stage
constexpr int kRowB = kStepK * 2;             // 128 B per LDS row
constexpr int kStageA = kTileCh * kRowB;      // 16 KB
constexpr int kStageB = kTileTok * kRowB;     // 32 KB
constexpr int kOutRowB = kTileCh * 2 + 16;    // bf16 output tile row in LDS, padded against bank conflicts
constexpr int kOutBytes = kTileTok * kOutRowB; // 69632
constexpr int kAngRowB = 64 * 8 + 16;          // one token's 64 (cos, sin) pairs in LDS, padded (16-byte rows)
constexpr int kAngBytes = kTileTok * kAngRowB; // 135168
constexpr int kXcds = 8;
constexpr int kTokGroup = 4;    // token tiles walked together with 8 channel tiles by one XCD's CUs

struct ProjTiles {
  int ch_tiles, tok_tiles, total, per_xcd;
  int wgs_per_xcd;   // work-groups launched per XCD (at most its 32 CUs)
};

struct TileLoader {   // scalars only
  const uint8_t* a_base;   // W + first channel row of the tile (wave-uniform)
  const uint8_t* b_base;   // x + first token row of the tile (wave-uniform)
  // per-lane byte offsets of the lane's chunk for load instruction t: row 8*wave + lane/8 + 64*t
  uint32_t a_off0, a_off1;
  uint32_t b_off0, b_off1, b_off2, b_off3;
  int lds_off;             // wave * 1024
};

// Copy reduction step kt of the W tile and of the x tile into one LDS stage.  Load
// instruction t of wave w covers tile rows 8*(w + 8t) .. +7 (1 KB of LDS): lane i carries the
// chunk that belongs at (row 8*(w+8t) + i/8, slot i%8).  ((row >> 1) & 7) = (i>>4) | 4*(w&1)
// does not depend on t.  Token rows past the end re-read the last token (clamped when the
// offsets are formed); their results are never stored.
// The copy is inline assembly, not the compiler's builtin: while a builtin copy is in flight
// the compiler turns every counted wait on an LDS read into a wait for all of them.  LDS
// address of lane i's 16 bytes: M0 + 16*i; M0 is an input operand bound to that register, the
// s_nop is the wait state required between its write and the copy.
__device__ __forceinline__ void copy16(const uint8_t* base /* wave-uniform */, uint32_t lane_off,
                                       uint8_t* lds_dst /* wave-uniform */) {
  const uint32_t m0 = __builtin_amdgcn_readfirstlane(LDS_ADDR(lds_dst));
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(lane_off), "s"(base), "{m0}"(m0) : "memory");
}

// PART 0, 1, 2: the W tile, the first and the second half of the x tile (two copies each); a
// step issues the three parts between its MFMA groups instead of all at once, so that the
// waves do not queue up behind the address unit right after the barrier.
template <int PART>
__device__ __forceinline__ void load_stage_part(const TileLoader& L, int kt, uint8_t* a_st, uint8_t* b_st) {
  const uint8_t* ap = L.a_base + (int64_t)kt * kRowB;
  const uint8_t* bp = L.b_base + (int64_t)kt * kRowB;
  if (PART == 0) {
    copy16(ap, L.a_off0, a_st + L.lds_off);
    copy16(ap, L.a_off1, a_st + L.lds_off + 8192);
  } else if (PART == 1) {
    copy16(bp, L.b_off0, b_st + L.lds_off);
    copy16(bp, L.b_off1, b_st + L.lds_off + 8192);
  } else {
    copy16(bp, L.b_off2, b_st + L.lds_off + 16384);
    copy16(bp, L.b_off3, b_st + L.lds_off + 24576);
  }
}
__device__ __forceinline__ void load_stage(const TileLoader& L, int kt, uint8_t* a_st, uint8_t* b_st) {
  load_stage_part<0>(L, kt, a_st, b_st);
  load_stage_part<1>(L, kt, a_st, b_st);
  load_stage_part<2>(L, kt, a_st, b_st);
}

struct Frags {
  bf16x8_t a[2], b[2];
};

__device__ __forceinline__ void read_frags(Frags& f, const uint8_t* a_st, const uint8_t* b_st, int a_off0,
                                           int b_off0, int kk) {
#pragma unroll
  for (int c = 0; c < 2; ++c)
    f.a[c] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(a_st + ((a_off0 ^ (kk << 5)) + c * 4096)));
#pragma unroll
  for (int t = 0; t < 2; ++t)
    f.b[t] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(b_st + ((b_off0 ^ (kk << 5)) + t * 4096)));
}

__device__ __forceinline__ void mfma4(f32x16_t (&acc)[2][2], const Frags& f) {
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int t = 0; t < 2; ++t) acc[c][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[c], f.b[t], acc[c][t], 0, 0, 0);
}

// Wait until at most VM copies of this wave are in flight (and, if LGKM0, every LDS read has
// returned), then a barrier WITHOUT the memory fence of __syncthreads(): the fence would wait
// for every copy in flight, also the ones into stages that are not needed yet.  The wait is
// the s_waitcnt builtin (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt
// 11:8), which the compiler's own wait-count bookkeeping understands.
template <int VM, bool LGKM0>
__device__ __forceinline__ void wait_and_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((VM & 15) | ((VM >> 4) << 14) | (7 << 4) | ((LGKM0 ? 0 : 15) << 8));
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// One reduction step, 16 MFMAs.  On entry f0 holds the fragments of sub-step 0 of stage
// `rd`, read after the barrier that closed the previous step.  The step starts the copy two
// steps ahead, runs sub-steps 0..2 while reading one sub-step ahead, then closes: waits for
// the next stage's copy, passes the barrier, reads the next stage's first fragments and
// only then issues the last four MFMAs, so that the LDS latency after the barrier is
// covered by matrix work.  Each wave has 6 copy instructions in flight per stage.
template <bool STEADY>   // STEADY: kt + 2 < n_kt is known, no conditions in the step
__device__ __forceinline__ void step(f32x16_t (&acc)[2][2], Frags& f0, Frags& f1, const TileLoader& L, int kt,
                                     int n_kt, const uint8_t* a_rd, const uint8_t* b_rd, uint8_t* a_ld,
                                     uint8_t* b_ld, const uint8_t* a_nx, const uint8_t* b_nx, int a_off0,
                                     int b_off0) {
  const bool prefetch = STEADY || kt + 2 < n_kt;
  read_frags(f1, a_rd, b_rd, a_off0, b_off0, 1);
  mfma4(acc, f0);
  if (prefetch) load_stage_part<0>(L, kt + 2, a_ld, b_ld);
  read_frags(f0, a_rd, b_rd, a_off0, b_off0, 2);
  mfma4(acc, f1);
  if (prefetch) load_stage_part<1>(L, kt + 2, a_ld, b_ld);
  read_frags(f1, a_rd, b_rd, a_off0, b_off0, 3);
  mfma4(acc, f0);
  if (prefetch) load_stage_part<2>(L, kt + 2, a_ld, b_ld);
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);   // DS reads one sub-step ahead
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);   // MFMA
  }
  // every read of stage rd has completed before any wave may overwrite it (two steps on)
  if (STEADY || kt + 2 < n_kt) wait_and_barrier<6, true>();
  else wait_and_barrier<0, true>();
  if (STEADY || kt + 1 < n_kt) read_frags(f0, a_nx, b_nx, a_off0, b_off0, 0);
  mfma4(acc, f1);
  if (STEADY) {
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
  }
}

// unit -> (channel tile, token tile).  Units are ordered so that 32 consecutive ones (what an
// XCD's 32 CUs hold at a time) form 8 channel tiles x 4 token tiles: their W and x tiles
// together stream through that XCD's L2 once.
__device__ __forceinline__ void unit_to_tile(const ProjTiles& pt, int unit, int& ch_tile, int& tok_tile) {
  const int per_group = kTokGroup * pt.ch_tiles;
  const int full_groups = pt.tok_tiles / kTokGroup;
  int grp = unit / per_group;
  int gs = kTokGroup;
  if (grp >= full_groups) { grp = full_groups; gs = pt.tok_tiles - kTokGroup * full_groups; }
  const int local = unit - grp * per_group;
  ch_tile = local / gs;
  tok_tile = kTokGroup * grp + local % gs;
}

template <bool PER_HEAD>
__global__ __attribute__((amdgpu_flat_work_group_size(512, 512), amdgpu_waves_per_eu(2, 2)))
void qkv_project_kernel(ProjArgs a, ProjTiles pt) {
  // three stages of (W tile 16 KB, x tile 32 KB); the epilogue reuses the space
  __shared__ __attribute__((aligned(1024))) uint8_t lds[3 * (kStageA + kStageB)];
  uint8_t* const a_lds0 = lds;
  uint8_t* const b_lds0 = lds + kStageA;
  uint8_t* const a_lds1 = lds + (kStageA + kStageB);
  uint8_t* const b_lds1 = a_lds1 + kStageA;
  uint8_t* const a_lds2 = lds + 2 * (kStageA + kStageB);
  uint8_t* const b_lds2 = a_lds2 + kStageA;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, g = lane >> 5;
  const int wc = wave & 1, wt = wave >> 1;   // channel half, token quarter of the tile

  // Persistent work-groups, one per CU: a work-group walks its XCD's run of the unit list in
  // strides of the XCD's CU count.  Not ending between tiles lets a tile's output stores drain
  // under the next tile's reduction instead of holding up the hand-over of the CU.
  for (int idx = (int)(blockIdx.x / kXcds); idx < pt.per_xcd; idx += pt.wgs_per_xcd) {
  const int unit = (int)(blockIdx.x % kXcds) * pt.per_xcd + idx;
  if (unit >= pt.total) break;   // wave-uniform; the whole work-group leaves together
  int ch_tile, tok_tile;
  unit_to_tile(pt, unit, ch_tile, tok_tile);
  const int tok0 = tok_tile * kTileTok;

  TileLoader L;
  {
    const int l_row = lane >> 3, l_slot = lane & 7;
    const int f = (lane >> 4) | ((wave & 1) << 2);
    const uint32_t chunk_bytes = (uint32_t)((l_slot ^ f) * 16);
    const int row = 8 * wave + l_row;
    const int64_t a_row_bytes = (int64_t)a.c_in * 2, b_row_bytes = a.x_tok * 2;
    L.a_base = reinterpret_cast<const uint8_t*>(a.w) + (int64_t)ch_tile * kTileCh * a_row_bytes;
    L.b_base = reinterpret_cast<const uint8_t*>(a.x) + (int64_t)tok0 * b_row_bytes;
    L.a_off0 = (uint32_t)(row * a_row_bytes) + chunk_bytes;
    L.a_off1 = (uint32_t)((row + 64) * a_row_bytes) + chunk_bytes;
    const int last = a.n_tokens - 1 - tok0;   // >= 0
    L.b_off0 = (uint32_t)(min(row, last) * b_row_bytes) + chunk_bytes;
    L.b_off1 = (uint32_t)(min(row + 64, last) * b_row_bytes) + chunk_bytes;
    L.b_off2 = (uint32_t)(min(row + 128, last) * b_row_bytes) + chunk_bytes;
    L.b_off3 = (uint32_t)(min(row + 192, last) * b_row_bytes) + chunk_bytes;
    L.lds_off = wave * 1024;
  }
  // fragment read offsets: row (64*w? + n), 16-byte chunk 2*kk + g -> slot ((2kk+g) ^ ((n>>1)&7))
  const int fl = (n >> 1) & 7;
  const int a_off0 = (64 * wc + n) * kRowB + ((g ^ fl) << 4);
  const int b_off0 = (64 * wt + n) * kRowB + ((g ^ fl) << 4);

  f32x16_t acc[2][2];
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[c][t][i] = 0.f;

  const int n_kt = a.c_in / kStepK;
  Frags f0, f1;
  load_stage(L, 0, a_lds0, b_lds0);
  if (n_kt > 1) {
    load_stage(L, 1, a_lds1, b_lds1);
    wait_and_barrier<6, false>();
  } else {
    wait_and_barrier<0, false>();
  }
  read_frags(f0, a_lds0, b_lds0, a_off0, b_off0, 0);
  // lgkmcnt(0): enter the loop with nothing pending, so that the loop's own waits are counted
  // ones (a pending scalar load would make the compiler wait for every LDS read instead)
  __builtin_amdgcn_s_waitcnt(0xC07F);
  int kt = 0;
  for (; kt + 4 < n_kt; kt += 3) {   // steady state: every step prefetches two steps ahead
    step<true>(acc, f0, f1, L, kt, n_kt, a_lds0, b_lds0, a_lds2, b_lds2, a_lds1, b_lds1, a_off0, b_off0);
    step<true>(acc, f0, f1, L, kt + 1, n_kt, a_lds1, b_lds1, a_lds0, b_lds0, a_lds2, b_lds2, a_off0, b_off0);
    step<true>(acc, f0, f1, L, kt + 2, n_kt, a_lds2, b_lds2, a_lds1, b_lds1, a_lds0, b_lds0, a_off0, b_off0);
  }
  for (; kt < n_kt; kt += 3) {       // the last (up to four) steps
    step<false>(acc, f0, f1, L, kt, n_kt, a_lds0, b_lds0, a_lds2, b_lds2, a_lds1, b_lds1, a_off0, b_off0);
    if (kt + 1 >= n_kt) break;
    step<false>(acc, f0, f1, L, kt + 1, n_kt, a_lds1, b_lds1, a_lds0, b_lds0, a_lds2, b_lds2, a_off0, b_off0);
    if (kt + 2 >= n_kt) break;
    step<false>(acc, f0, f1, L, kt + 2, n_kt, a_lds2, b_lds2, a_lds1, b_lds1, a_lds0, b_lds0, a_off0, b_off0);
  }

  // ------------------------------------------------------------------ epilogue
  // acc[c][t][i]: token tok0 + 64*wt + 32*t + n, channel 64*wc + 32*c + 8*(i/4) + 4*g + i%4 of the head.
  // The closing barrier of the last step has passed: every wave is done with the stages.  The
  // LDS now holds, in turn, the (cos, sin) rows of the tile's 256 tokens (gathered with pairs
  // on the lane axis, where a token's position is wave-uniform and its 64 pairs are three
  // contiguous runs of the tables, then read back with tokens on the lane axis at constant
  // offsets), the sums of squares, and the bf16 output tile, which leaves in whole 256-byte
  // (token, head) rows.
  uint8_t* const out_lds = lds;                                     // [256][kOutRowB]
  uint8_t* const ang_lds = lds;                                     // [256][kAngRowB]: 64 x (cos, sin)
  float* const ss_lds = reinterpret_cast<float*>(lds + kAngBytes);  // [wc][wt][t][32]
  const int which = ch_tile / a.n_heads;   // 0: q, 1: k, 2: v
  const int head = ch_tile - which * a.n_heads;
  // bias and gain of the lane's 32 channels: all loads issued together, ahead of their use
  float4 gv[2][4];
  if (which != 2) {
    const float* gp = (which == 0 ? a.gain_q : a.gain_k) + head * kHeadDim + 64 * wc + 4 * g;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int b = 0; b < 4; ++b) gv[c][b] = *reinterpret_cast<const float4*>(gp + 32 * c + 8 * b);
  }
  if (a.bias) {
    const float* bp = a.bias + (int64_t)ch_tile * kTileCh + 64 * wc + 4 * g;
    float4 bv[2][4];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int b = 0; b < 4; ++b) bv[c][b] = *reinterpret_cast<const float4*>(bp + 32 * c + 8 * b);
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          acc[c][t][4 * b + 0] += bv[c][b].x; acc[c][t][4 * b + 1] += bv[c][b].y;
          acc[c][t][4 * b + 2] += bv[c][b].z; acc[c][t][4 * b + 3] += bv[c][b].w;
        }
  }
  uint32_t packed[2][2][4][2];      // [t][c][b][pair of the 4 channels]
  uint32_t packed_lo[2][2][4][2];   // row-wide norm: bf16 of what the first rounding dropped

  if (which == 2) {   // v: one rounding
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          packed[t][c][b][0] = pack_bf16x2(acc[c][t][4 * b + 0], acc[c][t][4 * b + 1]);
          packed[t][c][b][1] = pack_bf16x2(acc[c][t][4 * b + 2], acc[c][t][4 * b + 3]);
        }
  } else {
    const int p_t = a.tl.pairs_t, p_h = a.tl.pairs_h, p_w = a.tl.pairs_w, p_th = p_t + p_h;
    const float2* tab2 = reinterpret_cast<const float2*>(a.table);
    // ---- gather: wave w fetches the rows of tile tokens 32w .. 32w+31.  Positions are decoded
    // with tokens on the lane axis; for the fetch the lane axis is the pair index (a token's
    // 64 pairs are three contiguous runs of the tables) and token rr's table row offsets are
    // broadcast from lane rr.  Lane j needs exactly one of the three offsets.
    {
      const int last_tok = a.n_tokens - 1;
      const int ig = a.token_offset + min(tok0 + 32 * wave + n, last_tok);   // past the end: last token's position
      const int hw = a.grid_h * a.grid_w;
      const int pf = ig / hw;
      const int rem = ig - pf * hw;
      const int ph = rem / a.grid_w;
      const int pw = rem - ph * a.grid_w;
      const int row_t = (a.start_frame + pf) * p_t, row_h = ph * p_h, row_w = pw * p_w;
      const int j = lane;
      const bool is_t = j < p_t, is_h = !is_t && j < p_th;
      const int m_t = is_t ? -1 : 0, m_h = is_h ? -1 : 0, m_w = (is_t || is_h) ? 0 : -1;
      const int cb = is_t ? (int)(a.tl.off_t / 2) + j
                          : is_h ? (int)(a.tl.off_h / 2) + (j - p_t) : (int)(a.tl.off_w / 2) + (j - p_th);
      uint8_t* dst = ang_lds + (32 * wave) * kAngRowB + lane * 8;
      float2 row[32];
#pragma unroll
      for (int rr = 0; rr < 32; ++rr) {
        const int st = __builtin_amdgcn_readlane(row_t, rr), sh = __builtin_amdgcn_readlane(row_h, rr),
                  sw = __builtin_amdgcn_readlane(row_w, rr);
        row[rr] = tab2[cb + ((st & m_t) | (sh & m_h) | (sw & m_w))];
      }
#pragma unroll
      for (int rr = 0; rr < 32; ++rr) *reinterpret_cast<float2*>(dst + rr * kAngRowB) = row[rr];
    }
    // ---- sums of squares over the head: lane-local, the other half of the wave, the other wave
    float tot[2];
    {
      float ss[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        float sq = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int i = 0; i < 16; ++i) sq = fmaf(acc[c][t][i], acc[c][t][i], sq);
        ss[t] = sum_across_halves(sq);
      }
      if (g == 0) {
        ss_lds[((wc * 4 + wt) * 2 + 0) * 32 + n] = ss[0];
        ss_lds[((wc * 4 + wt) * 2 + 1) * 32 + n] = ss[1];
      }
      __syncthreads();
#pragma unroll
      for (int t = 0; t < 2; ++t)
        tot[t] = ss_lds[((0 * 4 + wt) * 2 + t) * 32 + n] + ss_lds[((1 * 4 + wt) * 2 + t) * 32 + n];
    }
    float r[2];
    if (PER_HEAD) {
      r[0] = 1.0f / sqrtf(tot[0] * (1.0f / kHeadDim) + a.eps);
      r[1] = 1.0f / sqrtf(tot[1] * (1.0f / kHeadDim) + a.eps);
    } else {
      r[0] = r[1] = 1.0f;
      if (wc == 0 && g == 0) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int token = tok0 + 64 * wt + 32 * t + n;
          if (token < a.n_tokens) a.sumsq[((int64_t)which * a.n_tokens + token) * a.n_heads + head] = tot[t];
        }
      }
    }
    // ---- normalise, gain, rotate; the lane's pairs are 32*wc + 2*g + (16*c + 4*b + e)
    const uint8_t* ang_lane = ang_lds + (64 * wt + n) * kAngRowB + (32 * wc + 2 * g) * 8;
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const float4 cs = *reinterpret_cast<const float4*>(ang_lane + 32 * t * kAngRowB + (16 * c + 4 * b) * 8);
          const float xa0 = acc[c][t][4 * b + 0] * r[t] * gv[c][b].x, xb0 = acc[c][t][4 * b + 1] * r[t] * gv[c][b].y;
          const float xa1 = acc[c][t][4 * b + 2] * r[t] * gv[c][b].z, xb1 = acc[c][t][4 * b + 3] * r[t] * gv[c][b].w;
          const float z0 = xa0 * cs.x - xb0 * cs.y, z1 = xa0 * cs.y + xb0 * cs.x;
          const float z2 = xa1 * cs.z - xb1 * cs.w, z3 = xa1 * cs.w + xb1 * cs.z;
          const uint32_t h0 = pack_bf16x2(z0, z1), h1 = pack_bf16x2(z2, z3);
          packed[t][c][b][0] = h0;
          packed[t][c][b][1] = h1;
          if (!PER_HEAD) {
            packed_lo[t][c][b][0] = pack_bf16x2(z0 - bf16_lo(h0), z1 - bf16_hi(h0));
            packed_lo[t][c][b][1] = pack_bf16x2(z2 - bf16_lo(h1), z3 - bf16_hi(h1));
          }
        }
      }
    __syncthreads();   // every wave has read its angles: the output tile may overwrite them
  }

  // ---- the tile leaves in whole token rows: 16 lanes x 16 B = the 256 bytes of one (token, head)
  {
    uint8_t* out_lane = out_lds + (64 * wt + n) * kOutRowB + (64 * wc + 4 * g) * 2;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int b = 0; b < 4; ++b)
          *reinterpret_cast<uint2*>(out_lane + 32 * t * kOutRowB + (32 * c + 8 * b) * 2) =
              make_uint2(packed[t][c][b][0], packed[t][c][b][1]);
  }
  __syncthreads();
  {
    uint16_t* base;
    int64_t tstride;
    if (which == 0) { base = a.q_out + (int64_t)head * a.qo_head; tstride = a.qo_tok; }
    else {
      base = (which == 1 ? a.k_cache : a.v_cache) + a.dst_token * a.c_tok + (int64_t)head * a.c_head;
      tstride = a.c_tok;
    }
    const int chunk = tid & 15;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = (tid >> 4) + 32 * it;
      const int token = tok0 + row;
      if (token < a.n_tokens)
        *reinterpret_cast<uint4*>(base + (int64_t)token * tstride + chunk * 8) =
            *reinterpret_cast<const uint4*>(out_lds + row * kOutRowB + chunk * 16);
    }
  }
  __syncthreads();   // the output tile has been read: the next tile's copies may overwrite it
  if (!PER_HEAD && which != 2) {
    // the low parts take the same way out, into the workspace rows [which][token][head][128]
    uint8_t* out_lane = out_lds + (64 * wt + n) * kOutRowB + (64 * wc + 4 * g) * 2;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int b = 0; b < 4; ++b)
          *reinterpret_cast<uint2*>(out_lane + 32 * t * kOutRowB + (32 * c + 8 * b) * 2) =
              make_uint2(packed_lo[t][c][b][0], packed_lo[t][c][b][1]);
    __syncthreads();
    uint16_t* base = a.resid + ((int64_t)which * a.n_tokens * a.n_heads + head) * kHeadDim;
    const int64_t tstride = (int64_t)a.n_heads * kHeadDim;
    const int chunk = tid & 15;
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = (tid >> 4) + 32 * it;
      const int token = tok0 + row;
      if (token < a.n_tokens)
        *reinterpret_cast<uint4*>(base + (int64_t)token * tstride + chunk * 8) =
            *reinterpret_cast<const uint4*>(out_lds + row * kOutRowB + chunk * 16);
    }
    __syncthreads();
  }
  }   // next unit
}

// Second pass of the row-wide norm: one wave per (tensor, token) sums the per-head sums of
// squares in a fixed order, and replaces the stored high part of rotate(gain * y) by the bf16
// rounding of (high + low) / rms.
constexpr int kScaleWaves = 4;
__global__ __launch_bounds__(64 * kScaleWaves) void scale_rows_kernel(ProjArgs a) {
  const int lane = threadIdx.x & 63;
  const int tok = blockIdx.y * kScaleWaves + (threadIdx.x >> 6);
  if (tok >= a.n_tokens) return;
  const int which = blockIdx.x;   // 0: q, 1: k
  float s = lane < a.n_heads ? a.sumsq[((int64_t)which * a.n_tokens + tok) * a.n_heads + lane] : 0.f;
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
  const float r = 1.0f / sqrtf(s * (1.0f / (float)(a.n_heads * kHeadDim)) + a.eps);
  uint16_t* row = which == 0 ? a.q_out + (int64_t)tok * a.qo_tok : a.k_cache + (a.dst_token + tok) * a.c_tok;
  const int64_t hstride = which == 0 ? a.qo_head : a.c_head;
  const uint16_t* lo_row = a.resid + ((int64_t)which * a.n_tokens + tok) * a.n_heads * kHeadDim;
  const int n_chunks = a.n_heads * 16;
  for (int c = lane; c < n_chunks; c += 64) {
    uint4* p = reinterpret_cast<uint4*>(row + (int64_t)(c >> 4) * hstride + (c & 15) * 8);
    uint4 u = *p;
    const uint4 w = *reinterpret_cast<const uint4*>(lo_row + (int64_t)c * 8);
    u.x = pack_bf16x2((bf16_lo(u.x) + bf16_lo(w.x)) * r, (bf16_hi(u.x) + bf16_hi(w.x)) * r);
    u.y = pack_bf16x2((bf16_lo(u.y) + bf16_lo(w.y)) * r, (bf16_hi(u.y) + bf16_hi(w.y)) * r);
    u.z = pack_bf16x2((bf16_lo(u.z) + bf16_lo(w.z)) * r, (bf16_hi(u.z) + bf16_hi(w.z)) * r);
    u.w = pack_bf16x2((bf16_lo(u.w) + bf16_lo(w.w)) * r, (bf16_hi(u.w) + bf16_hi(w.w)) * r);
    *p = u;
  }
}

}  // namespace

// fp32 sums of squares [2][tokens][heads], rounded up to 256 bytes, then the bf16 low parts
// [2][tokens][heads][128]
static size_t sumsq_bytes(int n_tokens, int n_heads) {
  return (((size_t)2 * n_tokens * n_heads * sizeof(float)) + 255) & ~(size_t)255;
}
size_t project_workspace_bytes(int n_tokens, int n_heads, bool per_head_norm) {
  if (per_head_norm || n_tokens <= 0) return 0;
  return sumsq_bytes(n_tokens, n_heads) + (size_t)2 * n_tokens * n_heads * kHeadDim * sizeof(uint16_t);
}

hipError_t launch_project(const ProjArgs& a_in, hipStream_t st) {
  ProjArgs a = a_in;
  if (!a.per_head_norm)
    a.resid = reinterpret_cast<uint16_t*>(reinterpret_cast<uint8_t*>(a.sumsq) + sumsq_bytes(a.n_tokens, a.n_heads));
  ProjTiles pt;
  pt.ch_tiles = 3 * a.n_heads;
  pt.tok_tiles = (a.n_tokens + kTileTok - 1) / kTileTok;
  pt.total = pt.ch_tiles * pt.tok_tiles;
  pt.per_xcd = (pt.total + kXcds - 1) / kXcds;
  pt.wgs_per_xcd = pt.per_xcd < 32 ? pt.per_xcd : 32;
  const dim3 grid(pt.wgs_per_xcd * kXcds), block(512);
  if (a.per_head_norm) hipLaunchKernelGGL(qkv_project_kernel<true>, grid, block, 0, st, a, pt);
  else hipLaunchKernelGGL(qkv_project_kernel<false>, grid, block, 0, st, a, pt);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.per_head_norm) return e;
  hipLaunchKernelGGL(scale_rows_kernel, dim3(2, (a.n_tokens + kScaleWaves - 1) / kScaleWaves),
                     dim3(64 * kScaleWaves), 0, st, a);
  return hipGetLastError();
}

}  // namespace crope
