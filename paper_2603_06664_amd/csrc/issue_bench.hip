// Issue-level microbenchmark for gfx950, a measurement aid (not part of libcrope.so): what does
// it cost a wave to issue other instructions between its bf16 MFMAs?  Every kernel is a loop of
// eight independent v_mfma_f32_32x32x16_bf16 (eight accumulators, random bf16 operands in
// registers) with a chosen number of v_fma_f32, v_exp_f32, ds_read_b128 and ds_read_b64_tr_b16
// behind each MFMA, written as volatile inline assembly so that the order is exactly as given.
// One work-group per CU (96 KB of LDS each) with 4 waves (one per SIMD) or 8 (two per SIMD).
// Reported per case: shader clocks per MFMA per wave (s_memtime), the effective shader clock
// (s_memtime against the constant 100 MHz s_memrealtime) and the aggregate MFMA rate.  With
// two waves per SIMD the placement line shows how the hardware shares a SIMD between them.
//
//   hipcc --offload-arch=gfx950 -O3 issue_bench.hip -o issue_bench && ./issue_bench
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

// per MFMA: KF v_fma_f32, KE v_exp_f32, KL ds_read_b128, KT ds_read_b64_tr_b16 (x10: tenths, e.g. 15 = 1.5 per MFMA)
template <int KF10, int KE10, int KL10, int KT10, bool AGPR>
__global__ __attribute__((amdgpu_flat_work_group_size(64, 512)))
void k(const uint4* data, float* out, unsigned long long* t, int iters) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds[96 * 1024];
  const int lane = threadIdx.x & 63;
  for (int i = threadIdx.x; i < 96 * 1024 / 16; i += blockDim.x) reinterpret_cast<uint4*>(lds)[i] = data[i % 4096];
  __syncthreads();
  bf16x8 a[8], b[8];
  for (int j = 0; j < 8; ++j) { a[j] = __builtin_bit_cast(bf16x8, data[(threadIdx.x * 16 + j) % 4096]); b[j] = __builtin_bit_cast(bf16x8, data[(threadIdx.x * 16 + 8 + j + blockIdx.x) % 4096]); }
  f32x16 acc[8];
  for (int j = 0; j < 8; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  float x[16]; for (int i = 0; i < 16; ++i) x[i] = 0.001f * (threadIdx.x + i);
  float e[8]; for (int i = 0; i < 8; ++i) e[i] = -0.01f * (lane + i);
  f32x4 l128[4]; s16x4 ltr[4];
  for (int i = 0; i < 4; ++i) { l128[i] = f32x4{0, 0, 0, 0}; ltr[i] = s16x4{0, 0, 0, 0}; }
  const int g = lane >> 5, i16 = lane & 15, mh = (lane >> 4) & 1, kk = i16 >> 2, cc = i16 & 3, n = lane & 31;
  const uint32_t lbase = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) void*)lds) + (threadIdx.x >> 6) * 8192;
  const uint32_t a128 = lbase + n * 256 + ((g ^ (n & 15)) << 4);
  const uint32_t atr = lbase + (4 * g + kk) * 256 + (((0 ^ kk) + 4 * mh) << 5) + cc * 8;
  const float c1 = 0.9999f, c2 = 1e-7f;
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      if (AGPR) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[m]) : "v"(a[m]), "v"(b[(m + 3) & 7]));
      else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[m]) : "v"(a[m]), "v"(b[(m + 3) & 7]));
      const int nl = ((m + 1) * KL10) / 10 - (m * KL10) / 10, ntr = ((m + 1) * KT10) / 10 - (m * KT10) / 10;
      const int nf = ((m + 1) * KF10) / 10 - (m * KF10) / 10, ne = ((m + 1) * KE10) / 10 - (m * KE10) / 10;
#pragma unroll
      for (int r = 0; r < 4; ++r) if (r < nl) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(l128[(m + r) & 3]) : "v"(a128), "n"(2048) : "memory");
#pragma unroll
      for (int r = 0; r < 4; ++r) if (r < ntr) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(ltr[(m + r) & 3]) : "v"(atr), "n"(2048) : "memory");
#pragma unroll
      for (int r = 0; r < 8; ++r) if (r < nf) { const int i = (m * 5 + r) & 15; asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(c1), "v"(c2)); }
#pragma unroll
      for (int r = 0; r < 4; ++r) if (r < ne) { const int i = (m + r) & 7; asm volatile("v_exp_f32 %0, %0" : "+v"(e[i])); }
    }
    if (KL10 || KT10) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  const unsigned long long c1c = clock64(), w1 = wall_clock64();
  float s = 0.f;
  for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][7];
  for (int i = 0; i < 16; ++i) s += x[i];
  for (int i = 0; i < 8; ++i) s += e[i];
  for (int i = 0; i < 4; ++i) s += l128[i][0] + (float)ltr[i][0];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (lane == 0) {
    const int w = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    unsigned hw, xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    t[w * 2] = c1c - c0; t[w * 2 + 1] = w1 - w0;
    t[8192 + w * 4] = w0; t[8192 + w * 4 + 1] = w1; t[8192 + w * 4 + 2] = hw; t[8192 + w * 4 + 3] = xcc;
  }
}

struct Res { double cyc_per_mfma, ghz, tflops; };
template <int KF10, int KE10, int KL10, int KT10, bool AGPR>
Res run(const uint4* d, float* o, unsigned long long* t, int waves_per_cu, int iters) {
  const int blocks = 256, threads = 64 * waves_per_cu;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  hipLaunchKernelGGL((k<KF10, KE10, KL10, KT10, AGPR>), dim3(blocks), dim3(threads), 0, 0, d, o, t, iters / 10);   // warm
  CK(hipEventRecord(e0));
  hipLaunchKernelGGL((k<KF10, KE10, KL10, KT10, AGPR>), dim3(blocks), dim3(threads), 0, 0, d, o, t, iters);
  CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1));
  const int nw = blocks * waves_per_cu;
  std::vector<unsigned long long> ht(nw * 2); CK(hipMemcpy(ht.data(), t, nw * 16, hipMemcpyDeviceToHost));
  double c = 0, w = 0; for (int i = 0; i < nw; ++i) { c += ht[2 * i]; w += ht[2 * i + 1]; }
  if (waves_per_cu == 8 && KF10 + KE10 + KL10 + KT10 == 0) {
    std::vector<unsigned long long> hp(nw * 4); CK(hipMemcpy(hp.data(), t + 8192, nw * 32, hipMemcpyDeviceToHost));
    unsigned long long tmin = ~0ull; for (int i = 0; i < nw; ++i) tmin = std::min(tmin, hp[4 * i]);
    // waves per (xcc, se, sh?, cu, simd)
    std::vector<int> cnt(1 << 20, 0); int maxc = 0; int hist[16] = {0};
    double smin = 1e30, smax = 0, emin = 1e30, emax = 0;
    for (int i = 0; i < nw; ++i) {
      unsigned hw = (unsigned)hp[4 * i + 2], xcc = (unsigned)hp[4 * i + 3] & 0xf;
      unsigned simd = (hw >> 4) & 3, cu = (hw >> 8) & 0xf, sh = (hw >> 12) & 1, se = (hw >> 13) & 7;
      unsigned key = (((xcc * 8 + se) * 2 + sh) * 16 + cu) * 4 + simd;
      cnt[key]++;
      double st = (hp[4 * i] - tmin) / 100.0, en = (hp[4 * i + 1] - tmin) / 100.0;
      smin = std::min(smin, st); smax = std::max(smax, st); emin = std::min(emin, en); emax = std::max(emax, en);
    }
    int used = 0; for (int c : cnt) if (c) { ++used; hist[std::min(c, 15)]++; }
    printf("   placement: %d SIMDs used; waves per SIMD histogram:", used); for (int i = 1; i < 8; ++i) printf(" %d:%d", i, hist[i]);
    printf("; starts %.1f..%.1f us, ends %.1f..%.1f us, kernel %.1f us\n", smin, smax, emin, emax, ms * 1e3);
  }
  Res r; r.cyc_per_mfma = c / nw / iters / 8.0; r.ghz = c / w * 0.1; r.tflops = (double)nw * iters * 8 * 32768.0 / ms / 1e9;
  return r;
}
#define RUN(KF, KE, KL, KT, AG, W) do { Res r = run<KF, KE, KL, KT, AG>(d, o, t, W, 40000); \
  printf("waves/CU %d %s  per MFMA: fma %.1f exp %.1f ds128 %.1f dstr %.1f -> %6.1f clk per MFMA per wave, %5.2f GHz, %6.0f TFLOP/s\n", W, AG ? "agpr" : "vgpr", KF / 10.0, KE / 10.0, KL / 10.0, KT / 10.0, r.cyc_per_mfma, r.ghz, r.tflops); fflush(stdout); } while (0)
int main() {
  uint4* d; CK(hipMalloc(&d, 4096 * 16)); float* o; CK(hipMalloc(&o, 256 * 512 * 4));
  unsigned long long* t; CK(hipMalloc(&t, (8192 + 4096 * 4) * 8));
  std::vector<uint4> h(4096); unsigned s = 1;
  auto r16 = [&]() { s = s * 1664525u + 1013904223u; union { float f; unsigned u; } cv; cv.f = ((s >> 8) & 0xffff) / 8192.0f - 4.0f; return cv.u >> 16; };
  for (auto& x : h) { x.x = r16() | (r16() << 16); x.y = r16() | (r16() << 16); x.z = r16() | (r16() << 16); x.w = r16() | (r16() << 16); }
  CK(hipMemcpy(d, h.data(), 4096 * 16, hipMemcpyHostToDevice));
  // one wave per SIMD
  RUN(0, 0, 0, 0, false, 4); RUN(0, 0, 0, 0, true, 4);
  RUN(10, 0, 0, 0, false, 4); RUN(20, 0, 0, 0, false, 4); RUN(40, 0, 0, 0, false, 4); RUN(60, 0, 0, 0, false, 4);
  RUN(70, 0, 0, 0, false, 4); RUN(80, 0, 0, 0, false, 4);
  RUN(0, 10, 0, 0, false, 4); RUN(0, 20, 0, 0, false, 4); RUN(0, 30, 0, 0, false, 4); RUN(0, 40, 0, 0, false, 4);
  RUN(0, 0, 5, 0, false, 4); RUN(0, 0, 10, 0, false, 4); RUN(0, 0, 20, 0, false, 4);
  RUN(0, 0, 0, 10, false, 4); RUN(0, 0, 0, 20, false, 4); RUN(0, 0, 0, 40, false, 4);
  RUN(30, 10, 5, 10, false, 4);        // the attention kernel's mix per MFMA with the per-score fma and maximum
  RUN(10, 10, 5, 10, false, 4);        // ... with the softmax factor folded into q
  RUN(10, 10, 3, 5, false, 4);         // ... and 64 queries per wave (half the fragment reads)
  // two waves per SIMD
  RUN(0, 0, 0, 0, false, 8);
  RUN(20, 0, 0, 0, false, 8); RUN(40, 0, 0, 0, false, 8); RUN(60, 0, 0, 0, false, 8);
  RUN(0, 10, 0, 0, false, 8); RUN(0, 20, 0, 0, false, 8);
  RUN(0, 0, 5, 0, false, 8); RUN(0, 0, 10, 0, false, 8); RUN(0, 0, 0, 10, false, 8); RUN(0, 0, 0, 20, false, 8);
  RUN(0, 0, 5, 10, false, 8);
  RUN(30, 10, 5, 10, false, 8);
  RUN(10, 10, 5, 10, false, 8);
  return 0;
}
