// Measurement aids for the benchmark, NOT part of libcrope.so: two kernels that measure what
// this GPU sustains on the resources the hot-path kernels are bound by, so that their rates
// can be read against a measured ceiling next to the datasheet one.
//
//   ceiling_mfma:  every CU runs 8 waves (two per SIMD) that do nothing but issue
//                  v_mfma_f32_32x32x16_bf16 on random bf16 operands held in registers;
//                  consecutive instructions use different operands and four independent
//                  accumulators, so neither data dependencies nor memory limit the loop.
//   ceiling_copy:  a plain device-to-device copy, 16 bytes per lane, one launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kMfmaPerIter = 16;
constexpr int kWavesPerGroup = 4;
constexpr int kGroups = 512;   // 256 CUs x 2 work-groups of 4 waves

__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void mfma_loop_kernel(const uint4* __restrict__ operands, float* __restrict__ sink, int iters) {
  const int lane = threadIdx.x & 63;
  // 16 fragments per lane (8 A, 8 B), different for every wave of a work-group
  bf16x8_t a[8], b[8];
  const uint4* src = operands + ((threadIdx.x >> 6) * 16) * 64 + lane;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = __builtin_bit_cast(bf16x8_t, src[i * 64]);
    b[i] = __builtin_bit_cast(bf16x8_t, src[(8 + i) * 64]);
  }
  f32x16_t acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < kMfmaPerIter; ++m)
      acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(m * 3) & 7], b[(m + (m >> 3)) & 7], acc[m & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  if (s == 12345.678f) sink[blockIdx.x * blockDim.x + threadIdx.x] = s;   // keeps the loop alive
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

}  // namespace

extern "C" {

// bytes of random bf16 operands the MFMA loop reads once at its start
__attribute__((visibility("default"))) size_t ceiling_mfma_operand_bytes(void) {
  return (size_t)kWavesPerGroup * 16 * 64 * sizeof(uint4);
}

// floating-point operations of one launch with `iters` loop iterations
__attribute__((visibility("default"))) double ceiling_mfma_flops(int iters) {
  return (double)kGroups * kWavesPerGroup * (double)iters * kMfmaPerIter * (2.0 * 32 * 32 * 16);
}

// operands: device, ceiling_mfma_operand_bytes() of bf16 values; sink: device, >= 512*256 floats
// (never written in practice).  Returns the hipError_t of the launch.
__attribute__((visibility("default"))) int ceiling_mfma_launch(const void* operands, float* sink, int iters, void* stream) {
  if (!operands || !sink || iters <= 0) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(kGroups), dim3(64 * kWavesPerGroup), 0, (hipStream_t)stream,
                     (const uint4*)operands, sink, iters);
  return (int)hipGetLastError();
}

// copies `bytes` (a multiple of 16, both pointers 16-byte aligned) from src to dst on the device
__attribute__((visibility("default"))) int ceiling_copy_launch(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || bytes == 0 || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
    return (int)hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  const size_t blocks = (n16 + 255) / 256;
  if (blocks > 0x7fffffffu) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)dst,
                     (const uint4*)src, n16);
  return (int)hipGetLastError();
}

}  // extern "C"
