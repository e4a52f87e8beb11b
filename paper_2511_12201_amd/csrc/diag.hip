// Measurement aids behind the C ABI; none of them is part of the attention path.
//
//  * calibration_copy_kernel: a plain copy of a known number of bytes.  The HBM byte counters of
//    the profiler (FETCH_SIZE, WRITE_SIZE) are scaled by what they report for this kernel.
//  * mfma_rate_kernel: register-resident bf16 32x32x16 MFMAs and nothing else, with constant or
//    with pseudo-random operands.  The sustained rate with random operands is what the chip's
//    power management leaves of the nominal matrix-core peak for operands that toggle like real
//    data; the attention kernels are priced against both figures.  A third mode idles the matrix cores a
//    third of the time (all wavefronts of a workgroup sleep together after every 32 MFMAs): if the clock then
//    rises, the full-duty rate is set by the power limit and not by a fixed clock.
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

__global__ __launch_bounds__(256) void calibration_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                               long long n16) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__device__ __forceinline__ unsigned mix32(unsigned x) {
  x ^= x >> 16;
  x *= 0x7feb352dU;
  x ^= x >> 15;
  x *= 0x846ca68bU;
  x ^= x >> 16;
  return x;
}

constexpr int kRateFrags = 8;
constexpr int kRateMfmaPerIter = 4 * kRateFrags;

template <int RANDOM>
__global__ __launch_bounds__(512, 2) void mfma_rate_kernel(float* sink, long long* clocks, int iters) {
  bf16x8 a[kRateFrags], b[kRateFrags];
#pragma unroll
  for (int f = 0; f < kRateFrags; ++f)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (RANDOM) {
        const unsigned h1 = mix32(threadIdx.x * 977u + f * 131u + j * 17u + blockIdx.x * 7919u), h2 = mix32(h1 + 12345u);
        a[f][j] = (__bf16)(((h1 & 0xffff) / 32768.0f - 1.0f) * 2.0f);
        b[f][j] = (__bf16)(((h2 & 0xffff) / 32768.0f - 1.0f) * 2.0f);
      } else {
        a[f][j] = (__bf16)1.0f;
        b[f][j] = (__bf16)0.5f;
      }
    }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int r = 0; r < 16; ++r) c0[r] = c1[r] = c2[r] = c3[r] = 0.f;
  const long long t0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int f = 0; f < kRateFrags; ++f) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[f], b[f], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(f + 1) % kRateFrags], b[f], c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(f + 2) % kRateFrags], b[f], c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(f + 3) % kRateFrags], b[f], c3, 0, 0, 0);
    }
    if (RANDOM == 2) {                         // 2 x 32 MFMAs x 32 cycles per SIMD, then 17 x 64 idle cycles: 65 % duty
      __syncthreads();
      __builtin_amdgcn_s_sleep(17);
    }
    if (RANDOM && (it & 63) == 63) {           // keep the accumulators finite
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        c0[r] *= 1e-3f;
        c1[r] *= 1e-3f;
        c2[r] *= 1e-3f;
        c3[r] *= 1e-3f;
      }
    }
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  sink[(long long)blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    clocks[0] = t1 - t0;      // shader clock ticks
    clocks[1] = w1 - w0;      // constant 100 MHz ticks
  }
}

}  // namespace

int run_calibration_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  const long long n16 = (long long)(bytes / 16);
  hipLaunchKernelGGL(calibration_copy_kernel, dim3(256 * 8), dim3(256), 0, st, static_cast<const u32x4*>(src),
                     static_cast<u32x4*>(dst), n16);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

int run_mfma_rate(int random_operands, int iters, double* tflops, double* shader_mhz) {
  const int blocks = 256, threads = 512;
  float* sink = nullptr;
  long long* clocks = nullptr;
  OMNI_HIP_CHECK(hipMalloc(&sink, sizeof(float) * blocks * threads));
  if (hipMalloc(&clocks, 2 * sizeof(long long)) != hipSuccess) {
    (void)hipFree(sink);
    OMNI_FAIL(OMNI_ERR_HIP, "hipMalloc failed");
  }
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  auto launch = [&](int n) {
    if (random_operands == 2) hipLaunchKernelGGL(mfma_rate_kernel<2>, dim3(blocks), dim3(threads), 0, 0, sink, clocks, n);
    else if (random_operands) hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(blocks), dim3(threads), 0, 0, sink, clocks, n);
    else hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(blocks), dim3(threads), 0, 0, sink, clocks, n);
  };
  launch(16);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0, 0);
  launch(iters);
  (void)hipEventRecord(e1, 0);
  const hipError_t err = hipEventSynchronize(e1);
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  long long h[2] = {0, 1};
  (void)hipMemcpy(h, clocks, sizeof(h), hipMemcpyDeviceToHost);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  (void)hipFree(clocks);
  if (err != hipSuccess) OMNI_FAIL(OMNI_ERR_HIP, "mfma rate kernel: %s", hipGetErrorString(err));
  const double flops = (double)iters * kRateMfmaPerIter * 32768.0 * (threads / 64) * blocks;
  *tflops = flops / ((double)ms * 1e-3) / 1e12;
  *shader_mhz = (double)h[0] / ((double)h[1] / 100.0);
  return OMNI_OK;
}

}  // namespace omni
