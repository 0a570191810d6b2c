// libfa2_probe: MFMA-only throughput and engine clock on caller-supplied operands (see include/fa2_probe.h).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fa2_probe.h"

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(const u32x4* __restrict__ operands,
                                                            unsigned long long* __restrict__ ticks,
                                                            float* __restrict__ sink, int iters) {
  u32x4 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[threadIdx.x * 8 + i];
    b[i] = operands[threadIdx.x * 8 + 4 + i];
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        if (DT == 0)
          acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[(i + n) & 3]),
                                                          __builtin_bit_cast(f16x8, b[i]), acc[n], 0, 0, 0);
        else
          acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[(i + n) & 3]),
                                                           __builtin_bit_cast(bf16x8, b[i]), acc[n], 0, 0, 0);
      }
  }
  float res = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int v = 0; v < 16; ++v) res += acc[n][v];
  sink[blockIdx.x * 256 + threadIdx.x] = res;  // also orders the counters below after the last MFMA's result
  const unsigned long long c1 = clock64(), w1 = wall_clock64();
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    ticks[0] = c0;
    ticks[1] = c1;
    ticks[2] = w0;
    ticks[3] = w1;
  }
}

}  // namespace

extern "C" int fa2_probe_mfma(const void* operands, unsigned long long* ticks, float* sink, int dtype, int iters,
                              void* stream) {
  if (operands == nullptr || ticks == nullptr || sink == nullptr || iters < 1) return -1;
  if ((reinterpret_cast<uintptr_t>(operands) & 15) || (reinterpret_cast<uintptr_t>(ticks) & 7) ||
      (reinterpret_cast<uintptr_t>(sink) & 3))
    return -1;
  if (dtype != 0 && dtype != 1) return -1;
  const u32x4* ops = static_cast<const u32x4*>(operands);
  void* args[] = {&ops, &ticks, &sink, &iters};
  const void* fn = dtype == 0 ? reinterpret_cast<const void*>(mfma_probe_kernel<0>)
                              : reinterpret_cast<const void*>(mfma_probe_kernel<1>);
  const hipError_t err = hipLaunchKernel(fn, dim3(FA2_PROBE_WORKGROUPS), dim3(256), args, 0, static_cast<hipStream_t>(stream));
  return err == hipSuccess ? 0 : -3;
}
