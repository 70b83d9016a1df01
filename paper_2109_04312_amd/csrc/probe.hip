// Measurement aid, not part of the computation: a kernel that does nothing but issue independent
// 32x32x16 bf16 MFMAs (the instruction the attention and projection kernels use), so that the
// benchmark can time what the matrix cores of the box it runs on deliver under sustained load,
// next to the nominal peak.
#include <hip/hip_runtime.h>

#include "launch.h"
#include "mfma_common.h"

namespace mate {
namespace {

constexpr int kChains = 8;  // independent accumulators per wavefront: more than the pipe's depth

__global__ __launch_bounds__(256) void mfma_loop_kernel(float* __restrict__ sink, int iters) {
  // operands that the compiler cannot fold: small values derived from the lane index
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(0.001f * (float)((threadIdx.x + e) & 7));
    b[e] = (__bf16)(0.002f * (float)((threadIdx.x * 3 + e) & 7));
  }
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c) acc[c] = zero16();
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc[c] = mfma(a, b, acc[c]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[c][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_mfma_probe(float* sink, int workgroups, int iters, hipStream_t stream) {
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(workgroups), dim3(256), 0, stream, sink, iters);
  return hipGetLastError();
}

double mfma_probe_flop(int workgroups, int iters) {
  return (double)workgroups * 4.0 * (double)iters * kChains * 2.0 * 32 * 32 * 16;
}

}  // namespace mate
