// Measurement aid: a register-only loop of v_mfma_f32_32x32x16_bf16, the instruction the
// attention kernels are built on.  Timed by the caller, it gives the matrix-core rate this
// chip sustains at its own clock, to set beside the published 2.5 PFLOP/s.
#include "common.h"

namespace pisa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float* __restrict__ sink) {
  const int tid = threadIdx.x;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(0.001f * (float)((tid + e) & 7));
    b[e] = (__bf16)(0.002f * (float)((tid + 3 * e) & 7));
  }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = (f32x16){0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[(size_t)blockIdx.x * 256 + tid] = s;
}

}  // namespace

hipError_t launch_mfma_probe(int iters, float* sink, hipStream_t stream) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeWorkgroups), dim3(256), 0, stream, iters, sink);
  return hipGetLastError();
}

}  // namespace pisa
