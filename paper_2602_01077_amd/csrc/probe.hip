// Measurement aids.  (1) A register-only loop of v_mfma_f32_32x32x16_bf16, the instruction
// the attention kernels are built on: timed by the caller, it gives the matrix-core rate this
// chip sustains at its own clock, to set beside the published 2.5 PFLOP/s.  (2) A one-wave
// kernel that reads the shader-cycle counter and the constant-rate wall clock over a time
// window: launched on a second stream while another kernel runs, it tells the shader clock
// the chip holds under that kernel's load.
#include "common.h"

namespace pisa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ inline unsigned mix32(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// Operands are pseudo-random bf16 values in (-1, 1), four A and four B fragments per lane used
// in rotation, so that the switching activity in the operand paths resembles real data.
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float* __restrict__ sink) {
  const unsigned tid = blockIdx.x * 256u + threadIdx.x;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const unsigned ha = mix32(tid * 64u + u * 8 + e), hb = mix32(0x9e3779b9u + tid * 64u + u * 8 + e);
      a[u][e] = (__bf16)((float)((int)(ha & 0xffffu) - 32768) * (1.0f / 32768.f));
      b[u][e] = (__bf16)((float)((int)(hb & 0xffffu) - 32768) * (1.0f / 32768.f));
    }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = (f32x16){0};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + i) & 3], b[u], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// out[0] = shader cycles, out[1] = wall-clock ticks over (about) `ticks` wall-clock ticks.
// The wave sleeps between looks at the clock; `max_spins` bounds the loop whatever the clock does.
__global__ __launch_bounds__(64) void clock_probe_kernel(unsigned long long* __restrict__ out,
                                                         unsigned long long ticks, int max_spins) {
  const unsigned long long c0 = __builtin_amdgcn_s_memtime();
  const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();
  unsigned long long r1 = r0;
  for (int spins = 0; spins < max_spins && r1 - r0 < ticks; ++spins) {
    __builtin_amdgcn_s_sleep(127);
    r1 = __builtin_amdgcn_s_memrealtime();
  }
  const unsigned long long c1 = __builtin_amdgcn_s_memtime();
  if (threadIdx.x == 0) {
    out[0] = c1 - c0;
    out[1] = r1 - r0;
  }
}

}  // namespace

hipError_t launch_clock_probe(unsigned long long* out, unsigned long long ticks, hipStream_t stream) {
  hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, stream, out, ticks, 1 << 16);
  return hipGetLastError();
}

hipError_t launch_mfma_probe(int iters, float* sink, hipStream_t stream) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeWorkgroups), dim3(256), 0, stream, iters, sink);
  return hipGetLastError();
}

}  // namespace pisa
