// Device-side reduction of the per-chunk partial H matrices, shared by the translation units
// that launch it on its own and inside a fused launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>

namespace pisa {

// hsum[bh][e] = sum over chunks (in chunk order, so bit-reproducible) of partial_h[bh][chunk][e],
// e = a * D + b (key channel a, value channel b).
// hpack (optional): the same value split into two bf16 halves hi + lo (hi = x rounded to nearest
// even, lo = x - hi rounded), stored in the operand order of the attention kernel's first-order
// product: hpack[bh][part][ks][dt][lane][e8] with a = 16 ks + 8 (lane >> 5) + e8 and
// b = 32 dt + (lane & 31); part 0 = hi, part 1 = lo.
template <int E>
__device__ inline void reduce_h_elements(const float* __restrict__ partial_h, float* __restrict__ hsum,
                                         unsigned short* __restrict__ hpack, int n_chunks, int D, size_t bh,
                                         int e0, int stride) {
  // E elements e0, e0 + stride, ... per thread (those past D * D are skipped), their loads in
  // flight together.
  const int dd = D * D;
  const float* p = partial_h + bh * n_chunks * (size_t)dd;
  float acc[E];
#pragma unroll
  for (int i = 0; i < E; ++i) acc[i] = 0.f;
  int c = 0;
  for (; c + 8 <= n_chunks; c += 8) {         // eight loads per element in flight, added in chunk order
    float x[E][8];
#pragma unroll
    for (int i = 0; i < E; ++i)
#pragma unroll
      for (int u = 0; u < 8; ++u) x[i][u] = e0 + i * stride < dd ? p[(size_t)(c + u) * dd + e0 + i * stride] : 0.f;
#pragma unroll
    for (int i = 0; i < E; ++i)
#pragma unroll
      for (int u = 0; u < 8; ++u) acc[i] += x[i][u];
  }
  for (; c < n_chunks; ++c)
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] += e0 + i * stride < dd ? p[(size_t)c * dd + e0 + i * stride] : 0.f;
#pragma unroll
  for (int i = 0; i < E; ++i) {
    const int e = e0 + i * stride;
    if (e >= dd) continue;
    hsum[bh * dd + e] = acc[i];
    if (hpack) {
      const int a = e / D, b = e % D;
      const int ks = a >> 4, h = (a >> 3) & 1, e8 = a & 7, dt = b >> 5, lam = b & 31;
      const int o = (((ks * (D / 32) + dt) * 64) + 32 * h + lam) * 8 + e8;
      typedef float f32x2_t __attribute__((ext_vector_type(2)));
      typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
      const f32x2_t f = {acc[i], 0.f};
      const unsigned int hi = __builtin_bit_cast(unsigned int, __builtin_convertvector(f, bf16x2_t)) & 0xffffu;
      const f32x2_t g = {acc[i] - __uint_as_float(hi << 16), 0.f};
      const unsigned int lo = __builtin_bit_cast(unsigned int, __builtin_convertvector(g, bf16x2_t)) & 0xffffu;
      unsigned short* hp = hpack + bh * (size_t)(2 * dd);
      hp[o] = (unsigned short)hi;
      hp[dd + o] = (unsigned short)lo;
    }
  }
}

__device__ inline void reduce_h_element(const float* __restrict__ partial_h, float* __restrict__ hsum,
                                        unsigned short* __restrict__ hpack, int n_chunks, int D, size_t bh,
                                        int e) {
  reduce_h_elements<1>(partial_h, hsum, hpack, n_chunks, D, bh, e, 0);
}

}  // namespace pisa
