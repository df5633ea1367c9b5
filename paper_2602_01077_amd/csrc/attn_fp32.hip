// fp32 attention path (dense and PISA) on the vector ALUs.
//
// One workgroup of 256 threads per 64-row query tile; four threads share a query
// row: thread (r, qd) scores keys qd, qd+4, ... of a 64-key tile and owns the
// d/4-wide slice qd of the output row.  The three phases of Alg. 1 run inside one
// running-max softmax:
//   Phase 1  tiles of the selected blocks S_i (all tiles for dense attention)
//   Phase 2  tiles of 64 centroids: logit s q.kbar_j + ln B_j, selected columns and
//            columns past N masked, values vsum_j / B_j; the same mass also feeds l_tail
//   Phase 3  out = (O + (l_tail / L) (s q) hsum) / l
#include "common.h"

namespace pisa {
namespace {

struct P32 {
  const float* q;
  const float* k;
  const float* v;
  const float* kbar;
  const float* vsum;
  const float* hsum;
  const int32_t* idx;
  float* out;
  float* lse;
  int L, B, N, k_top;
  float scale;
  int dense;
};

template <int D>
__global__ __launch_bounds__(256) void attn_fp32_kernel(P32 p) {
  constexpr int DQ = D / 4;           // output channels per thread
  constexpr int KP = D + 4;           // padded key row
  __shared__ float Qs[kTile][D];
  __shared__ float Ks[kTile][KP];
  __shared__ float Vs[kTile][D];
  __shared__ float Ps[kTile][kTile + 1];
  __shared__ float bias[kTile];       // Phase 2: ln B_j, or -inf for masked columns
  __shared__ unsigned int chosen[128];   // bitmask over blocks (N <= 4096)

  const int tid = threadIdx.x;
  const int r = tid / 4, qd = tid % 4;
  const int qt = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int L = p.L, N = p.N;
  const float* qh = p.q + bh * (size_t)L * D;
  const float* kh = p.k + bh * (size_t)L * D;
  const float* vh = p.v + bh * (size_t)L * D;
  const int q_row = qt * kTile + r;
  const int tpb = p.B / kTile;
  const int qblock = qt / tpb;
  const int32_t* my_idx = p.dense ? nullptr : p.idx + (bh * N + qblock) * (size_t)p.k_top;

  for (int e = tid; e < kTile * D; e += 256) {
    const int n = e / D, c = e % D;
    const int row = qt * kTile + n;
    Qs[n][c] = row < L ? qh[(size_t)row * D + c] : 0.f;
  }
  if (tid < 128) chosen[tid] = 0u;
  __syncthreads();
  if (!p.dense)
    for (int t = tid; t < p.k_top; t += 256) {
      const int j = my_idx[t];
      if ((unsigned)j < (unsigned)N) atomicOr(&chosen[j >> 5], 1u << (j & 31));   // others are ignored
    }

  float o[DQ];
#pragma unroll
  for (int e = 0; e < DQ; ++e) o[e] = 0.f;
  float m = -INFINITY, l = 0.f, l_tail = 0.f;   // l, l_tail: this thread's share of the row sums

  // Scores one staged tile and folds it into the running state.
  auto absorb = [&](int nvalid, bool tail) {
    float s[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
    for (int c = 0; c < D; c += 4) {
      const float4 qv = *reinterpret_cast<const float4*>(&Qs[r][c]);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float4 kv = *reinterpret_cast<const float4*>(&Ks[qd + 4 * i][c]);
        s[i] = fmaf(qv.x, kv.x, s[i]);
        s[i] = fmaf(qv.y, kv.y, s[i]);
        s[i] = fmaf(qv.z, kv.z, s[i]);
        s[i] = fmaf(qv.w, kv.w, s[i]);
      }
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = qd + 4 * i;
      s[i] = tail ? s[i] * p.scale + bias[key] : (key < nvalid ? s[i] * p.scale : -INFINITY);
      tmax = fmaxf(tmax, s[i]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 1));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 2));
    const float m_new = fmaxf(m, tmax);
    float corr = 1.f, psum = 0.f;
    if (m_new == -INFINITY) {
#pragma unroll
      for (int i = 0; i < 16; ++i) Ps[r][qd + 4 * i] = 0.f;
    } else {
      corr = expf(m - m_new);          // m = -inf gives 0
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float pe = expf(s[i] - m_new);
        Ps[r][qd + 4 * i] = pe;
        psum += pe;
      }
    }
    m = m_new;
    l = l * corr + psum;
    l_tail = l_tail * corr + (tail ? psum : 0.f);
#pragma unroll
    for (int e = 0; e < DQ; ++e) o[e] *= corr;
    __syncthreads();
    for (int c = 0; c < kTile; ++c) {
      const float pe = Ps[r][c];
#pragma unroll
      for (int e = 0; e < DQ; e += 4) {
        const float4 vv = *reinterpret_cast<const float4*>(&Vs[c][qd * DQ + e]);
        o[e + 0] = fmaf(pe, vv.x, o[e + 0]);
        o[e + 1] = fmaf(pe, vv.y, o[e + 1]);
        o[e + 2] = fmaf(pe, vv.z, o[e + 2]);
        o[e + 3] = fmaf(pe, vv.w, o[e + 3]);
      }
    }
    __syncthreads();
  };

  // ---- Phase 1: exact tiles ----
  const int n_exact_tiles = p.dense ? (L + kTile - 1) / kTile : p.k_top * tpb;
  for (int t = 0; t < n_exact_tiles; ++t) {
    const int jsel = p.dense ? 0 : my_idx[t / tpb];
    if ((unsigned)jsel >= (unsigned)N) continue;          // uniform: entries outside [0, N) are ignored
    const int tile = p.dense ? t : jsel * tpb + t % tpb;
    const int row0 = tile * kTile;
    const int nvalid = min(kTile, L - row0);
    if (nvalid <= 0) continue;
    for (int e = tid; e < kTile * D / 4; e += 256) {
      const int n = e / (D / 4), c = (e % (D / 4)) * 4;
      float4 kv = make_float4(0.f, 0.f, 0.f, 0.f), vv = kv;
      if (n < nvalid) {
        kv = *reinterpret_cast<const float4*>(&kh[(size_t)(row0 + n) * D + c]);
        vv = *reinterpret_cast<const float4*>(&vh[(size_t)(row0 + n) * D + c]);
      }
      *reinterpret_cast<float4*>(&Ks[n][c]) = kv;
      *reinterpret_cast<float4*>(&Vs[n][c]) = vv;
    }
    __syncthreads();
    absorb(nvalid, false);
  }

  // ---- Phase 2: centroid tiles ----
  if (!p.dense && p.k_top < N && p.kbar) {
    const float* kb = p.kbar + bh * (size_t)N * D;
    const float* vsm = p.vsum + bh * (size_t)N * D;
    const int last_rows = L - (N - 1) * p.B;
    for (int g0 = 0; g0 < N; g0 += kTile) {
      __syncthreads();
      for (int e = tid; e < kTile * D / 4; e += 256) {
        const int n = e / (D / 4), c = (e % (D / 4)) * 4;
        const int j = g0 + n;
        float4 kv = make_float4(0.f, 0.f, 0.f, 0.f), vv = kv;
        if (j < N) {
          const float inv = 1.f / (float)(j == N - 1 ? last_rows : p.B);
          kv = *reinterpret_cast<const float4*>(&kb[(size_t)j * D + c]);
          vv = *reinterpret_cast<const float4*>(&vsm[(size_t)j * D + c]);
          vv.x *= inv; vv.y *= inv; vv.z *= inv; vv.w *= inv;
        }
        *reinterpret_cast<float4*>(&Ks[n][c]) = kv;
        *reinterpret_cast<float4*>(&Vs[n][c]) = vv;
      }
      if (tid < kTile) {
        const int j = g0 + tid;
        float b = -INFINITY;
        if (j < N && !((chosen[j >> 5] >> (j & 31)) & 1u))
          b = logf((float)(j == N - 1 ? last_rows : p.B));
        bias[tid] = b;
      }
      __syncthreads();
      absorb(kTile, true);
    }
  }

  // ---- Phase 3 and normalisation ----
  l += __shfl_xor(l, 1);
  l += __shfl_xor(l, 2);
  l_tail += __shfl_xor(l_tail, 1);
  l_tail += __shfl_xor(l_tail, 2);
  if (!p.dense && p.hsum && p.kbar && p.k_top < N) {
    const float* hs = p.hsum + bh * (size_t)D * D;
    const float w = l_tail / (float)L * p.scale;
    for (int a = 0; a < D; ++a) {
      const float qa = Qs[r][a] * w;
#pragma unroll
      for (int e = 0; e < DQ; e += 4) {
        const float4 hv = *reinterpret_cast<const float4*>(&hs[(size_t)a * D + qd * DQ + e]);
        o[e + 0] = fmaf(qa, hv.x, o[e + 0]);
        o[e + 1] = fmaf(qa, hv.y, o[e + 1]);
        o[e + 2] = fmaf(qa, hv.z, o[e + 2]);
        o[e + 3] = fmaf(qa, hv.w, o[e + 3]);
      }
    }
  }
  if (q_row < L) {
    const float inv_l = 1.f / l;
    float* orow = p.out + (bh * (size_t)L + q_row) * D + qd * DQ;
#pragma unroll
    for (int e = 0; e < DQ; e += 4)
      *reinterpret_cast<float4*>(&orow[e]) =
          make_float4(o[e] * inv_l, o[e + 1] * inv_l, o[e + 2] * inv_l, o[e + 3] * inv_l);
    if (p.lse && qd == 0) p.lse[bh * (size_t)L + q_row] = m + logf(l);
  }
}

}  // namespace

hipError_t launch_attention_fp32(const Dims& dm, const AttnArgs& a, hipStream_t stream) {
  P32 p;
  p.q = (const float*)a.q;
  p.k = (const float*)a.k;
  p.v = (const float*)a.v;
  p.kbar = a.kbar;
  p.vsum = a.vsum;
  p.hsum = a.hsum;
  p.idx = a.idx;
  p.out = (float*)a.out;
  p.lse = a.lse;
  p.L = dm.L;
  p.B = dm.B;
  p.N = dm.N;
  p.k_top = a.k_top;
  p.scale = dm.scale;
  p.dense = a.dense ? 1 : 0;
  dim3 grid((dm.L + kTile - 1) / kTile, dm.bh());
  if (dm.d == 64)
    hipLaunchKernelGGL((attn_fp32_kernel<64>), grid, dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL((attn_fp32_kernel<128>), grid, dim3(256), 0, stream, p);
  return hipGetLastError();
}

}  // namespace pisa
