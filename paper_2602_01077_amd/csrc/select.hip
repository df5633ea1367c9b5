// pisa_select: pooled block logits and top-k per query block (Alg. 1, "Select" step), with the
// optional log(M_j + eps) column bias of the covariance-aware score.
//
// Two kernels (one fused kernel when N <= 128).  (1) fp64 logits z[bh][i][j] = s * qbar_i . kbar_j on the fp64 matrix
// cores, one wave per 64x64 tile, written to scratch.  (2) One WAVE per row, the row's
// order-preserving 64-bit keys in registers: a bucket select narrows a key interval around
// the k-th largest logit (256 buckets per level over the tightened [min, max] of the
// surviving keys),
// ties at the threshold are granted to the lowest block indices, and the chosen indices
// are compacted in ascending order with wave ballots.  No workgroup barriers.
#include <algorithm>

#include "common.h"
#include "reduce_h.h"

namespace pisa {
namespace {

typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kZT = 64;   // logits tile edge (per wave)

// v_mfma_f64_16x16x4_f64: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16]; register r
// of the result holds D[4 * r + l / 16][l % 16].  A lane loads four consecutive channels
// of its row at once and feeds them to four successive instructions: both operands use the
// same channel for the same (instruction, l / 16), so the contraction covers every channel
// exactly once.
// col_bias (optional): [bh][N], added to every logit of key block j (covariance-aware score).
template <int D>
__global__ __launch_bounds__(256, 2) void logits_kernel(const double* __restrict__ qbar64,
                                                        const double* __restrict__ kbar64,
                                                        const double* __restrict__ col_bias,
                                                        double* __restrict__ z, int N, double scale) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t bh = blockIdx.z;
  const int i0 = blockIdx.y * kZT;
  const int j0 = (blockIdx.x * 4 + wave) * kZT;
  if (j0 >= N) return;                     // whole wave; the kernel has no barriers
  const int r = lane & 15, kk = lane >> 4;
  const double* qb = qbar64 + bh * (size_t)N * D;
  const double* kb = kbar64 + bh * (size_t)N * D;
  // Rows past N are clamped to N - 1: their products are computed and never stored.
  const double* qp[4];
  const double* kp[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    qp[a] = qb + (size_t)min(i0 + 16 * a + r, N - 1) * D + 4 * kk;
    kp[a] = kb + (size_t)min(j0 + 16 * a + r, N - 1) * D + 4 * kk;
  }
  f64x4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};

  f64x4 av[4], bv[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    av[a] = *reinterpret_cast<const f64x4*>(qp[a]);
    bv[a] = *reinterpret_cast<const f64x4*>(kp[a]);
  }
#pragma unroll 1
  for (int c0 = 0; c0 < D; c0 += 16) {
    f64x4 an[4], bn[4];
    const int cn = c0 + 16 < D ? c0 + 16 : c0;      // last step reloads in place, unused
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      an[a] = *reinterpret_cast<const f64x4*>(qp[a] + cn);
      bn[a] = *reinterpret_cast<const f64x4*>(kp[a] + cn);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[a][u], bv[b][u], acc[a][b], 0, 0, 0);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      av[a] = an[a];
      bv[a] = bn[a];
    }
  }
  double* zb = z + bh * (size_t)N * N;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int j = j0 + 16 * b + r;
    if (j >= N) continue;
    const double bias = col_bias ? col_bias[bh * N + j] : 0.0;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = i0 + 16 * a + 4 * e + kk;
        if (i < N) zb[(size_t)i * N + j] = scale * acc[a][b][e] + bias;
      }
  }
}

// The same product for short sequences, where 64x64 tiles would leave most of the chip
// idle: one wave per 16x16 tile, all operand loads issued up front.
template <int D>
__global__ __launch_bounds__(256) void logits_small_kernel(const double* __restrict__ qbar64,
                                                           const double* __restrict__ kbar64,
                                                           const double* __restrict__ col_bias,
                                                           double* __restrict__ z, int N, double scale) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t bh = blockIdx.z;
  const int i0 = blockIdx.y * 16;
  const int j0 = (blockIdx.x * 4 + wave) * 16;
  if (j0 >= N) return;                     // whole wave; the kernel has no barriers
  const int r = lane & 15, kk = lane >> 4;
  const double* qp = qbar64 + (bh * N + min(i0 + r, N - 1)) * (size_t)D + 4 * kk;
  const double* kp = kbar64 + (bh * N + min(j0 + r, N - 1)) * (size_t)D + 4 * kk;
  f64x4 av[D / 16], bv[D / 16];
#pragma unroll
  for (int c = 0; c < D / 16; ++c) {
    av[c] = *reinterpret_cast<const f64x4*>(qp + 16 * c);
    bv[c] = *reinterpret_cast<const f64x4*>(kp + 16 * c);
  }
  f64x4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = acc0;
#pragma unroll
  for (int c = 0; c < D / 16; ++c)
#pragma unroll
    for (int u = 0; u < 4; u += 2) {
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(av[c][u], bv[c][u], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(av[c][u + 1], bv[c][u + 1], acc1, 0, 0, 0);
    }
  const int j = j0 + r;
  if (j >= N) return;
  const double bias = col_bias ? col_bias[bh * N + j] : 0.0;
  double* zb = z + bh * (size_t)N * N;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int i = i0 + 4 * e + kk;
    if (i < N) zb[(size_t)i * N + j] = scale * (acc0[e] + acc1[e]) + bias;
  }
}

__device__ inline unsigned long long order_key(double x) {
  unsigned long long u = (unsigned long long)__double_as_longlong(x);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ inline double key_value(unsigned long long key) {
  unsigned long long u = (key >> 63) ? (key & 0x7fffffffffffffffull) : ~key;
  return __longlong_as_double((long long)u);
}

// Orders this wave's LDS traffic: writes before it are visible to every lane after it.
__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}
__device__ inline unsigned long long wave_min_u64(unsigned long long x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned long long y = __shfl_xor(x, off);
    x = y < x ? y : x;
  }
  return x;
}
__device__ inline unsigned long long wave_max_u64(unsigned long long x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned long long y = __shfl_xor(x, off);
    x = y > x ? y : x;
  }
  return x;
}
__device__ inline int lanes_below(unsigned long long mask) {   // set bits of mask below this lane
  return __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
}

// Top-k of one row by one wave.  Lane l holds keys l, l + 64, ... in registers (KPL of them,
// so N <= 64 * KPL); `hist` is the wave's own 256-bin histogram in LDS; `zr` may point into
// global memory or LDS; `gap` (optional) is this row's kth_gap slot.
template <int KPL>
__device__ inline void topk_row(const double* zr, int N, int k_top, int* hist, int32_t* __restrict__ out,
                                float* __restrict__ gap, int lane) {
  if (k_top == 0 || k_top == N) {
    for (int j = lane; j < k_top; j += 64) out[j] = j;
    if (gap && lane == 0) *gap = __int_as_float(0x7f800000);
    return;
  }
  unsigned long long key[KPL];
#pragma unroll
  for (int u = 0; u < KPL; ++u) key[u] = order_key(zr[min(lane + 64 * u, N - 1)]);
  const int n_mine = (N - lane + 63) / 64;       // slots u < n_mine hold keys of this row

  // ---- narrow [lo, hi] around the key of rank `want` (1-based, descending) among the keys
  // inside it.  Each level re-centres 256 buckets on the surviving keys' own [min, max], so
  // the shared sign / exponent bits of a row never produce a level that separates nothing.
  unsigned long long lo = 0ull, hi = ~0ull;
  int want = k_top;
  {  // split by sign first: mixed signs would put a whole row into two or three buckets
    int n_nonneg = 0;
#pragma unroll
    for (int u = 0; u < KPL; ++u)
      n_nonneg += __builtin_popcountll(__ballot(u < n_mine && (key[u] >> 63) != 0ull));
    if (want <= n_nonneg) {
      lo = 1ull << 63;
    } else {
      want -= n_nonneg;
      hi = (1ull << 63) - 1ull;
    }
  }
  unsigned long long thr;                  // the k-th largest key
  int take_equal;                          // how many keys equal to thr are selected
  for (;;) {
    unsigned long long kmin = ~0ull, kmax = 0ull;
#pragma unroll
    for (int u = 0; u < KPL; ++u)
      if (u < n_mine && key[u] >= lo && key[u] <= hi) {
        kmin = key[u] < kmin ? key[u] : kmin;
        kmax = key[u] > kmax ? key[u] : kmax;
      }
    kmin = wave_min_u64(kmin);
    kmax = wave_max_u64(kmax);
    const unsigned long long range = kmax - kmin;
    if (range == 0ull) {                   // every surviving key is the same value
      thr = kmin;
      take_equal = want;
      break;
    }
    const int sh = max(0, 56 - (int)__builtin_clzll(range));     // (range >> sh) <= 255
    reinterpret_cast<int4*>(hist)[lane] = make_int4(0, 0, 0, 0);
    wave_lds_sync();
#pragma unroll
    for (int u = 0; u < KPL; ++u)
      if (u < n_mine && key[u] >= kmin && key[u] <= kmax)
        atomicAdd(&hist[(int)((key[u] - kmin) >> sh)], 1);
    wave_lds_sync();
    // Walk the buckets from the top: lane l owns buckets 255-4l .. 252-4l; a wave prefix
    // sum over the per-lane totals finds the lane, then the lane finds its bucket.
    const int4 c = reinterpret_cast<const int4*>(hist)[63 - lane];   // c.w = bucket 255-4l
    const int mine = c.x + c.y + c.z + c.w;
    int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int up = __shfl_up(incl, off);
      if (lane >= off) incl += up;
    }
    const int before = incl - mine;        // keys in buckets above this lane's buckets
    const bool found = before < want && want <= incl;              // exactly one lane
    int w = want - before, bucket = 255 - 4 * lane, cnt = c.w;
    if (w > c.w) { w -= c.w; bucket -= 1; cnt = c.z;
      if (w > c.z) { w -= c.z; bucket -= 1; cnt = c.y;
        if (w > c.y) { w -= c.y; bucket -= 1; cnt = c.x; } } }
    const int src = __builtin_ctzll(__ballot(found));
    w = __shfl(w, src);
    bucket = __shfl(bucket, src);
    cnt = __shfl(cnt, src);
    wave_lds_sync();                       // histogram reads done before the next level clears it
    lo = kmin + ((unsigned long long)bucket << sh);
    const unsigned long long span = sh == 0 ? 0ull : (1ull << sh) - 1ull;
    hi = lo > ~0ull - span ? ~0ull : lo + span;
    want = w;
    if (cnt == want) {                     // the whole bucket is selected: keys >= lo
      thr = lo;
      take_equal = 0x7fffffff;
      break;
    }
    if (sh == 0) {                         // a bucket is one key value: ties at the threshold
      thr = lo;
      take_equal = want;
      break;
    }
  }

  // ---- ascending compaction, 64 consecutive indices per step ----
  int base = 0, eq_seen = 0;
  unsigned long long min_sel = ~0ull, max_unsel = 0ull;   // keys are never 0 for finite z
#pragma unroll
  for (int u = 0; u < KPL; ++u) {
    const bool valid = u < n_mine;
    const bool eq = valid && key[u] == thr;
    const unsigned long long eq_mask = __ballot(eq);
    const bool sel = valid && (key[u] > thr || (eq && eq_seen + lanes_below(eq_mask) < take_equal));
    const unsigned long long sel_mask = __ballot(sel);
    if (sel) {
      out[base + lanes_below(sel_mask)] = lane + 64 * u;
      min_sel = key[u] < min_sel ? key[u] : min_sel;
    } else if (valid) {
      max_unsel = key[u] > max_unsel ? key[u] : max_unsel;
    }
    base += __builtin_popcountll(sel_mask);
    eq_seen += __builtin_popcountll(eq_mask);
  }
  if (gap) {
    min_sel = wave_min_u64(min_sel);
    max_unsel = wave_max_u64(max_unsel);
    if (lane == 0) *gap = (float)(key_value(min_sel) - key_value(max_unsel));
  }
}

// One wave per (bh, query block i), four rows per workgroup.
template <int KPL>
__global__ __launch_bounds__(256) void topk_kernel(const double* __restrict__ z, int N, int k_top,
                                                   size_t n_rows, int32_t* __restrict__ idx,
                                                   float* __restrict__ kth_gap) {
  __shared__ int hist_all[4][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t row = (size_t)blockIdx.x * 4 + wave;
  if (row >= n_rows) return;               // whole wave; the kernel has no workgroup barriers
  topk_row<KPL>(z + row * (size_t)N, N, k_top, hist_all[wave], idx + row * (size_t)k_top,
                kth_gap ? kth_gap + row : nullptr, lane);
}

// Logits and top-k in one launch for N <= 128 (sequences of a few thousand tokens, where a
// launch costs as much as either kernel).  A workgroup of 16 waves takes 16 query blocks of
// one head: waves 0 .. ceil(N/16)-1 each compute one 16x16 logits tile exactly as
// logits_small_kernel does and park it in LDS, then every wave selects one row.
constexpr int kFusedMaxN = 128;
template <int D>
__device__ inline void select_small_body(const double* __restrict__ qbar64, const double* __restrict__ kbar64,
                                         const double* __restrict__ col_bias, int N, double scale, int k_top,
                                         int32_t* __restrict__ idx, float* __restrict__ kth_gap, int group,
                                         size_t bh) {
  __shared__ double zs[16][kFusedMaxN];
  __shared__ int hist_all[16][256];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i0 = group * 16;
  const int j0 = wave * 16;
  if (j0 < N) {                            // wave-uniform
    const int r = lane & 15, kk = lane >> 4;
    const double* qp = qbar64 + (bh * N + min(i0 + r, N - 1)) * (size_t)D + 4 * kk;
    const double* kp = kbar64 + (bh * N + min(j0 + r, N - 1)) * (size_t)D + 4 * kk;
    f64x4 av[D / 16], bv[D / 16];
#pragma unroll
    for (int c = 0; c < D / 16; ++c) {
      av[c] = *reinterpret_cast<const f64x4*>(qp + 16 * c);
      bv[c] = *reinterpret_cast<const f64x4*>(kp + 16 * c);
    }
    f64x4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = acc0;
#pragma unroll
    for (int c = 0; c < D / 16; ++c)
#pragma unroll
      for (int u = 0; u < 4; u += 2) {
        acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(av[c][u], bv[c][u], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(av[c][u + 1], bv[c][u + 1], acc1, 0, 0, 0);
      }
    const int j = j0 + r;
    if (j < N) {
      const double bias = col_bias ? col_bias[bh * N + j] : 0.0;
#pragma unroll
      for (int e = 0; e < 4; ++e) zs[4 * e + kk][j] = scale * (acc0[e] + acc1[e]) + bias;
    }
  }
  __syncthreads();
  const int i = i0 + wave;
  if (i >= N) return;
  const size_t row = bh * N + i;
  topk_row<kFusedMaxN / 64>(zs[wave], N, k_top, hist_all[wave], idx + row * (size_t)k_top,
                            kth_gap ? kth_gap + row : nullptr, lane);
}

template <int D>
__global__ __launch_bounds__(1024) void select_small_kernel(const double* __restrict__ qbar64,
                                                            const double* __restrict__ kbar64,
                                                            const double* __restrict__ col_bias, int N,
                                                            double scale, int k_top,
                                                            int32_t* __restrict__ idx,
                                                            float* __restrict__ kth_gap) {
  select_small_body<D>(qbar64, kbar64, col_bias, N, scale, k_top, idx, kth_gap, blockIdx.x, blockIdx.y);
}

// The same selection plus, in the workgroups past the first n_groups of a head, the reduction of
// the statistics pass's partial H sums (independent work on the same inputs' statistics: one
// launch instead of two on short sequences).
template <int D>
__global__ __launch_bounds__(1024) void select_small_reduce_kernel(
    const double* __restrict__ qbar64, const double* __restrict__ kbar64, const double* __restrict__ col_bias,
    int N, double scale, int k_top, int32_t* __restrict__ idx, float* __restrict__ kth_gap, int n_groups,
    const float* __restrict__ partial_h, float* __restrict__ hsum, unsigned short* __restrict__ hpack,
    int n_chunks) {
  if ((int)blockIdx.x < n_groups) {
    select_small_body<D>(qbar64, kbar64, col_bias, N, scale, k_top, idx, kth_gap, blockIdx.x, blockIdx.y);
  } else {
    // four elements per thread, 1024 apart (consecutive threads stay on consecutive addresses):
    // few workgroups, so that the whole launch is resident at once
    const int e0 = ((int)blockIdx.x - n_groups) * 4096 + (int)threadIdx.x;
    reduce_h_elements<4>(partial_h, hsum, hpack, n_chunks, D, blockIdx.y, e0, 1024);
  }
}

}  // namespace

size_t select_workspace_bytes(const Dims& dm) {
  return (size_t)dm.bh() * dm.N * dm.N * sizeof(double);
}

bool select_fuses_reduce(const Dims& dm) { return dm.N <= kFusedMaxN; }

hipError_t launch_select(const Dims& dm, const double* qbar64, const double* kbar64,
                         const double* col_bias, int k_top, int32_t* idx, float* kth_gap, double* zbuf,
                         const PendingReduce* pending, hipStream_t stream) {
  const int nt = (dm.N + kZT - 1) / kZT;
  if (pending && !select_fuses_reduce(dm)) return hipErrorInvalidValue;   // the caller checks first
  if (dm.N <= kFusedMaxN && pending) {                    // selection and H reduction in one launch
    const int n_groups = (dm.N + 15) / 16;
    const dim3 fgrid(n_groups + (dm.d * dm.d + 4095) / 4096, dm.bh());
    if (dm.d == 64)
      hipLaunchKernelGGL(select_small_reduce_kernel<64>, fgrid, dim3(1024), 0, stream, qbar64, kbar64, col_bias,
                         dm.N, (double)dm.scale, k_top, idx, kth_gap, n_groups, pending->partial_h,
                         pending->hsum, (unsigned short*)pending->hpack, pending->n_chunks);
    else
      hipLaunchKernelGGL(select_small_reduce_kernel<128>, fgrid, dim3(1024), 0, stream, qbar64, kbar64, col_bias,
                         dm.N, (double)dm.scale, k_top, idx, kth_gap, n_groups, pending->partial_h,
                         pending->hsum, (unsigned short*)pending->hpack, pending->n_chunks);
    return hipGetLastError();
  }
  if (dm.N <= kFusedMaxN) {                               // one launch for short sequences
    const dim3 fgrid((dm.N + 15) / 16, dm.bh());
    if (dm.d == 64)
      hipLaunchKernelGGL(select_small_kernel<64>, fgrid, dim3(1024), 0, stream, qbar64, kbar64, col_bias, dm.N,
                         (double)dm.scale, k_top, idx, kth_gap);
    else
      hipLaunchKernelGGL(select_small_kernel<128>, fgrid, dim3(1024), 0, stream, qbar64, kbar64, col_bias, dm.N,
                         (double)dm.scale, k_top, idx, kth_gap);
    return hipGetLastError();
  }
  if ((size_t)nt * nt * dm.bh() < 1024) {                 // too few 64x64 tiles to fill the chip
    const int nt16 = (dm.N + 15) / 16;
    const dim3 sgrid((nt16 + 3) / 4, nt16, dm.bh());
    if (dm.d == 64)
      hipLaunchKernelGGL(logits_small_kernel<64>, sgrid, dim3(256), 0, stream, qbar64, kbar64, col_bias, zbuf,
                         dm.N, (double)dm.scale);
    else
      hipLaunchKernelGGL(logits_small_kernel<128>, sgrid, dim3(256), 0, stream, qbar64, kbar64, col_bias, zbuf,
                         dm.N, (double)dm.scale);
  } else {
    const dim3 zgrid((nt + 3) / 4, nt, dm.bh());
    if (dm.d == 64)
      hipLaunchKernelGGL(logits_kernel<64>, zgrid, dim3(256), 0, stream, qbar64, kbar64, col_bias, zbuf, dm.N,
                         (double)dm.scale);
    else
      hipLaunchKernelGGL(logits_kernel<128>, zgrid, dim3(256), 0, stream, qbar64, kbar64, col_bias, zbuf, dm.N,
                         (double)dm.scale);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const size_t n_rows = (size_t)dm.bh() * dm.N;
  const dim3 grid((unsigned)((n_rows + 3) / 4));
  if (dm.N <= 64 * 8)
    hipLaunchKernelGGL(topk_kernel<8>, grid, dim3(256), 0, stream, zbuf, dm.N, k_top, n_rows, idx, kth_gap);
  else if (dm.N <= 64 * 20)
    hipLaunchKernelGGL(topk_kernel<20>, grid, dim3(256), 0, stream, zbuf, dm.N, k_top, n_rows, idx, kth_gap);
  else if (dm.N <= 64 * 32)
    hipLaunchKernelGGL(topk_kernel<32>, grid, dim3(256), 0, stream, zbuf, dm.N, k_top, n_rows, idx, kth_gap);
  else
    hipLaunchKernelGGL(topk_kernel<64>, grid, dim3(256), 0, stream, zbuf, dm.N, k_top, n_rows, idx, kth_gap);
  return hipGetLastError();
}

}  // namespace pisa
