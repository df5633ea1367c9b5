// pisa_select: pooled block logits and top-k per query block (Alg. 1 line 2), with the
// optional log(M_j + eps) column bias of the covariance-aware score.
//
// Two kernels.  (1) fp64 logits z[bh][i][j] = s * qbar_i . kbar_j, register-tiled
// on the vector ALUs, written to scratch.  (2) One workgroup per row: an MSB-first
// radix select on order-preserving 64-bit keys finds the k-th largest logit, ties at
// the threshold are granted to the lowest block indices, and the chosen indices are
// compacted in ascending order with a prefix sum.
#include "common.h"

namespace pisa {
namespace {

constexpr int kZT = 64;   // logits tile edge
constexpr int kZC = 16;   // channels staged per step

// col_bias (optional): [bh][N], added to every logit of key block j (covariance-aware score).
__global__ __launch_bounds__(256) void logits_kernel(const double* __restrict__ qbar64,
                                                     const double* __restrict__ kbar64,
                                                     const double* __restrict__ col_bias,
                                                     double* __restrict__ z, int N, int D, double scale) {
  __shared__ double qs[kZC][kZT + 1];
  __shared__ double ks[kZC][kZT + 1];
  const int tid = threadIdx.x;
  const size_t bh = blockIdx.z;
  const int i0 = blockIdx.y * kZT, j0 = blockIdx.x * kZT;
  const double* qb = qbar64 + bh * (size_t)N * D;
  const double* kb = kbar64 + bh * (size_t)N * D;
  const int ti = tid / 16, tj = tid % 16;
  double acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;

  const int lr = tid / 4, lc = (tid % 4) * 4;   // loader: row, first channel of 4
  for (int c0 = 0; c0 < D; c0 += kZC) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int qi = i0 + lr, kj = j0 + lr;
      qs[lc + u][lr] = qi < N ? qb[(size_t)qi * D + c0 + lc + u] : 0.0;
      ks[lc + u][lr] = kj < N ? kb[(size_t)kj * D + c0 + lc + u] : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kZC; ++c) {
      double qa[4], kk[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) qa[a] = qs[c][ti * 4 + a];
#pragma unroll
      for (int b = 0; b < 4; ++b) kk[b] = ks[c][tj * 4 + b];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = fma(qa[a], kk[b], acc[a][b]);
    }
    __syncthreads();
  }
  double* zb = z + bh * (size_t)N * N;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int i = i0 + ti * 4 + a;
    if (i >= N) continue;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int j = j0 + tj * 4 + b;
      if (j < N) zb[(size_t)i * N + j] = scale * acc[a][b] + (col_bias ? col_bias[bh * N + j] : 0.0);
    }
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

// Exclusive prefix sum of one int per thread over a 256-thread workgroup.
__device__ inline int block_exclusive_scan(int x, int* scratch /*[256]*/, int* total) {
  const int tid = threadIdx.x;
  scratch[tid] = x;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    int add = tid >= off ? scratch[tid - off] : 0;
    __syncthreads();
    scratch[tid] += add;
    __syncthreads();
  }
  const int incl = scratch[tid];
  *total = scratch[255];
  __syncthreads();
  return incl - x;
}

// One workgroup per (bh, query block i).  Dynamic LDS: N keys of 8 bytes.
__global__ __launch_bounds__(256) void topk_kernel(const double* __restrict__ z, int N, int k_top,
                                                   int32_t* __restrict__ idx, float* __restrict__ kth_gap) {
  extern __shared__ unsigned long long keys[];
  __shared__ int hist[256];
  __shared__ int scan_buf[256];
  __shared__ unsigned long long s_prefix;
  __shared__ int s_want;
  __shared__ unsigned long long s_red[256];

  const int tid = threadIdx.x;
  const size_t row = (size_t)blockIdx.y * N + blockIdx.x;
  const double* zr = z + row * (size_t)N;
  for (int j = tid; j < N; j += 256) keys[j] = order_key(zr[j]);
  if (tid == 0) {
    s_prefix = 0ull;
    s_want = k_top;
  }
  __syncthreads();

  if (k_top == 0 || k_top == N) {
    for (int j = tid; j < k_top; j += 256) idx[row * (size_t)k_top + j] = j;
    if (kth_gap && tid == 0) kth_gap[row] = __int_as_float(0x7f800000);
    return;
  }

  // ---- radix select: key of rank k_top (1-based, descending) ----
  for (int shift = 56; shift >= 0; shift -= 8) {
    hist[tid] = 0;
    __syncthreads();
    const unsigned long long prefix = s_prefix;
    const unsigned long long himask = shift == 56 ? 0ull : (~0ull << (shift + 8));
    for (int j = tid; j < N; j += 256) {
      const unsigned long long key = keys[j];
      if ((key & himask) == prefix) atomicAdd(&hist[(int)((key >> shift) & 0xff)], 1);
    }
    __syncthreads();
    // Wave 0 walks the 256 bins from the top: lane l owns bins 255-4l .. 252-4l, a wave
    // prefix sum over the per-lane totals finds the lane, then the lane finds its bin.
    if (tid < 64) {
      const int want = s_want;
      const int b0 = 255 - 4 * tid;
      const int c0 = hist[b0], c1 = hist[b0 - 1], c2 = hist[b0 - 2], c3 = hist[b0 - 3];
      const int mine = c0 + c1 + c2 + c3;
      int incl = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (tid >= off) incl += up;
      }
      const int before = incl - mine;               // keys in bins above this lane's bins
      if (before < want && want <= incl) {          // exactly one lane
        int w = want - before, digit = b0;
        if (w > c0) { w -= c0; digit = b0 - 1;
          if (w > c1) { w -= c1; digit = b0 - 2;
            if (w > c2) { w -= c2; digit = b0 - 3; } } }
        s_want = w;
        s_prefix = prefix | ((unsigned long long)digit << shift);
      }
    }
    __syncthreads();
  }
  const unsigned long long thr = s_prefix;   // the k-th largest key
  const int take_equal = s_want;             // how many keys equal to thr are selected

  // ---- ascending compaction: each thread owns a contiguous index range ----
  const int per = (N + 255) / 256;
  const int lo = min(N, tid * per), hi = min(N, lo + per);
  int n_eq = 0;
  for (int j = lo; j < hi; ++j) n_eq += keys[j] == thr;
  int total;
  const int eq_base = block_exclusive_scan(n_eq, scan_buf, &total);
  int n_sel = 0, eq_seen = eq_base;
  for (int j = lo; j < hi; ++j) {
    const unsigned long long key = keys[j];
    if (key > thr) ++n_sel;
    else if (key == thr) n_sel += (eq_seen++ < take_equal);
  }
  const int out_base = block_exclusive_scan(n_sel, scan_buf, &total);
  int32_t* out = idx + row * (size_t)k_top;
  int w = out_base;
  eq_seen = eq_base;
  unsigned long long best_unsel = 0ull;       // largest key left out (keys are never 0 for finite z)
  for (int j = lo; j < hi; ++j) {
    const unsigned long long key = keys[j];
    bool sel = key > thr;
    if (key == thr) sel = (eq_seen++ < take_equal);
    if (sel) out[w++] = j;
    else best_unsel = key > best_unsel ? key : best_unsel;
  }
  if (kth_gap) {
    s_red[tid] = best_unsel;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
      if (tid < off) s_red[tid] = s_red[tid] > s_red[tid + off] ? s_red[tid] : s_red[tid + off];
      __syncthreads();
    }
    if (tid == 0) kth_gap[row] = (float)(key_value(thr) - key_value(s_red[0]));
  }
}

}  // namespace

size_t select_workspace_bytes(const Dims& dm) {
  return (size_t)dm.bh() * dm.N * dm.N * sizeof(double);
}

hipError_t launch_select(const Dims& dm, const double* qbar64, const double* kbar64,
                         const double* col_bias, int k_top, int32_t* idx, float* kth_gap, double* zbuf,
                         hipStream_t stream) {
  const int nt = (dm.N + kZT - 1) / kZT;
  hipLaunchKernelGGL(logits_kernel, dim3(nt, nt, dm.bh()), dim3(256), 0, stream, qbar64, kbar64, col_bias,
                     zbuf, dm.N, dm.d, (double)dm.scale);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topk_kernel, dim3(dm.N, dm.bh()), dim3(256), (size_t)dm.N * 8, stream, zbuf,
                     dm.N, k_top, idx, kth_gap);
  return hipGetLastError();
}

}  // namespace pisa
