// pisa_block_heterogeneity: M_j = || H_j - Hbar ||, Hbar = (1/N) sum_j H_j, and the column
// bias log(M_j + eps) of the covariance-aware selection score (Methodology,
// "Covariance-Aware Block Selection"; H_j from "Global First-Order Correction").
//
// Everything here is fp64 on the vector ALUs: the bias is added to fp64 pooled logits and
// has to keep their accuracy.  Two passes over K and V, no per-block matrices in memory:
//   (1) hsum64_kernel   one workgroup per chunk of blocks accumulates sum_j H_j; the partial
//                       sums are added in chunk order and divided by N (hbar64_kernel);
//   (2) hetero_kernel   one workgroup per block rebuilds H_j, subtracts Hbar and takes the
//                       Frobenius norm, or the spectral norm by power iteration on D^T D.
// A thread owns an R x R patch (R = d/16) of the d x d matrix.
#include <hip/hip_bf16.h>

#include "common.h"

namespace pisa {
namespace {

template <typename T> __device__ inline double to_f64(T x);
template <> __device__ inline double to_f64<float>(float x) { return (double)x; }
template <> __device__ inline double to_f64<__hip_bfloat16>(__hip_bfloat16 x) { return (double)__bfloat162float(x); }

// h += sum over the rows of block j of (k_n - kbar_j)^T v_n.  kc / vs: LDS staging.
template <typename T, int D>
__device__ inline void add_block_H(double (&h)[D / 16][D / 16], const T* kh, const T* vh,
                                   const double* kmean /* kbar64 row of block j */, int row0, int rows,
                                   double (*kc)[D], float (*vs)[D]) {
  constexpr int R = D / 16;
  const int tid = threadIdx.x, ta = tid / 16, tb = tid % 16;
  for (int sub = 0; sub < rows; sub += kTile) {
    const int nv = min(kTile, rows - sub);
    __syncthreads();
    for (int e = tid; e < nv * D; e += 256) {
      const int n = e / D, c = e % D;
      const size_t off = (size_t)(row0 + sub + n) * D + c;
      kc[n][c] = to_f64(kh[off]) - kmean[c];
      vs[n][c] = (float)to_f64(vh[off]);
    }
    __syncthreads();
    for (int n = 0; n < nv; ++n) {
      double ka[R], vb[R];
#pragma unroll
      for (int a = 0; a < R; ++a) ka[a] = kc[n][ta * R + a];
#pragma unroll
      for (int b = 0; b < R; ++b) vb[b] = (double)vs[n][tb * R + b];
#pragma unroll
      for (int a = 0; a < R; ++a)
#pragma unroll
        for (int b = 0; b < R; ++b) h[a][b] = fma(ka[a], vb[b], h[a][b]);
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void hsum64_kernel(const T* __restrict__ k, const T* __restrict__ v,
                                                     const double* __restrict__ kbar64,
                                                     double* __restrict__ partial, int L, int B, int N,
                                                     int chunk_blocks, int n_chunks) {
  constexpr int R = D / 16;
  __shared__ double kc[kTile][D];
  __shared__ float vs[kTile][D];
  const int tid = threadIdx.x, ta = tid / 16, tb = tid % 16;
  const int chunk = blockIdx.x;
  const size_t bh = blockIdx.y;
  const T* kh = k + bh * (size_t)L * D;
  const T* vh = v + bh * (size_t)L * D;
  double h[R][R];
#pragma unroll
  for (int a = 0; a < R; ++a)
#pragma unroll
    for (int b = 0; b < R; ++b) h[a][b] = 0.0;
  const int j_end = min(N, (chunk + 1) * chunk_blocks);
  for (int j = chunk * chunk_blocks; j < j_end; ++j)
    add_block_H<T, D>(h, kh, vh, kbar64 + (bh * N + j) * D, j * B, min(B, L - j * B), kc, vs);
  double* ph = partial + (bh * n_chunks + chunk) * (size_t)D * D;
#pragma unroll
  for (int a = 0; a < R; ++a)
#pragma unroll
    for (int b = 0; b < R; ++b) ph[(size_t)(ta * R + a) * D + tb * R + b] = h[a][b];
}

// hbar64[bh][e] = (sum over chunks, in chunk order, of partial[bh][chunk][e]) / N
__global__ __launch_bounds__(256) void hbar64_kernel(const double* __restrict__ partial,
                                                     double* __restrict__ hbar64, int n_chunks, int dd, int N) {
  const size_t bh = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= dd) return;
  const double* p = partial + bh * n_chunks * (size_t)dd + e;
  double acc = 0.0;
  for (int c = 0; c < n_chunks; ++c) acc += p[(size_t)c * dd];
  hbar64[bh * dd + e] = acc / (double)N;
}

// Sum of one double per thread over the first D threads of the workgroup (D = 64 or 128).
template <int D>
__device__ inline double sum_first_threads(double x, double* scratch /* [2] */) {
  const int tid = threadIdx.x;
  if (tid >= D) x = 0.0;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  __syncthreads();
  if (tid == 0) scratch[0] = x;
  if (tid == 64) scratch[1] = x;
  __syncthreads();
  return D > 64 ? scratch[0] + scratch[1] : scratch[0];
}

template <typename T, int D>
__global__ __launch_bounds__(256) void hetero_kernel(const T* __restrict__ k, const T* __restrict__ v,
                                                     const double* __restrict__ kbar64,
                                                     const double* __restrict__ hbar64,
                                                     double* __restrict__ log_m, int L, int B, int N,
                                                     int spectral, int n_iter, double eps) {
  constexpr int R = D / 16;
  __shared__ double kc[kTile][D];          // staging; reused as the partial-product board
  __shared__ float vs[kTile][D];
  __shared__ double xs[D], ys[D];
  __shared__ double red[2];
  const int tid = threadIdx.x, ta = tid / 16, tb = tid % 16;
  const int j = blockIdx.x;
  const size_t bh = blockIdx.y;
  double dm[R][R];
#pragma unroll
  for (int a = 0; a < R; ++a)
#pragma unroll
    for (int b = 0; b < R; ++b) dm[a][b] = 0.0;
  add_block_H<T, D>(dm, k + bh * (size_t)L * D, v + bh * (size_t)L * D, kbar64 + (bh * N + j) * D, j * B,
                    min(B, L - j * B), kc, vs);
  const double* hb = hbar64 + bh * (size_t)D * D;
#pragma unroll
  for (int a = 0; a < R; ++a)
#pragma unroll
    for (int b = 0; b < R; ++b) dm[a][b] -= hb[(size_t)(ta * R + a) * D + tb * R + b];

  double m_norm;
  if (!spectral) {
    double ss = 0.0;
#pragma unroll
    for (int a = 0; a < R; ++a)
#pragma unroll
      for (int b = 0; b < R; ++b) ss = fma(dm[a][b], dm[a][b], ss);
    // all 256 threads contribute: two-level sum over the four waves
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    __syncthreads();
    if ((tid & 63) == 0) xs[tid >> 6] = ss;
    __syncthreads();
    m_norm = sqrt((xs[0] + xs[1]) + (xs[2] + xs[3]));
  } else {
    // Power iteration on D^T D: x <- D^T (D x) / ||.||; then M = ||D x||.
    double (*board)[16] = reinterpret_cast<double (*)[16]>(&kc[0][0]);   // [D][16] partial products
    __syncthreads();
    if (tid < D) xs[tid] = 1.0 + 0.5 * sin(1.0 + 0.37 * (double)tid);    // fixed, generic start
    __syncthreads();
    {
      const double n2 = sum_first_threads<D>(tid < D ? xs[tid] * xs[tid] : 0.0, red);
      if (tid < D) xs[tid] /= sqrt(n2);
    }
    for (int it = 0; it <= n_iter; ++it) {
      __syncthreads();
      // y = D x
#pragma unroll
      for (int a = 0; a < R; ++a) {
        double pa = 0.0;
#pragma unroll
        for (int b = 0; b < R; ++b) pa = fma(dm[a][b], xs[tb * R + b], pa);
        board[ta * R + a][tb] = pa;
      }
      __syncthreads();
      double yv = 0.0;
      if (tid < D) {
#pragma unroll
        for (int t = 0; t < 16; ++t) yv += board[tid][t];
        ys[tid] = yv;
      }
      if (it == n_iter) {                      // final: M = ||D x||
        m_norm = sqrt(sum_first_threads<D>(yv * yv, red));
        break;
      }
      __syncthreads();
      // z = D^T y
#pragma unroll
      for (int b = 0; b < R; ++b) {
        double pb = 0.0;
#pragma unroll
        for (int a = 0; a < R; ++a) pb = fma(dm[a][b], ys[ta * R + a], pb);
        board[tb * R + b][ta] = pb;
      }
      __syncthreads();
      double zv = 0.0;
      if (tid < D) {
#pragma unroll
        for (int t = 0; t < 16; ++t) zv += board[tid][t];
      }
      const double n2 = sum_first_threads<D>(zv * zv, red);
      if (tid < D) xs[tid] = n2 > 0.0 ? zv / sqrt(n2) : xs[tid];
    }
  }
  if (tid == 0) log_m[bh * N + j] = log(m_norm + eps);
}

}  // namespace

size_t hetero_workspace_bytes(const Dims& dm) {
  const StatsPlan plan = stats_plan(dm);
  return (size_t)dm.bh() * (plan.n_chunks + 1) * dm.d * dm.d * sizeof(double);
}

hipError_t launch_block_heterogeneity(const Dims& dm, const void* k, const void* v, const double* kbar64,
                                      int spectral, int n_iter, double eps, double* log_m,
                                      double* workspace, hipStream_t stream) {
  const StatsPlan plan = stats_plan(dm);
  const int dd = dm.d * dm.d;
  double* partial = workspace;
  double* hbar = workspace + (size_t)dm.bh() * plan.n_chunks * dd;
  const dim3 g1(plan.n_chunks, dm.bh()), g2((dd + 255) / 256, dm.bh()), g3(dm.N, dm.bh());
#define PISA_HET(T, DD)                                                                                \
  do {                                                                                                  \
    hipLaunchKernelGGL((hsum64_kernel<T, DD>), g1, dim3(256), 0, stream, (const T*)k, (const T*)v,      \
                       kbar64, partial, dm.L, dm.B, dm.N, plan.chunk_blocks, plan.n_chunks);            \
    hipLaunchKernelGGL(hbar64_kernel, g2, dim3(256), 0, stream, partial, hbar, plan.n_chunks, dd, dm.N); \
    hipLaunchKernelGGL((hetero_kernel<T, DD>), g3, dim3(256), 0, stream, (const T*)k, (const T*)v,      \
                       kbar64, hbar, log_m, dm.L, dm.B, dm.N, spectral, n_iter, eps);                   \
  } while (0)
  if (dm.dtype == PISA_BF16)
    PISA_HET(__hip_bfloat16, 128);
  else if (dm.d == 64)
    PISA_HET(float, 64);
  else
    PISA_HET(float, 128);
#undef PISA_HET
  return hipGetLastError();
}

}  // namespace pisa
