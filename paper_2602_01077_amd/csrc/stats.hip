// pisa_block_stats: block means of Q and K, block sums of V, and the global
// first-order statistic  hsum = sum_j sum_n (k_{j,n} - kbar_j)^T v_{j,n}
// (Alg. 1, "Prepare" step; H_j as defined in the "Global First-Order Correction" paragraph).
//
// Grid: (n_chunks, batch*heads).  A workgroup walks `chunk_blocks` consecutive
// blocks of one head, keeps its share of H in registers, and writes one partial
// d x d matrix; a second kernel adds the partials in chunk order, so hsum is
// bit-identical from run to run.
#include "common.h"
#include "reduce_h.h"

namespace pisa {
namespace {

template <typename T> __device__ inline float to_f32(T x);
template <> __device__ inline float to_f32<float>(float x) { return x; }

// Vector-ALU statistics kernel (the fp32 build; bf16 inputs take the matrix-core kernel).
//   LDS: kc[64][D] centred keys, vs[64][D] values, column-sum scratch.
template <typename T, int D>
__global__ __launch_bounds__(256) void stats_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
    float* __restrict__ qbar, float* __restrict__ kbar, float* __restrict__ vsum,
    double* __restrict__ qbar64, double* __restrict__ kbar64, float* __restrict__ partial_h,
    int L, int B, int N, int chunk_blocks, int n_chunks) {
  constexpr int R = D / 16;           // each thread owns an R x R patch of H
  constexpr int P = 256 / D;          // row-parts per column in the sum pass
  __shared__ float kc[kTile][D];
  __shared__ float vs[kTile][D];
  __shared__ double psum[3][P][D];
  __shared__ double kmean[D];

  const int tid = threadIdx.x;
  const int chunk = blockIdx.x;
  const size_t bh = blockIdx.y;
  const T* qh = q + bh * (size_t)L * D;
  const T* kh = k + bh * (size_t)L * D;
  const T* vh = v + bh * (size_t)L * D;

  const int ta = tid / 16, tb = tid % 16;
  float h[R][R];
#pragma unroll
  for (int a = 0; a < R; ++a)
#pragma unroll
    for (int b = 0; b < R; ++b) h[a][b] = 0.f;

  const int j_begin = chunk * chunk_blocks;
  const int j_end = min(N, j_begin + chunk_blocks);
  for (int j = j_begin; j < j_end; ++j) {
    const int row0 = j * B;
    const int rows = min(B, L - row0);
    // ---- column sums in fp64 ----
    {
      const int col = tid % D, part = tid / D;
      double sq = 0.0, sk = 0.0, sv = 0.0;
      for (int n = part; n < rows; n += P) {
        const size_t off = (size_t)(row0 + n) * D + col;
        sq += (double)to_f32(qh[off]);
        sk += (double)to_f32(kh[off]);
        sv += (double)to_f32(vh[off]);
      }
      psum[0][part][col] = sq;
      psum[1][part][col] = sk;
      psum[2][part][col] = sv;
    }
    __syncthreads();
    if (tid < D) {
      double sq = 0.0, sk = 0.0, sv = 0.0;
#pragma unroll
      for (int p = 0; p < P; ++p) {
        sq += psum[0][p][tid];
        sk += psum[1][p][tid];
        sv += psum[2][p][tid];
      }
      const double inv = 1.0 / (double)rows;
      const double qm = sq / (double)rows, km = sk / (double)rows;
      (void)inv;
      const size_t o = (bh * N + j) * D + tid;
      qbar[o] = (float)qm;
      kbar[o] = (float)km;
      vsum[o] = (float)sv;
      if (qbar64) qbar64[o] = qm;
      if (kbar64) kbar64[o] = km;
      kmean[tid] = km;
    }
    __syncthreads();
    // ---- H_j accumulated in 64-row sub-tiles ----
    for (int sub = 0; sub < rows; sub += kTile) {
      const int nv = min(kTile, rows - sub);
      for (int e = tid; e < kTile * D; e += 256) {
        const int n = e / D, c = e % D;
        float kv = 0.f, vv = 0.f;
        if (n < nv) {
          const size_t off = (size_t)(row0 + sub + n) * D + c;
          kv = (float)((double)to_f32(kh[off]) - kmean[c]);
          vv = to_f32(vh[off]);
        }
        kc[n][c] = kv;
        vs[n][c] = vv;
      }
      __syncthreads();
      for (int n = 0; n < nv; ++n) {
        float ka[R], vb[R];
#pragma unroll
        for (int a = 0; a < R; ++a) ka[a] = kc[n][ta * R + a];
#pragma unroll
        for (int b = 0; b < R; ++b) vb[b] = vs[n][tb * R + b];
#pragma unroll
        for (int a = 0; a < R; ++a)
#pragma unroll
          for (int b = 0; b < R; ++b) h[a][b] = fmaf(ka[a], vb[b], h[a][b]);
      }
      __syncthreads();
    }
  }
  float* ph = partial_h + (bh * n_chunks + chunk) * (size_t)D * D;
#pragma unroll
  for (int a = 0; a < R; ++a)
#pragma unroll
    for (int b = 0; b < R; ++b) ph[(size_t)(ta * R + a) * D + tb * R + b] = h[a][b];
}

// hsum (and, if asked for, its packed bf16 split) from the per-chunk partial sums: one thread
// per matrix element.
__global__ __launch_bounds__(256) void reduce_h_kernel(const float* __restrict__ partial_h,
                                                       float* __restrict__ hsum,
                                                       unsigned short* __restrict__ hpack, int n_chunks, int D) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= D * D) return;
  reduce_h_element(partial_h, hsum, hpack, n_chunks, D, blockIdx.y, e);
}

}  // namespace

hipError_t launch_block_stats_bf16(const Dims& dm, const void* q, const void* k, const void* v,
                                       float* qbar, float* kbar, float* vsum,
                                       double* qbar64, double* kbar64, float* partial_h,
                                       void* kcen, void* vbar, const StatsPlan& plan, hipStream_t stream);

hipError_t launch_block_stats(const Dims& dm, const void* q, const void* k, const void* v,
                              float* qbar, float* kbar, float* vsum, float* hsum,
                              double* qbar64, double* kbar64, float* partial_h,
                              const StatsExtras& extra, hipStream_t stream) {
  const StatsPlan plan = stats_plan(dm);
  dim3 grid(plan.n_chunks, dm.bh());
#define PISA_STATS(T, DD)                                                                          \
  hipLaunchKernelGGL((stats_kernel<T, DD>), grid, dim3(256), 0, stream, (const T*)q, (const T*)k, \
                     (const T*)v, qbar, kbar, vsum, qbar64, kbar64, partial_h, dm.L, dm.B, dm.N,   \
                     plan.chunk_blocks, plan.n_chunks)
  if (dm.dtype == PISA_BF16) {
    hipError_t e = launch_block_stats_bf16(dm, q, k, v, qbar, kbar, vsum, qbar64, kbar64,
                                           partial_h, extra.kcen, extra.vbar, plan, stream);
    if (e != hipSuccess) return e;
  } else if (dm.d == 64) {
    PISA_STATS(float, 64);
  } else {
    PISA_STATS(float, 128);
  }
#undef PISA_STATS
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (extra.defer_reduce) return hipSuccess;   // the caller reduces the partial sums in a later launch
  const int dd = dm.d * dm.d;
  hipLaunchKernelGGL(reduce_h_kernel, dim3((dd + 255) / 256, dm.bh()), dim3(256), 0, stream,
                     partial_h, hsum, (unsigned short*)extra.hpack, plan.n_chunks, dm.d);
  return hipGetLastError();
}

}  // namespace pisa
