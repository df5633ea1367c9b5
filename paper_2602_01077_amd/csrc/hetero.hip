// pisa_block_heterogeneity: M_j = || H_j - Hbar ||, Hbar = (1/N) sum_j H_j, and the column
// bias log(M_j + eps) of the covariance-aware selection score (Methodology,
// "Covariance-Aware Block Selection"; H_j from "Global First-Order Correction").
//
// Everything here is fp64: the bias is added to fp64 pooled logits and has to keep their
// accuracy.  Two passes over K and V, no per-block matrices in memory:
//   (1) hsum64_kernel   one workgroup per chunk of blocks accumulates sum_j H_j on the fp64
//                       matrix cores; the partial sums are added in chunk order and divided
//                       by N (hbar64_kernel).  A caller that accepts Hbar at fp32 accuracy hands
//                       in the hsum of the statistics pass instead and saves this pass;
//   (2) frob_kernel     one workgroup per block rebuilds H_j the same way, subtracts Hbar and
//                       takes the Frobenius norm; or
//       hetero_kernel   (spectral norm) rebuilds H_j on the vector ALUs, a thread owning an
//                       R x R patch (R = d/16), and finds the largest eigenvalue of D^T D by a
//                       locally optimal three-term iteration run to a relative residual.
#include <hip/hip_bf16.h>

#include "common.h"

namespace pisa {
namespace {

template <typename T> __device__ inline double to_f64(T x);
template <> __device__ inline double to_f64<float>(float x) { return (double)x; }
template <> __device__ inline double to_f64<__hip_bfloat16>(__hip_bfloat16 x) { return (double)__bfloat162float(x); }

// h += sum over the rows of block j of (k_n - kbar_j)^T v_n.  kc / vs: LDS staging of kSubV
// tokens at a time (two workgroups per CU fit their LDS).
constexpr int kSubV = 32;
template <typename T, int D>
__device__ inline void add_block_H(double (&h)[D / 16][D / 16], const T* kh, const T* vh,
                                   const double* kmean /* kbar64 row of block j */, int row0, int rows,
                                   double (*kc)[D], float (*vs)[D]) {
  constexpr int R = D / 16;
  const int tid = threadIdx.x, ta = tid / 16, tb = tid % 16;
  for (int sub = 0; sub < rows; sub += kSubV) {
    const int nv = min(kSubV, rows - sub);
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

typedef double f64x4 __attribute__((ext_vector_type(4)));

// Matrix-core version of add_block_H.  The d x d matrix is split over the four waves in
// quadrants; wave w holds TR x TR tiles of 16 x 16 (TR = d/32) as v_mfma_f64_16x16x4_f64
// accumulators: acc[a][b][e] <-> H[rb + 16a + 4e + l/16][cb + 16b + l%16], rb = (d/2)(w/2),
// cb = (d/2)(w%2).  Per step of four tokens a lane supplies A[l%16][l/16] = centred key
// channel rb + 16a + l%16 of token l/16 and B[l/16][l%16] = value channel cb + 16b + l%16.
// Rows of the LDS staging are padded by 16 elements so the four token rows of a step fall
// on different banks; tokens are staged 32 at a time with 16-byte loads.
constexpr int kSub = 32;   // tokens staged at a time (two workgroups per CU fit their LDS)
template <int D> struct HStage {
  static constexpr int P = D + 16;
  double kc[kSub][P];
  float vs[kSub][P];
};

// 16 bytes of consecutive channels of one row, widened to fp64.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ inline void load(const float* p, double (&out)[4]) {
    const float4 x = *reinterpret_cast<const float4*>(p);
    out[0] = x.x; out[1] = x.y; out[2] = x.z; out[3] = x.w;
  }
};
template <> struct Vec16<__hip_bfloat16> {
  static constexpr int N = 8;
  static __device__ inline void load(const __hip_bfloat16* p, double (&out)[8]) {
    const uint4 x = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = (double)__uint_as_float(w[i] << 16);
      out[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

template <typename T, int D>
__device__ inline void add_block_H_mfma(f64x4 (&acc)[D / 32][D / 32], const T* kh, const T* vh,
                                        const double* kmean, int row0, int rows, HStage<D>& sh) {
  constexpr int TR = D / 32;
  constexpr int EPV = Vec16<T>::N;           // channels per 16-byte load
  constexpr int CPR = D / EPV;               // loads per row; divides 256, so a thread keeps its channels
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kk = lane >> 4;
  const int rb = (D / 2) * (wave >> 1), cb = (D / 2) * (wave & 1);
  const int c0 = (tid % CPR) * EPV;
  double mean[EPV];
#pragma unroll
  for (int i = 0; i < EPV; ++i) mean[i] = kmean[c0 + i];
  for (int sub = 0; sub < rows; sub += kSub) {
    const int nv = min(kSub, rows - sub);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kSub * CPR / 256; ++it) {
      const int n = (it * 256 + tid) / CPR;
      double kv[EPV], vv[EPV];
#pragma unroll
      for (int i = 0; i < EPV; ++i) kv[i] = vv[i] = 0.0;
      if (n < nv) {                          // rows past the block contribute zeros
        const size_t off = (size_t)(row0 + sub + n) * D + c0;
        Vec16<T>::load(kh + off, kv);
        Vec16<T>::load(vh + off, vv);
#pragma unroll
        for (int i = 0; i < EPV; ++i) kv[i] -= mean[i];
      }
#pragma unroll
      for (int i = 0; i < EPV; ++i) {
        sh.kc[n][c0 + i] = kv[i];
        sh.vs[n][c0 + i] = (float)vv[i];
      }
    }
    __syncthreads();
    const int steps = (nv + 3) / 4;
    for (int s4 = 0; s4 < steps; ++s4) {
      const int n = 4 * s4 + kk;
      double af[TR], bf[TR];
#pragma unroll
      for (int a = 0; a < TR; ++a) af[a] = sh.kc[n][rb + 16 * a + i16];
#pragma unroll
      for (int b = 0; b < TR; ++b) bf[b] = (double)sh.vs[n][cb + 16 * b + i16];
#pragma unroll
      for (int a = 0; a < TR; ++a)
#pragma unroll
        for (int b = 0; b < TR; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[a], bf[b], acc[a][b], 0, 0, 0);
    }
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256, 2) void hsum64_kernel(const T* __restrict__ k, const T* __restrict__ v,
                                                     const double* __restrict__ kbar64,
                                                     double* __restrict__ partial, int L, int B, int N,
                                                     int chunk_blocks, int n_chunks) {
  constexpr int TR = D / 32;
  __shared__ HStage<D> sh;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = blockIdx.x;
  const size_t bh = blockIdx.y;
  const T* kh = k + bh * (size_t)L * D;
  const T* vh = v + bh * (size_t)L * D;
  f64x4 acc[TR][TR];
#pragma unroll
  for (int a = 0; a < TR; ++a)
#pragma unroll
    for (int b = 0; b < TR; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};
  const int j_end = min(N, (chunk + 1) * chunk_blocks);
  for (int j = chunk * chunk_blocks; j < j_end; ++j)
    add_block_H_mfma<T, D>(acc, kh, vh, kbar64 + (bh * N + j) * D, j * B, min(B, L - j * B), sh);
  double* ph = partial + (bh * n_chunks + chunk) * (size_t)D * D;
  const int rb = (D / 2) * (wave >> 1), cb = (D / 2) * (wave & 1);
#pragma unroll
  for (int a = 0; a < TR; ++a)
#pragma unroll
    for (int b = 0; b < TR; ++b)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        ph[(size_t)(rb + 16 * a + 4 * e + (lane >> 4)) * D + cb + 16 * b + (lane & 15)] = acc[a][b][e];
}

// M_j = || H_j - Hbar ||_F for one block per workgroup.
template <typename T, int D>
__global__ __launch_bounds__(256, 2) void frob_kernel(const T* __restrict__ k, const T* __restrict__ v,
                                                   const double* __restrict__ kbar64,
                                                   const double* __restrict__ hbar64,
                                                   double* __restrict__ log_m, int L, int B, int N, double eps) {
  constexpr int TR = D / 32;
  __shared__ HStage<D> sh;
  __shared__ double red[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = blockIdx.x;
  const size_t bh = blockIdx.y;
  f64x4 acc[TR][TR];
#pragma unroll
  for (int a = 0; a < TR; ++a)
#pragma unroll
    for (int b = 0; b < TR; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};
  add_block_H_mfma<T, D>(acc, k + bh * (size_t)L * D, v + bh * (size_t)L * D, kbar64 + (bh * N + j) * D,
                         j * B, min(B, L - j * B), sh);
  const double* hb = hbar64 + bh * (size_t)D * D;
  const int rb = (D / 2) * (wave >> 1), cb = (D / 2) * (wave & 1);
  double ss = 0.0;
#pragma unroll
  for (int a = 0; a < TR; ++a)
#pragma unroll
    for (int b = 0; b < TR; ++b)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const double dv =
            acc[a][b][e] - hb[(size_t)(rb + 16 * a + 4 * e + (lane >> 4)) * D + cb + 16 * b + (lane & 15)];
        ss = fma(dv, dv, ss);
      }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if (lane == 0) red[wave] = ss;
  __syncthreads();
  if (tid == 0) log_m[bh * N + j] = log(sqrt((red[0] + red[1]) + (red[2] + red[3])) + eps);
}

// hbar64[bh][e] = hsum[bh][e] / N from the fp32 sum the statistics pass has already produced.
__global__ __launch_bounds__(256) void hbar_from_hsum_kernel(const float* __restrict__ hsum,
                                                             double* __restrict__ hbar64, size_t total, int N) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e < total) hbar64[e] = (double)hsum[e] / (double)N;
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

template <typename T, int D>
__global__ __launch_bounds__(256, 2) void hetero_kernel(const T* __restrict__ k, const T* __restrict__ v,
                                                     const double* __restrict__ kbar64,
                                                     const double* __restrict__ hbar64,
                                                     double* __restrict__ log_m, int L, int B, int N,
                                                     int spectral, int n_iter, double eps) {
  constexpr int R = D / 16;
  __shared__ double kc[kSubV][D];          // staging; reused as the partial-product board
  __shared__ float vs[kSubV][D];
  static_assert(sizeof(double) * kSubV * D >= sizeof(double) * D * 16, "the board must fit the staging area");
  __shared__ double xs[D], ys[D];
  __shared__ double dots[2][8];
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
    // Largest eigenvalue theta of A = D^T D by a locally optimal three-term iteration: each step
    // takes the best vector (Rayleigh-Ritz) in the span of the iterate x, its residual
    // r = A x - theta x and the previous step direction p -- the convergence of a Krylov method,
    // which the closely spaced leading singular values of these matrices need (a plain power
    // iteration is still 1-2 % short after 48 steps), with three vectors of state.  It stops
    // once ||r|| <= kRelResidual * theta: some eigenvalue of A then lies within ||r|| of theta,
    // so M = sqrt(theta) is within kRelResidual / 2 relative of a singular value, and in
    // practice (the error of a Ritz value is quadratic in the residual) exact to rounding.
    // Thread t < D holds component t of every vector; all 256 threads share the two products.
    double (*board)[16] = reinterpret_cast<double (*)[16]>(&kc[0][0]);   // [D][16] partial products
    auto apply_A = [&](double vin) -> double {               // component tid of D^T (D v)
      __syncthreads();
      if (tid < D) xs[tid] = vin;
      __syncthreads();
#pragma unroll
      for (int a = 0; a < R; ++a) {
        double pa = 0.0;
#pragma unroll
        for (int b = 0; b < R; ++b) pa = fma(dm[a][b], xs[tb * R + b], pa);
        board[ta * R + a][tb] = pa;
      }
      __syncthreads();
      if (tid < D) {
        double yv = 0.0;
#pragma unroll
        for (int t = 0; t < 16; ++t) yv += board[tid][t];
        ys[tid] = yv;
      }
      __syncthreads();
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
      return zv;
    };
    // sums of NV per-thread products over the first D threads, the same value in every thread
    auto reduce = [&](auto& vals) {
      constexpr int NV = sizeof(vals) / sizeof(double);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        double x = tid < D ? vals[i] : 0.0;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
        vals[i] = x;
      }
      __syncthreads();
      if ((tid & 63) == 0 && tid < 128) {
#pragma unroll
        for (int i = 0; i < NV; ++i) dots[tid >> 6][i] = vals[i];
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NV; ++i) vals[i] = D > 64 ? dots[0][i] + dots[1][i] : dots[0][i];
    };

    double x = tid < D ? 1.0 + 0.5 * sin(1.0 + 0.37 * (double)tid) : 0.0;    // fixed, generic start
    {
      double n2[1] = {x * x};
      reduce(n2);
      x /= sqrt(n2[0]);
    }
    double ax = apply_A(x);
    double pv = 0.0, apv = 0.0;                 // previous direction and its image (none yet)
    bool have_p = false;
    double theta;
    {
      double t1[1] = {x * ax};
      reduce(t1);
      theta = t1[0];
    }
    for (int it = 0; it < n_iter; ++it) {
      const double r = ax - theta * x;
      double d2[4] = {r * r, pv * r, pv * x, pv * pv};
      reduce(d2);
      const double rn = sqrt(d2[0]);
      if (!(rn > kRelResidual * theta)) break;             // converged (also ends on theta = 0 or NaN)
      const double q2 = r / rn;
      const double aq2 = apply_A(q2);
      // p made orthogonal to x and q2 (x is a unit vector and r is orthogonal to it)
      const double c1 = d2[2], c2 = d2[1] / rn;
      double q3 = pv - c1 * x - c2 * q2;
      double aq3 = apv - c1 * ax - c2 * aq2;
      double g[6] = {x * aq2, x * aq3, q2 * aq2, q2 * aq3, q3 * aq3, q3 * q3};
      reduce(g);
      const bool use_p = have_p && g[5] > 1e-24 * d2[3] && g[5] > 0.0;
      double g01 = g[0], g02 = 0.0, g11 = g[2], g12 = 0.0, g22 = 0.0;
      if (use_p) {
        const double inv = 1.0 / sqrt(g[5]);
        q3 *= inv;
        aq3 *= inv;
        g02 = g[1] * inv;
        g12 = g[3] * inv;
        g22 = g[4] * inv * inv;
      }
      // Largest eigenpair of the symmetric 3 x 3 (or 2 x 2) matrix G = Q^T A Q, Q = [x q2 q3]:
      // Newton on the characteristic polynomial from an upper bound of the spectrum falls
      // monotonically onto the largest root; the eigenvector is the largest cross product of
      // two rows of G - lambda I.
      const double g00 = theta;
      double lam = g00 + g11 + g22;                         // trace >= largest eigenvalue (G is positive semi-definite)
      double e0, e1, e2;
      if (use_p) {
        const double tr = g00 + g11 + g22;
        const double m2 = g00 * g11 + g00 * g22 + g11 * g22 - g01 * g01 - g02 * g02 - g12 * g12;
        const double det = g00 * (g11 * g22 - g12 * g12) - g01 * (g01 * g22 - g12 * g02) +
                           g02 * (g01 * g12 - g11 * g02);
        for (int nt = 0; nt < 60; ++nt) {
          const double f = ((lam - tr) * lam + m2) * lam - det;
          const double fp = (3.0 * lam - 2.0 * tr) * lam + m2;
          if (!(fp > 0.0)) break;
          const double step = f / fp;
          lam -= step;
          if (!(fabs(step) > 1e-16 * fabs(lam))) break;
        }
        const double a00 = g00 - lam, a11 = g11 - lam, a22 = g22 - lam;
        // cross products of row pairs (0,1), (0,2), (1,2)
        const double u0 = g01 * g12 - g02 * a11, u1 = g02 * g01 - a00 * g12, u2 = a00 * a11 - g01 * g01;
        const double v0 = g01 * a22 - g02 * g12, v1 = g02 * g02 - a00 * a22, v2 = a00 * g12 - g01 * g02;
        const double w0 = a11 * a22 - g12 * g12, w1 = g12 * g02 - g01 * a22, w2 = g01 * g12 - a11 * g02;
        const double nu = u0 * u0 + u1 * u1 + u2 * u2, nv = v0 * v0 + v1 * v1 + v2 * v2,
                     nw = w0 * w0 + w1 * w1 + w2 * w2;
        if (nu >= nv && nu >= nw) { e0 = u0; e1 = u1; e2 = u2; }
        else if (nv >= nw) { e0 = v0; e1 = v1; e2 = v2; }
        else { e0 = w0; e1 = w1; e2 = w2; }
        const double en = sqrt(e0 * e0 + e1 * e1 + e2 * e2);
        if (!(en > 0.0)) { e0 = 1.0; e1 = e2 = 0.0; }       // G is a multiple of the identity
        else { e0 /= en; e1 /= en; e2 /= en; }
      } else {
        const double half = 0.5 * (g00 - g11);
        lam = 0.5 * (g00 + g11) + sqrt(half * half + g01 * g01);
        e0 = g01;
        e1 = lam - g00;
        if (fabs(lam - g11) > fabs(e1)) { e0 = lam - g11; e1 = g01; }
        e2 = 0.0;
        const double en = sqrt(e0 * e0 + e1 * e1);
        if (!(en > 0.0)) { e0 = 1.0; e1 = 0.0; }
        else { e0 /= en; e1 /= en; }
      }
      if (e0 < 0.0) { e0 = -e0; e1 = -e1; e2 = -e2; }
      // new iterate; the part of it outside the old x is the next direction
      pv = e1 * q2 + e2 * q3;
      apv = e1 * aq2 + e2 * aq3;
      x = e0 * x + pv;
      ax = e0 * ax + apv;
      have_p = true;
      // theta = x.Ax / x.x of the vector actually held (x drifts off unit length by rounding only);
      // the residual of the next step is orthogonal to x only with this theta
      double t2[2] = {x * ax, x * x};
      reduce(t2);
      const double inv = 1.0 / sqrt(t2[1]);
      x *= inv;
      ax *= inv;
      theta = t2[0] / t2[1];
    }
    m_norm = theta > 0.0 ? sqrt(theta) : 0.0;
  }
  if (tid == 0) log_m[bh * N + j] = log(m_norm + eps);
}

}  // namespace

size_t hetero_workspace_bytes(const Dims& dm) {
  const StatsPlan plan = stats_plan(dm);
  return (size_t)dm.bh() * (plan.n_chunks + 1) * dm.d * dm.d * sizeof(double);
}

hipError_t launch_block_heterogeneity(const Dims& dm, const void* k, const void* v, const double* kbar64,
                                      const float* hsum, int spectral, int n_iter, double eps, double* log_m,
                                      double* workspace, hipStream_t stream) {
  const StatsPlan plan = stats_plan(dm);
  const int dd = dm.d * dm.d;
  double* partial = workspace;
  double* hbar = workspace + (size_t)dm.bh() * plan.n_chunks * dd;
  const dim3 g1(plan.n_chunks, dm.bh()), g2((dd + 255) / 256, dm.bh()), g3(dm.N, dm.bh());
#define PISA_HET(T, DD)                                                                                \
  do {                                                                                                  \
    if (hsum) {                                                                                         \
      const size_t total = (size_t)dm.bh() * dd;                                                        \
      hipLaunchKernelGGL(hbar_from_hsum_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, \
                         hsum, hbar, total, dm.N);                                                      \
    } else {                                                                                            \
      hipLaunchKernelGGL((hsum64_kernel<T, DD>), g1, dim3(256), 0, stream, (const T*)k, (const T*)v,    \
                         kbar64, partial, dm.L, dm.B, dm.N, plan.chunk_blocks, plan.n_chunks);          \
      hipLaunchKernelGGL(hbar64_kernel, g2, dim3(256), 0, stream, partial, hbar, plan.n_chunks, dd, dm.N); \
    }                                                                                                   \
    if (spectral)                                                                                       \
      hipLaunchKernelGGL((hetero_kernel<T, DD>), g3, dim3(256), 0, stream, (const T*)k, (const T*)v,    \
                         kbar64, hbar, log_m, dm.L, dm.B, dm.N, spectral, n_iter, eps);                 \
    else                                                                                                \
      hipLaunchKernelGGL((frob_kernel<T, DD>), g3, dim3(256), 0, stream, (const T*)k, (const T*)v,      \
                         kbar64, hbar, log_m, dm.L, dm.B, dm.N, eps);                                   \
  } while (0)
  if (dm.dtype == PISA_BF16 && dm.d == 64)
    PISA_HET(__hip_bfloat16, 64);
  else if (dm.dtype == PISA_BF16)
    PISA_HET(__hip_bfloat16, 128);
  else if (dm.d == 64)
    PISA_HET(float, 64);
  else
    PISA_HET(float, 128);
#undef PISA_HET
  return hipGetLastError();
}

}  // namespace pisa
