// pisa_block_stats for bf16 inputs, head_dim 128 or 64, block 64 or 128: one streaming pass
// (Alg. 1, "Prepare" step).  Written out for head_dim 128; the differences at 64 are noted where they occur.
//
// Grid (n_chunks, batch*heads); a workgroup of 4 waves walks `chunk_blocks` consecutive
// blocks of one head.  Per 64-token (sub-)block:
//   * wave w loads rows 16w..16w+15 of the Q, K and V tiles, one 4-byte channel pair per
//     lane (a wave-load is one 256-byte row), one sub-block ahead of their use, and adds
//     them in fp64 (exact for bf16 data);
//     the four waves' partial column sums meet in LDS and are added in wave order;
//   * K is centred on the block mean in registers, split into bf16 hi + lo parts and
//     written to LDS together with V (rows swizzled for conflict-free transposed reads);
//   * H += Kc^T V on the matrix cores: wave w owns the 32 key channels 32w..32w+31 and all
//     128 value channels (four 32x32 accumulators); both operands are contracted over
//     tokens, so both come from ds_read_b64_tr_b16.
// The partial H of the chunk goes to scratch; partials are added in chunk order by the
// caller's reduction kernel, so hsum is run-to-run identical.
#include "common.h"

namespace pisa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));
#define LDS_PTR(T) __attribute__((address_space(3))) T*


__device__ inline unsigned int pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(unsigned int, b);
}

// Swizzle of a staged [token][channel] tile: the 32-byte chunk index of row n is XORed with
// this value, which makes the transposed reads below bank-conflict free (256-byte rows: a
// 3-bit pattern; 128-byte rows, two to a bank line: bit 1 flipped for every other row pair).
template <int D> __device__ inline int swz3(int n) {
  return D == 128 ? (((n & 3) << 1) | ((n >> 2) & 1)) : (((n >> 1) & 1) << 1);
}

// Byte address of channel pair `c2` (channels 2 c2, 2 c2 + 1) of row n in a swizzled tile.
template <int D> __device__ inline int swz_pair(int n, int c2) {
  const int byte = c2 * 4;
  return n * (2 * D) + ((((byte >> 5) ^ swz3<D>(n)) << 5) | (byte & 31));
}

// A / B operand of v_mfma_f32_32x32x16_bf16 for contraction step `step` (16 tokens) and
// channel tile `ct` (32 channels), read transposed from a swizzled [token][channel] tile.
template <int D>
__device__ inline bf16x8 read_operand(LDS_PTR(const unsigned char) tile, int lane, int step, int ct) {
  constexpr int ROWB = 2 * D;
  const int j16 = lane & 15, h = lane >> 5, lhalf = (lane >> 4) & 1;
  const int kq = 4 * h + (j16 >> 2);
  const int off = (16 * step + kq) * ROWB + 8 * (j16 & 3) + (((2 * ct + lhalf) ^ swz3<D>(kq)) << 5);
  LDS_PTR(unsigned char) p = const_cast<LDS_PTR(unsigned char)>(tile) + off;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_PTR(s16x4)>(p));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_PTR(s16x4)>(p + 8 * ROWB));
  const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
  const u32x4 w = {l2.x, l2.y, h2.x, h2.y};
  return __builtin_bit_cast(bf16x8, w);
}

// TPB = tiles (64-token sub-blocks) per block: 1 for block 64, 2 for block 128.  With two
// sub-blocks each is centred on its OWN mean c_s for the matrix-core contraction, and the
// block's H_j follows from  sum_n (k_n - c_s)^T v_n = sum_n (k_n - kbar_j)^T v_n + (kbar_j - c_s)^T Vhat_s :
//   H_j = sum_s [ A_s + (c_s - kbar_j)^T Vhat_s ],
// a small rank-one correction per sub-block (c_s is close to kbar_j, so nothing cancels).
// Head_dim 64: a 256-byte wave-load is two rows (lane = row parity x channel pair), a lane
// holds 8 rows per tensor instead of 16, the two row parities are added with one lane
// exchange, and the 64 x 64 matrix H is four 32 x 32 tiles, one per wave.
//
// HETERO: the same walk used for the covariance-aware score instead of the statistics: every
// block's H_j is rebuilt exactly as above (same centring, same hi/lo split, same products, so
// the same bits that went into hsum), kept per block instead of summed over the chunk, and
// reduced to log(||H_j - hsum / N||_F + eps); nothing else is written and Q is not read.
template <int D, int TPB, bool HETERO>
__global__ __launch_bounds__(256, 2) void stats_bf16_kernel(
    const unsigned int* __restrict__ q, const unsigned int* __restrict__ k, const unsigned int* __restrict__ v,
    float* __restrict__ qbar, float* __restrict__ kbar, float* __restrict__ vsum,
    double* __restrict__ qbar64, double* __restrict__ kbar64, float* __restrict__ partial_h,
    unsigned short* __restrict__ kcen, unsigned short* __restrict__ vbar, int npad,
    int L, int N, int chunk_blocks, int n_chunks,
    const float* __restrict__ hsum, double eps, double* __restrict__ log_m) {
  constexpr int B = TPB * kTile;
  constexpr int TILEB = kTile * 2 * D;
  constexpr int LPR = D / 2;            // lanes per row (one channel pair each)
  constexpr int RPW = 64 / LPR;         // rows per wave-load
  constexpr int NR = 16 / RPW;          // loads per lane and tensor
  constexpr int NB = D / 32 / (D == 128 ? 1 : 2);   // value tiles per wave: 4, or 1
  __shared__ __attribute__((aligned(1024))) unsigned char khi_s[TILEB];
  __shared__ __attribute__((aligned(1024))) unsigned char klo_s[TILEB];
  __shared__ __attribute__((aligned(1024))) unsigned char v_s[TILEB];
  __shared__ __attribute__((aligned(16))) double red[3][4][D];
  __shared__ double tot[3][D];          // block totals over the sub-blocks (q, k, v)
  __shared__ double csub[2][D];         // sub-block key means c_s
  __shared__ float vsub[2][D];          // sub-block value sums Vhat_s
  __shared__ float dks[2][D];           // c_s - kbar_j
  __shared__ float kmean_s[D];
  __shared__ double hnorm_s[4];         // HETERO: per-wave sums of squares

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: row addresses stay scalar
  const int chunk = blockIdx.x;
  const size_t bh = blockIdx.y;
  const size_t head_words = (size_t)L * (D / 2);
  const unsigned int* qh = q + bh * head_words;
  const unsigned int* kh = k + bh * head_words;
  const unsigned int* vh = v + bh * head_words;
  LDS_PTR(unsigned char) khi = (LDS_PTR(unsigned char))khi_s;
  LDS_PTR(unsigned char) klo = (LDS_PTR(unsigned char))klo_s;
  LDS_PTR(unsigned char) vt = (LDS_PTR(unsigned char))v_s;
  const int lam = lane & 31, h = lane >> 5;
  const int rp = lane / LPR, cp = lane % LPR;        // row parity inside a wave-load, channel pair
  const int ktile = D == 128 ? wave : (wave & 1);    // this wave's 32 key channels of H
  const int vtile0 = D == 128 ? 0 : (wave >> 1);     // its first 32-value-channel tile

  f32x16 acc[NB];
#pragma unroll
  for (int bt = 0; bt < NB; ++bt) acc[bt] = (f32x16){0};

  // HETERO: 1 / N, and this head's hsum (read per block from L2: 64 more registers would not fit)
  const float inv_n = 1.f / (float)N;
  const float* hs_head = HETERO ? hsum + bh * (size_t)D * D : nullptr;

  // Optional second form of the block outputs, for the attention kernel's centroid phase: the
  // key mean and the value mean of block j as bf16 rows of tiles [bh][npad][D] (the fp32
  // values just written, rounded to nearest even; rows N .. npad - 1 are zero).  Called by
  // the threads tid < D.
  auto centroid_rows = [&](int j, float kmean, float vs, int rows_in_block) {
    if (!kcen) return;
    const size_t o = (bh * (size_t)npad + j) * D + tid;
    kcen[o] = (unsigned short)pack_bf16(kmean, 0.f);
    vbar[o] = (unsigned short)pack_bf16(vs * (1.f / (float)rows_in_block), 0.f);
    if (j == N - 1)
      for (int jj = N; jj < npad; ++jj) {
        const size_t oz = (bh * (size_t)npad + jj) * D + tid;
        kcen[oz] = 0;
        vbar[oz] = 0;
      }
  };

  // This wave's 16 rows of one 64-token sub-block, one channel pair per lane.  Rows past the
  // end repeat the last valid row (the users mask them), so the loads carry no conditions.
  auto load_rows = [&](const unsigned int* src, int row0, int rows, unsigned int (&x)[NR]) {
    if (rows <= 0) return;
#pragma unroll
    for (int i = 0; i < NR; ++i)
      x[i] = src[(size_t)(row0 + min(16 * wave + RPW * i + rp, rows - 1)) * (D / 2) + cp];
  };

  const int j_begin = chunk * chunk_blocks;
  const int j_end = min(N, j_begin + chunk_blocks);
  // The rows of sub-block t + 1 are requested while sub-block t is worked on (K and V at its
  // start into a second register set, Q into its own registers once its sums are taken), so a
  // wave always has 8 to 12 KB of loads in flight.
  unsigned int kx[NR] = {}, vx[NR] = {}, qx[NR] = {}, kn[NR] = {}, vn[NR] = {};
  if (j_begin < j_end) {
    const int rows = min(kTile, L - j_begin * B);
    if (!HETERO) load_rows(qh, j_begin * B, rows, qx);
    load_rows(kh, j_begin * B, rows, kx);
    load_rows(vh, j_begin * B, rows, vx);
  }
  for (int j = j_begin; j < j_end; ++j) {
    const int block_rows = min(B, L - j * B);
    int n_sub = 0;
    for (int sub = 0; sub < TPB; ++sub) {
      const int row0 = j * B + sub * kTile;
      const int rows = min(kTile, L - row0);
      if (rows <= 0) break;                       // uniform: the block ends inside its first half
      n_sub = sub + 1;
      int next_row0, next_rows;
      {
        int nj = j, ns = sub + 1;
        if (ns == TPB || j * B + ns * kTile >= L) {
          nj = j + 1;
          ns = 0;
        }
        next_row0 = nj * B + ns * kTile;
        next_rows = nj < j_end ? min(kTile, L - next_row0) : 0;
        load_rows(kh, next_row0, next_rows, kn);
        load_rows(vh, next_row0, next_rows, vn);
      }
      // ---- fp64 column sums of the 16 rows (absent rows are zeroed first) ----
      double sq0 = 0, sq1 = 0, sk0 = 0, sk1 = 0, sv0 = 0, sv1 = 0;
#pragma unroll
      for (int i = 0; i < NR; ++i) {
        if (16 * wave + RPW * i + rp >= rows) {   // uniform at head_dim 128
          qx[i] = kx[i] = vx[i] = 0u;
        }
        sq0 += (double)__uint_as_float(qx[i] << 16);
        sq1 += (double)__uint_as_float(qx[i] & 0xffff0000u);
        sk0 += (double)__uint_as_float(kx[i] << 16);
        sk1 += (double)__uint_as_float(kx[i] & 0xffff0000u);
        sv0 += (double)__uint_as_float(vx[i] << 16);
        sv1 += (double)__uint_as_float(vx[i] & 0xffff0000u);
      }
      if (RPW == 2) {                             // the other row parity of the same channels
        sq0 += __shfl_xor(sq0, 32); sq1 += __shfl_xor(sq1, 32);
        sk0 += __shfl_xor(sk0, 32); sk1 += __shfl_xor(sk1, 32);
        sv0 += __shfl_xor(sv0, 32); sv1 += __shfl_xor(sv1, 32);
      }
      if (lane < LPR) {
        *reinterpret_cast<f64x2*>(&red[0][wave][2 * cp]) = (f64x2){sq0, sq1};
        *reinterpret_cast<f64x2*>(&red[1][wave][2 * cp]) = (f64x2){sk0, sk1};
        *reinterpret_cast<f64x2*>(&red[2][wave][2 * cp]) = (f64x2){sv0, sv1};
      }
      if (!HETERO) load_rows(qh, next_row0, next_rows, qx);    // Q(t) is used up
      __syncthreads();
      if (tid < D) {
        const double sq = ((red[0][0][tid] + red[0][1][tid]) + red[0][2][tid]) + red[0][3][tid];
        const double sk = ((red[1][0][tid] + red[1][1][tid]) + red[1][2][tid]) + red[1][3][tid];
        const double sv = ((red[2][0][tid] + red[2][1][tid]) + red[2][2][tid]) + red[2][3][tid];
        const double cm = sk / (double)rows;
        if (TPB == 1) {
          if (!HETERO) {
            const double qm = sq / (double)rows;
            const size_t o = (bh * N + j) * D + tid;
            qbar[o] = (float)qm;
            kbar[o] = (float)cm;
            vsum[o] = (float)sv;
            if (qbar64) qbar64[o] = qm;
            if (kbar64) kbar64[o] = cm;
            centroid_rows(j, (float)cm, (float)sv, rows);
          }
        } else {
          tot[0][tid] = sub == 0 ? sq : tot[0][tid] + sq;
          tot[1][tid] = sub == 0 ? sk : tot[1][tid] + sk;
          tot[2][tid] = sub == 0 ? sv : tot[2][tid] + sv;
          csub[sub][tid] = cm;
          vsub[sub][tid] = (float)sv;
        }
        kmean_s[tid] = (float)cm;
      }
      __syncthreads();
      // ---- centre K on the sub-block mean, split hi/lo, stage with V ----
      {
        const float m0 = kmean_s[2 * cp], m1 = kmean_s[2 * cp + 1];
#pragma unroll
        for (int i = 0; i < NR; ++i) {
          const int n = 16 * wave + RPW * i + rp;
          unsigned int hi = 0u, lo = 0u;
          if (n < rows) {
            const float c0 = __uint_as_float(kx[i] << 16) - m0;
            const float c1 = __uint_as_float(kx[i] & 0xffff0000u) - m1;
            hi = pack_bf16(c0, c1);
            lo = pack_bf16(c0 - __uint_as_float(hi << 16), c1 - __uint_as_float(hi & 0xffff0000u));
          }
          const int a = swz_pair<D>(n, cp);
          *reinterpret_cast<LDS_PTR(unsigned int)>(khi + a) = hi;
          *reinterpret_cast<LDS_PTR(unsigned int)>(klo + a) = lo;
          *reinterpret_cast<LDS_PTR(unsigned int)>(vt + a) = vx[i];
        }
      }
      __syncthreads();
      // ---- H[32 ktile .. +32][this wave's value tiles] += Kc^T V over the 64 tokens ----
#pragma unroll
      for (int step = 0; step < 4; ++step) {
        const bf16x8 ahi = read_operand<D>(khi, lane, step, ktile);
        const bf16x8 alo = read_operand<D>(klo, lane, step, ktile);
#pragma unroll
        for (int bt = 0; bt < NB; ++bt) {
          const bf16x8 b = read_operand<D>(vt, lane, step, vtile0 + bt);
          acc[bt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, b, acc[bt], 0, 0, 0);
          acc[bt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(alo, b, acc[bt], 0, 0, 0);
        }
      }
      // the next sub-block's LDS writes are separated from these reads by its two barriers
#pragma unroll
      for (int i = 0; i < NR; ++i) {
        kx[i] = kn[i];
        vx[i] = vn[i];
      }
    }
    if (TPB == 2) {
      // ---- block outputs from the sub-block totals, then the rank-one corrections ----
      if (tid < D) {
        const double qm = tot[0][tid] / (double)block_rows, km = tot[1][tid] / (double)block_rows;
        if (!HETERO) {
          const size_t o = (bh * N + j) * D + tid;
          qbar[o] = (float)qm;
          kbar[o] = (float)km;
          vsum[o] = (float)tot[2][tid];
          if (qbar64) qbar64[o] = qm;
          if (kbar64) kbar64[o] = km;
          centroid_rows(j, (float)km, (float)tot[2][tid], block_rows);
        }
        for (int sub = 0; sub < n_sub; ++sub) dks[sub][tid] = (float)(csub[sub][tid] - km);
      }
      __syncthreads();
      for (int sub = 0; sub < n_sub; ++sub) {
#pragma unroll
        for (int bt = 0; bt < NB; ++bt) {
          const float vb = vsub[sub][32 * (vtile0 + bt) + lam];
#pragma unroll
          for (int r = 0; r < 16; ++r)
            acc[bt][r] = fmaf(dks[sub][32 * ktile + (r / 4) * 8 + 4 * h + (r % 4)], vb, acc[bt][r]);
        }
      }
      __syncthreads();                            // dks / vsub / tot are rewritten by the next block
    }
    if (HETERO) {
      // acc holds H_j; this lane's elements sit at fixed positions of the matrix
      double ss = 0.0;
      const float* hp = hs_head;
      asm volatile("" : "+s"(hp));    // keeps the 64 loads below inside the block loop (hoisted, they spill)
#pragma unroll
      for (int bt = 0; bt < NB; ++bt) {
        float hb[16];                 // the elements of hsum at this lane's accumulator positions (see the store below)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          hb[r] = hp[(size_t)(32 * ktile + (r / 4) * 8 + 4 * h + (r % 4)) * D + 32 * (vtile0 + bt) + lam];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const double dlt = (double)fmaf(-hb[r], inv_n, acc[bt][r]);   // both terms carry fp32 rounding already
          ss = fma(dlt, dlt, ss);
          acc[bt][r] = 0.f;
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
      if (lane == 0) hnorm_s[wave] = ss;
      __syncthreads();
      if (tid == 0)
        log_m[bh * N + j] = log(sqrt(((hnorm_s[0] + hnorm_s[1]) + hnorm_s[2]) + hnorm_s[3]) + eps);
      // hnorm_s is written again only after the next block's barriers
    }
  }
  if (HETERO) return;
  // acc[bt][r] = H[32 ktile + (r/4)*8 + 4h + r%4][32 (vtile0 + bt) + lam]
  float* ph = partial_h + (bh * n_chunks + chunk) * (size_t)D * D;
#pragma unroll
  for (int bt = 0; bt < NB; ++bt)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      ph[(size_t)(32 * ktile + (r / 4) * 8 + 4 * h + (r % 4)) * D + 32 * (vtile0 + bt) + lam] = acc[bt][r];
}

}  // namespace

hipError_t launch_block_stats_bf16(const Dims& dm, const void* q, const void* k, const void* v,
                                   float* qbar, float* kbar, float* vsum,
                                   double* qbar64, double* kbar64, float* partial_h,
                                   void* kcen, void* vbar, const StatsPlan& plan, hipStream_t stream) {
  const int npad = ((dm.N + kTile - 1) / kTile) * kTile;
  const dim3 grid(plan.n_chunks, dm.bh());
#define PISA_STATS_BF16(DD, TPB)                                                                           \
  hipLaunchKernelGGL((stats_bf16_kernel<DD, TPB, false>), grid, dim3(256), 0, stream, (const unsigned int*)q, \
                     (const unsigned int*)k, (const unsigned int*)v, qbar, kbar, vsum, qbar64, kbar64,     \
                     partial_h, (unsigned short*)kcen, (unsigned short*)vbar, npad, dm.L, dm.N,                \
                     plan.chunk_blocks, plan.n_chunks, nullptr, 0.0, nullptr)
  if (dm.d == 128 && dm.B == kTile) PISA_STATS_BF16(128, 1);
  else if (dm.d == 128) PISA_STATS_BF16(128, 2);
  else if (dm.B == kTile) PISA_STATS_BF16(64, 1);
  else PISA_STATS_BF16(64, 2);
#undef PISA_STATS_BF16
  return hipGetLastError();
}

// log(||H_j - hsum / N||_F + eps) per block with H_j rebuilt on the bf16 matrix cores (fp32-level
// accuracy, the accuracy hsum itself has).
hipError_t launch_block_heterogeneity_fast(const Dims& dm, const void* k, const void* v, const float* hsum,
                                           double eps, double* log_m, hipStream_t stream) {
  const StatsPlan plan = stats_plan(dm);
  const dim3 grid(plan.n_chunks, dm.bh());
#define PISA_HET_FAST(DD, TPB)                                                                              \
  hipLaunchKernelGGL((stats_bf16_kernel<DD, TPB, true>), grid, dim3(256), 0, stream, nullptr,               \
                     (const unsigned int*)k, (const unsigned int*)v, nullptr, nullptr, nullptr, nullptr,    \
                     nullptr, nullptr, nullptr, nullptr, 0, dm.L, dm.N, plan.chunk_blocks, plan.n_chunks,   \
                     hsum, eps, log_m)
  if (dm.d == 128 && dm.B == kTile) PISA_HET_FAST(128, 1);
  else if (dm.d == 128) PISA_HET_FAST(128, 2);
  else if (dm.B == kTile) PISA_HET_FAST(64, 1);
  else PISA_HET_FAST(64, 2);
#undef PISA_HET_FAST
  return hipGetLastError();
}

}  // namespace pisa
