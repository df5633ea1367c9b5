// bf16 attention path (dense and PISA) on the gfx950 matrix cores, head_dim 128.
//
// One workgroup (4 wavefronts) per 64-row query tile.  Wave w = (kh, qh): query half
// qh (32 rows) x key half kh (32 of the 64 keys of every tile).  Each wave keeps its own
// online-softmax state; the two key halves are merged through LDS at the end.
//
// Everything is computed transposed, with v_mfma_f32_32x32x16_bf16:
//     S^T (keys x queries) = K_tile (keys x d)  *  Q^T (d x queries)
//     O^T (d    x queries) = V_tile^T (d x keys) * P^T (keys x queries)
// so that a lane owns one query column: row max / row sum are in-lane reductions plus one
// cross-half exchange, the rescale factor is a per-lane scalar, and the fp32 S^T
// accumulator converts in place into the bf16 B operand of the second product (the key
// order inside a contraction step is permuted identically on the V side).
// V is staged row-major; a lane reads 8 bytes = channels 4*lane..4*lane+3 of one key and
// byte-permutes eight such reads into the four A operands whose row `lane` stands for
// channel 4*lane + dt (dt = 0..3), i.e. output tile dt holds channels = dt (mod 4).
//
// The three phases of Alg. 1 share the tile routine:
//   Phase 1  K/V tiles of the selected blocks (all tiles for dense attention), global ->
//            registers -> LDS, double buffered;
//   Phase 2  tiles of 64 centroids: kbar split into bf16 hi + lo parts (two MFMA chains, so
//            the centroid logits keep fp32-level accuracy), logit + log2 B_j, selected
//            columns masked, values vsum_j / B_j; the mass also accumulates into l_tail;
//   Phase 3  O += (l_tail / L) s Q hsum with hsum split hi + lo, then division by l.
#include "common.h"

namespace pisa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;
constexpr int KPITCH = 272;                 // bytes per staged key row (256 + 16 pad)
constexpr int VPITCH = 256;                 // bytes per staged value row
constexpr int KBYTES = kTile * KPITCH;      // 17408
constexpr int VBYTES = kTile * VPITCH;      // 16384
constexpr int BUFBYTES = KBYTES + VBYTES;   // one (K, V) stage
constexpr int MASK_WORDS = 128;             // bitmask over blocks, N <= 4096
constexpr int SMEM_BYTES = 2 * BUFBYTES + MASK_WORDS * 4;
constexpr int MRG_STRIDE = 68;              // floats per lane in the merge buffer (64 + m, l, l_tail)
static_assert(2 * KBYTES + VBYTES + 256 <= 2 * BUFBYTES, "phase-2 staging must fit");
static_assert(2 * 64 * MRG_STRIDE * 4 <= 2 * BUFBYTES, "merge buffer must fit");

struct PB {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  const float* kbar;
  const float* vsum;
  const float* hsum;
  const int32_t* idx;
  __bf16* out;
  float* lse;
  int L, B, N, k_top, nqt, total;
  float scale;
  int dense;
};

__device__ inline unsigned int pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(unsigned int, b);
}
__device__ inline float bf16_bits_to_f32(unsigned int bits16) { return __uint_as_float(bits16 << 16); }

// Splits x into bf16 hi + bf16 lo (x ~ hi + lo); returns hi in the low 16 bits, lo in the high.
__device__ inline void split_bf16(float x, unsigned int& hi, unsigned int& lo) {
  const unsigned int p = pack_bf16(x, 0.f);
  hi = p & 0xffffu;
  const float r = x - bf16_bits_to_f32(hi);
  lo = pack_bf16(r, 0.f) & 0xffffu;
}

struct State {
  f32x16 ot[4];      // O^T tiles: ot[dt][r] <-> channel 4*rho + dt, rho = (r/4)*8 + 4h + r%4
  float m;           // running max (log2 domain, includes the scale)
  float l;           // this lane's share of the row sum
  float l_tail;      // this lane's share of the tail mass
};

// One 64-key tile.  kA/kB: staged key rows (TAIL: hi and lo parts), vS: staged value rows.
// bias (TAIL only): 64 floats, log2 B_j or -inf.  nvalid: valid keys in the tile (Phase 1).
template <bool TAIL>
__device__ inline void absorb_tile(State& st, const bf16x8 (&qreg)[8], const unsigned char* kA,
                                   const unsigned char* kB, const unsigned char* vS,
                                   const float* bias, int nvalid, float c, int lam, int h, int kh) {
  f32x16 s = {0};
  const unsigned char* krow = kA + (32 * kh + lam) * KPITCH + 16 * h;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(krow + 32 * ks);
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], s, 0, 0, 0);
  }
  if (TAIL) {
    const unsigned char* krow2 = kB + (32 * kh + lam) * KPITCH + 16 * h;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(krow2 + 32 * ks);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], s, 0, 0, 0);
    }
  }
  // ---- logits in the log2 domain, masks ----
  float x[16];
  if (TAIL) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 b = *reinterpret_cast<const float4*>(bias + 32 * kh + 8 * g + 4 * h);
      x[4 * g + 0] = fmaf(s[4 * g + 0], c, b.x);
      x[4 * g + 1] = fmaf(s[4 * g + 1], c, b.y);
      x[4 * g + 2] = fmaf(s[4 * g + 2], c, b.z);
      x[4 * g + 3] = fmaf(s[4 * g + 3], c, b.w);
    }
  } else {
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = s[r] * c;
    if (nvalid < kTile) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 32 * kh + (r / 4) * 8 + 4 * h + (r % 4);
        if (key >= nvalid) x[r] = -INFINITY;
      }
    }
  }
  float tmax = x[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, x[r]);
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
  const float m_new = fmaxf(st.m, tmax);
  const float m_safe = m_new == -INFINITY ? 0.f : m_new;
  if (__any(m_new != st.m)) {
    const float corr = __builtin_amdgcn_exp2f(st.m - m_safe);
    st.l *= corr;
    st.l_tail *= corr;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) st.ot[dt] *= corr;
    st.m = m_new;
  }
  float pe[16];
  float psum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    pe[r] = __builtin_amdgcn_exp2f(x[r] - m_safe);
    psum += pe[r];
  }
  st.l += psum;
  if (TAIL) st.l_tail += psum;
  // ---- O^T += V^T P^T ----
#pragma unroll
  for (int s2 = 0; s2 < 2; ++s2) {
    u32x4 pw;
#pragma unroll
    for (int i = 0; i < 4; ++i) pw[i] = pack_bf16(pe[8 * s2 + 2 * i], pe[8 * s2 + 2 * i + 1]);
    const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
    u32x2 vr[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int key = 32 * kh + (2 * s2 + e / 4) * 8 + 4 * h + (e % 4);
      vr[e] = *reinterpret_cast<const u32x2*>(vS + key * VPITCH + lam * 8);
    }
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      u32x4 aw;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const unsigned int w0 = (dt >> 1) ? vr[2 * i].y : vr[2 * i].x;
        const unsigned int w1 = (dt >> 1) ? vr[2 * i + 1].y : vr[2 * i + 1].x;
        aw[i] = __builtin_amdgcn_perm(w1, w0, (dt & 1) ? 0x07060302u : 0x05040100u);
      }
      st.ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), pb,
                                                          st.ot[dt], 0, 0, 0);
    }
  }
}

__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(PB p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned int* chosen = reinterpret_cast<unsigned int*>(smem + 2 * BUFBYTES);

  // XCD-aware order: consecutive workgroup ids land on different XCDs, so give each of
  // the 8 XCDs a contiguous range of (head, query tile) items; its L2 then sees one head.
  const int wg = blockIdx.x;
  const int per_xcd = (p.total + 7) / 8;
  const int item = (wg % 8) * per_xcd + wg / 8;
  if (item >= p.total) return;
  const size_t bh = item / p.nqt;
  const int qt = item % p.nqt;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lam = lane & 31, h = lane >> 5;
  const int qh = wave & 1, kh = wave >> 1;
  const int L = p.L, N = p.N;
  const __bf16* qg = p.q + bh * (size_t)L * D;
  const __bf16* kg = p.k + bh * (size_t)L * D;
  const __bf16* vg = p.v + bh * (size_t)L * D;
  const int tpb = p.B / kTile;
  const int32_t* my_idx = p.dense ? nullptr : p.idx + (bh * N + qt / tpb) * (size_t)p.k_top;
  const float c = p.scale * 1.44269504088896340736f;

  // ---- Q^T operand: this lane's query row, 8 channel slices ----
  const int q_row = qt * kTile + 32 * qh + lam;
  bf16x8 qreg[8];
  {
    const u32x4 zero = {0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 w = zero;
      if (q_row < L) w = *reinterpret_cast<const u32x4*>(qg + (size_t)q_row * D + 16 * ks + 8 * h);
      qreg[ks] = __builtin_bit_cast(bf16x8, w);
    }
  }
  if (tid < MASK_WORDS) chosen[tid] = 0u;

  State st;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) st.ot[dt] = (f32x16){0};
  st.m = -INFINITY;
  st.l = 0.f;
  st.l_tail = 0.f;

  // ---- Phase 1 ----
  const int n1 = p.dense ? (L + kTile - 1) / kTile : p.k_top * tpb;
  auto tile_of = [&](int t) -> int { return p.dense ? t : my_idx[t / tpb] * tpb + (t % tpb); };
  u32x4 kr[4], vr[4];
  auto fetch = [&](int tile) {
    const int row0 = tile * kTile;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int ch = it * 256 + tid;
      const int row = row0 + (ch >> 4), col = ch & 15;
      const u32x4 zero = {0, 0, 0, 0};
      kr[it] = zero;
      vr[it] = zero;
      if (row < L) {
        kr[it] = *reinterpret_cast<const u32x4*>(kg + (size_t)row * D + col * 8);
        vr[it] = *reinterpret_cast<const u32x4*>(vg + (size_t)row * D + col * 8);
      }
    }
  };
  auto stage = [&](int buf) {
    unsigned char* kS = smem + buf * BUFBYTES;
    unsigned char* vS = kS + KBYTES;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int ch = it * 256 + tid;
      const int row = ch >> 4, col = ch & 15;
      *reinterpret_cast<u32x4*>(kS + row * KPITCH + col * 16) = kr[it];
      *reinterpret_cast<u32x4*>(vS + row * VPITCH + col * 16) = vr[it];
    }
  };
  int tile_cur = 0;
  if (n1 > 0) {
    tile_cur = tile_of(0);
    fetch(tile_cur);
    stage(0);
  }
  __syncthreads();
  if (!p.dense) {
    for (int t = tid; t < p.k_top; t += 256) {
      const int j = my_idx[t];
      atomicOr(&chosen[j >> 5], 1u << (j & 31));
    }
  }
  for (int t = 0; t < n1; ++t) {
    const int buf = t & 1;
    int tile_next = 0;
    if (t + 1 < n1) {
      tile_next = tile_of(t + 1);
      fetch(tile_next);
    }
    const unsigned char* kS = smem + buf * BUFBYTES;
    const int nvalid = min(kTile, L - tile_cur * kTile);
    absorb_tile<false>(st, qreg, kS, nullptr, kS + KBYTES, nullptr, nvalid, c, lam, h, kh);
    if (t + 1 < n1) stage(buf ^ 1);
    tile_cur = tile_next;
    __syncthreads();
  }

  // ---- Phase 2 ----
  const bool approx = !p.dense && p.k_top < N;
  if (approx) {
    unsigned char* kHi = smem;
    unsigned char* kLo = smem + KBYTES;
    unsigned char* vS = smem + 2 * KBYTES;
    float* bias = reinterpret_cast<float*>(smem + 2 * KBYTES + VBYTES);
    const float* kb = p.kbar + bh * (size_t)N * D;
    const float* vs = p.vsum + bh * (size_t)N * D;
    const int last_rows = L - (N - 1) * p.B;
    for (int g0 = 0; g0 < N; g0 += kTile) {
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int ch = it * 256 + tid;            // float4 chunk: row = ch / 32, col4 = ch % 32
        const int n = ch >> 5, c4 = (ch & 31) * 4;
        const int j = g0 + n;
        float4 kv = make_float4(0.f, 0.f, 0.f, 0.f), vv = kv;
        if (j < N) {
          const float inv = 1.f / (float)(j == N - 1 ? last_rows : p.B);
          kv = *reinterpret_cast<const float4*>(kb + (size_t)j * D + c4);
          vv = *reinterpret_cast<const float4*>(vs + (size_t)j * D + c4);
          vv.x *= inv; vv.y *= inv; vv.z *= inv; vv.w *= inv;
        }
        unsigned int h0, l0, h1, l1, h2, l2, h3, l3;
        split_bf16(kv.x, h0, l0);
        split_bf16(kv.y, h1, l1);
        split_bf16(kv.z, h2, l2);
        split_bf16(kv.w, h3, l3);
        u32x2 hi = {h0 | (h1 << 16), h2 | (h3 << 16)};
        u32x2 lo = {l0 | (l1 << 16), l2 | (l3 << 16)};
        u32x2 vb = {pack_bf16(vv.x, vv.y), pack_bf16(vv.z, vv.w)};
        *reinterpret_cast<u32x2*>(kHi + n * KPITCH + c4 * 2) = hi;
        *reinterpret_cast<u32x2*>(kLo + n * KPITCH + c4 * 2) = lo;
        *reinterpret_cast<u32x2*>(vS + n * VPITCH + c4 * 2) = vb;
      }
      if (tid < kTile) {
        const int j = g0 + tid;
        float b = -INFINITY;
        if (j < N && !((chosen[j >> 5] >> (j & 31)) & 1u))
          b = __builtin_amdgcn_logf((float)(j == N - 1 ? last_rows : p.B));   // log2
        bias[tid] = b;
      }
      __syncthreads();
      absorb_tile<true>(st, qreg, kHi, kLo, vS, bias, kTile, c, lam, h, kh);
      __syncthreads();
    }
  }

  // ---- merge the two key halves ----
  st.l += __shfl_xor(st.l, 32);
  st.l_tail += __shfl_xor(st.l_tail, 32);
  float* mrg = reinterpret_cast<float*>(smem) + qh * 64 * MRG_STRIDE;
  if (kh == 1) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mrg[(dt * 16 + r) * 64 + lane] = st.ot[dt][r];
    mrg[64 * 64 + lane] = st.m;
    mrg[65 * 64 + lane] = st.l;
    mrg[66 * 64 + lane] = st.l_tail;
  }
  __syncthreads();
  if (kh == 1) return;
  {
    const float m1 = mrg[64 * 64 + lane], l1 = mrg[65 * 64 + lane], t1 = mrg[66 * 64 + lane];
    const float ms = fmaxf(st.m, m1);
    const float a0 = __builtin_amdgcn_exp2f(st.m - ms), a1 = __builtin_amdgcn_exp2f(m1 - ms);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        st.ot[dt][r] = st.ot[dt][r] * a0 + mrg[(dt * 16 + r) * 64 + lane] * a1;
    st.l = st.l * a0 + l1 * a1;
    st.l_tail = st.l_tail * a0 + t1 * a1;
    st.m = ms;
  }

  // ---- Phase 3: R^T = hsum^T (d_out x d_in) * Q^T (d_in x queries), weight l_tail/L * s ----
  if (approx && p.hsum) {
    const float* hs = p.hsum + bh * (size_t)D * D;
    f32x16 rt[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) rt[dt] = (f32x16){0};
    for (int ks = 0; ks < 8; ++ks) {
      float4 hv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e)
        hv[e] = *reinterpret_cast<const float4*>(hs + (size_t)(16 * ks + 8 * h + e) * D + 4 * lam);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        u32x4 ahi, alo;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float x0 = dt == 0 ? hv[2 * i].x : dt == 1 ? hv[2 * i].y : dt == 2 ? hv[2 * i].z : hv[2 * i].w;
          const float x1 = dt == 0 ? hv[2 * i + 1].x : dt == 1 ? hv[2 * i + 1].y
                         : dt == 2 ? hv[2 * i + 1].z : hv[2 * i + 1].w;
          unsigned int h0, l0, h1, l1;
          split_bf16(x0, h0, l0);
          split_bf16(x1, h1, l1);
          ahi[i] = h0 | (h1 << 16);
          alo[i] = l0 | (l1 << 16);
        }
        rt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ahi), qreg[ks],
                                                         rt[dt], 0, 0, 0);
        rt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, alo), qreg[ks],
                                                         rt[dt], 0, 0, 0);
      }
    }
    const float w = st.l_tail / (float)L * p.scale;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) st.ot[dt] += rt[dt] * w;
  }

  // ---- normalise and store ----
  if (q_row < L) {
    const float inv_l = 1.f / st.l;
    __bf16* orow = p.out + (bh * (size_t)L + q_row) * D;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      // registers 4g..4g+3 of the four tiles: channels 32g + 16h + 0..15
      u32x4 w0, w1;
#pragma unroll
      for (int rr = 0; rr < 2; ++rr) {
        const int r = 4 * g + rr;
        w0[2 * rr] = pack_bf16(st.ot[0][r] * inv_l, st.ot[1][r] * inv_l);
        w0[2 * rr + 1] = pack_bf16(st.ot[2][r] * inv_l, st.ot[3][r] * inv_l);
        const int r2 = 4 * g + 2 + rr;
        w1[2 * rr] = pack_bf16(st.ot[0][r2] * inv_l, st.ot[1][r2] * inv_l);
        w1[2 * rr + 1] = pack_bf16(st.ot[2][r2] * inv_l, st.ot[3][r2] * inv_l);
      }
      *reinterpret_cast<u32x4*>(orow + 32 * g + 16 * h) = w0;
      *reinterpret_cast<u32x4*>(orow + 32 * g + 16 * h + 8) = w1;
    }
    if (p.lse && h == 0)
      p.lse[bh * (size_t)L + q_row] =
          (st.m + __builtin_amdgcn_logf(st.l)) * 0.69314718055994530942f;
  }
}

}  // namespace

hipError_t launch_attention_bf16(const Dims& dm, const AttnArgs& a, hipStream_t stream) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  PB p;
  p.q = (const __bf16*)a.q;
  p.k = (const __bf16*)a.k;
  p.v = (const __bf16*)a.v;
  p.kbar = a.kbar;
  p.vsum = a.vsum;
  p.hsum = a.hsum;
  p.idx = a.idx;
  p.out = (__bf16*)a.out;
  p.lse = a.lse;
  p.L = dm.L;
  p.B = dm.B;
  p.N = dm.N;
  p.k_top = a.k_top;
  p.nqt = (dm.L + kTile - 1) / kTile;
  p.total = p.nqt * dm.bh();
  p.scale = dm.scale;
  p.dense = a.dense ? 1 : 0;
  const int grid = ((p.total + 7) / 8) * 8;
  hipLaunchKernelGGL(attn_bf16_kernel, dim3(grid), dim3(256), SMEM_BYTES, stream, p);
  return hipGetLastError();
}

}  // namespace pisa
