// bf16 attention path (dense and PISA) on the gfx950 matrix cores, head_dim 128 or 64
// (everything below is a template over the head dimension D).
//
// Workgroup = 4 wavefronts = 128 query rows (two adjacent 64-row query blocks, or one
// 128-row block); wave w owns rows 32w..32w+31 and sees every key of a staged tile.
// Two workgroups fit a CU (2 x 75 KB LDS at D = 128, <= 256 VGPRs), so barrier stalls of one
// are covered by the other.
//
// Everything is computed transposed with v_mfma_f32_32x32x16_bf16:
//     S^T (keys x queries) = K_tile (keys x d)   *  Q^T (d x queries)
//     O^T (d    x queries) = V_tile^T (d x keys) *  P^T (keys x queries)
// A lane therefore owns one query column: row max / row sum are in-lane reductions plus
// one exchange with lane^32, the rescale factor is a per-lane scalar, and the fp32 S^T
// accumulator converts in place into the bf16 B operand of the second product (the key
// order inside a contraction step is permuted identically on the V side).
//
// Staging: K and V tiles (64 rows x 2 D bytes) go global -> LDS with global_load_lds_dwordx4
// (no registers in between), double buffered, one barrier per tile.  A wave-load writes
// 1 KB of consecutive LDS, so bank conflicts are avoided by permuting which global chunk
// each lane fetches: K rows XOR their 16-byte chunk index with a function of the row
// (conflict-free ds_read_b128 of one chunk from 16 different rows); V rows XOR their 32-byte
// chunk index with another (conflict-free ds_read_b64_tr_b16, which hands a 16-lane group a
// 16-channel x 4-key transposed fragment, i.e. the V^T operand straight from row-major V).
//
// Tile loop: one barrier per trip; after it the loads of K(t+2) and V(t+1) go out, then the
// softmax of trip t, O^T += V(t)^T P(t)^T, and S^T(t+1) into the score registers the softmax
// has just consumed.  The running maximum is lazy: a full exact tile is exponentiated against
// the maximum as it stands and the exact step (new maximum, rescale) runs only when a tile sum
// nears overflow or on a wave's first tile.
//
// PISA, block 64: the index rows of the workgroup's two query blocks are merged into a trip
// list in LDS.  A tile both blocks selected is one full trip; the tiles only one block selected
// are paired (i-th of the first block with i-th of the second) and each pair is walked as two
// split trips in which the stage holds 32 keys of either tile and each block's waves take their
// half, so no wave sits a trip out and every unshared tile is still loaded once.  A workgroup
// whose rows coincide runs the loop without the half guards (the dense kernel's code).
// Phase 2 streams bf16 centroid tiles (kbar_j rounded to bf16, the precision the keys
// themselves arrive in; vsum_j / B_j), written by a small pre-pass or, in the one-call entry
// point, by the statistics kernels; Phase 3 multiplies by the pre-packed hi/lo split of hsum,
// staged through LDS once per workgroup.
#include <mutex>
#include <type_traits>

#include "common.h"

namespace pisa {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T) __attribute__((address_space(3))) T*
#define GLB_PTR(T) const __attribute__((address_space(1))) T*

// Geometry of a head dimension D (128 or 64): a staged K or V tile is 64 rows of 2 D bytes.
template <int D> struct Geo {
  static constexpr int ROWB = 2 * D;               // bytes per staged row
  static constexpr int TILEB = kTile * ROWB;       // one staged K or V tile (16 KB / 8 KB)
  static constexpr int NKS = D / 16;               // contraction steps of S^T = K Q^T
  static constexpr int NDT = D / 32;               // 32-channel tiles of O^T
  static constexpr int CPR = ROWB / 16;            // 16-byte chunks per row
  static constexpr int RPL = 1024 / ROWB;          // rows a wave-load (1 KB) covers
  static constexpr int NLD = kTile / (4 * RPL);    // loads per wave and tile
};
constexpr int QROWS = 128;                   // query rows per workgroup
constexpr int MASK_WORDS = kMaxBlocks / 32;  // 128 words per block bitmask

struct PB {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  const __bf16* kcen;     // [bh][npad][D] kbar_j rounded to bf16    (pre-pass)
  const __bf16* vbar;     // [bh][npad][D] vsum_j / B_j
  const __bf16* hpack;    // [bh][2][D/16 ks][D/32 dt][64 lanes][8] hsum^T hi / lo in A-operand order
  const int32_t* idx;
  __bf16* out;
  float* lse;
  int L, B, N, k_top, npad, n_super, total;
  float scale;
  int first_order;
  const int32_t* pair;    // block 64 only, may be null: [bh][2 * n_super] query blocks of each workgroup (-1: none)
};

__device__ inline unsigned int pack_bf16(float lo, float hi) {
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(unsigned int, b);
}
__device__ inline float bf16_bits_to_f32(unsigned int bits16) { return __uint_as_float(bits16 << 16); }
__device__ inline void split_bf16(float x, unsigned int& hi, unsigned int& lo) {
  hi = pack_bf16(x, 0.f) & 0xffffu;
  lo = pack_bf16(x - bf16_bits_to_f32(hi), 0.f) & 0xffffu;
}

// ---------------------------------------------------------------------------------
// Pre-pass for PISA: centroid tiles and hsum in the forms the main kernel consumes.
// grid (npad/64 + kPackBlocks, bh); the extra blocks of each head pack hsum.
// ---------------------------------------------------------------------------------
constexpr int kPackBlocks = 8;
template <int D>
__global__ __launch_bounds__(256) void attn_prep_kernel(
    const float* __restrict__ kbar, const float* __restrict__ vsum, const float* __restrict__ hsum,
    __bf16* __restrict__ kcen, __bf16* __restrict__ vbar,
    __bf16* __restrict__ hpack, int L, int B, int N, int npad) {
  const int tid = threadIdx.x;
  const size_t bh = blockIdx.y;
  const int g = blockIdx.x;
  constexpr int ROWB = Geo<D>::ROWB, NDT = Geo<D>::NDT;
  const int last_rows = L - (N - 1) * B;
  if (g < npad / kTile) {
    const float* kb = kbar + bh * (size_t)N * D;
    const float* vs = vsum + bh * (size_t)N * D;
    unsigned char* ok = reinterpret_cast<unsigned char*>(kcen + bh * (size_t)npad * D);
    unsigned char* ov = reinterpret_cast<unsigned char*>(vbar + bh * (size_t)npad * D);
#pragma unroll
    for (int it = 0; it < kTile * (D / 4) / 256; ++it) {
      const int ch = it * 256 + tid;
      const int n = ch / (D / 4), c4 = (ch % (D / 4)) * 4;
      const int j = g * kTile + n;
      float4 kv = make_float4(0.f, 0.f, 0.f, 0.f), vv = kv;
      if (j < N) {
        const float inv = 1.f / (float)(j == N - 1 ? last_rows : B);
        kv = *reinterpret_cast<const float4*>(kb + (size_t)j * D + c4);
        vv = *reinterpret_cast<const float4*>(vs + (size_t)j * D + c4);
        vv.x *= inv; vv.y *= inv; vv.z *= inv; vv.w *= inv;
      }
      const u32x2 kc = {pack_bf16(kv.x, kv.y), pack_bf16(kv.z, kv.w)};
      const u32x2 vb = {pack_bf16(vv.x, vv.y), pack_bf16(vv.z, vv.w)};
      const size_t o = (size_t)j * ROWB + c4 * 2;
      *reinterpret_cast<u32x2*>(ok + o) = kc;
      *reinterpret_cast<u32x2*>(ov + o) = vb;
    }
  } else if (hsum) {
    // hpack[part][ks][dt][lane][e] = part(hsum[d_in = 16 ks + 8 h + e][d_out = 32 dt + lam]);
    // each of the kPackBlocks extra blocks of a head packs one slice of the d x d matrix.
    const float* hs = hsum + bh * (size_t)D * D;
    __bf16* hp = hpack + bh * (size_t)(2 * D * D);
    constexpr int PER = D * D / kPackBlocks / 256;      // elements per thread
    const int o0 = (g - npad / kTile) * (D * D / kPackBlocks) + tid;
    float x[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int o = o0 + 256 * u;
      const int e = o & 7, lane = (o >> 3) & 63, dt = (o >> 9) % NDT, ks = (o >> 9) / NDT;
      const int lam = lane & 31, h = lane >> 5;
      x[u] = hs[(size_t)(16 * ks + 8 * h + e) * D + 32 * dt + lam];
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int o = o0 + 256 * u;
      unsigned int hi, lo;
      split_bf16(x[u], hi, lo);
      reinterpret_cast<unsigned short*>(hp)[o] = (unsigned short)hi;
      reinterpret_cast<unsigned short*>(hp)[D * D + o] = (unsigned short)lo;
    }
  }
}

// ---------------------------------------------------------------------------------
// Main kernel
// ---------------------------------------------------------------------------------
template <int D> struct State {
  f32x16 ot[D / 32]; // O^T tiles: ot[dt][r] <-> channel 32 dt + (r/4)*8 + 4h + r%4
  float m;           // running max (log2 domain, scale included)
  float l;           // this lane's share of the row sum (keys with its h)
  float l_tail;      // this lane's share of the tail mass
};

// Per-lane constants of the staging layout, computed once per kernel.
// LDS-DMA: a staged tile is kTile * ROWB / 1024 pieces of 1 KB (RPL rows each); wave w fills
// the NLD consecutive pieces NLD w .. NLD w + NLD - 1, i.e. tile rows 16 w .. 16 w + 15, with
// NLD instructions that differ only in their immediate offset (i KB), which the hardware adds
// to the global address and to the LDS address alike: one scalar base and one M0 value serve
// all of a wave's loads of a tile.  The bank swizzle depends on the row, so each load has its
// own per-lane byte offset (position inside its 1 KB piece).
struct LaneCtx {
  unsigned dma_k[4], dma_v[4];   // per-lane byte offset inside piece i of a global tile: K format / V format
  int dma_r0;              // tile row of the first load (load i: row dma_r0 + RPL i)
  unsigned wave;           // wave index (uniform)
  LDS_PTR(const unsigned char) kbase;   // K operand address of contraction step 0
  LDS_PTR(const unsigned char) vbase;   // V^T operand address of channel tile 0
  int h;
};

// One LDS-DMA instruction: 64 lanes x 16 bytes, global (base + voff + IMM) -> LDS (M0 + IMM +
// 16 lane).  It goes through inline asm on purpose: the compiler then does not track it and
// puts no vmcnt wait in front of LDS reads of the other stage; completion is enforced by
// wait_async_loads() + barrier before a stage is read.  M0 is written by the caller.
template <int IMM>
__device__ inline void dma_1kb(unsigned voff, const unsigned char* base /* wave-uniform */) {
  static_assert(IMM >= 0 && IMM < 4096, "13-bit signed immediate offset");
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(voff), "s"(base), "n"(IMM) : "memory");
}
// The instruction takes its LDS base from M0; a scalar write of M0 needs one wait state before
// an LDS-DMA instruction reads it, and the compiler cannot see inside the asm string, so the
// s_nop is written out.
__device__ inline void set_dma_lds_base(unsigned lds_byte_address /* wave-uniform */) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(lds_byte_address) : "memory", "m0");
}

// Asynchronous global -> LDS load of one 64-row tile starting at `tile_base` (wave-uniform):
// this wave's NLD pieces.  rows_avail < 64: rows past the end are replaced by the last valid
// row (finite data; such keys are masked by the caller).
template <int D, bool KFMT>
__device__ inline void load_tile_async(const LaneCtx& lc, const unsigned char* tile_base, int rows_avail,
                                       unsigned lds_stage /* LDS byte address of the destination tile */) {
  constexpr int NLD = Geo<D>::NLD, RPL = Geo<D>::RPL, ROWB = Geo<D>::ROWB;
  const unsigned piece0 = __builtin_amdgcn_readfirstlane(lc.wave * (NLD * 1024));
  set_dma_lds_base(lds_stage + piece0);
  if (rows_avail >= kTile) {
    const unsigned char* base = tile_base + piece0;
    dma_1kb<0>(KFMT ? lc.dma_k[0] : lc.dma_v[0], base);
    dma_1kb<1024>(KFMT ? lc.dma_k[1] : lc.dma_v[1], base);
    if (NLD == 4) {
      dma_1kb<2048>(KFMT ? lc.dma_k[2] : lc.dma_v[2], base);
      dma_1kb<3072>(KFMT ? lc.dma_k[3] : lc.dma_v[3], base);
    }
  } else {
    // per-lane source rows, stepped back to the last valid one; the immediate offset still
    // moves the LDS side, so it is taken off the global address again
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int r = lc.dma_r0 + RPL * i;
      const int back = max(r - (rows_avail - 1), 0);                    // rows to step back
      const unsigned voff = KFMT ? lc.dma_k[i] : lc.dma_v[i];
      const unsigned char* src = tile_base + piece0 + (long long)voff - (long long)back * ROWB;
      if (i == 0) asm volatile("global_load_lds_dwordx4 %0, off" : : "v"(src) : "memory");
      if (i == 1) asm volatile("global_load_lds_dwordx4 %0, off offset:1024" : : "v"(src) : "memory");
      if (i == 2) asm volatile("global_load_lds_dwordx4 %0, off offset:2048" : : "v"(src) : "memory");
      if (i == 3) asm volatile("global_load_lds_dwordx4 %0, off offset:3072" : : "v"(src) : "memory");
    }
  }
}

// One trip of the Phase-1 walk fills a 64-row stage in two halves of 32 rows: `lo` and `hi`
// are the byte offsets (from the head's K or V base) of the sources of stage rows 0..31 and
// 32..63.  Both halves of one tile (hi = lo + half a tile) make an ordinary full-tile trip;
// in a split trip the two halves come from different tiles (see the trip list in the kernel).
struct Trip {
  int lo, hi;
};

// This wave's share of a stage: waves 0, 1 fill stage rows 0..31 from `lo`, waves 2, 3 rows
// 32..63 from `hi`; one source address and one M0 value per wave.
template <int D, bool KFMT>
__device__ inline void load_stage(const LaneCtx& lc, const unsigned char* g, const Trip t, unsigned lds_stage) {
  constexpr int NLD = Geo<D>::NLD;
  const unsigned piece0 = __builtin_amdgcn_readfirstlane(lc.wave * (NLD * 1024));
  const int off = __builtin_amdgcn_readfirstlane((lc.wave < 2 ? t.lo : t.hi) + (int)(lc.wave & 1) * (NLD * 1024));
  const unsigned char* base = g + off;
  set_dma_lds_base(lds_stage + piece0);
  dma_1kb<0>(KFMT ? lc.dma_k[0] : lc.dma_v[0], base);
  dma_1kb<1024>(KFMT ? lc.dma_k[1] : lc.dma_v[1], base);
  if (NLD == 4) {
    dma_1kb<2048>(KFMT ? lc.dma_k[2] : lc.dma_v[2], base);
    dma_1kb<3072>(KFMT ? lc.dma_k[3] : lc.dma_v[3], base);
  }
}

// V-format swizzle: the 32-byte chunk index of row r is XORed with this 3-bit value.  The
// four consecutive rows a 16-lane group reads together get 0,2,4,6 (or 1,3,5,7), so the two
// groups of a half-wave (chunk indices differing in bit 0) hit disjoint banks: measured
// 2.2 clk per ds_read_b64_tr_b16 against 4.2 clk with a plain (r & 7) XOR.
// At D = 64 a row has four 32-byte chunks and two rows share a bank line: rows 2m and 2m + 1
// flip chunk bit 1 by m & 1, which again spreads the eight 32-byte pieces of a half-wave over
// eight distinct bank groups.
template <int D> __device__ inline int vswz(int r) {
  return D == 128 ? (((r & 3) << 1) | ((r >> 2) & 1)) : (((r >> 1) & 1) << 1);
}
// K-format swizzle of the 16-byte chunk index: 16 rows of a ds_read_b128 pass must fall on 16
// different bank groups (256-byte rows: row & 15; 128-byte rows pair up in a bank line:
// (row >> 1) & 7).
template <int D> __device__ inline int kswz(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }

// The staging area is 1 KB aligned, so flipping address bits 4..6 (4..7 at D = 128) stays inside a row.
__device__ inline LDS_PTR(const unsigned char) xor_ptr(LDS_PTR(const unsigned char) p, unsigned bits) {
  return (LDS_PTR(const unsigned char))(unsigned long long)((unsigned)(unsigned long long)p ^ bits);
}

// s_waitcnt vmcnt(0) with the other counters left alone (gfx9 encoding).
__device__ inline void wait_async_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// s_waitcnt vmcnt(N): returns once at most the N youngest of this wave's loads are still in
// flight (they complete in the order issued).  gfx9 encoding: vmcnt in bits 3..0 and 15..14.
template <int N> __device__ inline void wait_older_loads() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// ---- the three stages of one 64-key tile ------------------------------------------------
// LDS offsets (KOFF, VOFF) are compile-time and relative to the staging origin the
// LaneCtx pointers refer to.

// S^T = K_tile Q^T.
template <int D, int KOFF>
__device__ inline void qk_tile(f32x16& s0, f32x16& s1, const bf16x8 (&qreg)[D / 16], const LaneCtx& lc) {
  constexpr int ROWB = Geo<D>::ROWB;
  s0 = (f32x16){0};
  s1 = (f32x16){0};
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    LDS_PTR(const unsigned char) kp = xor_ptr(lc.kbase, ks << 5);
    const bf16x8 a0 = *reinterpret_cast<LDS_PTR(const bf16x8)>(kp + KOFF);
    const bf16x8 a1 = *reinterpret_cast<LDS_PTR(const bf16x8)>(kp + KOFF + 32 * ROWB);
    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qreg[ks], s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qreg[ks], s1, 0, 0, 0);
  }
}

// One half of it: the 32 keys of stage rows ROW0 .. ROW0 + 31 (ROW0 = 0 or 32).
template <int D, int KOFF, int ROW0>
__device__ inline void qk_rows(f32x16& s, const bf16x8 (&qreg)[D / 16], const LaneCtx& lc) {
  constexpr int ROWB = Geo<D>::ROWB;
  s = (f32x16){0};
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    LDS_PTR(const unsigned char) kp = xor_ptr(lc.kbase, ks << 5);
    const bf16x8 a = *reinterpret_cast<LDS_PTR(const bf16x8)>(kp + KOFF + ROW0 * ROWB);
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], s, 0, 0, 0);
  }
}

// Online softmax in the log2 domain, in two steps so that the only branch (the rescale of O
// when some row maximum moved) sits in front of the straight-line exponential part.
// Register r of S^T half kk <-> key 32 kk + (r/4)*8 + 4h + r%4.
//   bias (TAIL only): 64 floats in LDS: log2 B_j, or -inf for masked / absent columns.
//   RAGGED: keys >= nvalid contribute nothing (their staged rows hold finite filler).

// Step 1: new running max; rescales l, l_tail and O if it moved.  Returns the (finite)
// value to subtract.  TAIL: s0, s1 are turned into biased log2-domain logits in place.
template <int D, bool TAIL>
__device__ inline float softmax_max(State<D>& st, f32x16& s0, f32x16& s1, const LaneCtx& lc,
                                    LDS_PTR(const float) bias, float c) {
  float tmax;
  if (TAIL) {
    const int h = lc.h;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 b0 = *reinterpret_cast<LDS_PTR(const f32x4)>(bias + 8 * g + 4 * h);
      const f32x4 b1 = *reinterpret_cast<LDS_PTR(const f32x4)>(bias + 32 + 8 * g + 4 * h);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s0[4 * g + e] = fmaf(s0[4 * g + e], c, b0[e]);
        s1[4 * g + e] = fmaf(s1[4 * g + e], c, b1[e]);
      }
    }
  }
  // max over the accumulators (raw ones when !TAIL: the scale is positive); filler keys of a
  // ragged tile may take part: any bound >= the valid logits keeps the softmax exact.
  float t = s0[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) t = fmaxf(t, s0[r]);
#pragma unroll
  for (int r = 0; r < 16; ++r) t = fmaxf(t, s1[r]);
  tmax = TAIL ? t : t * c;
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
  const float m_new = fmaxf(st.m, tmax);
  const float m_safe = m_new == -INFINITY ? 0.f : m_new;
  if (__any(m_new != st.m)) {
    const float corr = __builtin_amdgcn_exp2f(st.m - m_safe);
    st.l *= corr;
    st.l_tail *= corr;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) st.ot[dt] *= corr;
    st.m = m_new;
  }
  return m_safe;
}

// Step 2: probabilities, row-sum update, bf16 B operands pb[step] (16 keys each).
template <int D, bool TAIL, bool RAGGED>
__device__ inline void softmax_exp(State<D>& st, const f32x16& s0, const f32x16& s1, float m_safe,
                                   bf16x8 (&pb)[4], const LaneCtx& lc, int nvalid, float c) {
  float x[32];
  const float nm = -m_safe;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    x[r] = __builtin_amdgcn_exp2f(TAIL ? s0[r] + nm : fmaf(s0[r], c, nm));
    x[16 + r] = __builtin_amdgcn_exp2f(TAIL ? s1[r] + nm : fmaf(s1[r], c, nm));
  }
  if (RAGGED) {
    const int h = lc.h;
#pragma unroll
    for (int r = 0; r < 32; ++r) {
      const int key = 32 * (r >> 4) + ((r & 15) / 4) * 8 + 4 * h + (r % 4);
      if (key >= nvalid) x[r] = 0.f;
    }
  }
  float psum = 0.f;
#pragma unroll
  for (int r = 0; r < 32; ++r) psum += x[r];
  st.l += psum;
  if (TAIL) st.l_tail += psum;
#pragma unroll
  for (int step = 0; step < 4; ++step) {            // keys 16 step .. 16 step + 15
    u32x4 pw;
#pragma unroll
    for (int i = 0; i < 4; ++i) pw[i] = pack_bf16(x[8 * step + 2 * i], x[8 * step + 2 * i + 1]);
    pb[step] = __builtin_bit_cast(bf16x8, pw);
  }
}

// Fast step for full exact keys: probabilities against the running max AS IT STANDS (no
// new maximum is taken, so no cross-lane exchange and no rescale), packed to bf16, with
// their row-sum.  fp32 and bf16 share their exponent range, so a stale maximum costs no
// accuracy until 2^(logit - max) nears overflow: the caller falls back to the exact step
// (the true maximum, then this again) when some lane's sum is not below kStaleLimit.  Sums stay
// below 2^60 between refreshes, so l and O (at most a few 10^5 keys of bounded values) stay
// far from the fp32 limit.  A wave that has absorbed nothing yet (max = -inf) gets +inf
// everywhere and therefore always falls back on its first tile; NaN falls back as well.
// The work comes in halves of 32 keys (one S^T accumulator -> two B operands of 16 keys), so
// that a wave can take either half of a stage or both; pa / pc carry the two partial sums
// through the halves in a fixed order.
constexpr float kStaleLimit = 0x1p60f;
__device__ inline void exp_rows(const f32x16& s, float c, float nm, bf16x8& p0, bf16x8& p1, float& pa, float& pc) {
#pragma unroll
  for (int step = 0; step < 2; ++step) {            // keys 16 step .. 16 step + 15 of the half
    u32x4 pw;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 8 * step + 2 * i;
      const float x0 = __builtin_amdgcn_exp2f(fmaf(s[r], c, nm));
      const float x1 = __builtin_amdgcn_exp2f(fmaf(s[r + 1], c, nm));
      pw[i] = pack_bf16(x0, x1);
      if (i & 1) pc += x0 + x1;
      else pa += x0 + x1;
    }
    if (step == 0) p0 = __builtin_bit_cast(bf16x8, pw);
    else p1 = __builtin_bit_cast(bf16x8, pw);
  }
}
// Largest raw accumulator of one half.
__device__ inline float max_rows(const f32x16& s) {
  float t = s[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) t = fmaxf(t, s[r]);
  return t;
}
// Exact step: the running max takes in `tmax` (this lane's largest new logit, log2 domain);
// l, l_tail and O are rescaled if some lane's max moved.
template <int D>
__device__ inline void raise_max(State<D>& st, float tmax) {
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
  const float m_new = fmaxf(st.m, tmax);
  const float m_safe = m_new == -INFINITY ? 0.f : m_new;
  if (__any(m_new != st.m)) {
    const float corr = __builtin_amdgcn_exp2f(st.m - m_safe);
    st.l *= corr;
    st.l_tail *= corr;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) st.ot[dt] *= corr;
    st.m = m_new;
  }
}

// O^T += V^T P^T: four contraction steps of 16 keys.  Transposed LDS read: lane j of a
// 16-lane group points at 4 channels of key (j >> 2) and receives channel (group base + j)
// of the group's four keys.
template <int D, int VOFF>
__device__ inline void pv_tile(State<D>& st, const bf16x8 (&pb)[4], const LaneCtx& lc) {
  constexpr int ROWB = Geo<D>::ROWB;
#pragma unroll
  for (int step = 0; step < 4; ++step) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
      LDS_PTR(unsigned char) vp =
          const_cast<LDS_PTR(unsigned char)>(xor_ptr(lc.vbase, dt << 6)) + VOFF + 16 * step * ROWB;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_PTR(s16x4)>(vp));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_PTR(s16x4)>(vp + 8 * ROWB));
      const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
      const u32x4 aw = {l2.x, l2.y, h2.x, h2.y};
      st.ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), pb[step],
                                                          st.ot[dt], 0, 0, 0);
    }
  }
}

// Two of those contraction steps: the 32 keys of stage rows ROW0 .. ROW0 + 31.
template <int D, int VOFF, int ROW0>
__device__ inline void pv_rows(State<D>& st, const bf16x8& p0, const bf16x8& p1, const LaneCtx& lc) {
  constexpr int ROWB = Geo<D>::ROWB;
#pragma unroll
  for (int step = 0; step < 2; ++step) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
      LDS_PTR(unsigned char) vp =
          const_cast<LDS_PTR(unsigned char)>(xor_ptr(lc.vbase, dt << 6)) + VOFF + (ROW0 + 16 * step) * ROWB;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_PTR(s16x4)>(vp));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_PTR(s16x4)>(vp + 8 * ROWB));
      const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
      const u32x4 aw = {l2.x, l2.y, h2.x, h2.y};
      st.ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw), step == 0 ? p0 : p1,
                                                          st.ot[dt], 0, 0, 0);
    }
  }
}

// One staged tile, start to finish (ragged tile, centroid tiles).
template <int D, bool TAIL, bool RAGGED, int KOFF, int VOFF>
__device__ inline void absorb_tile(State<D>& st, const bf16x8 (&qreg)[D / 16], const LaneCtx& lc,
                                   LDS_PTR(const float) bias, int nvalid, float c) {
  f32x16 s0, s1;
  bf16x8 pb[4];
  qk_tile<D, KOFF>(s0, s1, qreg, lc);
  const float m_safe = softmax_max<D, TAIL>(st, s0, s1, lc, bias, c);
  softmax_exp<D, TAIL, RAGGED>(st, s0, s1, m_safe, pb, lc, nvalid, c);
  pv_tile<D, VOFF>(st, pb, lc);
}

// LDS map of the staging area (byte offsets): K stages | V stages; Phase 2 reuses it as
// centroid keys (K stage 0) and centroid values (V stage 0).
// Three workgroups per CU at head_dim 64 (168 VGPRs, 33 KB LDS each), two at 128.
// TPB: 64-key tiles per block of the selection (1: block 64, two query blocks per workgroup;
// 2: block 128, one); the dense kernel is built with TPB = 2 (it has no block lists).
template <int D, bool DENSE, int TPB>
__global__ __launch_bounds__(256, D == 64 ? 3 : 2) void attn_bf16_kernel(PB p) {
  constexpr int ROWB = Geo<D>::ROWB, TILEB = Geo<D>::TILEB, NKS = Geo<D>::NKS, NDT = Geo<D>::NDT;
  constexpr int CPR = Geo<D>::CPR, RPL = Geo<D>::RPL;
  constexpr int KST0 = 0, KST1 = TILEB, VST0 = 2 * TILEB, VST1 = 3 * TILEB;
  __shared__ __attribute__((aligned(1024))) unsigned char stage[4 * TILEB];   // K0 | K1 | V0 | V1
  __shared__ unsigned int chosen[2][MASK_WORDS];
  __shared__ __attribute__((aligned(16))) float bias_s[2][2][kTile];          // [stage parity][query block][centroid]
  __shared__ unsigned short trip_list[DENSE || TPB == 2 ? 2 : kMaxBlocks + 2];          // Phase-1 walk of a block-64 workgroup
  __shared__ unsigned short pre_s[DENSE || TPB == 2 ? 1 : MASK_WORDS + 1], pre_a[DENSE || TPB == 2 ? 1 : MASK_WORDS + 1],
      pre_b[DENSE || TPB == 2 ? 1 : MASK_WORDS + 1];                                   // tiles below each mask word, by class

  // Workgroup ids are dealt round-robin to the 8 XCDs.  Dense attention gives each XCD a
  // contiguous range of (head, query tile) items, so one XCD's L2 serves one head whose tiles
  // all its workgroups walk in the same order.  PISA workgroups walk different tile lists and
  // mostly miss L2, so there all XCDs work on the same head at the same time instead: the
  // misses of all 8 XCDs then fall on one or two heads' K/V (39 MB each), which the 256 MB
  // Infinity Cache holds, rather than on eight heads at once.
  const int wg = blockIdx.x;
  int item = ((wg >> 6) << 6) + ((wg & 7) << 3) + ((wg >> 3) & 7);   // 8 neighbours per XCD
  if (DENSE) {
    // The grid is rounded up, so ids with wg / 8 >= per_xcd would spill into the next XCD's
    // range and redo its first items: they leave.
    const int per_xcd = (p.total + 7) / 8;
    if (wg / 8 >= per_xcd) return;
    item = (wg % 8) * per_xcd + wg / 8;
  }
  if (item >= p.total) return;
  const size_t bh = item / p.n_super;
  const int sg = item % p.n_super;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lam = lane & 31, h = lane >> 5;
  const int L = p.L, N = p.N;
  const unsigned char* kg = reinterpret_cast<const unsigned char*>(p.k + bh * (size_t)L * D);
  const unsigned char* vg = reinterpret_cast<const unsigned char*>(p.v + bh * (size_t)L * D);
  constexpr int tpb = TPB;                           // tiles per block: 1 or 2
  const int qb = tpb == 1 ? (wave >> 1) : 0;         // which of the workgroup's query blocks
  const float c = p.scale * 1.44269504088896340736f;
  LDS_PTR(unsigned char) lds = (LDS_PTR(unsigned char)) & stage[0];
  const unsigned lds_addr = (unsigned)(unsigned long long)lds;

  LaneCtx lc;
  lc.h = h;
  lc.wave = __builtin_amdgcn_readfirstlane(wave);
  {
    const int pos = lane % CPR;                  // 16-byte slot inside the LDS row
    lc.dma_r0 = RPL * Geo<D>::NLD * wave + lane / CPR;   // tile row of this lane's first DMA load
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = lc.dma_r0 + RPL * i;         // tile row of load i; its offset is relative to piece i
      const int in_piece = (lane / CPR) * ROWB;
      lc.dma_k[i] = in_piece + ((pos ^ kswz<D>(r)) << 4);
      lc.dma_v[i] = in_piece + (((((pos >> 1) ^ vswz<D>(r)) << 1) | (pos & 1)) << 4);
    }
    const int j16 = lane & 15;
    const int kq = 4 * h + (j16 >> 2);           // key offset of this lane's V pointer (= key & 7)
    const int lhalf = (lane >> 4) & 1;
    lc.kbase = lds + lam * ROWB + ((kswz<D>(lam) ^ h) << 4);
    lc.vbase = lds + kq * ROWB + 8 * (j16 & 3) + ((lhalf ^ vswz<D>(kq)) << 5);
  }

  // The two query blocks of a block-64 workgroup: neighbours 2 sg, 2 sg + 1, or whatever the
  // pairing table says (blocks paired by the similarity of their index rows share more tiles).
  int blk[2] = {tpb == 1 ? 2 * sg : sg, 2 * sg + 1};
  if (!DENSE && tpb == 1 && p.pair) {
    blk[0] = p.pair[(bh * p.n_super + sg) * 2];
    blk[1] = p.pair[(bh * p.n_super + sg) * 2 + 1];
  }
  blk[0] = __builtin_amdgcn_readfirstlane(blk[0]);
  blk[1] = __builtin_amdgcn_readfirstlane(blk[1]);

  // The first 256 entries of each block's index row are requested before anything else: they
  // head the chain index row -> trip list -> first tile load, and the Q operand loads queue
  // up behind them.
  constexpr int nqb = (!DENSE && tpb == 1) ? 2 : 1;
  int j_first[nqb];
  if (!DENSE) {
#pragma unroll
    for (int b = 0; b < nqb; ++b) {
      const int i = blk[b];
      j_first[b] = -1;
      if (i >= 0 && i < N && tid < p.k_top) j_first[b] = p.idx[(bh * N + i) * (size_t)p.k_top + tid];
    }
  }

  // ---- Q^T operand: this lane's query row, D/16 channel slices of 16 ----
  const int my_blk = (!DENSE && tpb == 1) ? blk[wave >> 1] : -1;
  const int q_row = (!DENSE && tpb == 1) ? (my_blk < 0 ? L : my_blk * kTile + 32 * (wave & 1) + lam)
                                         : sg * QROWS + 32 * wave + lam;
  bf16x8 qreg[NKS];
  {
    const __bf16* qg = p.q + bh * (size_t)L * D;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      u32x4 w = {0, 0, 0, 0};
      if (q_row < L) w = *reinterpret_cast<const u32x4*>(qg + (size_t)q_row * D + 16 * ks + 8 * h);
      qreg[ks] = __builtin_bit_cast(bf16x8, w);
    }
  }

  State<D> st;
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt) st.ot[dt] = (f32x16){0};
  st.m = -INFINITY;
  st.l = 0.f;
  st.l_tail = 0.f;

  // ---- block bitmasks of the workgroup's query block(s) ----
  const int nwords = (N + 31) / 32;
  if (!DENSE) {
    for (int w = tid; w < 2 * MASK_WORDS; w += 256) (&chosen[0][0])[w] = 0u;
    __syncthreads();
#pragma unroll
    for (int b = 0; b < nqb; ++b) {
      const int i = blk[b];
      if (i >= 0 && i < N) {
        const int32_t* row = p.idx + (bh * N + i) * (size_t)p.k_top;
        int j = j_first[b];
        for (int t = tid; t < p.k_top; t += 256) {
          if (t != tid) j = row[t];
          if ((unsigned)j < (unsigned)N)          // entries outside [0, N) are ignored
            atomicOr(&chosen[b][j >> 5], 1u << (j & 31));
        }
      }
    }
    __syncthreads();
  }

  // ---- Phase 1: the walk over full exact tiles (a ragged last tile is folded in afterwards) ----
  const int n_tiles = L / kTile;
  constexpr int HALFB = TILEB / 2;

  // Block 64, PISA: the two query blocks' lists are merged into one trip list in LDS.  A tile
  // both blocks selected becomes one full trip in which every wave takes all 64 keys.  The
  // tiles only the first block selected and those only the second selected are paired up in
  // ascending order (i-th with i-th; both blocks hold k entries, so the two sets are equally
  // long unless an entry was out of range or the ragged tile is in one list only).  A pair
  // becomes two split trips, one per 32-key half of the two tiles: stage rows 0..31 hold the
  // half of the first block's tile, rows 32..63 the half of the second block's, and each
  // block's waves take the 32 keys that are theirs, so no wave sits a trip out.  Entries are
  // ordered by tile index, a pair by the larger of its two, so the walk stays ascending; tiles
  // left without a partner follow at the end as split trips with one block idle.
  // Entry: bits 0..12 tile, bits 13..15 kind (0 shared, 1 member of a pair: first-block tile
  // then second-block tile, 2 / 3 unpaired tile of the first / second block).
  int n_entries = 0;
  if (!DENSE && TPB == 1) {
    // scratch inside the (still unused) staging area
    LDS_PTR(unsigned int) w_s = (LDS_PTR(unsigned int))(lds);                       // [128] shared words
    LDS_PTR(unsigned int) w_a = w_s + MASK_WORDS;                                    // first block only
    LDS_PTR(unsigned int) w_b = w_a + MASK_WORDS;                                    // second block only
    LDS_PTR(unsigned short) l_s = (LDS_PTR(unsigned short))(w_b + MASK_WORDS);       // [4096] compacted
    LDS_PTR(unsigned short) l_a = l_s + kMaxBlocks;
    LDS_PTR(unsigned short) l_b = l_a + kMaxBlocks;
    static_assert(3 * MASK_WORDS * 4 + 3 * kMaxBlocks * 2 <= 4 * Geo<64>::TILEB, "list scratch must fit the staging area");
    if (wave == 0) {
      // lane l owns mask words 2l, 2l + 1: split them, count, exclusive scan over the lanes
      unsigned ws[2], wa[2], wb[2];
      unsigned cs = 0, cab = 0, cs0 = 0, cab0 = 0;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int w = 2 * lane + u;
        unsigned c0 = 0u, c1 = 0u;
        if (w < nwords) {
          const int first = 32 * w;                      // tiles >= n_tiles (the ragged one) stay out
          const unsigned lim = first + 32 <= n_tiles ? 0xffffffffu
                               : (first >= n_tiles ? 0u : ((1u << (n_tiles - first)) - 1u));
          c0 = chosen[0][w] & lim;
          c1 = chosen[1][w] & lim;
        }
        ws[u] = c0 & c1;
        wa[u] = c0 & ~c1;
        wb[u] = c1 & ~c0;
        w_s[w] = ws[u];
        w_a[w] = wa[u];
        w_b[w] = wb[u];
        if (u == 0) {
          cs0 = __builtin_popcount(ws[0]);
          cab0 = __builtin_popcount(wa[0]) | (__builtin_popcount(wb[0]) << 16);
        }
        cs += __builtin_popcount(ws[u]);
        cab += __builtin_popcount(wa[u]) | (__builtin_popcount(wb[u]) << 16);
      }
      unsigned is = cs, iab = cab;                       // inclusive scans (counts <= 4096: 16-bit halves never carry)
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const unsigned ts = __shfl_up(is, off), tab = __shfl_up(iab, off);
        if (lane >= off) {
          is += ts;
          iab += tab;
        }
      }
      const unsigned es = is - cs, eab = iab - cab;      // exclusive prefix of this lane's first word
      pre_s[2 * lane] = (unsigned short)es;
      pre_s[2 * lane + 1] = (unsigned short)(es + cs0);
      pre_a[2 * lane] = (unsigned short)(eab & 0xffffu);
      pre_a[2 * lane + 1] = (unsigned short)((eab + cab0) & 0xffffu);
      pre_b[2 * lane] = (unsigned short)(eab >> 16);
      pre_b[2 * lane + 1] = (unsigned short)((eab + cab0) >> 16);
      if (lane == 63) {
        pre_s[MASK_WORDS] = (unsigned short)is;
        pre_a[MASK_WORDS] = (unsigned short)(iab & 0xffffu);
        pre_b[MASK_WORDS] = (unsigned short)(iab >> 16);
      }
      // compaction: this lane's tiles, ascending, at their ranks
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int w = 2 * lane + u;
        unsigned rs = u == 0 ? es : es + cs0;
        unsigned ra = (u == 0 ? eab : eab + cab0) & 0xffffu;
        unsigned rb = (u == 0 ? eab : eab + cab0) >> 16;
        for (unsigned m = ws[u]; m; m &= m - 1u) l_s[rs++] = (unsigned short)(32 * w + __builtin_ctz(m));
        for (unsigned m = wa[u]; m; m &= m - 1u) l_a[ra++] = (unsigned short)(32 * w + __builtin_ctz(m));
        for (unsigned m = wb[u]; m; m &= m - 1u) l_b[rb++] = (unsigned short)(32 * w + __builtin_ctz(m));
      }
    }
    __syncthreads();
    const int n_s = pre_s[MASK_WORDS], n_a = pre_a[MASK_WORDS], n_b = pre_b[MASK_WORDS];
    const int n_pairs = min(n_a, n_b);
    for (int i = tid; i < n_pairs; i += 256) {           // pair i sits behind the shared tiles below its larger member
      const int ta = l_a[i], tb = l_b[i];
      const int key = max(ta, tb);
      const int below = pre_s[key >> 5] + __builtin_popcount(w_s[key >> 5] & ((1u << (key & 31)) - 1u));
      trip_list[2 * i + below] = (unsigned short)(ta | (1 << 13));
      trip_list[2 * i + below + 1] = (unsigned short)(tb | (1 << 13));
    }
    for (int m = tid; m < n_s; m += 256) {               // shared tile m sits behind the pairs that lie wholly below it
      const int t = l_s[m];
      const unsigned low = (1u << (t & 31)) - 1u;
      const int na = pre_a[t >> 5] + __builtin_popcount(w_a[t >> 5] & low);
      const int nb = pre_b[t >> 5] + __builtin_popcount(w_b[t >> 5] & low);
      trip_list[m + 2 * min(na, nb)] = (unsigned short)t;
    }
    const int base = n_s + 2 * n_pairs;
    for (int i = n_pairs + tid; i < n_a; i += 256) trip_list[base + i - n_pairs] = (unsigned short)(l_a[i] | (2 << 13));
    for (int i = n_pairs + tid; i < n_b; i += 256) trip_list[base + i - n_pairs] = (unsigned short)(l_b[i] | (3 << 13));
    n_entries = __builtin_amdgcn_readfirstlane(base + (n_a - n_pairs) + (n_b - n_pairs));
    if (tid < 2) trip_list[n_entries + tid] = 0;
    __syncthreads();                                     // list complete; the staging area is free again
  }

  // The trip generator (wave-uniform state in scalar registers).  A trip is handed around as
  // three plain integers: lo, hi (see Trip) and a work mask wm, in which bit 2 b + e says that
  // the waves of query block b take stage half e (keys 32 e .. 32 e + 31).
  int li = 0, split_left = 0, split_lo = 0, split_hi = 0, split_wm = 0, w_word = -1, pend = -1, dense_t = 0;
  unsigned int w_bits = 0u;
  auto next_trip = [&](int& lo, int& hi, int& wm) -> bool {
    if (DENSE) {
      if (dense_t >= n_tiles) return false;
      lo = dense_t * TILEB;
      hi = lo + HALFB;
      wm = 15;
      ++dense_t;
      return true;
    }
    if (TPB == 2) {                                      // one 128-token block per workgroup: two tiles per entry
      int tile;
      if (pend >= 0) {
        tile = pend;
        pend = -1;
      } else {
        while (w_bits == 0u) {
          if (++w_word >= nwords) return false;
          w_bits = __builtin_amdgcn_readfirstlane(chosen[0][w_word]);
        }
        const int j = w_word * 32 + __builtin_ctz(w_bits);
        w_bits &= w_bits - 1u;
        tile = 2 * j;
        if (tile >= n_tiles) return false;               // only the ragged tile is left
        if (tile + 1 < n_tiles) pend = tile + 1;
      }
      lo = tile * TILEB;
      hi = lo + HALFB;
      wm = 15;
      return true;
    }
    if (split_left) {                                    // second half of a split pair
      lo = split_lo;
      hi = split_hi;
      wm = split_wm;
      split_left = 0;
      return true;
    }
    if (li >= n_entries) return false;
    const unsigned e0 = __builtin_amdgcn_readfirstlane((unsigned)trip_list[li]);
    const unsigned e1 = __builtin_amdgcn_readfirstlane((unsigned)trip_list[li + 1]);
    const int kind = e0 >> 13, tile = e0 & 0x1fff;
    if (kind == 0) {
      ++li;
      lo = tile * TILEB;
      hi = lo + HALFB;
      wm = 15;
      return true;
    }
    const int tb = kind == 1 ? (int)(e1 & 0x1fff) : tile;
    li += kind == 1 ? 2 : 1;
    lo = tile * TILEB;                                   // first block's tile  -> stage rows 0..31
    hi = tb * TILEB;                                     // second block's tile -> stage rows 32..63
    wm = kind == 1 ? 9 : (kind == 2 ? 1 : 8);            // first block: half 0; second block: half 1
    split_lo = lo + HALFB;
    split_hi = hi + HALFB;
    split_wm = wm;
    split_left = 1;
    return true;
  };

  // Software pipeline over trips t = 0, 1, ...: K runs one trip ahead of V.  One barrier per
  // trip; after it K(t+1) and V(t) have landed and K stage t&1 / V stage (t+1)&1 are free, so
  // the loads of K(t+2) and V(t+1) go out.  The wave then runs the softmax of trip t,
  // O^T += V(t)^T P(t)^T, and last S^T(t+1), which takes over the score registers the softmax
  // has just consumed.  Where trips can be split (block 64, PISA) every step comes in two halves
  // of 32 keys, each guarded by its bit of the trip's work mask (both set in a full trip).
  // A block-64 workgroup whose two lists coincide has no split trip at all: it runs the copy of
  // the loop without the guards (the code the dense kernel runs), so that r = 0 costs what the
  // dense kernel costs.
  const int my_shift = (int)(lc.wave >> 1) * 2;
  f32x16 sc0, sc1;                       // S^T of the current trip: stage rows 0..31 / 32..63
  auto walk = [&](auto splits_tag) {
    constexpr bool SPLITS = decltype(splits_tag)::value;
    int lo0 = 0, hi0 = 0, wm0 = 0, lo1 = 0, hi1 = 0, wm1 = 0, lo2 = 0, hi2 = 0, wm2 = 0;
    bool have0 = next_trip(lo0, hi0, wm0);
    bool have1 = false, have2 = false;
    auto scores = [&](auto koff_tag, int wm) {
      constexpr int KOFF = decltype(koff_tag)::value;
      if (!SPLITS) {
        qk_tile<D, KOFF>(sc0, sc1, qreg, lc);
      } else {
        if ((wm >> my_shift) & 1) qk_rows<D, KOFF, 0>(sc0, qreg, lc);
        if ((wm >> my_shift) & 2) qk_rows<D, KOFF, 32>(sc1, qreg, lc);
      }
    };
    if (have0) {
      load_stage<D, true>(lc, kg, Trip{lo0, hi0}, lds_addr + KST0);
      have1 = next_trip(lo1, hi1, wm1);
      wait_async_loads();
      __syncthreads();
      if (have1) load_stage<D, true>(lc, kg, Trip{lo1, hi1}, lds_addr + KST1);
      load_stage<D, false>(lc, vg, Trip{lo0, hi0}, lds_addr + VST0);
      scores(std::integral_constant<int, KST0>{}, wm0);
    }
    auto trip = [&](auto parity_tag) {
      constexpr int P = decltype(parity_tag)::value;       // parity of the current trip
      constexpr int K_NEXT = P ? KST0 : KST1, K_FREE = P ? KST1 : KST0;
      constexpr int V_CUR = P ? VST1 : VST0, V_FREE = P ? VST0 : VST1;
      have2 = have1 && next_trip(lo2, hi2, wm2);
      wait_async_loads();
      __syncthreads();
      // Past the end of the walk the loads repeat trip 0's sources into the free stages (harmless).
      load_stage<D, true>(lc, kg, Trip{have2 ? lo2 : lo0, have2 ? hi2 : hi0}, lds_addr + K_FREE);
      load_stage<D, false>(lc, vg, Trip{have1 ? lo1 : lo0, have1 ? hi1 : hi0}, lds_addr + V_FREE);
      const bool do_lo = !SPLITS || ((wm0 >> my_shift) & 1), do_hi = !SPLITS || ((wm0 >> my_shift) & 2);
      if (do_lo || do_hi) {
        bf16x8 pb[4];
        float nm = -st.m, pa = 0.f, pc = 0.f;
        if (do_lo) exp_rows(sc0, c, nm, pb[0], pb[1], pa, pc);
        if (do_hi) exp_rows(sc1, c, nm, pb[2], pb[3], pa, pc);
        if (__any(!(pa + pc < kStaleLimit))) {         // first keys of this wave, or a maximum that ran away
          float t = -INFINITY;
          if (do_lo) t = max_rows(sc0);
          if (do_hi) t = fmaxf(t, max_rows(sc1));
          raise_max<D>(st, t * c);
          nm = -st.m;
          pa = pc = 0.f;
          if (do_lo) exp_rows(sc0, c, nm, pb[0], pb[1], pa, pc);
          if (do_hi) exp_rows(sc1, c, nm, pb[2], pb[3], pa, pc);
        }
        st.l += pa + pc;
        if (do_lo) pv_rows<D, V_CUR, 0>(st, pb[0], pb[1], lc);
        if (do_hi) pv_rows<D, V_CUR, 32>(st, pb[2], pb[3], lc);
      }
      if (have1) scores(std::integral_constant<int, K_NEXT>{}, wm1);
      lo0 = lo1; hi0 = hi1; wm0 = wm1; have0 = have1;
      lo1 = lo2; hi1 = hi2; wm1 = wm2; have1 = have2;
    };
    while (have0) {
      trip(std::integral_constant<int, 0>{});
      if (!have0) break;
      trip(std::integral_constant<int, 1>{});
    }
  };
  if (!DENSE && TPB == 1) {
    const bool any_split = n_entries != __builtin_amdgcn_readfirstlane((int)pre_s[MASK_WORDS]);
    if (any_split) walk(std::true_type{});
    else walk(std::false_type{});
  } else {
    walk(std::false_type{});
  }
  wait_async_loads();                      // the last trips' repeated loads

  // ---- ragged last tile (L not a multiple of 64), if this workgroup attends it ----
  if (L % kTile != 0) {
    const int tile = n_tiles, jb = tile / tpb;
    const unsigned inm = DENSE ? 3u
                               : (((chosen[0][jb >> 5] >> (jb & 31)) & 1u) |
                                  (tpb == 1 ? (((chosen[1][jb >> 5] >> (jb & 31)) & 1u) << 1) : 0u));
    if (inm) {            // uniform over the workgroup
      __syncthreads();
      load_tile_async<D, true>(lc, kg + (size_t)tile * TILEB, L - tile * kTile, lds_addr + KST0);
      load_tile_async<D, false>(lc, vg + (size_t)tile * TILEB, L - tile * kTile, lds_addr + VST0);
      wait_async_loads();
      __syncthreads();
      if ((inm >> qb) & 1)
        absorb_tile<D, false, true, KST0, VST0>(st, qreg, lc, nullptr, L - tile * kTile, c);
    }
  }

  // ---- Phase 2: centroid tiles (keys, values) ----
  const bool approx = !DENSE && p.k_top < N && p.kcen != nullptr;   // kcen == nullptr: keep-or-drop
  if (approx) {
    const unsigned char* kcg = reinterpret_cast<const unsigned char*>(p.kcen + bh * (size_t)p.npad * D);
    const unsigned char* vbg = reinterpret_cast<const unsigned char*>(p.vbar + bh * (size_t)p.npad * D);
    // Double buffered: tile g + 1 (and its column bias) is fetched while tile g is absorbed.
    const float log2_full = __builtin_amdgcn_logf((float)p.B);
    const float log2_last = __builtin_amdgcn_logf((float)(L - (N - 1) * p.B));
    auto fetch = [&](int g0, auto parity_tag) {
      constexpr int P = decltype(parity_tag)::value;
      load_tile_async<D, true>(lc, kcg + (size_t)g0 * ROWB, kTile, lds_addr + (P ? KST1 : KST0));
      load_tile_async<D, false>(lc, vbg + (size_t)g0 * ROWB, kTile, lds_addr + (P ? VST1 : VST0));
      if (tid < 2 * kTile) {
        const int b = tid >> 6, j = g0 + (tid & 63);
        const bool masked =
            (tpb == 2 && b == 1) ? true : ((chosen[b][(j >> 5) & (MASK_WORDS - 1)] >> (j & 31)) & 1u);
        // log2 B_j for a centroid that stands for its block; computed here (two values per
        // call), so that no ordinary load, and with it no wait on the tile loads just issued,
        // sits in this step
        bias_s[P][b][tid & 63] = (masked || j >= N) ? -INFINITY : (j == N - 1 ? log2_last : log2_full);
      }
    };
    auto absorb = [&](int g0, auto parity_tag) {
      constexpr int P = decltype(parity_tag)::value;
      wait_async_loads();
      __syncthreads();                         // tile g has landed; tile g - 1 is fully consumed
      if (g0 + kTile < N) fetch(g0 + kTile, std::integral_constant<int, 1 - P>{});
      absorb_tile<D, true, false, (P ? KST1 : KST0), (P ? VST1 : VST0)>(
          st, qreg, lc, (LDS_PTR(const float)) & bias_s[P][qb][0], kTile, c);
    };
    __syncthreads();                           // the stages are free (Phase 1 and the ragged tile are done)
    fetch(0, std::integral_constant<int, 0>{});
    for (int g0 = 0; g0 < N; g0 += 2 * kTile) {
      absorb(g0, std::integral_constant<int, 0>{});
      if (g0 + kTile < N) absorb(g0 + kTile, std::integral_constant<int, 1>{});
    }
  }

  // ---- combine the two lane halves (keys with h = 0 / h = 1) ----
  st.l += __shfl_xor(st.l, 32);
  st.l_tail += __shfl_xor(st.l_tail, 32);

  // ---- Phase 3: R^T = hsum^T (d_out x d_in) * Q^T (d_in x queries), weight l_tail / L * s ----
  // The packed matrix (hi and lo halves, 4 D^2 bytes: the size of the staging area at head_dim
  // 128) goes through LDS once per workgroup instead of once per wave from L2: it is stored in
  // operand order, 16 bytes per lane, so the copy is a straight LDS-DMA and the reads are
  // conflict-free ds_read_b128.
  if (approx && p.first_order) {
    const unsigned char* hp = reinterpret_cast<const unsigned char*>(p.hpack + bh * (size_t)(2 * D * D));
    constexpr int HP_BYTES = 4 * D * D, HP_LOADS = HP_BYTES / (4 * 1024);     // 1 KB wave-loads per wave
    static_assert(HP_BYTES <= 4 * TILEB, "the packed matrix must fit the staging area");
    __syncthreads();                            // every wave is done with the centroid stages
#pragma unroll
    for (int i = 0; i < HP_LOADS; ++i) {
      const unsigned off = (unsigned)__builtin_amdgcn_readfirstlane((int)((lc.wave * HP_LOADS + i) * 1024));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(lds_addr + off), "v"((unsigned)(lane * 16)), "s"(hp + off)
                   : "memory", "m0");
    }
    wait_async_loads();
    __syncthreads();
    LDS_PTR(const unsigned char) hl = lds + lane * 16;
    f32x16 rt[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) rt[dt] = (f32x16){0};
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int dt = 0; dt < NDT; ++dt) {
        const bf16x8 ahi = *reinterpret_cast<LDS_PTR(const bf16x8)>(hl + (ks * NDT + dt) * 1024);
        const bf16x8 alo = *reinterpret_cast<LDS_PTR(const bf16x8)>(hl + 2 * D * D + (ks * NDT + dt) * 1024);
        rt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, qreg[ks], rt[dt], 0, 0, 0);
        rt[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(alo, qreg[ks], rt[dt], 0, 0, 0);
      }
    const float w = st.l_tail / (float)L * p.scale;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) st.ot[dt] += rt[dt] * w;
  }

  // ---- normalise and store: register group g of tile dt = channels 32 dt + 8 g + 4 h + 0..3 ----
  if (q_row < L) {
    const float inv_l = 1.f / st.l;
    __bf16* orow = p.out + (bh * (size_t)L + q_row) * D;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const u32x2 w = {pack_bf16(st.ot[dt][4 * g] * inv_l, st.ot[dt][4 * g + 1] * inv_l),
                         pack_bf16(st.ot[dt][4 * g + 2] * inv_l, st.ot[dt][4 * g + 3] * inv_l)};
        *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * g + 4 * h) = w;
      }
    if (p.lse && h == 0)
      p.lse[bh * (size_t)L + q_row] = (st.m + __builtin_amdgcn_logf(st.l)) * 0.69314718055994530942f;
  }
}

}  // namespace

// The kernels that walk two tiles per block without a trip list: dense_attention and block 128.
template <int D> static hipError_t launch_attention_two_tiles(const PB& p, bool dense, int grid, hipStream_t stream) {
  if (dense) hipLaunchKernelGGL((attn_bf16_kernel<D, true, 2>), dim3(grid), dim3(256), 0, stream, p);
  else hipLaunchKernelGGL((attn_bf16_kernel<D, false, 2>), dim3(grid), dim3(256), 0, stream, p);
  return hipGetLastError();
}

size_t attention_workspace_bytes(const Dims& dm) {
  if (dm.dtype != PISA_BF16) return 0;
  const size_t npad = (size_t)((dm.N + kTile - 1) / kTile) * kTile;
  const size_t D = dm.d;
  return (size_t)dm.bh() * (2 * npad * D * 2 + 2 * D * D * 2) + pairing_workspace_bytes(dm);
}

void attention_workspace_carve(const Dims& dm, void* workspace, void** kcen, void** vbar, void** hpack) {
  const size_t npad = (size_t)((dm.N + kTile - 1) / kTile) * kTile;
  const size_t tile_elems = (size_t)dm.bh() * npad * dm.d;
  __bf16* kc = static_cast<__bf16*>(workspace);
  *kcen = kc;
  *vbar = kc + tile_elems;
  *hpack = kc + 2 * tile_elems;
}

template <int D>
static hipError_t launch_attention_bf16_d(const Dims& dm, const AttnArgs& a, hipStream_t stream) {
  PB p{};
  p.q = (const __bf16*)a.q;
  p.k = (const __bf16*)a.k;
  p.v = (const __bf16*)a.v;
  p.idx = a.idx;
  p.out = (__bf16*)a.out;
  p.lse = a.lse;
  p.L = dm.L;
  p.B = dm.B;
  p.N = dm.N;
  p.k_top = a.k_top;
  p.npad = ((dm.N + kTile - 1) / kTile) * kTile;
  p.n_super = (dm.L + QROWS - 1) / QROWS;
  p.total = p.n_super * dm.bh();
  p.scale = dm.scale;
  p.first_order = a.hsum != nullptr;

  const int grid = ((p.total + 63) / 64) * 64;
  if (a.dense) return launch_attention_two_tiles<D>(p, true, grid, stream);
  if (a.k_top < dm.N && a.kbar) {
    void *kcen_v, *vbar_v, *hpack_v;                      // kcen | vbar | hpack
    attention_workspace_carve(dm, a.workspace, &kcen_v, &vbar_v, &hpack_v);
    __bf16* kcen = static_cast<__bf16*>(kcen_v);
    __bf16* vbar = static_cast<__bf16*>(vbar_v);
    __bf16* hpack = static_cast<__bf16*>(hpack_v);
    if (!a.prepared) {
      hipLaunchKernelGGL(attn_prep_kernel<D>, dim3(p.npad / kTile + kPackBlocks, dm.bh()), dim3(256), 0, stream,
                         a.kbar, a.vsum, a.hsum, kcen, vbar, hpack, dm.L, dm.B, dm.N, p.npad);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    p.kcen = kcen;
    p.vbar = vbar;
    p.hpack = hpack;
  }
  if (pairing_pays(dm, a.k_top) && a.workspace) {
    // the pairing scratch follows the pre-pass results (whether or not those are in use)
    unsigned char* after = static_cast<unsigned char*>(a.workspace) +
                           (size_t)dm.bh() * (2 * (size_t)p.npad * D * 2 + 2 * D * D * 2);
    hipError_t e = launch_pair_blocks(dm, a.idx, a.k_top, after, &p.pair, stream);
    if (e != hipSuccess) return e;
  }
  if (dm.B != kTile) return launch_attention_two_tiles<D>(p, false, grid, stream);
  hipLaunchKernelGGL((attn_bf16_kernel<D, false, 1>), dim3(grid), dim3(256), 0, stream, p);
  return hipGetLastError();
}

// Device scratch for callers that cannot hand over a workspace (pisa_attention_static): the
// centroid tiles and the packed hsum of one call.  Every device the library
// runs on holds its own copy of the array until the process ends.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code `scratch` is only a handle: the array's device address is looked up once per
// device (with that device current) and kept; kernels and copies get that pointer.
hipError_t static_scratch_ptr(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

hipError_t launch_attention_bf16(const Dims& dm, const AttnArgs& a, hipStream_t stream) {
  return dm.d == 64 ? launch_attention_bf16_d<64>(dm, a, stream) : launch_attention_bf16_d<128>(dm, a, stream);
}

}  // namespace pisa
