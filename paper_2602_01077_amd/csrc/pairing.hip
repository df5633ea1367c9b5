// Which two 64-row query blocks share a workgroup of the block-64 attention kernel.
//
// The kernel stages every tile that either of its two query blocks selected (Alg. 1, Phase 1:
// the exact blocks S_i), so a workgroup's tile traffic and trip count are set by the UNION of
// the two index rows.  Neighbouring blocks 2s, 2s + 1 share about 58 % of their rows at the
// paper's video shapes; pairing each block with the block whose row overlaps its own most,
// within a window of neighbours, shares more (union 252 -> 241 tiles at the Wan shape, about 270 ->
// 258 at the Hunyuan shape) and costs three small launches (0.09 ms at the Wan shape).  Any pairing gives the same attention
// output up to the order of the fp32 sums; the table only decides which blocks travel together.
//
// Three small launches:
//   1. row_masks_kernel: the bitmask of every index row (global scratch, ceil(N/32) x N words,
//      word-major so that the lanes of a wave, which look at consecutive blocks, read
//      consecutive words);
//   2. pair_candidates_kernel: one wave per block: its overlap (popcount of the ANDed masks)
//      with each of the 2 x kPairWindow blocks around it, and the kPairCandidates best of them
//      in order (larger overlap first, ties to the lower index);
//   3. match_kernel, one workgroup per (batch, head): rounds of mutual-best matching over
//      those lists (every unmatched block proposes to its first unmatched candidate; two
//      blocks that propose to each other are paired), then the blocks still unmatched are
//      paired in index order, and the pairs are written in the order of their lower member, so
//      that consecutive workgroups still work on neighbouring parts of the sequence.
#include <cstdlib>

#include "common.h"

namespace pisa {
namespace {

constexpr int kPairWindow = 64;     // candidates: the 64 blocks before and the 64 after
constexpr int kPairCandidates = 8;  // kept per block, best first
constexpr int kPairRounds = 12;
constexpr int kPairThreads = 1024;

// 1. one wave per index row: the lanes read the row's entries side by side and set their bits
// in an LDS copy of the row's mask, which is then written out word-major.  Entries outside
// [0, N) are ignored, like everywhere else.
__global__ __launch_bounds__(256) void row_masks_kernel(const int32_t* __restrict__ idx, int N, int k_top,
                                                        unsigned int* __restrict__ masks) {
  __shared__ unsigned int row_mask[4][kMaxBlocks / 32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t bh = blockIdx.y;
  const int i = blockIdx.x * 4 + wave;
  if (i >= N) return;                            // whole wave; the kernel has no workgroup barriers
  const int W32 = (N + 31) / 32;
  unsigned int* mine = row_mask[wave];
  for (int w = lane; w < W32; w += 64) mine[w] = 0u;
  const int32_t* row = idx + (bh * N + i) * (size_t)k_top;
  for (int t = lane; t < k_top; t += 64) {
    const int j = row[t];
    if ((unsigned)j < (unsigned)N) atomicOr(&mine[j >> 5], 1u << (j & 31));
  }
  // a wave's LDS operations complete in order, so the words are final when it reads them back
  unsigned int* mk = masks + bh * (size_t)N * W32;
  for (int w = lane; w < W32; w += 64) mk[(size_t)w * N + i] = mine[w];
}

// 2. one wave per block i; lane l looks at blocks i - 64 + l and i + 1 + l.
__global__ __launch_bounds__(256) void pair_candidates_kernel(const unsigned int* __restrict__ masks, int N,
                                                              int32_t* __restrict__ cand) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t bh = blockIdx.y;
  const int i = blockIdx.x * 4 + wave;
  if (i >= N) return;                            // whole wave
  const int W32 = (N + 31) / 32;
  const unsigned int* mk = masks + bh * (size_t)N * W32;
  const int j0 = i - kPairWindow + lane, j1 = i + 1 + lane;
  const bool ok0 = j0 >= 0, ok1 = j1 < N;
  const int c0 = ok0 ? j0 : i, c1 = ok1 ? j1 : i;      // harmless stand-ins
  int ov0 = 0, ov1 = 0;
#pragma unroll 4
  for (int w = 0; w < W32; ++w) {
    const unsigned int mi = mk[(size_t)w * N + i];
    ov0 += __popc(mi & mk[(size_t)w * N + c0]);
    ov1 += __popc(mi & mk[(size_t)w * N + c1]);
  }
  // key = overlap * 8192 + (8191 - j): largest overlap first, then the lower index
  int k0 = ok0 ? ov0 * 8192 + (8191 - j0) : -1;
  int k1 = ok1 ? ov1 * 8192 + (8191 - j1) : -1;
  int32_t* out = cand + (bh * N + i) * (size_t)kPairCandidates;
  for (int t = 0; t < kPairCandidates; ++t) {
    int m = max(k0, k1);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = max(m, __shfl_xor(m, o));
    if (lane == 0) out[t] = m < 0 ? -1 : 8191 - (m & 8191);
    if (k0 == m) k0 = -1;                        // keys are distinct (distinct j), so one lane drops one key
    if (k1 == m) k1 = -1;
  }
}

// Exclusive prefix sum of one value per thread over the workgroup (1024 threads = 16 waves);
// `total` receives the sum.  wave_sums: 16 ints of LDS.
__device__ inline int block_exclusive_scan(int v, int* wave_sums, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();                       // wave_sums may still be read from an earlier call
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kPairThreads / 64; ++w) {
    const int s = wave_sums[w];
    if (w < wave) before += s;
    all += s;
  }
  total = all;
  return before + incl - v;
}

// 3. matching over the candidate lists.
__global__ __launch_bounds__(kPairThreads) void match_kernel(const int32_t* __restrict__ cand, int N,
                                                             int32_t* __restrict__ pair, int n_super) {
  __shared__ int partner[kMaxBlocks];    // -1: unmatched
  __shared__ int best[kMaxBlocks];       // this round's proposal; later the list of unmatched blocks
  __shared__ int wave_sums[kPairThreads / 64];
  const int tid = threadIdx.x;
  const size_t bh = blockIdx.x;
  const int32_t* cd = cand + bh * (size_t)N * kPairCandidates;
  for (int i = tid; i < N; i += kPairThreads) partner[i] = -1;
  // thread t proposes for blocks t, t + 1024, ...: their candidate lists stay in registers
  constexpr int kOwn = kMaxBlocks / kPairThreads;
  int list[kOwn][kPairCandidates];
#pragma unroll
  for (int u = 0; u < kOwn; ++u) {
    const int i = tid + u * kPairThreads;
#pragma unroll
    for (int t = 0; t < kPairCandidates; ++t) list[u][t] = i < N ? cd[(size_t)i * kPairCandidates + t] : -1;
  }
  __syncthreads();
  for (int round = 0; round < kPairRounds; ++round) {
#pragma unroll
    for (int u = 0; u < kOwn; ++u) {
      const int i = tid + u * kPairThreads;
      if (i >= N) continue;
      int choice = -1;
      if (partner[i] < 0) {
#pragma unroll
        for (int t = kPairCandidates - 1; t >= 0; --t) {       // the first unmatched candidate wins
          const int j = list[u][t];
          if (j >= 0 && j < N && partner[j] < 0) choice = j;
        }
      }
      best[i] = choice;
    }
    __syncthreads();
    for (int i = tid; i < N; i += kPairThreads) {
      const int j = best[i];
      if (j > i && best[j] == i) {       // the lower member of a mutual pair writes both
        partner[i] = j;
        partner[j] = i;
      }
    }
    __syncthreads();
  }

  // 3. the rest, in index order: thread t owns blocks 4 t .. 4 t + 3
  int mine[4], n_mine = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = 4 * tid + u;
    mine[u] = (i < N && partner[i] < 0) ? 1 : 0;
    n_mine += mine[u];
  }
  int n_free = 0;
  int rank = block_exclusive_scan(n_mine, wave_sums, n_free);
  __syncthreads();                       // every thread has read partner[] and best[] of the rounds
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (mine[u]) best[rank++] = 4 * tid + u;        // best[] now lists the unmatched blocks
  __syncthreads();
  for (int r = tid; r < n_free; r += kPairThreads) {
    const int i = best[r];
    partner[i] = (r ^ 1) < n_free ? best[r ^ 1] : -1;   // an odd one out stays single
  }
  __syncthreads();

  // 4. pairs in the order of their lower member
  int heads = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = 4 * tid + u;
    mine[u] = (i < N && (partner[i] > i || partner[i] < 0)) ? 1 : 0;
    heads += mine[u];
  }
  int n_heads = 0;
  int pid = block_exclusive_scan(heads, wave_sums, n_heads);
  int32_t* out = pair + bh * (size_t)n_super * 2;
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (mine[u] && pid < n_super) {
      out[2 * pid] = 4 * tid + u;
      out[2 * pid + 1] = partner[4 * tid + u];
      ++pid;
    }
  // N blocks make ceil(N / 2) = n_super pairs (at most one of them single), so the table is full
}

}  // namespace

bool pairing_pays(const Dims& dm, int k_top) {
  // block 64 only (a block-128 workgroup holds one block); on short sequences the launches cost
  // more than the shared tiles save, and above a density of 20 % neighbouring rows overlap so
  // much already that nothing was gained (measured at 25 % and 50 %)
  // PISA_NO_PAIRING=1 in the environment (read once) keeps the neighbour pairing: for studies that
  // need two launches to walk the same trips
  static const bool off = [] {
    const char* e = std::getenv("PISA_NO_PAIRING");
    return e != nullptr && e[0] == '1';
  }();
  return !off && dm.dtype == PISA_BF16 && dm.B == kTile && k_top > 0 && k_top * 5 <= dm.N && dm.N >= 256;
}

size_t pairing_workspace_bytes(const Dims& dm) {
  if (dm.dtype != PISA_BF16 || dm.B != kTile || dm.N < 256) return 0;
  const size_t w32 = (dm.N + 31) / 32, n_super = (dm.N + 1) / 2;
  return (size_t)dm.bh() * ((size_t)dm.N * w32 * sizeof(unsigned int) +
                            (size_t)dm.N * kPairCandidates * sizeof(int32_t) + 2 * n_super * sizeof(int32_t));
}

hipError_t launch_pair_blocks(const Dims& dm, const int32_t* idx, int k_top, void* workspace, const int32_t** pair,
                              hipStream_t stream) {
  const size_t w32 = (dm.N + 31) / 32, n_super = (dm.N + 1) / 2;
  unsigned int* masks = static_cast<unsigned int*>(workspace);
  int32_t* cand = reinterpret_cast<int32_t*>(masks + (size_t)dm.bh() * dm.N * w32);
  int32_t* table = cand + (size_t)dm.bh() * dm.N * kPairCandidates;
  hipLaunchKernelGGL(row_masks_kernel, dim3((dm.N + 3) / 4, dm.bh()), dim3(256), 0, stream, idx, dm.N, k_top, masks);
  hipLaunchKernelGGL(pair_candidates_kernel, dim3((dm.N + 3) / 4, dm.bh()), dim3(256), 0, stream, masks, dm.N, cand);
  hipLaunchKernelGGL(match_kernel, dim3(dm.bh()), dim3(kPairThreads), 0, stream, cand, dm.N, table, (int)n_super);
  *pair = table;
  return hipGetLastError();
}

}  // namespace pisa
