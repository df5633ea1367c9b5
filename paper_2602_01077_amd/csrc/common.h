// Internal declarations shared by the translation units of libpisa.
// Host-side only: problem dimensions, error reporting, launcher prototypes.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pisa.h"

namespace pisa {

// Resolved problem dimensions (shape after validation).
struct Dims {
  int batch, heads, L, d, B, N;   // N = ceil(L / B)
  int dtype;                      // PISA_FP32 / PISA_BF16
  float scale;                    // resolved softmax scale
  int bh() const { return batch * heads; }
};

// Key/value tiles are always 64 rows; a block of 128 tokens is walked as two tiles.
constexpr int kTile = 64;
// Largest block count the selection and the Phase-2 column mask are sized for.
constexpr int kMaxBlocks = 4096;
// Spectral norm of the block heterogeneity: the eigenvalue iteration on D^T D stops at this
// relative residual (||A x - theta x|| <= kRelResidual * theta), or after kSpectralMaxSteps steps.
constexpr double kRelResidual = 1e-7;
constexpr int kSpectralMaxSteps = 300;

// Records the message returned by pisa_last_error() and returns `code`.
int32_t fail(int32_t code, const char* fmt, ...);

// Chunking of the block axis used by the statistics kernels: each workgroup
// accumulates H over `chunk_blocks` consecutive blocks of one head, and the
// partial sums are reduced in chunk order afterwards.
struct StatsPlan {
  int chunk_blocks;
  int n_chunks;
};
StatsPlan stats_plan(const Dims& dm);

// What the fused forward call asks of the statistics launches beyond the plain outputs (all
// optional; bf16 only): the centroid tiles and the packed hsum in the form the attention kernel
// reads (they replace its pre-pass), and leaving the reduction of the partial H sums to a later
// launch.
struct StatsExtras {
  void* kcen = nullptr;          // bf16 [bh][npad][d]: kbar_j
  void* vbar = nullptr;          // bf16 [bh][npad][d]: vsum_j / B_j
  void* hpack = nullptr;         // bf16 [bh][2][d*d]: hsum split hi / lo in operand order
  bool defer_reduce = false;
};
// The reduction a deferred statistics launch left undone, for launch_select to run in its launch.
struct PendingReduce {
  const float* partial_h = nullptr;
  float* hsum = nullptr;
  void* hpack = nullptr;
  int n_chunks = 0;
};

// Launchers (each returns hipGetLastError() after its launches).
hipError_t launch_block_stats(const Dims& dm, const void* q, const void* k, const void* v,
                              float* qbar, float* kbar, float* vsum, float* hsum,
                              double* qbar64, double* kbar64, float* partial_h,
                              const StatsExtras& extra, hipStream_t stream);
size_t select_workspace_bytes(const Dims& dm);
// True if launch_select would take `pending` into its own (single) launch for this shape.
bool select_fuses_reduce(const Dims& dm);
hipError_t launch_select(const Dims& dm, const double* qbar64, const double* kbar64,
                         const double* col_bias, int k_top, int32_t* idx, float* kth_gap, double* zbuf,
                         const PendingReduce* pending, hipStream_t stream);
size_t hetero_workspace_bytes(const Dims& dm);
hipError_t launch_block_heterogeneity(const Dims& dm, const void* k, const void* v, const double* kbar64,
                                      const float* hsum, int spectral, int n_iter, double eps, double* log_m,
                                      double* workspace, hipStream_t stream);

hipError_t launch_block_heterogeneity_fast(const Dims& dm, const void* k, const void* v, const float* hsum,
                                           double eps, double* log_m, hipStream_t stream);

// Arguments of the attention kernels (dense and PISA share them).
struct AttnArgs {
  const void* q;
  const void* k;
  const void* v;
  const float* kbar;     // null for dense
  const float* vsum;     // null for dense
  const float* hsum;     // null: no first-order term
  const int32_t* idx;    // null for dense
  int k_top;
  void* out;
  float* lse;            // may be null
  bool dense;
  void* workspace;       // scratch for the bf16 PISA pre-pass (null for dense / fp32)
  bool prepared = false; // the workspace already holds the pre-pass results (fused forward call)
};
size_t attention_workspace_bytes(const Dims& dm);
// Where the bf16 attention pre-pass results sit inside a workspace of that size.
void attention_workspace_carve(const Dims& dm, void* workspace, void** kcen, void** vbar, void** hpack);
// Pairing of the query blocks that share a block-64 workgroup by the overlap of their index rows
// (one launch; the table it writes lives in `workspace`, pairing_workspace_bytes large).
bool pairing_pays(const Dims& dm, int k_top);
size_t pairing_workspace_bytes(const Dims& dm);
hipError_t launch_pair_blocks(const Dims& dm, const int32_t* idx, int k_top, void* workspace, const int32_t** pair,
                              hipStream_t stream);
// Size of the file-scope device array behind pisa_attention_static, and its address on the
// current device (resolved on first use, once per device).
constexpr size_t kStaticScratchBytes = PISA_STATIC_SCRATCH_BYTES;
hipError_t static_scratch_ptr(void** out);
hipError_t launch_attention_fp32(const Dims& dm, const AttnArgs& a, hipStream_t stream);
hipError_t launch_attention_bf16(const Dims& dm, const AttnArgs& a, hipStream_t stream);

// Matrix-core rate probe: kProbeWorkgroups workgroups of 4 waves, 16 MFMAs per wave and iteration.
constexpr int kProbeWorkgroups = 1024;
hipError_t launch_mfma_probe(int iters, float* sink, hipStream_t stream);
// Shader-clock probe: one wave, out = {shader cycles, wall-clock ticks} over `ticks` ticks.
hipError_t launch_clock_probe(unsigned long long* out, unsigned long long ticks, hipStream_t stream);

}  // namespace pisa
