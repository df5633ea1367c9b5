// C-ABI entry points of libpisa: argument validation and dispatch.
// Validation runs before any device call, so bad arguments are reported on a
// host without a GPU too.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>

#include <initializer_list>

#include "common.h"

namespace pisa {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static int32_t hip_fail(const char* what, hipError_t e) {
  return fail(PISA_HIP_ERROR, "%s: %s (%d)", what, hipGetErrorName(e), (int)e);
}

// Validates a shape and resolves it.  Returns PISA_OK or an error code.
static int32_t resolve(const pisa_shape* s, Dims* dm) {
  if (!s) return fail(PISA_INVALID_ARG, "shape is NULL");
  if (s->batch < 1 || s->heads < 1 || s->seq_len < 1)
    return fail(PISA_INVALID_ARG, "batch, heads and seq_len must be >= 1 (got %d, %d, %d)",
                s->batch, s->heads, s->seq_len);
  if (s->dtype != PISA_FP32 && s->dtype != PISA_BF16)
    return fail(PISA_INVALID_ARG, "dtype must be PISA_FP32 (0) or PISA_BF16 (1), got %d", s->dtype);
  if (s->block != 64 && s->block != 128)
    return fail(PISA_INVALID_ARG, "block must be 64 or 128, got %d", s->block);
  if (s->head_dim != 64 && s->head_dim != 128)
    return fail(PISA_INVALID_ARG, "head_dim must be 64 or 128, got %d", s->head_dim);
  if (!(s->scale == s->scale) || std::isinf(s->scale))
    return fail(PISA_INVALID_ARG, "scale is not finite");
  if ((long long)s->batch * s->heads > 65535)     // several kernels put batch * heads on a 16-bit grid axis
    return fail(PISA_UNSUPPORTED, "batch * heads = %lld exceeds 65535", (long long)s->batch * s->heads);
  long long rows = (long long)s->batch * s->heads * s->seq_len;
  if (rows * s->head_dim >= (1LL << 40))
    return fail(PISA_UNSUPPORTED, "tensor too large");
  dm->batch = s->batch;
  dm->heads = s->heads;
  dm->L = s->seq_len;
  dm->d = s->head_dim;
  dm->B = s->block;
  dm->N = (s->seq_len + s->block - 1) / s->block;
  dm->dtype = s->dtype;
  dm->scale = s->scale > 0.f ? s->scale : 1.0f / std::sqrt((float)s->head_dim);
  return PISA_OK;
}

StatsPlan stats_plan(const Dims& dm) {
  // The streaming kernels keep two workgroups on each of the 256 compute units, and all
  // their workgroups take about the same time: the launch should be a whole number of rounds
  // of 512, never a few workgroups more.  Aim at two rounds (one when that still leaves a
  // workgroup only a handful of blocks, to halve the partial sums written and re-read).
  const int kSlots = 512;
  int target = 2 * kSlots;
  if ((long long)dm.N * dm.bh() <= 8LL * kSlots) target = kSlots;
  int want = target / dm.bh();
  if (want < 1) want = 1;
  if (want > dm.N) want = dm.N;
  StatsPlan p;
  p.chunk_blocks = (dm.N + want - 1) / want;
  p.n_chunks = (dm.N + p.chunk_blocks - 1) / p.chunk_blocks;
  return p;
}

static size_t stats_workspace_bytes(const Dims& dm) {
  StatsPlan p = stats_plan(dm);
  return (size_t)dm.bh() * p.n_chunks * dm.d * dm.d * sizeof(float);
}

}  // namespace pisa

using namespace pisa;

// The kernels move 16 bytes per lane: every tensor pointer has to sit on a 16-byte boundary.
static bool misaligned(std::initializer_list<const void*> ptrs) {
  for (const void* p : ptrs)
    if (reinterpret_cast<uintptr_t>(p) & 15u) return true;
  return false;
}
#define PISA_CHECK_ALIGN(...)                                                                   \
  if (misaligned({__VA_ARGS__})) return fail(PISA_INVALID_ARG, "tensor and workspace pointers must be 16-byte aligned")

extern "C" {

int32_t pisa_num_blocks(int32_t seq_len, int32_t block) {
  if (seq_len < 1 || block < 1) return -1;
  return (seq_len + block - 1) / block;
}

int32_t pisa_topk_count(int32_t num_blocks, double sparsity) {
  if (num_blocks < 0 || !(sparsity == sparsity)) return -1;
  double approx = std::floor(sparsity * (double)num_blocks + 1e-9);
  double k = (double)num_blocks - approx;
  if (k < 0) k = 0;
  if (k > num_blocks) k = num_blocks;
  return (int32_t)k;
}

size_t pisa_workspace_bytes(const pisa_shape* shape) {
  Dims dm;
  if (resolve(shape, &dm) != PISA_OK) return 0;
  return std::max({stats_workspace_bytes(dm), select_workspace_bytes(dm), attention_workspace_bytes(dm),
                   hetero_workspace_bytes(dm)});
}

int32_t pisa_block_stats(const pisa_shape* shape, const void* q, const void* k, const void* v,
                         float* qbar, float* kbar, float* vsum, float* hsum,
                         double* qbar64, double* kbar64,
                         void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  int32_t rc = resolve(shape, &dm);
  if (rc != PISA_OK) return rc;
  if (!q || !k || !v) return fail(PISA_INVALID_ARG, "q, k, v must not be NULL");
  if (!qbar || !kbar || !vsum || !hsum)
    return fail(PISA_INVALID_ARG, "qbar, kbar, vsum, hsum must not be NULL");
  PISA_CHECK_ALIGN(q, k, v, qbar, kbar, vsum, hsum, qbar64, kbar64, workspace);
  size_t need = stats_workspace_bytes(dm);
  if (!workspace) return fail(PISA_INVALID_ARG, "workspace is NULL (need %zu bytes)", need);
  if (workspace_bytes < need)
    return fail(PISA_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, need %zu", workspace_bytes, need);
  hipError_t e = launch_block_stats(dm, q, k, v, qbar, kbar, vsum, hsum, qbar64, kbar64,
                                    (float*)workspace, StatsExtras{}, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("pisa_block_stats", e);
  return PISA_OK;
}

int32_t pisa_block_heterogeneity(const pisa_shape* shape, const void* k, const void* v,
                                 const double* kbar64, const float* hsum, int32_t norm_kind, double eps,
                                 double* log_m,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  int32_t rc = resolve(shape, &dm);
  if (rc != PISA_OK) return rc;
  if (norm_kind != PISA_NORM_SPECTRAL && norm_kind != PISA_NORM_FROBENIUS && norm_kind != PISA_NORM_FROBENIUS_FAST)
    return fail(PISA_INVALID_ARG, "norm_kind must be PISA_NORM_SPECTRAL (0), PISA_NORM_FROBENIUS (1) or "
                                  "PISA_NORM_FROBENIUS_FAST (2)");
  if (!(eps >= 0.0)) return fail(PISA_INVALID_ARG, "eps must be >= 0");
  PISA_CHECK_ALIGN(k, v, kbar64, hsum, log_m, workspace);
  if (norm_kind == PISA_NORM_FROBENIUS_FAST) {
    if (!k || !v || !log_m) return fail(PISA_INVALID_ARG, "k, v, log_m must not be NULL");
    if (dm.dtype != PISA_BF16)
      return fail(PISA_UNSUPPORTED, "PISA_NORM_FROBENIUS_FAST runs on the bf16 matrix cores: bf16 inputs only");
    if (!hsum) return fail(PISA_INVALID_ARG, "PISA_NORM_FROBENIUS_FAST needs hsum (as written by pisa_block_stats)");
    hipError_t e = launch_block_heterogeneity_fast(dm, k, v, hsum, eps, log_m, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail("pisa_block_heterogeneity", e);
    return PISA_OK;
  }
  if (!k || !v || !kbar64 || !log_m) return fail(PISA_INVALID_ARG, "k, v, kbar64, log_m must not be NULL");
  size_t need = hetero_workspace_bytes(dm);
  if (!workspace) return fail(PISA_INVALID_ARG, "workspace is NULL (need %zu bytes)", need);
  if (workspace_bytes < need)
    return fail(PISA_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, need %zu", workspace_bytes, need);
  hipError_t e = launch_block_heterogeneity(dm, k, v, kbar64, hsum, norm_kind == PISA_NORM_SPECTRAL,
                                            kSpectralMaxSteps, eps, log_m, (double*)workspace,
                                            (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("pisa_block_heterogeneity", e);
  return PISA_OK;
}

int32_t pisa_select(const pisa_shape* shape, const double* qbar64, const double* kbar64,
                    const double* col_bias, int32_t k_top, int32_t* idx, float* kth_gap,
                    void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  int32_t rc = resolve(shape, &dm);
  if (rc != PISA_OK) return rc;
  if (!qbar64 || !kbar64) return fail(PISA_INVALID_ARG, "qbar64 and kbar64 must not be NULL");
  if (k_top < 0 || k_top > dm.N)
    return fail(PISA_INVALID_ARG, "k_top = %d outside [0, N = %d]", k_top, dm.N);
  if (k_top > 0 && !idx) return fail(PISA_INVALID_ARG, "idx is NULL but k_top > 0");
  PISA_CHECK_ALIGN(qbar64, kbar64, col_bias, idx, kth_gap, workspace);
  if (dm.N > kMaxBlocks)
    return fail(PISA_UNSUPPORTED, "at most %d blocks are supported (N = %d)", kMaxBlocks, dm.N);
  size_t need = select_workspace_bytes(dm);
  if (!workspace) return fail(PISA_INVALID_ARG, "workspace is NULL (need %zu bytes)", need);
  if (workspace_bytes < need)
    return fail(PISA_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, need %zu", workspace_bytes, need);
  hipError_t e = launch_select(dm, qbar64, kbar64, col_bias, k_top, idx, kth_gap, (double*)workspace,
                               nullptr, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("pisa_select", e);
  return PISA_OK;
}

static int32_t run_attention(const Dims& dm, const AttnArgs& a, void* stream, const char* who) {
  // the bf16 kernels address a head's K and V tiles with 32-bit byte offsets
  if (dm.dtype == PISA_BF16 && (long long)dm.L * dm.d * 2 >= (1LL << 31))
    return fail(PISA_UNSUPPORTED, "%s: one head of K or V must stay below 2 GiB (seq_len * head_dim * 2 = %lld bytes)",
                who, (long long)dm.L * dm.d * 2);
  hipError_t e = dm.dtype == PISA_BF16 ? launch_attention_bf16(dm, a, (hipStream_t)stream)
                                       : launch_attention_fp32(dm, a, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(who, e);
  return PISA_OK;
}

int32_t pisa_attention(const pisa_shape* shape, const void* q, const void* k, const void* v,
                       const float* kbar, const float* vsum, const float* hsum,
                       const int32_t* idx, int32_t k_top,
                       void* out, float* lse,
                       void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  int32_t rc = resolve(shape, &dm);
  if (rc != PISA_OK) return rc;
  if (!q || !k || !v || !out) return fail(PISA_INVALID_ARG, "q, k, v, out must not be NULL");
  if (k_top < 0 || k_top > dm.N)
    return fail(PISA_INVALID_ARG, "k_top = %d outside [0, N = %d]", k_top, dm.N);
  if (k_top > 0 && !idx) return fail(PISA_INVALID_ARG, "idx is NULL but k_top > 0");
  if ((kbar == nullptr) != (vsum == nullptr))
    return fail(PISA_INVALID_ARG, "kbar and vsum must both be given or both be NULL");
  if (!kbar && k_top == 0)
    return fail(PISA_INVALID_ARG, "keep-or-drop mode (kbar == vsum == NULL) needs k_top >= 1");
  PISA_CHECK_ALIGN(q, k, v, kbar, vsum, hsum, idx, out, lse, workspace);
  if (dm.N > kMaxBlocks)
    return fail(PISA_UNSUPPORTED, "at most %d blocks are supported (N = %d)", kMaxBlocks, dm.N);
  if (k_top < dm.N && kbar) {
    size_t need = attention_workspace_bytes(dm);
    if (need > 0 && !workspace) return fail(PISA_INVALID_ARG, "workspace is NULL (need %zu bytes)", need);
    if (workspace_bytes < need)
      return fail(PISA_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, need %zu", workspace_bytes, need);
  } else if (workspace && workspace_bytes < attention_workspace_bytes(dm)) {
    workspace = nullptr;       // not needed in this mode; too small for the optional pairing of query blocks
  }
  AttnArgs a{q, k, v, kbar, vsum, hsum, idx, k_top, out, lse, false, workspace};
  return run_attention(dm, a, stream, "pisa_attention");
}

int32_t pisa_attention_static(const pisa_shape* shape, const void* q, const void* k, const void* v,
                              const float* kbar, const float* vsum, const float* hsum,
                              const int32_t* idx, int32_t k_top, void* out, float* lse, void* stream) {
  Dims dm;
  int32_t rc = resolve(shape, &dm);
  if (rc != PISA_OK) return rc;
  if (!q || !k || !v || !out) return fail(PISA_INVALID_ARG, "q, k, v, out must not be NULL");
  if (k_top < 0 || k_top > dm.N)
    return fail(PISA_INVALID_ARG, "k_top = %d outside [0, N = %d]", k_top, dm.N);
  if (k_top > 0 && !idx) return fail(PISA_INVALID_ARG, "idx is NULL but k_top > 0");
  if ((kbar == nullptr) != (vsum == nullptr))
    return fail(PISA_INVALID_ARG, "kbar and vsum must both be given or both be NULL");
  if (!kbar && k_top == 0)
    return fail(PISA_INVALID_ARG, "keep-or-drop mode (kbar == vsum == NULL) needs k_top >= 1");
  PISA_CHECK_ALIGN(q, k, v, kbar, vsum, hsum, idx, out, lse);
  if (dm.N > kMaxBlocks)
    return fail(PISA_UNSUPPORTED, "at most %d blocks are supported (N = %d)", kMaxBlocks, dm.N);
  void* ws = nullptr;
  const size_t need = attention_workspace_bytes(dm);
  if (k_top < dm.N && kbar && need > kStaticScratchBytes)
    return fail(PISA_WORKSPACE_TOO_SMALL,
                "this shape needs %zu bytes of scratch, the built-in array holds %zu: use pisa_attention "
                "with a caller-owned workspace", need, (size_t)kStaticScratchBytes);
  if (need > 0 && need <= kStaticScratchBytes) {     // (in the modes that need no scratch it still serves the pairing)
    hipError_t e = static_scratch_ptr(&ws);
    if (e != hipSuccess) return hip_fail("pisa_attention_static (address of the scratch array)", e);
  }
  AttnArgs a{q, k, v, kbar, vsum, hsum, idx, k_top, out, lse, false, ws};
  return run_attention(dm, a, stream, "pisa_attention_static");
}

// Layout of the workspace of pisa_forward: every intermediate of the three stages, each region
// on a 256-byte boundary.
namespace {
struct ForwardCarve {
  size_t qbar, kbar, vsum, hsum, qbar64, kbar64, idx, partial, logits, attn, total;
};
ForwardCarve forward_carve(const Dims& dm, int k_top) {
  ForwardCarve c{};
  size_t at = 0;
  auto take = [&](size_t bytes) {
    const size_t here = at;
    at += (bytes + 255) & ~(size_t)255;
    return here;
  };
  const size_t nd = (size_t)dm.bh() * dm.N * dm.d;
  c.qbar = take(nd * sizeof(float));
  c.kbar = take(nd * sizeof(float));
  c.vsum = take(nd * sizeof(float));
  c.hsum = take((size_t)dm.bh() * dm.d * dm.d * sizeof(float));
  c.qbar64 = take(nd * sizeof(double));
  c.kbar64 = take(nd * sizeof(double));
  c.idx = take((size_t)dm.bh() * dm.N * (size_t)std::max(k_top, 1) * sizeof(int32_t));
  c.partial = take(stats_workspace_bytes(dm));
  c.logits = take(select_fuses_reduce(dm) ? 0 : select_workspace_bytes(dm));
  c.attn = take(attention_workspace_bytes(dm));
  c.total = at;
  return c;
}
}  // namespace

size_t pisa_forward_workspace_bytes(const pisa_shape* shape, int32_t k_top) {
  Dims dm;
  if (resolve(shape, &dm) != PISA_OK) return 0;
  if (k_top < 0 || k_top > dm.N) return 0;
  return forward_carve(dm, k_top).total;
}

int32_t pisa_forward(const pisa_shape* shape, const void* q, const void* k, const void* v, int32_t k_top,
                     void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  int32_t rc = resolve(shape, &dm);
  if (rc != PISA_OK) return rc;
  if (!q || !k || !v || !out) return fail(PISA_INVALID_ARG, "q, k, v, out must not be NULL");
  if (k_top < 0 || k_top > dm.N)
    return fail(PISA_INVALID_ARG, "k_top = %d outside [0, N = %d]", k_top, dm.N);
  PISA_CHECK_ALIGN(q, k, v, out, lse, workspace);
  if (dm.N > kMaxBlocks)
    return fail(PISA_UNSUPPORTED, "at most %d blocks are supported (N = %d)", kMaxBlocks, dm.N);
  const ForwardCarve c = forward_carve(dm, k_top);
  if (!workspace) return fail(PISA_INVALID_ARG, "workspace is NULL (need %zu bytes)", c.total);
  if (workspace_bytes < c.total)
    return fail(PISA_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, need %zu", workspace_bytes, c.total);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  float* qbar = reinterpret_cast<float*>(ws + c.qbar);
  float* kbar = reinterpret_cast<float*>(ws + c.kbar);
  float* vsum = reinterpret_cast<float*>(ws + c.vsum);
  float* hsum = reinterpret_cast<float*>(ws + c.hsum);
  double* qbar64 = reinterpret_cast<double*>(ws + c.qbar64);
  double* kbar64 = reinterpret_cast<double*>(ws + c.kbar64);
  int32_t* idx = reinterpret_cast<int32_t*>(ws + c.idx);
  float* partial = reinterpret_cast<float*>(ws + c.partial);
  const hipStream_t st = (hipStream_t)stream;

  // bf16: the statistics launches also write what the attention kernel's pre-pass would (the
  // centroid tiles from the statistics kernel, the packed hsum from the reduction), and on short
  // sequences the reduction rides in the selection's single launch: three launches in all.
  StatsExtras extra;
  const bool fused = dm.dtype == PISA_BF16;
  if (fused) {
    attention_workspace_carve(dm, ws + c.attn, &extra.kcen, &extra.vbar, &extra.hpack);
    extra.defer_reduce = k_top > 0 && select_fuses_reduce(dm);
  }
  hipError_t e = launch_block_stats(dm, q, k, v, qbar, kbar, vsum, hsum, qbar64, kbar64, partial, extra, st);
  if (e != hipSuccess) return hip_fail("pisa_forward (statistics)", e);
  if (k_top > 0) {
    PendingReduce pending;
    pending.partial_h = partial;
    pending.hsum = hsum;
    pending.hpack = extra.hpack;
    pending.n_chunks = stats_plan(dm).n_chunks;
    e = launch_select(dm, qbar64, kbar64, nullptr, k_top, idx, nullptr, reinterpret_cast<double*>(ws + c.logits),
                      extra.defer_reduce ? &pending : nullptr, st);
    if (e != hipSuccess) return hip_fail("pisa_forward (selection)", e);
  }
  AttnArgs a{q, k, v, kbar, vsum, hsum, k_top > 0 ? idx : nullptr, k_top, out, lse, false, ws + c.attn};
  a.prepared = fused;
  return run_attention(dm, a, stream, "pisa_forward (attention)");
}

int32_t dense_attention(const pisa_shape* shape, const void* q, const void* k, const void* v,
                        void* out, float* lse, void* stream) {
  Dims dm;
  int32_t rc = resolve(shape, &dm);
  if (rc != PISA_OK) return rc;
  if (!q || !k || !v || !out) return fail(PISA_INVALID_ARG, "q, k, v, out must not be NULL");
  PISA_CHECK_ALIGN(q, k, v, out, lse);
  AttnArgs a{q, k, v, nullptr, nullptr, nullptr, nullptr, dm.N, out, lse, true, nullptr};
  return run_attention(dm, a, stream, "dense_attention");
}

int32_t pisa_probe_mfma_rate(int32_t iters, float* sink, size_t sink_floats, double* flop, void* stream) {
  if (iters < 1 || iters > (1 << 24)) return fail(PISA_INVALID_ARG, "iters = %d outside [1, 2^24]", iters);
  if (!sink || !flop) return fail(PISA_INVALID_ARG, "sink and flop must not be NULL");
  const size_t need = (size_t)kProbeWorkgroups * 256;
  if (sink_floats < need) return fail(PISA_WORKSPACE_TOO_SMALL, "sink has %zu floats, need %zu", sink_floats, need);
  PISA_CHECK_ALIGN(sink);
  *flop = (double)kProbeWorkgroups * 4.0 * (double)iters * 16.0 * (2.0 * 32 * 32 * 16);
  hipError_t e = launch_mfma_probe(iters, sink, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("pisa_probe_mfma_rate", e);
  return PISA_OK;
}

int32_t pisa_probe_shader_clock(double window_ms, uint64_t* counts, double* wall_clock_hz, void* stream) {
  if (!(window_ms > 0.0) || window_ms > 50.0)
    return fail(PISA_INVALID_ARG, "window_ms = %g outside (0, 50]", window_ms);
  if (!counts || !wall_clock_hz) return fail(PISA_INVALID_ARG, "counts and wall_clock_hz must not be NULL");
  PISA_CHECK_ALIGN(counts);
  int dev = 0, khz = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev);
  if (e != hipSuccess) return hip_fail("pisa_probe_shader_clock", e);
  if (khz <= 0) return fail(PISA_UNSUPPORTED, "the device reports no wall-clock rate");
  *wall_clock_hz = 1e3 * (double)khz;
  const unsigned long long ticks = (unsigned long long)(window_ms * (double)khz);
  e = launch_clock_probe(reinterpret_cast<unsigned long long*>(counts), ticks, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail("pisa_probe_shader_clock", e);
  return PISA_OK;
}

const char* pisa_last_error(void) { return pisa::g_err; }

}  // extern "C"
