/*
 * libpisa -- forward pass of Piecewise Sparse Attention (PISA) for AMD MI355X (gfx950).
 *
 * C ABI.  Every entry point below follows one step of the paper's forward-pass
 * algorithm (Methodology, "Hardware-aware Kernel Implementation", Alg. 1):
 *
 *   pisa_block_stats   Alg. 1, "Prepare" step (block means, block value sums, global H)
 *   pisa_select        Alg. 1, "Select" step (block-wise top-k of pooled scores)
 *   pisa_block_heterogeneity   "Covariance-Aware Block Selection": log(M_j + eps)
 *   pisa_attention     Alg. 1, the loop over query blocks: Phase 1 exact, Phase 2 zeroth-order
 *                      scan, Phase 3 global first-order term, one online softmax
 *   pisa_attention_static      the same for callers that cannot allocate (built-in scratch)
 *   pisa_forward       the three steps in one call (fewer launches on short sequences)
 *   dense_attention    Preliminaries, first equation (softmax(QK^T/sqrt d)V), the
 *                      speed-up baseline, written with the same tile loop
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never
 *     allocates, frees or synchronises.  Work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream).  Every tensor and
 *     workspace pointer must be 16-byte aligned (PISA_INVALID_ARG otherwise).
 *   - Layout: Q, K, V, O are dense [batch, heads, seq_len, head_dim], head_dim contiguous.
 *     Blocks are consecutive runs of `block` tokens; N = ceil(seq_len / block); the last
 *     block may be ragged (B_j < block rows) -- statistics run over its valid rows.
 *   - Supported: dtype PISA_BF16 with head_dim 128 or 64 (MFMA path); dtype PISA_FP32 with
 *     head_dim 64 or 128 (fp32 path); block 64 or 128; batch * heads <= 65535.
 *   - Every function returns a status code; pisa_last_error() gives the message of the
 *     last failure on the calling thread.  Arguments are validated before any device
 *     call, so argument errors are reported on a host without a GPU as well.
 */
#ifndef PISA_H_
#define PISA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  PISA_OK = 0,
  PISA_INVALID_ARG = 1,          /* null pointer, non-positive size, k outside [0, N], ... */
  PISA_UNSUPPORTED = 2,          /* dtype / head_dim / block combination not built        */
  PISA_WORKSPACE_TOO_SMALL = 3,
  PISA_HIP_ERROR = 4             /* a launch failed; message carries the hipError_t name   */
};

enum { PISA_FP32 = 0, PISA_BF16 = 1 };
enum { PISA_NORM_SPECTRAL = 0, PISA_NORM_FROBENIUS = 1, PISA_NORM_FROBENIUS_FAST = 2 };

typedef struct pisa_shape {
  int32_t batch;      /* >= 1 */
  int32_t heads;      /* >= 1 */
  int32_t seq_len;    /* L >= 1 */
  int32_t head_dim;   /* d: 64 or 128 */
  int32_t block;      /* B: 64 or 128 (query and key/value side alike) */
  int32_t dtype;      /* PISA_FP32 or PISA_BF16: element type of Q, K, V, O */
  float   scale;      /* softmax scale s; <= 0 selects 1/sqrt(head_dim) */
} pisa_shape;

/* Alg. 1 (the loop over query blocks i = 1 .. ceil(L / B)): the number of blocks
 * N = ceil(seq_len / block) on the query and on the key/value side alike.
 * Returns -1 on non-positive arguments. */
int32_t pisa_num_blocks(int32_t seq_len, int32_t block);

/* Number k of exactly-attended blocks at sparsity r (Experiments, "Implementation
 * Details": sparsity = share of blocks handled by the approximation):
 * k = N - floor(r*N + 1e-9), clamped to [0, N].  Returns -1 if N < 0 or r is NaN. */
int32_t pisa_topk_count(int32_t num_blocks, double sparsity);

/* Bytes of device scratch that pisa_block_stats, pisa_block_heterogeneity, pisa_select and
 * pisa_attention each need
 * for this shape (the largest of: partial sums of H, reduced in a fixed order so the result
 * is run-to-run identical; the N x N fp64 pooled logits per head; the bf16 centroid tiles
 * and the packed hsum the attention kernel streams).  One buffer of this size serves all
 * three calls when they run one after the other on a stream.  0 on a bad shape. */
size_t pisa_workspace_bytes(const pisa_shape* shape);

/*
 * Alg. 1, "Prepare" step.  For every (batch, head):
 *   qbar[i,:]  = mean of the rows of query block i            fp32 [batch,heads,N,d]
 *   kbar[j,:]  = mean of the rows of key block j  (centroid)  fp32 [batch,heads,N,d]
 *   vsum[j,:]  = sum  of the rows of value block j            fp32 [batch,heads,N,d]
 *   hsum       = sum_j sum_n (k_{j,n} - kbar_j)^T v_{j,n}     fp32 [batch,heads,d,d]
 *                (the UN-normalised sum over all N blocks of the per-block H_j of the
 *                "Global First-Order Correction" paragraph; hsum[a][b] pairs key channel a
 *                with value channel b)
 *   qbar64, kbar64: the same means in fp64 [batch,heads,N,d] (block sums are accumulated
 *                in fp64, so for bf16 inputs they are exact); pisa_select ranks with these.
 *                Either may be NULL when the caller does not need it.
 * Outputs are written, never read.  `workspace` must hold pisa_workspace_bytes(shape).
 */
int32_t pisa_block_stats(const pisa_shape* shape, const void* q, const void* k, const void* v,
                         float* qbar, float* kbar, float* vsum, float* hsum,
                         double* qbar64, double* kbar64,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * Methodology, "Covariance-Aware Block Selection": per key block j the heterogeneity
 *   M_j = || H_j - Hbar ||,  H_j = sum_n (k_{j,n} - kbar_j)^T v_{j,n},  Hbar = (1/N) sum_j H_j,
 * and the column bias log(M_j + eps) that the selection score adds to the pooled logit.
 *   norm_kind  PISA_NORM_SPECTRAL: operator 2-norm (the norm of the paper's error analysis):
 *              the largest eigenvalue theta of (H_j - Hbar)^T (H_j - Hbar) by a Krylov-type
 *              iteration from a fixed start vector, run until the residual of the eigenpair is
 *              below 1e-7 theta (at most 300 steps), M_j = sqrt(theta): within 5e-8 relative of a
 *              singular value by construction, in practice equal to the largest one to rounding;
 *              PISA_NORM_FROBENIUS: exact (fp64), cheaper, an upper bound of the spectral norm.
 *              PISA_NORM_FROBENIUS_FAST (bf16 inputs only, needs hsum): the Frobenius norm with H_j
 *              rebuilt the way pisa_block_stats builds it (bf16 matrix cores, K centred and split
 *              hi + lo, fp32 accumulation: the very bits that were summed into hsum) instead of
 *              in fp64: one pass at the cost of the statistics pass; M_j within 1e-6 of the
 *              largest M_j of the head (1e-7 measured).  kbar64 and workspace are not used and may be NULL.
 *   kbar64     fp64 [batch,heads,N,d] as written by pisa_block_stats
 *   hsum       NULL: Hbar is accumulated here in fp64 (one more pass over K and V), and M_j matches
 *              a plain fp64 evaluation to rounding.  Or fp32 [batch,heads,d,d] as written by
 *              pisa_block_stats: Hbar = hsum / N is taken from it, which saves that pass; Hbar then
 *              carries the fp32 rounding of hsum (about 1e-6 of its largest entry), and M_j an
 *              error of about 1e-7 relative, since ||Hbar|| is a fraction of ||H_j - Hbar||.
 *   log_m      fp64 [batch,heads,N], written
 * All arithmetic is fp64 except in the FAST kind.  `workspace` must hold pisa_workspace_bytes(shape).
 * The paper enables this score for image models only; pass log_m as `col_bias` to pisa_select.
 */
int32_t pisa_block_heterogeneity(const pisa_shape* shape, const void* k, const void* v,
                                 const double* kbar64, const float* hsum, int32_t norm_kind, double eps,
                                 double* log_m,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Alg. 1, "Select" step.  For every (batch, head, query block i): logits z_ij = s * qbar_i . kbar_j
 * (+ col_bias[j] if given: the selection-score equation with or without its covariance term;
 * softmax is monotone so the logits are ranked directly), and the k_top largest are kept;
 * equal logits go to the lower block index.
 *   col_bias fp64 [batch,heads,N] or NULL
 *   idx      int32 [batch,heads,N,k_top], ascending and unique within a row
 *   kth_gap  fp32  [batch,heads,N]: z of rank k_top minus z of rank k_top+1 (+inf when
 *            k_top is 0 or N); may be NULL.  Rows with a tiny gap are the only ones where
 *            another index set is equally valid.
 * k_top == 0 is legal (idx may then be NULL).  N up to 4096 blocks.
 * `workspace` must hold pisa_workspace_bytes(shape); its contents are overwritten.
 */
int32_t pisa_select(const pisa_shape* shape, const double* qbar64, const double* kbar64,
                    const double* col_bias, int32_t k_top, int32_t* idx, float* kth_gap,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Alg. 1, the loop over query blocks (its three phases) for every (batch, head, query block i), rows t of the block:
 *   D_t = sum_{j in S_i} sum_n exp(s q_t k_{j,n}^T)  +  sum_{j in U_i} B_j exp(s q_t kbar_j^T)
 *   N_t = sum_{j in S_i} sum_n exp(s q_t k_{j,n}^T) v_{j,n}
 *       + sum_{j in U_i} exp(s q_t kbar_j^T) vsum_j
 *       + (T_t / L) (s q_t) hsum ,   T_t = sum_{j in U_i} B_j exp(s q_t kbar_j^T)
 *   out_t = N_t / D_t                         (hybrid equations; the last step of Alg. 1)
 * with S_i = idx[i, :], U_i its complement, all inside one running-max softmax.
 *   kbar, vsum, hsum: as written by pisa_block_stats.  hsum == NULL drops the first-order
 *            term (the zeroth-order variant of the ablation study).  kbar == vsum == NULL
 *            drops the approximation altogether: plain block-sparse "keep-or-drop" attention
 *            over S_i (Preliminaries, second equation; the ablation's baseline curve);
 *            k_top must then be >= 1.
 *   idx      int32 [batch,heads,N,k_top]; expected in range, ascending and unique within a
 *            row (as pisa_select writes it).  The kernels never index memory with an entry
 *            outside [0, N): such entries are ignored (the row then attends fewer blocks
 *            exactly).  Order does not matter to the bf16 build; a repeated entry is
 *            harmless there and counts the block twice in the fp32 build.
 *   out      [batch,heads,seq_len,d] in shape->dtype
 *   lse      fp32 [batch,heads,seq_len]: log D_t; may be NULL.
 * k_top == N reproduces dense_attention; k_top == 0 is the pure approximation.
 * N up to 4096 blocks.  `workspace` must hold pisa_workspace_bytes(shape) when k_top < N and
 * kbar is given (it may be NULL otherwise); its contents are overwritten.
 * bf16, block 64, N >= 256, density k_top / N at most 20 %, workspace given: which two 64-row
 * query blocks travel in one workgroup is decided from idx (blocks whose rows overlap most are
 * paired, three small launches ahead of the attention kernel), which changes the order of the
 * fp32 sums and nothing else; every entry point decides the same way for the same idx.
 * (PISA_NO_PAIRING=1 in the environment, read once per process, keeps neighbours together.)
 */
int32_t pisa_attention(const pisa_shape* shape, const void* q, const void* k, const void* v,
                       const float* kbar, const float* vsum, const float* hsum,
                       const int32_t* idx, int32_t k_top,
                       void* out, float* lse,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * pisa_attention for callers that cannot allocate or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and the same result bit for bit; the scratch (bf16 centroid tiles, packed hsum,
 * the tables of the query-block pairing)
 * lives in a device array inside the library of PISA_STATIC_SCRATCH_BYTES, which
 * every GPU the library runs on holds until the process ends.  The call allocates and frees
 * nothing and does not synchronise.
 *   - Shapes whose scratch need (batch * heads * (4 * ceil(N / 64) * 64 * d + 4 * d * d) bytes, plus
 *     batch * heads * (4 * N * ceil(N / 32) + 32 * N + 8 * ceil(N / 2)) at block 64 with N >= 256; bf16 path) exceeds the array return PISA_WORKSPACE_TOO_SMALL before
 *     any device work; the three bf16 shapes of the paper's models fit.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 *     (different streams, or threads) race on it.  Calls on one stream are ordered and safe.
 *     Nothing in the array has to be cleared between calls: each call rewrites all it reads.
 *   - The array's address is looked up on the first call on each device; make that call
 *     outside a stream capture.
 */
#define PISA_STATIC_SCRATCH_BYTES (40u << 20)
int32_t pisa_attention_static(const pisa_shape* shape, const void* q, const void* k, const void* v,
                              const float* kbar, const float* vsum, const float* hsum,
                              const int32_t* idx, int32_t k_top,
                              void* out, float* lse, void* stream);

/*
 * Alg. 1 from its first line to its last in one call: block statistics, selection of the k_top
 * exact blocks per query block (plain pooled-logit score, no covariance term), and the fused
 * three-phase attention, with every intermediate kept in the workspace.  The result (out, lse)
 * is bit for bit what pisa_block_stats + pisa_select + pisa_attention give on the same inputs.
 * What it saves is launches, which is what short sequences pay for (the paper's remark on
 * 4K-token inputs): on the bf16 path the statistics kernels write the attention kernel's
 * centroid tiles and packed hsum directly (no pre-pass), and for N <= 128 blocks the reduction
 * of the partial H sums shares the selection's launch: three launches instead of five.
 *   q, k, v    device, shape->dtype, [batch,heads,seq_len,head_dim]
 *   k_top      number of exact blocks per query block, 0 .. N (pisa_topk_count)
 *   out, lse   as for pisa_attention (lse may be NULL)
 *   workspace  device, pisa_forward_workspace_bytes(shape, k_top) bytes, 16-byte aligned,
 *              caller-owned; contents on return: the intermediates, in no documented layout
 * Errors as for the three calls; nothing is enqueued if validation fails.
 */
size_t pisa_forward_workspace_bytes(const pisa_shape* shape, int32_t k_top);   /* 0 for an invalid shape or k_top */
int32_t pisa_forward(const pisa_shape* shape, const void* q, const void* k, const void* v, int32_t k_top,
                     void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* Preliminaries, first equation: out = softmax(s Q K^T) V with an online softmax over
 * 64-key tiles; lse as above (may be NULL).  shape->block only sets the tile walk. */
int32_t dense_attention(const pisa_shape* shape, const void* q, const void* k, const void* v,
                        void* out, float* lse, void* stream);

/*
 * Measurement aid, not a step of the method: enqueues a register-only loop of the bf16
 * matrix instruction the attention kernels use (1024 workgroups x 4 waves x iters x 16
 * MFMAs of 32x32x16, on pseudo-random operands in (-1, 1)) and stores the floating-point
 * operation count in *flop (host memory).
 * The caller times the launch on `stream`; flop / time is the matrix-core rate the chip
 * sustains at its own clock, to quote beside the published peak.  `sink` is device memory of
 * at least 262144 floats (overwritten).  iters in [1, 2^24].
 */
int32_t pisa_probe_mfma_rate(int32_t iters, float* sink, size_t sink_floats, double* flop, void* stream);

/*
 * Measurement aid, not a step of the method: enqueues a one-wave kernel that reads the shader
 * cycle counter and the device's constant-rate wall clock at the start and the end of a window
 * of about window_ms milliseconds (in (0, 50]; the wave sleeps in between) and stores
 * counts[0] = shader cycles, counts[1] = wall-clock ticks (device memory, 16-byte aligned,
 * two entries).  *wall_clock_hz (host memory) receives the wall clock's rate, so that
 * counts[0] / counts[1] * wall_clock_hz is the shader clock held during the window.  Launched
 * on a second stream while an attention call runs, it reports the clock under that load.
 */
int32_t pisa_probe_shader_clock(double window_ms, uint64_t* counts, double* wall_clock_hz, void* stream);

/* Message of the last failure on this thread ("" if none).  Never NULL. */
const char* pisa_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PISA_H_ */
