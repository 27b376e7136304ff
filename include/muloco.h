/*
 * muloco.h -- C ABI of the MI355X (gfx950) MuLoCo optimizer hot path.
 *
 * Three operations, named after the method they implement:
 *   newton_schulz       quintic Newton-Schulz orthogonalisation of a batch of matrices
 *   muloco_inner_step   one Muon step (momentum, look-ahead, orthogonalisation, update)
 *   muloco_outer_step   one DiLoCo outer step over K resident worker replicas
 * plus muloco_quantize_delta, the compressor of the outer step as a call of its own.
 *
 * Conventions shared by every call
 *   - Every data pointer is a DEVICE pointer owned by the caller and 16-byte aligned.
 *     Arrays of structs and arrays of pointers (groups, worker lists) are HOST memory and
 *     are only read during the call.
 *   - A "group" is `count` row-major matrices of one shape, contiguous: [count][m][n].
 *   - bf16 buffers hold IEEE bfloat16 bit patterns (uint16_t); conversions from fp32
 *     round to nearest, ties to even.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue kernels on it; they never allocate, free or synchronise.  Work spaces are
 *     passed in by the caller and may be reused by the next call on the same stream.
 *   - Return value: MLC_OK or a negative MLC_ERR_* code.  Arguments are validated on the
 *     host before anything is enqueued; on an argument error no buffer is touched.
 *   - The library keeps no mutable state apart from the optional timing recorder.
 *   - Buffers must not overlap unless a parameter is documented as in/out or aliasable.
 */
#ifndef MULOCO_H_
#define MULOCO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MLC_F32 = 0, MLC_BF16 = 1 } mlc_dtype;

enum {
  MLC_OK = 0,
  MLC_ERR_NULL = -1,        /* a required pointer is NULL */
  MLC_ERR_SHAPE = -2,       /* count/m/n < 1, overflow, odd row length for 4-bit codes */
  MLC_ERR_DTYPE = -3,       /* not an mlc_dtype */
  MLC_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned or too small */
  MLC_ERR_ARG = -5,         /* scalar argument out of range (iters < 0, K < 1, ...) */
  MLC_ERR_LAUNCH = -6,      /* the HIP runtime refused a launch */
  MLC_ERR_UNSUPPORTED = -7, /* valid request this build does not implement */
  MLC_ERR_SCRATCH = -8      /* one matrix does not fit the library's built-in scratch buffer */
};

#define MLC_MAX_WORKERS 32  /* largest K accepted by the outer step */

/* Human-readable name of a return code (static string, never NULL). */
const char* muloco_strerror(int code);

/* ------------------------------------------------------------------------------------
 * Newton-Schulz orthogonalisation (paper Sec. 2, paragraph "Muon").
 *
 * For each of the `count` matrices U (m x n):
 *     X_0 = U / (||U||_F + eps)
 *     X_j = a X_{j-1} + b (X X^T) X_{j-1} + c (X X^T)^2 X_{j-1},   j = 1..iters
 *     out = X_iters
 * i.e. the odd quintic p(s) = a s + b s^3 + c s^5 applied to the singular values,
 * approximating the polar factor U V^T.  The paper uses (a, b, c) = (3.4445, -4.7750,
 * 2.0315) and iters = 5.  The products run on the bf16 matrix cores with fp32
 * accumulation; X, X X^T and the polynomial are held in bf16 between products, so the
 * result carries about 1e-2 relative Frobenius error with respect to exact arithmetic.
 * Tall matrices (m > n) use the algebraically identical n x n form with X^T X.
 *
 * in, out     [count][m][n] of `io` dtype; `out` may alias `in`.
 * iters       >= 0; 0 returns the normalised input.
 * workspace   at least newton_schulz_workspace_bytes(count, m, n) bytes, 256-byte
 *             aligned.  A smaller work space that still holds one matrix is accepted;
 *             the batch is then processed in several chunks.
 * An all-zero matrix gives an all-zero result (for every eps >= 0).
 */
size_t newton_schulz_workspace_bytes(int64_t count, int64_t m, int64_t n);
/* Smallest accepted work space (one matrix per chunk). */
size_t newton_schulz_workspace_min_bytes(int64_t m, int64_t n);
int newton_schulz(const void* in, void* out, int io_dtype,
                  int64_t count, int64_t m, int64_t n,
                  int iters, float a, float b, float c, float eps,
                  void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * newton_schulz for callers that cannot allocate device memory or hand over a work space:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 *
 * Same operation, arguments and results as newton_schulz, but the work space is a buffer of
 * MLC_STATIC_SCRATCH_BYTES that is part of the library's code object (each GPU the library
 * runs on holds its own copy until the process ends).  The call allocates and frees
 * nothing.  The batch is processed in as many chunks as the buffer requires; a shape whose
 * single matrix needs more (newton_schulz_workspace_min_bytes(m, n) >
 * MLC_STATIC_SCRATCH_BYTES; 2048 x 2048 still fits, 2048 x 8192 does not) is refused with
 * MLC_ERR_SCRATCH before anything is enqueued.  Every call on a GPU uses that GPU's one
 * buffer: calls on different streams of one GPU must not overlap (they would race), calls
 * on one stream are ordered and need no clearing in between (every byte that is read has
 * been written earlier in the same call).
 */
#define MLC_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int newton_schulz_static_scratch(const void* in, void* out, int io_dtype,
                                 int64_t count, int64_t m, int64_t n,
                                 int iters, float a, float b, float c, float eps, void* stream);

/* ------------------------------------------------------------------------------------
 * Muon inner step (paper Sec. 2 "Muon"; Sec. 4.1 eq. 1; Algorithm 1, the Muon line;
 * Sec. 5 "MuLoCo" for the per-shape learning-rate rescale).
 *
 * Per matrix W with gradient g and momentum accumulator mom:
 *     mom <- beta * mom + g
 *     U    = g + beta * mom            if nesterov, else U = mom
 *     O    = newton_schulz(U)          (as above)
 *     W   <- W - eta * lr_scale * O - eta * weight_decay * W
 * The paper asks for lr_scale = sqrt(n/m) for an m x n matrix; the caller supplies it.
 * For bf16 W with m and n multiples of 128 (and matrices larger than 128 x 512) the last line
 * is the epilogue of the last Newton-Schulz product: O is then used unrounded (fp32) and never
 * stored; otherwise O is rounded to bf16 and a separate pass applies it.
 */
typedef struct {
  int64_t count, m, n;
  void* param;           /* W, in/out, [count][m][n] of param_dtype                    */
  int param_dtype;       /* mlc_dtype                                                  */
  const void* grad;      /* g, in, same shape, grad_dtype                              */
  int grad_dtype;        /* mlc_dtype                                                  */
  float* momentum;       /* mom, fp32, in/out, same shape                              */
  float lr_scale;        /* multiplies eta on the orthogonalised term only             */
} mlc_inner_group;

typedef struct {
  float eta;             /* inner learning rate                                        */
  float weight_decay;    /* lambda, decoupled: the decay term is eta * lambda * W      */
  float beta;            /* momentum coefficient                                       */
  int nesterov;          /* 1: U = g + beta * mom_t ; 0: U = mom_t                     */
  int ns_iters;          /* Newton-Schulz iterations (paper: 5)                        */
  float ns_a, ns_b, ns_c;/* polynomial coefficients (paper: 3.4445, -4.7750, 2.0315)   */
  float ns_eps;          /* added to the Frobenius norm (1e-7)                         */
} mlc_muon_hparams;

/* Work space that holds every group at once, each as a single batch (the sum over groups).
 * With it the groups go through Newton-Schulz side by side and products of equal depth share
 * launches; with less (down to the minimum below) the groups are processed one after the
 * other, in chunks that fit.  The results are the same bit for bit. */
size_t muloco_inner_workspace_bytes(const mlc_inner_group* groups, int n_groups);
/* Smallest accepted work space (every group processed one matrix at a time). */
size_t muloco_inner_workspace_min_bytes(const mlc_inner_group* groups, int n_groups);
/* groups: host array.  Same-shape matrices of a group are batched into each launch. */
int muloco_inner_step(const mlc_inner_group* groups, int n_groups,
                      const mlc_muon_hparams* hp,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * DiLoCo outer step (paper Sec. 4.1 eqs. 2-3; Algorithm 1, the four lines after the
 * inner loop; Algorithm 2, "compress parameter delta", for the quantised path).
 *
 * Per element, with K worker replicas resident on this GPU:
 *     Delta_k = theta_g - theta_k
 *     Delta_k = dequantise(quantise(Delta_k))        only if quant_bits != 0
 *     Psi     = (1/K) sum_k Delta_k
 *     u      <- mu * u + eta_out * Psi
 *     theta_g<- theta_g - mu * u - eta_out * Psi     (nesterov = 1)
 *     theta_g<- theta_g - u                          (nesterov = 0)
 *     theta_k<- theta_g for every k                  (write_back = 1)
 *
 * Quantiser (quant_bits = 2, 4 or 8): row-wise linear, symmetric, defined in IEEE fp32 so
 * that codes are reproducible bit for bit.  With qmax = 2^(bits-1) - 1 (1, 7, 127), for each
 * row (length n) of each matrix:
 *     delta = fl32(theta_g) - fl32(theta_k);  amax = max |delta|;  scale = amax / qmax
 *     q = clamp(rint(delta / scale), -qmax, qmax) (ties to even), q = 0 when amax = 0
 *     code = q + 2^(bits-1); a byte holds 8 / bits codes, the lowest column in the lowest
 *     bits (4 bit: byte i of a row = code[2i] | code[2i+1] << 4)
 *     dequantised value = (float)q * scale
 * n must be a multiple of 8 / bits.
 *
 * Offset form (quant_offset = 1; the linear quantiser of paper Sec. 2 "Compressed
 * Communication" in its general shape): the range is [lo, hi] = [min, max] of the values, L = 2^bits - 1,
 *     scale = fl32(hi - lo) / L;  q = clamp(rint(fl32(delta - lo) / scale), 0, L), 0 if scale = 0
 *     code = q;  dequantised value = fl32(fl32((float)q * scale) + lo);  lo goes to offsets.
 * Scope (quant_per_matrix = 1; the paper's global variant): one range per matrix instead of
 * one per row; scales[k] and offsets[k] then hold count entries, and the call makes one more
 * pass over the deltas to find the ranges.
 *
 * Error feedback (paper Sec. 2 "Compressed Communication"; Algorithm 2, EF branch), with
 * error_feedback = 1 and one fp32 residual E_k per worker, also fixed in fp32:
 *     e   = fl32(fl32(ef_beta * E_k) + delta)      (product, then sum; not fused)
 *     the row of e is quantised as above and its dequantised values are what is averaged
 *     E_k <- fl32(e - (float)q * scale)
 * It needs a compressor: error_feedback = 1 with quant_bits = 0 is MLC_ERR_ARG.
 *
 * Second quantisation (paper Sec. 2 "Collectives": one dequantise-reduce-quantise between
 * the all-to-all reduce-scatter and the all-gather), with second_quantisation = 1: the mean
 *     Psi = fl32(((s_1 + s_2) + ... + s_K) * fl32(1 / K)),  s_k the dequantised values, fp32
 * is quantised row-wise again with the same bit width, and eq. 3 uses its dequantised
 * value.  Its codes and scales are written to mean_codes / mean_scales when these are not
 * NULL.  Rows longer than 24576 or not a multiple of 8 are MLC_ERR_UNSUPPORTED, and so are
 * the pair of fp32 workers with a bf16 global copy and the per-matrix scope.
 * A "fragment" for streaming synchronisation is simply a call with a subset of groups.
 */
typedef struct {
  int64_t count, m, n;           /* rows for the quantiser: count * m rows of length n */
  void* const* worker_params;    /* HOST array of K device pointers theta_k; read, and
                                    written when write_back = 1                        */
  int worker_dtype;              /* mlc_dtype                                          */
  void* global_param;            /* theta_g, in/out                                    */
  int global_dtype;              /* mlc_dtype                                          */
  float* outer_momentum;         /* u, fp32, in/out                                    */
  uint8_t* const* codes;         /* HOST array of K device pointers, each
                                    [count*m][n*bits/8] packed codes; needed iff
                                    quant_bits                                         */
  float* const* scales;          /* HOST array of K device pointers, each [count*m]
                                    ([count] with quant_per_matrix)                    */
  float* const* residuals;       /* HOST array of K device pointers E_k, fp32
                                    [count][m][n], in/out; needed iff error_feedback   */
  uint8_t* mean_codes;           /* device, [count*m][n*bits/8], or NULL: codes of the
                                    second quantisation                                */
  float* mean_scales;            /* device, [count*m], or NULL                         */
  float* const* offsets;         /* HOST array of K device pointers like scales: lower
                                    ends of the ranges; needed iff quant_offset        */
  float* mean_offsets;           /* device, [count*m], or NULL (second quantisation in
                                    the offset form)                                   */
} mlc_outer_group;

typedef struct {
  int K;                 /* number of worker replicas, 1..MLC_MAX_WORKERS              */
  float eta_out;         /* outer learning rate                                        */
  float mu;              /* outer momentum                                             */
  int nesterov;          /* 1: eq. 3 as printed ; 0: theta_g <- theta_g - u            */
  int quant_bits;        /* 0: exchange fp32 deltas ; 2, 4, 8: row-wise linear codes   */
  int write_back;        /* 1: copy the new theta_g into every worker replica          */
  int error_feedback;    /* 1: compress beta E + Delta and keep what was not sent      */
  float ef_beta;         /* decay of the residual (1 = keep all of it)                 */
  int second_quantisation; /* 1: quantise the mean again before the outer update       */
  int quant_offset;      /* 1: range [min, max] with an offset instead of [-amax, amax] */
  int quant_per_matrix;  /* 1: one range per matrix instead of one per row             */
} mlc_outer_hparams;

/* Needs no work space.  With quant_bits != 0 it first writes codes/scales (and with
 * error feedback the residuals), exactly what muloco_quantize_delta writes, and then
 * consumes them. */
int muloco_outer_step(const mlc_outer_group* groups, int n_groups,
                      const mlc_outer_hparams* hp, void* stream);

/* Only the compressor: fills codes[k] and scales[k] for every worker and, with error
 * feedback, updates the residuals; nothing else is written.  hp->quant_bits must be 2, 4
 * or 8. */
int muloco_quantize_delta(const mlc_outer_group* groups, int n_groups,
                          const mlc_outer_hparams* hp, void* stream);

/* ------------------------------------------------------------------------------------
 * Outer step with top-k sparsification of the pseudogradients (paper Sec. 2 "Compressed
 * Communication": the k% entries of a weight matrix with the largest magnitude are kept,
 * the rest set to zero; sparsified once per worker, then averaged).
 *
 * For every worker k and every matrix [m][n] of a group, with N = m * n:
 *     v     = Delta_k, or with error feedback fl32(fl32(ef_beta * E_k) + Delta_k)
 *     kept  = ceil(fraction * N) (in double), at least 1, at most N
 *     tau   = the kept-th largest |v| of the matrix
 *     sent  = v where |v| >= tau, else 0      (entries that tie with tau are all kept)
 *     E_k  <- v - sent                        (error feedback only)
 * and the outer update of muloco_outer_step runs on the mean of the K sent tensors.
 * hp->quant_bits must be 0.  If groups[i].scales is not NULL it receives tau: K device
 * pointers to [count] floats.  workspace: device memory, 16-byte aligned, at least
 * muloco_topk_workspace_bytes(groups, n_groups, hp->K) bytes; its contents need not be
 * initialised and are not needed afterwards.
 */
size_t muloco_topk_workspace_bytes(const mlc_outer_group* groups, int n_groups, int K);
int muloco_topk_outer_step(const mlc_outer_group* groups, int n_groups, const mlc_outer_hparams* hp,
                           double fraction, void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------
 * AdamW step for the parameters Muon does not cover: embeddings, norms, biases (paper
 * Sec. 4, "AdamW inner updates and induced pseudogradient"; Sec. 2 "Muon" applies Muon to
 * the hidden matrices only).  Per element, in fp32:
 *     m     <- beta1 * m + (1 - beta1) * g
 *     v     <- beta2 * v + (1 - beta2) * g * g
 *     theta <- theta - lr * m^ / (sqrt(v^) + eps) - lr * weight_decay * theta
 * with m^ = m, v^ = v as printed, or m^ = m / (1 - beta1^step), v^ = v / (1 - beta2^step)
 * when bias_correction = 1 (step counts from 1).  Tensors are flat; every pointer is a
 * device pointer aligned to 16 bytes; m and v are fp32 and updated in place.
 */
typedef struct {
  int64_t count;          /* number of elements                                        */
  void* param;            /* theta, in/out                                             */
  int param_dtype;        /* mlc_dtype                                                 */
  const void* grad;       /* g                                                         */
  int grad_dtype;         /* mlc_dtype                                                 */
  float* exp_avg;         /* m, in/out                                                 */
  float* exp_avg_sq;      /* v, in/out                                                 */
} mlc_adamw_group;

typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  int bias_correction;    /* 0: as printed ; 1: divide by 1 - beta^step                 */
  int step;               /* 1-based step count, used only with bias_correction        */
} mlc_adamw_hparams;

int muloco_adamw_step(const mlc_adamw_group* groups, int n_groups, const mlc_adamw_hparams* hp,
                      void* stream);

/* ------------------------------------------------------------------------------------
 * Optional timing recorder (for benchmarks; not part of the method).
 *
 * While enabled, every kernel launch of this library is bracketed by HIP events on the
 * stream it is launched on.  muloco_timing_read waits for the recorded events, adds
 * each launch's duration to its kernel family and clears the record.  Enabling creates
 * HIP events (host-side objects); it never allocates device memory.
 */
enum {
  MLC_KERNEL_NS_GEMM = 0,     /* batched bf16 MFMA product of Newton-Schulz            */
  MLC_KERNEL_MOMENTUM = 1,    /* momentum + look-ahead + sum of squares                */
  MLC_KERNEL_NORM = 2,        /* per-matrix 1 / (norm + eps)                           */
  MLC_KERNEL_UPDATE = 3,      /* parameter update                                      */
  MLC_KERNEL_OUTER = 4,       /* fused pseudogradient / average / outer update         */
  MLC_KERNEL_QUANTIZE = 5,    /* row-wise quantiser (stand-alone compressor)           */
  MLC_KERNEL_DEQUANT_OUTER = 6,/* (quantise +) dequantise + average + outer update     */
  MLC_KERNEL_CONVERT = 7,     /* layout / dtype conversion around newton_schulz        */
  MLC_KERNEL_ADAMW = 8,       /* AdamW step of the non-matrix parameters               */
  MLC_KERNEL_TOPK = 9,        /* top-k selection passes + sparsified outer update      */
  MLC_KERNEL_FAMILIES = 10
};
typedef struct {
  int64_t launches;      /* launches recorded since the last read                      */
  double total_ms;       /* sum of their durations                                     */
  double flops;          /* matrix-core FLOP executed by those launches (0 if n/a)     */
  double bytes;          /* algorithmic HBM bytes of those launches (0 if n/a)         */
} mlc_kernel_timing;

int muloco_timing_enable(int on);
/* out: HOST array of MLC_KERNEL_FAMILIES entries.  Synchronises with recorded events. */
int muloco_timing_read(mlc_kernel_timing* out);

#ifdef __cplusplus
}
#endif
#endif /* MULOCO_H_ */
