/*
 * fp4_linear.h -- C ABI of the FP4 (E2M1) quantized linear layer for MI355X (gfx950).
 *
 * The library implements the hot path of FP4 training as described in
 * arXiv 2501.17116: for a linear layer Y = A W with A [M x K] (tokens x input
 * channels) and W [K x N] (input x output channels), both operands are absmax-scaled
 * along their non-contracted axis, rounded to the 16-value E2M1 grid, multiplied on
 * the FP4 matrix cores and the two scale vectors divided back out (Sec. 2 Eq. 1;
 * Fig. 2; Sec. 4.1; App. C.2).  Activations are first clamped at per-tensor quantile
 * thresholds and the clamped-away part is added back through a sparse high-precision
 * product (Sec. 3.2).  The weight gradient is multiplied element-wise by the capped
 * derivative of the differentiable quantization surrogate (Sec. 3.1 Eq. 8).
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller unless a parameter
 *     says "host".  Matrices are row-major.  The library allocates no memory, keeps no
 *     state between calls and never synchronizes: every call only enqueues kernels on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream), and on no
 *     other stream, so every entry point may be called while `stream` is being captured
 *     into a graph.
 *   - Return value: FP4_OK (0) or a negative fp4_status.  Arguments are validated on
 *     the host before anything is enqueued; on error nothing has been enqueued, except
 *     FP4_ERR_HIP which reports a failed launch of the call's own kernels.
 *   - Inputs must be finite.  Tensor base pointers must be 16-byte aligned and leading
 *     dimensions (in elements) multiples of 8.
 *   - Packed FP4 tensors ("codes"): two 4-bit codes per byte along the contracted axis,
 *     element 2t in bits 3:0 and element 2t+1 in bits 7:4, rows densely packed
 *     (cols/2 bytes per row).  Code = sign, 2 exponent bits, 1 mantissa bit (App. A
 *     table): 0..7 -> 0, .5, 1, 1.5, 2, 3, 4, 6; 8..15 the negatives; 1000 is never
 *     produced.
 *   - Rounding to the grid follows the comparison chain printed in App. A: nearest
 *     value, a midpoint goes to its upper neighbour (towards +inf) for either sign,
 *     magnitudes above 6 saturate.
 *   - Scales are multiplicative, gamma = fl32(6 / absmax) (Eq. 1); gamma = 1 for an
 *     all-zero vector or when 6/absmax is not finite.  The scaled value is the single
 *     fp32 product x * gamma.
 *   - Every GEMM contracts over an axis whose length is a multiple of 32.
 *   - Workspaces: query with fp4_workspace_bytes(); contents on entry are ignored and
 *     on exit undefined.  Two calls may share a workspace only if stream order
 *     serializes them.  The query does not know alpha: it provides for residual
 *     densities up to 20 %, i.e. alpha >= 0.9 (the paper uses 0.97 .. 0.999, Sec. 4.3).
 *     An alpha in (0.5, 0.9) is refused with FP4_ERR_ARG; outside (0.5, 1] likewise.
 *   - Residual capacity: the library never writes beyond `capacity` entries and never
 *     uses more than the workspaces provide for, whatever larger capacity is passed.
 */
#ifndef FP4_LINEAR_H
#define FP4_LINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FP4_OK = 0,
  FP4_ERR_NULL = -1,      /* a required pointer is NULL                                   */
  FP4_ERR_SHAPE = -2,     /* a dimension <= 0 where not allowed, odd packed length,
                             contraction length not a multiple of 32, ld too small        */
  FP4_ERR_DTYPE = -3,     /* unknown fp4_dtype / fp4_axis / op                            */
  FP4_ERR_ARG = -4,       /* alpha outside [0.9, 1] (see below), dge_cap <= 0, misaligned
                             pointer                                                      */
  FP4_ERR_WORKSPACE = -5, /* workspace NULL or smaller than fp4_workspace_bytes()         */
  FP4_ERR_CAPACITY = -6,  /* residual buffers smaller than 2*floor((1-alpha)*rows*cols)   */
  FP4_ERR_HIP = -7,       /* a kernel launch failed (hipGetLastError)                     */
  FP4_ERR_LIMIT = -8      /* problem larger than the built-in scratch of an entry point
                             that allocates nothing                                       */
} fp4_status;

typedef enum { FP4_F32 = 0, FP4_BF16 = 1 } fp4_dtype;

/* Operand formats of the mixed-format ablations (Sec. 4.3): E2M1 as above; E4M3 = the OCP FP8
 * format (bias 7, largest magnitude 448, no infinities), one code per byte, rounded to nearest
 * with ties to even, sign kept, saturating, scaled with gamma = fl32(448 / absmax). */
typedef enum { FP4_FMT_E2M1 = 0, FP4_FMT_E4M3 = 1 } fp4_format;

typedef enum {
  FP4_AXIS_ROW = 0,   /* one scale per row;    codes [rows x cols/2], cols contiguous       */
  FP4_AXIS_COL = 1,   /* one scale per column; codes TRANSPOSED [cols x rows/2]             */
  FP4_AXIS_TENSOR = 2 /* one scale for the whole tensor (the coarse granularity of the Sec. 4.3
                         ablation; App. C.2 with a scalar sf): codes as ROW, gamma [1]        */
} fp4_axis;

/* Scope of the clamp thresholds of Sec. 3.2 (the paper does not name the axis of the quantile):
 * TENSOR: one {lo, hi} pair for the whole activation operand (the default reading);
 * TOKEN:  one pair per token (row), each the order statistics of that row alone with
 *         k = floor((1-alpha)*cols) elements allowed per tail; rows of at most 16384 elements. */
typedef enum { FP4_OCC_TENSOR = 0, FP4_OCC_TOKEN = 1 } fp4_occ_scope;

typedef enum {
  FP4_OP_QUANTIZE = 0, /* (M=rows, K=cols, N ignored)                                     */
  FP4_OP_OCC = 1,      /* (M=rows, K=cols, N ignored)                                     */
  FP4_OP_FWD = 2,
  FP4_OP_DGRAD = 3,
  FP4_OP_WGRAD = 4,
  FP4_OP_SPMM = 5,     /* (M=P rows of S, K=Q, N)                                        */
  FP4_OP_PREPARE = 6,  /* fp4_prepare_weights (M ignored)                                 */
  FP4_OP_FWD_MIXED = 7,/* fp4_linear_fwd_mixed                                            */
  FP4_OP_BWD = 8       /* fp4_linear_bwd                                                  */
} fp4_op;

/* What the forward pass leaves for the weight-gradient pass (Sec. 3.1 needs the
 * forward's per-output-channel scales for f'(W_scaled); Sec. 3.2 needs the thresholds
 * and the residual).  All members are caller-allocated device buffers. */
typedef struct {
  float*   gamma_W;    /* [N]   forward scales of W, one per output channel               */
  float*   thresholds; /* [2]   {lo, hi}; {-inf, +inf} when alpha == 1.  scope TOKEN:
                          [2 M] {lo_i, hi_i} of every token                               */
  int64_t* row_ptr;    /* [M+1] CSR of Delta_A = A - clamp(A): row starts                 */
  int32_t* col_idx;    /* [capacity] column of each entry, ascending inside a row         */
  float*   val;        /* [capacity] fl32(A[i,c] - threshold)                             */
  int64_t  capacity;   /* entries available; >= 2*floor((1-alpha)*M*K)                    */
  int64_t* nnz;        /* [1]   number of entries                                         */
  int32_t  scope;      /* fp4_occ_scope, set by the caller before the forward pass; with
                          TOKEN capacity >= fp4_occ_capacity_token(M, K, alpha) suffices   */
} fp4_fwd_ctx;

const char* fp4_status_string(int status);

/* Bytes of device workspace an operation needs for the given problem. 0 for a bad op. */
size_t fp4_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, fp4_dtype dt);

/* Entries the residual buffers must hold: 2*floor((1-alpha)*rows*cols) (Sec. 3.2; the
 * density 2(1-alpha) is stated in App. B). */
int64_t fp4_occ_capacity(int64_t rows, int64_t cols, double alpha);

/* Vector-wise absmax quantization (Sec. 2 Eq. 1; Sec. 4.1: token-wise for A,
 * channel-wise for W).
 *   x      [rows x cols] of dtype dt, leading dimension ld (elements)
 *   axis   ROW: gamma[rows], codes [rows x cols/2]   (cols must be even)
 *          COL: gamma[cols], codes [cols x rows/2]   (rows must be even)
 *   rows or cols == 0 is allowed and does nothing. */
int fp4_quantize(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                 fp4_axis axis, uint8_t* codes, float* gamma,
                 void* workspace, size_t workspace_bytes, void* stream);

/* fp4_quantize for callers that cannot allocate or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * bit for bit, no workspace: the column-wise path keeps its partial column maxima in a
 * file-scope device array of FP4_NOALLOC_SCRATCH_BYTES (one copy per GPU the library runs on,
 * held until the process ends), which bounds the problem: ceil(rows/128) * cols * 4 bytes must
 * fit, else FP4_ERR_LIMIT and nothing is enqueued (16384 x 12288 needs 6 MiB).  The row-wise
 * path needs no scratch and has no limit.  The call allocates nothing and frees nothing; its
 * first call on a device looks up the array's address (not a stream operation: make that call
 * outside a capture).  All calls on one GPU share the array: calls that may overlap there --
 * different streams without an ordering between them -- race; stream order is enough. */
#define FP4_NOALLOC_SCRATCH_BYTES (8u << 20)
int fp4_quantize_noalloc(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                         fp4_axis axis, uint8_t* codes, float* gamma, void* stream);

/* Outlier clamping and compensation on one tensor (Sec. 3.2).
 *   thresholds (out, [2]): lo = v[k], hi = v[n-1-k] of the ascending-sorted values,
 *       k = floor((1-alpha)*rows*cols) evaluated in double, no interpolation.
 *   x_clamped (optional out, dtype dt, leading dimension ld): clamp(x, lo, hi).
 *   codes/gamma (optional out, both or neither): row-wise quantization of the clamped
 *       tensor, as fp4_quantize(axis = ROW) would produce from x_clamped.
 *   row_ptr/col_idx/val/nnz (out): CSR of x - x_clamped; an entry exists exactly where
 *       x < lo or x > hi, val = fl32(x - threshold).  capacity as in fp4_occ_capacity. */
int occ_clamp_residual(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                       double alpha, float* thresholds, uint8_t* codes, float* gamma,
                       void* x_clamped, int64_t* row_ptr, int32_t* col_idx, float* val,
                       int64_t capacity, int64_t* nnz,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The same with per-token thresholds (FP4_OCC_TOKEN): thresholds (out, [2 rows]) = {lo_i, hi_i},
 * the (k+1)-th smallest and (k+1)-th largest element of row i, k = floor((1-alpha)*cols); every
 * row holds at most 2k entries, exactly 2k when no element ties with a threshold.  The tensor is
 * read once.  cols <= 16384.  capacity >= fp4_occ_capacity_token(rows, cols, alpha) = rows * 2k.
 * Workspace as occ_clamp_residual. */
int64_t fp4_occ_capacity_token(int64_t rows, int64_t cols, double alpha);
int occ_clamp_residual_token(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                             double alpha, float* thresholds, uint8_t* codes, float* gamma,
                             void* x_clamped, int64_t* row_ptr, int32_t* col_idx, float* val,
                             int64_t capacity, int64_t* nnz,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Forward: Y = dequant(Q(A_c) Q(W)) + Delta_A W   (Fig. 2; Sec. 3.2; App. C.2).
 *   A [M x K], W [K x N], Y [M x N], all dtype dt, dense (ld = row length).
 *   A_c = A clamped at the alpha / 1-alpha order statistics of the whole tensor and
 *   quantized per token; W quantized per output channel; the residual product uses the
 *   unquantized W with fp32 accumulation and is added before the single rounding of Y.
 *   alpha == 1 switches OCC off.  `saved` is filled for fp4_linear_bwd_wgrad; saved->scope
 *   selects per-tensor (default) or per-token thresholds. */
int fp4_linear_fwd(const void* A, const void* W, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
                   double alpha, void* Y, const fp4_fwd_ctx* saved,
                   void* workspace, size_t workspace_bytes, void* stream);

/* The two quantizations of W that a training step needs (Sec. 4.1: scales live on the
 * non-contracted axis of each GEMM, so the forward pass and the activation gradient each need
 * their own).  W only changes at an optimizer step: with several micro-batches per step the
 * caller prepares them once per weight version and passes them to the *_cached entry points,
 * which then launch no quantization of W.  All members are caller-allocated device buffers. */
typedef struct {
  uint8_t* qWt;      /* [N x K/2] codes per output channel, transposed: forward's right operand */
  float*   gamma_W;  /* [N]       their scales (the ones the DGE factor uses)                   */
  uint8_t* qWk;      /* [K x N/2] codes per input channel: the activation gradient's operand    */
  float*   gamma_Wk; /* [K]       their scales                                                  */
} fp4_weight_cache;

/* Fills *wq from W [K x N] (K, N multiples of 32).  Bit-identical to what fp4_linear_fwd and
 * fp4_linear_bwd_dgrad compute internally.  Workspace: fp4_workspace_bytes(FP4_OP_PREPARE, 0, K, N, dt). */
int fp4_prepare_weights(const void* W, fp4_dtype dt, int64_t K, int64_t N, const fp4_weight_cache* wq,
                        void* workspace, size_t workspace_bytes, void* stream);

/* fp4_linear_fwd / fp4_linear_bwd_dgrad with W's quantizations taken from *wq (read only).  The
 * forward still needs the unquantized W for the residual product.  saved->gamma_W receives a copy of
 * wq->gamma_W unless it is the same pointer.  Workspaces as for the plain entry points. */
int fp4_linear_fwd_cached(const void* A, const void* W, const fp4_weight_cache* wq, fp4_dtype dt,
                          int64_t M, int64_t K, int64_t N, double alpha, void* Y, const fp4_fwd_ctx* saved,
                          void* workspace, size_t workspace_bytes, void* stream);
int fp4_linear_bwd_dgrad_cached(const void* dY, const fp4_weight_cache* wq, fp4_dtype dt,
                                int64_t M, int64_t K, int64_t N, void* dA,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Activation gradient: dA = dY W^T as an FP4 GEMM contracting over output channels,
 * dY scaled per token and W per input channel (scales on the non-contracted axes,
 * Sec. 4.1).  dY [M x N], W [K x N], dA [M x K], dtype dt.  No DGE term (Sec. 3). */
int fp4_linear_bwd_dgrad(const void* dY, const void* W, fp4_dtype dt,
                         int64_t M, int64_t K, int64_t N, void* dA,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Weight gradient: dW = (A^T dY) (.) min(dge_cap, f'(W gamma_W))
 * (Sec. 3.1 Eq. 3-6 and 8; App. C.2 Eq. 22).  A^T dY is an FP4 GEMM contracting over
 * tokens: A clamped at saved->thresholds and scaled per input channel, dY scaled per
 * output channel, plus Delta_A^T dY from the saved residual in fp32.  f' uses the
 * forward's saved->gamma_W.  dge_k <= 0 selects the straight-through estimator (f' = 1).
 * dW is fp32 [K x N], overwritten. */
int fp4_linear_bwd_wgrad(const void* A, const void* dY, const void* W, fp4_dtype dt,
                         int64_t M, int64_t K, int64_t N, const fp4_fwd_ctx* saved,
                         float dge_k, float dge_cap, float* dW,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Both gradients in one call, bit-identical to fp4_linear_bwd_dgrad followed by
 * fp4_linear_bwd_wgrad.  The axis rule of Sec. 4.1 makes dY's scales per token in one GEMM and per
 * output channel in the other; here dY is read once for its row-wise codes and the column maxima
 * together (bf16 masters, N <= 16384; other cases run the two passes), so the column-wise
 * quantization that follows needs no absmax pass.  wq: optional cache of W's quantizations (NULL:
 * W is quantized per input channel here).  M, N multiples of 32, K of 8.
 * Workspace: fp4_workspace_bytes(FP4_OP_BWD, M, K, N, dt). */
int fp4_linear_bwd(const void* dY, const void* A, const void* W, const fp4_weight_cache* wq, fp4_dtype dt,
                   int64_t M, int64_t K, int64_t N, const fp4_fwd_ctx* saved, float dge_k, float dge_cap,
                   void* dA, float* dW, void* workspace, size_t workspace_bytes, void* stream);

/* ---- building blocks, exported for parity tests and per-kernel measurement ---- */

/* out[P x Q] = (codes_l[P x Kc/2] . codes_rt[Q x Kc/2]^T) / (gamma_l[p] gamma_r[q]) (+ addend),
 * the FP4 GEMM with scale dequantization (Fig. 2).  gamma_l / gamma_r NULL = raw fp32
 * accumulator (then out must be fp32).  addend: optional fp32 [P x Q] (same ld as out)
 * added before rounding; may alias out when out is fp32. */
int fp4_gemm(const uint8_t* codes_l, const float* gamma_l, const uint8_t* codes_rt,
             const float* gamma_r, int64_t P, int64_t Q, int64_t Kc,
             const float* addend, void* out, fp4_dtype out_dt, int64_t ldo, void* stream);

/* ---- mixed formats: W4A8 / W8A4 (Sec. 4.3) ----
 * fp8_quantize: as fp4_quantize with E4M3 codes, one per byte: ROW: codes [rows x cols];
 *   COL: codes TRANSPOSED [cols x rows].  Workspace as fp4_quantize (COL only).
 * fp4_gemm_mixed: as fp4_gemm with exactly one operand in E4M3 ([rows x Kc] bytes) and the other
 *   in E2M1 ([rows x Kc/2] bytes); Kc a multiple of 128.  The fp32 accumulator of a mixed product is
 *   not exact (products are multiples of 2^-10 up to 2688), so results are compared under the
 *   tolerance of the scaled outputs.
 * fp4_linear_fwd_mixed: the forward pass with one operand in 8 bits.  act_fmt = E4M3, wgt_fmt =
 *   E2M1 (W4A8): activations E4M3 per token, no clamp (alpha must be 1), weights E2M1 per output
 *   channel.  act_fmt = E2M1, wgt_fmt = E4M3 (W8A4): activations E2M1 per token with the clamp and
 *   residual of Sec. 3.2, weights E4M3 per output channel.  saved as in fp4_linear_fwd (gamma_W
 *   then holds the 8-bit scales in the W8A4 case).  K a multiple of 128.  Workspace:
 *   fp4_workspace_bytes(FP4_OP_FWD_MIXED, M, K, N, dt).  The backward passes stay FP4. */
int fp8_quantize(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld, fp4_axis axis,
                 uint8_t* codes, float* gamma, void* workspace, size_t workspace_bytes, void* stream);
int fp4_gemm_mixed(const uint8_t* codes_l, fp4_format fmt_l, const float* gamma_l,
                   const uint8_t* codes_rt, fp4_format fmt_r, const float* gamma_r,
                   int64_t P, int64_t Q, int64_t Kc, const float* addend, void* out, fp4_dtype out_dt,
                   int64_t ldo, void* stream);
int fp4_linear_fwd_mixed(const void* A, const void* W, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
                         fp4_format act_fmt, fp4_format wgt_fmt, double alpha, void* Y,
                         const fp4_fwd_ctx* saved, void* workspace, size_t workspace_bytes, void* stream);

/* ---- granularity: tensor-wise scaling (Sec. 4.3 "Granularity") ----
 * fp4_linear_fwd with the scale of the activations and / or of the weights taken over the whole tensor
 * instead of per token / per output channel (fp4_quantize offers the same as FP4_AXIS_TENSOR):
 * gamma_A = 6 / max|A_c| over the clamped activation tensor, gamma_W = 6 / max|W|.  Clamp, residual and
 * everything else as in fp4_linear_fwd with per-tensor thresholds (a per-token saved->scope together with
 * act_tensorwise is refused with FP4_ERR_ARG).  saved->gamma_W receives the scales used, N copies of the
 * scalar when wgt_tensorwise.  Workspace: fp4_workspace_bytes(FP4_OP_FWD, M, K, N, dt).  The backward
 * passes stay vector-wise. */
int fp4_linear_fwd_granularity(const void* A, const void* W, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
                               int act_tensorwise, int wgt_tensorwise, double alpha, void* Y,
                               const fp4_fwd_ctx* saved, void* workspace, size_t workspace_bytes, void* stream);

/* One 4-bit code per output byte (for inspecting packed tensors). */
int fp4_unpack(const uint8_t* codes, int64_t rows, int64_t cols, uint8_t* one_per_byte,
               void* stream);

/* dW[k, n] = G[k, n] * min(cap, f'(W[k, n] * gamma_W[n])): the DGE factor as a
 * stand-alone pass (Sec. 3.1 Eq. 8).  G and dW fp32 [K x N] (may alias), W dtype dt. */
int fp4_dge_apply(const float* G, const void* W, fp4_dtype dt, const float* gamma_W,
                  int64_t K, int64_t N, float dge_k, float dge_cap, float* dW, void* stream);

/* R[P x N] (fp32, overwritten) = S D with S a P x Q CSR matrix (fp32 values) and D
 * [Q x N] dense of dtype dt: the high-precision sparse product of Sec. 3.2.  Column indices
 * must ascend inside a row.  Workspace: fp4_workspace_bytes(FP4_OP_SPMM, P, Q, N, dt). */
int fp4_residual_spmm(const int64_t* row_ptr, const int32_t* col_idx, const float* val,
                      int64_t P, int64_t Q, const void* D, fp4_dtype dt, int64_t N,
                      float* R, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FP4_LINEAR_H */
