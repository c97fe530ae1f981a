// Host side of the C ABI: argument validation, workspace carving and the kernel sequences of
// the three layer passes (Fig. 2; Sec. 3.1; Sec. 3.2; Sec. 4.1).  Nothing here allocates device
// memory or synchronizes; every buffer is the caller's, every kernel goes to the caller's stream,
// and the library keeps no state between calls.
#include "fp4_common.h"

#include <algorithm>
#include <cmath>
#include <limits>

// launchers defined next to their kernels
int fp4_launch_gemm(const uint8_t* L, const float* gl, const uint8_t* Rt, const float* gr, int64_t P,
                    int64_t Q, int64_t Kc, const float* addend, void* out, int out_bf16, int64_t ldo,
                    const void* W, int w_bf16, int64_t ldw, const float* gamma_w, float dge_k,
                    float dge_cap, hipStream_t stream);
int fp4_launch_quantize_rows(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld,
                             uint8_t* codes, float* gamma, hipStream_t s);
int fp4_launch_occ_count(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, const float* thr,
                         int32_t* row_cnt, hipStream_t s);
int fp4_launch_occ_rows(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, const float* thr,
                        uint8_t* codes, float* gamma, void* x_clamped, int32_t* col_idx, float* val,
                        int32_t* tmp_col, float* tmp_val, const int64_t* row_ptr, int64_t capacity, const float* gamma_in,
                        hipStream_t s);
int64_t fp4_tensor_gamma_scratch_words();
int fp4_launch_tensor_gamma(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, const float* thr,
                            uint32_t* scratch, float* scalar, float* bcast, int64_t n, hipStream_t s);
int fp4_launch_quantize_rows_fixed(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, const float* gamma_in,
                                   uint8_t* codes, float* gamma, hipStream_t s);
int fp4_launch_quantize_cols_given_gamma(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld,
                                         uint8_t* codes_t, float* gamma, hipStream_t s);
int fp4_launch_quantize_cols(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld,
                             const float* clamp_thr, int per_row_thr, uint8_t* codes_t, float* gamma,
                             uint32_t* amax_scratch, hipStream_t s);
int fp4_launch_occ_rows_token(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, int64_t tail_k,
                              float* thr_out, uint8_t* codes, float* gamma, void* x_clamped, int32_t* tmp_col,
                              float* tmp_val, int32_t* row_cnt, hipStream_t s);
int64_t fp4_dual_axis_part_elems(int64_t rows, int64_t cols);
int fp4_launch_quantize_rows_colmax(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, uint8_t* codes,
                                    float* gamma, uint16_t* part, hipStream_t s);
int fp4_launch_quantize_cols_known_max(const void* x, int64_t rows, int64_t cols, int64_t ld, const uint16_t* part,
                                       uint8_t* codes_t, float* gamma, hipStream_t s);
int fp4_launch_compact_rows(const int32_t* tmp_col, const float* tmp_val, const int32_t* row_cnt, int64_t stride,
                            const int64_t* row_ptr, int64_t rows, int64_t capacity, int32_t* col_idx, float* val,
                            hipStream_t s);
int64_t fp4_quantize_cols_scratch_words(int64_t rows, int64_t cols);
size_t fp4_select_scratch_bytes();
int fp4_launch_thresholds(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, int64_t k,
                          float* thresholds, void* scratch, unsigned long long* total, hipStream_t s);
int fp4_launch_scan_rows(const int32_t* row_cnt, int64_t rows, int64_t* row_ptr, int64_t* nnz, hipStream_t s);
int fp4_launch_csr_gather(const int32_t* tmp_col, const float* tmp_val, int64_t rows, int64_t capacity,
                          const int64_t* row_ptr, int32_t* col_idx, float* val, hipStream_t s);
int fp4_launch_csr_transpose(const int64_t* row_ptr, const int32_t* col_idx, const float* val,
                             const int64_t* nnz, int64_t P, int64_t Q, int64_t capacity, int64_t* t_ptr,
                             int32_t* t_idx, float* t_val, int32_t* u_idx, float* u_val, int32_t* scratch,
                             hipStream_t s);
int64_t fp4_spmm_long_list_cap(int64_t capacity);
int fp8_launch_quantize_rows(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, uint8_t* codes,
                             float* gamma, hipStream_t s);
int fp8_launch_quantize_cols(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, uint8_t* codes_t,
                             float* gamma, uint32_t* amax_scratch, hipStream_t s);
int fp4_launch_gemm_mixed(const uint8_t* L, const float* gl, const uint8_t* Rt, const float* gr, int l_fp8, int64_t P,
                          int64_t Q, int64_t Kc, const float* addend, void* out, int out_bf16, int64_t ldo,
                          hipStream_t stream);
int64_t fp4_csr_transpose_scratch_words(int64_t P, int64_t Q);
int fp4_launch_order_rows(const int64_t* row_ptr, int64_t rows, int64_t nidx, int64_t capacity,
                          const int32_t* u_idx, const float* u_val, int32_t* idx, float* val, hipStream_t s);
int64_t fp4_spmm_scratch_words(int64_t list_cap, int64_t Q, int64_t N);
int fp4_launch_spmm(const int64_t* row_ptr, const int32_t* col_idx, const float* val, int64_t capacity,
                    int64_t P, int64_t Q, const void* D, int bf16, int64_t N, float* R, int32_t* scratch,
                    int64_t list_cap, hipStream_t s);

namespace {

__global__ void init_no_occ_kernel(float* thr, int64_t* row_ptr, int64_t rows, int64_t* nnz) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (row_ptr && i <= rows) row_ptr[i] = 0;
  if (i == 0) {
    if (thr) { thr[0] = -INFINITY; thr[1] = INFINITY; }
    if (nnz) *nnz = 0;
  }
}

// Bump allocator over the caller's workspace; every block 256-byte aligned.
struct Carver {
  uint8_t* base;
  size_t off = 0;
  explicit Carver(void* p) : base(reinterpret_cast<uint8_t*>(p)) {}
  template <class T>
  T* take(size_t count) {
    T* r = reinterpret_cast<T*>(base ? base + off : nullptr);
    off += align_up(count * sizeof(T), 256);
    return r;
  }
};

inline bool dtype_ok(fp4_dtype dt) { return dt == FP4_F32 || dt == FP4_BF16; }
inline size_t esize(fp4_dtype dt) { return dt == FP4_BF16 ? 2 : 4; }

int64_t tail_count(int64_t n, double alpha) { return (int64_t)std::floor((1.0 - alpha) * (double)n); }
// Residual entries the workspaces provide for: the workspace query does not know alpha, so it
// sizes for alpha >= 0.9 (density up to 20 %); a smaller alpha is refused with FP4_ERR_ARG.
int64_t provisioned_entries(int64_t rows, int64_t cols) { return 2 * tail_count(rows * cols, 0.9); }

struct OccTemps {
  void* select;
  int32_t* tmp_col;
  float* tmp_val;
  int64_t* row_start;
  int32_t* row_cnt;
  unsigned long long* total;
};
OccTemps carve_occ(Carver& c, int64_t rows, int64_t capacity) {
  OccTemps t;
  t.select = c.take<uint8_t>(fp4_select_scratch_bytes());
  t.tmp_col = c.take<int32_t>((size_t)capacity);
  t.tmp_val = c.take<float>((size_t)capacity);
  t.row_start = c.take<int64_t>((size_t)rows);
  t.row_cnt = c.take<int32_t>((size_t)rows);
  t.total = c.take<unsigned long long>(1);
  return t;
}

struct FwdWs {
  uint8_t* qA; float* gA; uint8_t* qWt; uint32_t* amax; OccTemps occ; float* R; int32_t* sp_scratch;
  uint32_t* tg;   // tensor-wise scaling: partial maxima, then (at word TG_SCALAR) the scale itself
};
const int64_t TG_SCALAR = fp4_tensor_gamma_scratch_words() - 32;
FwdWs carve_fwd(Carver& c, int64_t M, int64_t K, int64_t N, fp4_dtype dt) {
  FwdWs w;
  w.qA = c.take<uint8_t>((size_t)(M * K / 2));
  w.gA = c.take<float>((size_t)M);
  w.qWt = c.take<uint8_t>((size_t)(N * K / 2));
  w.amax = c.take<uint32_t>((size_t)fp4_quantize_cols_scratch_words(K, N));
  // sized for the densest residual the entry points accept (alpha > 0.5 -> fewer than M*K entries);
  // the workspace query does not know alpha, so it provides for alpha >= 0.9
  w.occ = carve_occ(c, M, provisioned_entries(M, K));
  w.R = dt == FP4_BF16 ? c.take<float>((size_t)(M * N)) : nullptr;
  w.sp_scratch = c.take<int32_t>((size_t)fp4_spmm_scratch_words(fp4_spmm_long_list_cap(provisioned_entries(M, K)), K, N));
  w.tg = c.take<uint32_t>((size_t)fp4_tensor_gamma_scratch_words());
  return w;
}

// forward with one 8-bit operand: as FwdWs with room for one code per byte on either side
FwdWs carve_fwd_mixed(Carver& c, int64_t M, int64_t K, int64_t N, fp4_dtype dt) {
  FwdWs w;
  w.qA = c.take<uint8_t>((size_t)(M * K));
  w.gA = c.take<float>((size_t)M);
  w.qWt = c.take<uint8_t>((size_t)(N * K));
  w.amax = c.take<uint32_t>((size_t)fp4_quantize_cols_scratch_words(K, N));
  w.occ = carve_occ(c, M, provisioned_entries(M, K));
  w.R = dt == FP4_BF16 ? c.take<float>((size_t)(M * N)) : nullptr;
  w.sp_scratch = c.take<int32_t>((size_t)fp4_spmm_scratch_words(fp4_spmm_long_list_cap(provisioned_entries(M, K)), K, N));
  w.tg = nullptr;
  return w;
}

struct DgradWs { uint8_t* qdY; float* gdY; uint8_t* qW; float* gWk; };
DgradWs carve_dgrad(Carver& c, int64_t M, int64_t K, int64_t N) {
  DgradWs w;
  w.qdY = c.take<uint8_t>((size_t)(M * N / 2));
  w.gdY = c.take<float>((size_t)M);
  w.qW = c.take<uint8_t>((size_t)(K * N / 2));
  w.gWk = c.take<float>((size_t)K);
  return w;
}

struct WgradWs {
  uint8_t* qAt; float* gAk; uint8_t* qdYt; float* gdYn; uint32_t* amax;
  int64_t* t_ptr; int32_t* t_idx; float* t_val; int32_t* u_idx; float* u_val; int32_t* t_scratch;
  int32_t* sp_scratch;
};
WgradWs carve_wgrad(Carver& c, int64_t M, int64_t K, int64_t N) {
  WgradWs w;
  w.qAt = c.take<uint8_t>((size_t)(K * M / 2));
  w.gAk = c.take<float>((size_t)K);
  w.qdYt = c.take<uint8_t>((size_t)(N * M / 2));
  w.gdYn = c.take<float>((size_t)N);
  w.amax = c.take<uint32_t>((size_t)fp4_quantize_cols_scratch_words(M, std::max(K, N)));
  const int64_t cap = provisioned_entries(M, K);
  w.t_ptr = c.take<int64_t>((size_t)(K + 1));
  w.t_idx = c.take<int32_t>((size_t)cap);
  w.t_val = c.take<float>((size_t)cap);
  w.u_idx = c.take<int32_t>((size_t)cap);
  w.u_val = c.take<float>((size_t)cap);
  w.t_scratch = c.take<int32_t>((size_t)fp4_csr_transpose_scratch_words(M, K));
  w.sp_scratch = c.take<int32_t>((size_t)fp4_spmm_scratch_words(fp4_spmm_long_list_cap(cap), M, N));
  return w;
}

}  // namespace

extern "C" const char* fp4_status_string(int status) {
  switch (status) {
    case FP4_OK: return "ok";
    case FP4_ERR_NULL: return "null pointer";
    case FP4_ERR_SHAPE: return "bad shape";
    case FP4_ERR_DTYPE: return "bad dtype, axis or op";
    case FP4_ERR_ARG: return "bad argument";
    case FP4_ERR_WORKSPACE: return "workspace too small";
    case FP4_ERR_CAPACITY: return "residual capacity too small";
    case FP4_ERR_HIP: return "kernel launch failed";
    case FP4_ERR_LIMIT: return "problem exceeds the built-in scratch of the no-allocation entry point";
    default: return "unknown status";
  }
}

extern "C" int64_t fp4_occ_capacity(int64_t rows, int64_t cols, double alpha) {
  if (rows < 0 || cols < 0 || !(alpha > 0.5) || !(alpha <= 1.0)) return -1;
  return 2 * tail_count(rows * cols, alpha);
}

extern "C" size_t fp4_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, fp4_dtype dt) {
  if (M < 0 || K < 0 || N < 0 || !dtype_ok(dt)) return 0;
  Carver c(nullptr);
  switch (op) {
    case FP4_OP_QUANTIZE:   // partial column maxima, or the partial maxima of the tensor-wise scale
      c.take<uint32_t>((size_t)std::max(fp4_quantize_cols_scratch_words(M, K), fp4_tensor_gamma_scratch_words()));
      break;
    case FP4_OP_OCC: carve_occ(c, M, provisioned_entries(M, K)); break;
    case FP4_OP_FWD: carve_fwd(c, M, K, N, dt); break;
    case FP4_OP_DGRAD: carve_dgrad(c, M, K, N); break;
    case FP4_OP_WGRAD: carve_wgrad(c, M, K, N); break;
    case FP4_OP_PREPARE: c.take<uint32_t>((size_t)fp4_quantize_cols_scratch_words(K, N)); break;
    case FP4_OP_FWD_MIXED: carve_fwd_mixed(c, M, K, N, dt); break;
    case FP4_OP_BWD:
      carve_dgrad(c, M, K, N);
      carve_wgrad(c, M, K, N);
      c.take<uint16_t>((size_t)fp4_dual_axis_part_elems(M, N));
      break;
    case FP4_OP_SPMM: c.take<int32_t>((size_t)fp4_spmm_scratch_words(M + 2, K, N)); break;   // long-row list: at most M rows
    default: return 0;
  }
  return c.off + 256;
}

namespace {
constexpr int64_t TOKEN_MAX_COLS = 16384;   // a row must fit the registers of one workgroup

// The per-token chain: one fused pass (thresholds, clamp, codes, entries at a fixed stride per row),
// the scan of the rows' entry counts, and the compaction into CSR.
int occ_token_chain(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, int64_t k_row, float* thresholds,
                    uint8_t* codes, float* gamma, void* x_clamped, int64_t* row_ptr, int32_t* col_idx, float* val,
                    int64_t capacity, int64_t* nnz, const OccTemps& t, hipStream_t s) {
  int rc = fp4_launch_occ_rows_token(x, bf16, rows, cols, ld, k_row, thresholds, codes, gamma, x_clamped, t.tmp_col,
                                     t.tmp_val, t.row_cnt, s);
  if (rc) return rc;
  rc = fp4_launch_scan_rows(t.row_cnt, rows, row_ptr, nnz, s);
  if (rc) return rc;
  return fp4_launch_compact_rows(t.tmp_col, t.tmp_val, t.row_cnt, 2 * k_row, row_ptr, rows, capacity, col_idx, val, s);
}
}  // namespace

extern "C" int64_t fp4_occ_capacity_token(int64_t rows, int64_t cols, double alpha) {
  if (rows < 0 || cols < 0 || !(alpha > 0.5) || !(alpha <= 1.0)) return -1;
  return rows * 2 * tail_count(cols, alpha);
}

extern "C" int occ_clamp_residual_token(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                        double alpha, float* thresholds, uint8_t* codes, float* gamma,
                                        void* x_clamped, int64_t* row_ptr, int32_t* col_idx, float* val,
                                        int64_t capacity, int64_t* nnz, void* workspace, size_t workspace_bytes,
                                        void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (rows <= 0 || cols <= 0 || ld < cols || (cols & 1) || cols > TOKEN_MAX_COLS) return FP4_ERR_SHAPE;
  if (!(alpha > 0.5) || !(alpha <= 1.0)) return FP4_ERR_ARG;
  if (!x || !thresholds || !row_ptr || !nnz) return FP4_ERR_NULL;
  if ((codes == nullptr) != (gamma == nullptr)) return FP4_ERR_NULL;
  const int64_t k_row = tail_count(cols, alpha);
  if (2 * k_row >= cols) return FP4_ERR_ARG;
  if (capacity < rows * 2 * k_row) return FP4_ERR_CAPACITY;
  if (capacity > 0 && (!col_idx || !val)) return FP4_ERR_NULL;
  if (!aligned16(x) || (ld % 8) != 0 || (codes && !aligned16(codes)) || (x_clamped && !aligned16(x_clamped)))
    return FP4_ERR_ARG;
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_OCC, rows, cols, 0, dt)) return FP4_ERR_WORKSPACE;
  if (rows * 2 * k_row > provisioned_entries(rows, cols)) return FP4_ERR_ARG;  // alpha below 0.9 is not provisioned
  Carver c(reinterpret_cast<void*>(align_up((size_t)(uintptr_t)workspace, 256)));
  OccTemps t = carve_occ(c, rows, provisioned_entries(rows, cols));
  return occ_token_chain(x, dt == FP4_BF16, rows, cols, ld, k_row, thresholds, codes, gamma, x_clamped, row_ptr, col_idx,
                         val, capacity, nnz, t, (hipStream_t)stream);
}

extern "C" int occ_clamp_residual(const void* x, fp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                  double alpha, float* thresholds, uint8_t* codes, float* gamma,
                                  void* x_clamped, int64_t* row_ptr, int32_t* col_idx, float* val,
                                  int64_t capacity, int64_t* nnz, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (rows <= 0 || cols <= 0 || ld < cols || (cols & 1)) return FP4_ERR_SHAPE;
  if (!(alpha > 0.5) || !(alpha <= 1.0)) return FP4_ERR_ARG;
  if (!x || !thresholds || !row_ptr || !nnz) return FP4_ERR_NULL;
  if ((codes == nullptr) != (gamma == nullptr)) return FP4_ERR_NULL;
  const int64_t k = tail_count(rows * cols, alpha);
  if (capacity < 2 * k) return FP4_ERR_CAPACITY;
  if (capacity > 0 && (!col_idx || !val)) return FP4_ERR_NULL;
  if (!aligned16(x) || (ld % 8) != 0 || (codes && !aligned16(codes)) || (x_clamped && !aligned16(x_clamped)))
    return FP4_ERR_ARG;
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_OCC, rows, cols, 0, dt)) return FP4_ERR_WORKSPACE;
  if (2 * k > provisioned_entries(rows, cols)) return FP4_ERR_ARG;  // alpha below 0.9 is not provisioned
  hipStream_t s = (hipStream_t)stream;
  Carver c(reinterpret_cast<void*>(align_up((size_t)(uintptr_t)workspace, 256)));
  OccTemps t = carve_occ(c, rows, provisioned_entries(rows, cols));
  capacity = std::min(capacity, provisioned_entries(rows, cols));  // never beyond the temporaries
  int rc = fp4_launch_thresholds(x, dt == FP4_BF16, rows, cols, ld, k, thresholds, t.select, t.total, s);
  if (rc) return rc;
  rc = fp4_launch_occ_count(x, dt == FP4_BF16, rows, cols, ld, thresholds, t.row_cnt, s);
  if (rc) return rc;
  rc = fp4_launch_scan_rows(t.row_cnt, rows, row_ptr, nnz, s);
  if (rc) return rc;
  rc = fp4_launch_occ_rows(x, dt == FP4_BF16, rows, cols, ld, thresholds, codes, gamma, x_clamped, col_idx, val,
                           t.tmp_col, t.tmp_val, row_ptr, capacity, nullptr, s);
  if (rc == 1) {   // streamed rows: entries unordered in the temporaries
    rc = fp4_launch_order_rows(row_ptr, rows, cols, capacity, t.tmp_col, t.tmp_val, col_idx, val, s);
    if (rc == 1) rc = fp4_launch_csr_gather(t.tmp_col, t.tmp_val, rows, capacity, row_ptr, col_idx, val, s);
  }
  return rc;
}

namespace {
__global__ void copy_f32_kernel(const float* src, float* dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

bool cache_ok(const fp4_weight_cache* wq) {
  return wq && wq->qWt && wq->gamma_W && wq->qWk && wq->gamma_Wk && aligned16(wq->qWt) && aligned16(wq->qWk);
}

// Forward pass; wq == nullptr: W is quantized here, into the workspace and saved->gamma_W.
// act_tensor / wgt_tensor: one scale for the whole operand instead of one per token / output channel
// (granularity ablation); everything else, clamp and residual included, is the same path.
int fwd_impl(const void* A, const void* W, const fp4_weight_cache* wq, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
             double alpha, void* Y, const fp4_fwd_ctx* saved, void* workspace, size_t workspace_bytes, void* stream,
             bool act_tensor = false, bool wgt_tensor = false) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (M <= 0 || K <= 0 || N <= 0 || (K % 32) != 0 || (N % 8) != 0) return FP4_ERR_SHAPE;
  if (!(alpha > 0.5) || !(alpha <= 1.0)) return FP4_ERR_ARG;
  if (!A || !W || !Y || !saved || !saved->gamma_W) return FP4_ERR_NULL;
  if (!aligned16(A) || !aligned16(W) || !aligned16(Y)) return FP4_ERR_ARG;
  const bool occ = alpha < 1.0;
  if (saved->scope != FP4_OCC_TENSOR && saved->scope != FP4_OCC_TOKEN) return FP4_ERR_DTYPE;
  const bool token = occ && saved->scope == FP4_OCC_TOKEN;
  if (token && act_tensor) return FP4_ERR_ARG;      // one scale per tensor goes with the per-tensor clamp
  const int64_t k = tail_count(M * K, alpha);       // per tail of the tensor
  const int64_t k_row = tail_count(K, alpha);       // per tail of a token
  const int64_t need = token ? M * 2 * k_row : 2 * k;
  if (occ) {
    if (!saved->thresholds || !saved->row_ptr || !saved->nnz) return FP4_ERR_NULL;
    if (token && (K > TOKEN_MAX_COLS || 2 * k_row >= K)) return FP4_ERR_SHAPE;
    if (saved->capacity < need) return FP4_ERR_CAPACITY;
    if (saved->capacity > 0 && (!saved->col_idx || !saved->val)) return FP4_ERR_NULL;
    if (need > provisioned_entries(M, K)) return FP4_ERR_ARG;   // alpha below 0.9 is not provisioned
  }
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_FWD, M, K, N, dt)) return FP4_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int bf16 = dt == FP4_BF16;
  Carver c(reinterpret_cast<void*>(align_up((size_t)(uintptr_t)workspace, 256)));
  FwdWs w = carve_fwd(c, M, K, N, dt);

  // W per output channel -> codes [N x K/2], scales kept for the DGE term of the backward pass;
  // from the cache when the caller prepared one (W does not change between micro-batches)
  int rc = FP4_OK;
  const uint8_t* qWt = w.qWt;
  if (wq) {
    qWt = wq->qWt;
    if (saved->gamma_W != wq->gamma_W) {
      hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, s, wq->gamma_W, saved->gamma_W, N);
      if (hipGetLastError() != hipSuccess) return FP4_ERR_HIP;
    }
  } else if (wgt_tensor) {
    rc = fp4_launch_tensor_gamma(W, bf16, K, N, N, nullptr, w.tg, nullptr, saved->gamma_W, N, s);
    if (!rc) rc = fp4_launch_quantize_cols_given_gamma(W, bf16, K, N, N, w.qWt, saved->gamma_W, s);
    if (rc) return rc;
  } else {
    rc = fp4_launch_quantize_cols(W, bf16, K, N, N, nullptr, 0, w.qWt, saved->gamma_W, w.amax, s);
    if (rc) return rc;
  }
  const float* addend = nullptr;
  if (occ) {
    const int64_t cap = std::min(saved->capacity, provisioned_entries(M, K));  // never beyond the temporaries
    if (token) {
      rc = occ_token_chain(A, bf16, M, K, K, k_row, saved->thresholds, w.qA, w.gA, nullptr, saved->row_ptr,
                           saved->col_idx, saved->val, cap, saved->nnz, w.occ, s);
    } else {
      rc = fp4_launch_thresholds(A, bf16, M, K, K, k, saved->thresholds, w.occ.select, w.occ.total, s);
      if (rc) return rc;
      rc = fp4_launch_occ_count(A, bf16, M, K, K, saved->thresholds, w.occ.row_cnt, s);
      if (rc) return rc;
      rc = fp4_launch_scan_rows(w.occ.row_cnt, M, saved->row_ptr, saved->nnz, s);
      if (rc) return rc;
      const float* g_all = nullptr;   // tensor-wise activations: one scale, from the clamped tensor's absmax
      if (act_tensor) {
        rc = fp4_launch_tensor_gamma(A, bf16, M, K, K, saved->thresholds, w.tg, reinterpret_cast<float*>(w.tg + TG_SCALAR),
                                     nullptr, 0, s);
        if (rc) return rc;
        g_all = reinterpret_cast<const float*>(w.tg + TG_SCALAR);
      }
      rc = fp4_launch_occ_rows(A, bf16, M, K, K, saved->thresholds, w.qA, w.gA, nullptr, saved->col_idx, saved->val,
                               w.occ.tmp_col, w.occ.tmp_val, saved->row_ptr, cap, g_all, s);
      if (rc == 1) {   // streamed rows: entries unordered in the temporaries
        rc = fp4_launch_order_rows(saved->row_ptr, M, K, cap, w.occ.tmp_col, w.occ.tmp_val, saved->col_idx, saved->val, s);
        if (rc == 1)
          rc = fp4_launch_csr_gather(w.occ.tmp_col, w.occ.tmp_val, M, cap, saved->row_ptr, saved->col_idx, saved->val, s);
      }
    }
    if (rc) return rc;
    // Delta_A W with the unquantized W, fp32; lands where the GEMM epilogue picks it up
    float* R = bf16 ? w.R : reinterpret_cast<float*>(Y);
    rc = fp4_launch_spmm(saved->row_ptr, saved->col_idx, saved->val, cap, M, K, W, bf16, N, R, w.sp_scratch,
                         fp4_spmm_long_list_cap(provisioned_entries(M, K)), s);
    if (rc) return rc;
    addend = R;
  } else {
    if (act_tensor) {
      float* const g_all = reinterpret_cast<float*>(w.tg + TG_SCALAR);
      rc = fp4_launch_tensor_gamma(A, bf16, M, K, K, nullptr, w.tg, g_all, nullptr, 0, s);
      if (!rc) rc = fp4_launch_quantize_rows_fixed(A, bf16, M, K, K, g_all, w.qA, w.gA, s);
    } else {
      rc = fp4_launch_quantize_rows(A, bf16, M, K, K, w.qA, w.gA, s);
    }
    if (rc) return rc;
    if (saved->thresholds || saved->row_ptr || saved->nnz) {
      hipLaunchKernelGGL(init_no_occ_kernel, dim3((unsigned)((M + 1 + 255) / 256)), dim3(256), 0, s,
                         saved->thresholds, saved->row_ptr, M, saved->nnz);
      if (hipGetLastError() != hipSuccess) return FP4_ERR_HIP;
    }
  }
  return fp4_launch_gemm(w.qA, w.gA, qWt, saved->gamma_W, M, N, K, addend, Y, bf16, N, nullptr, 0, 0,
                         nullptr, 0.0f, 0.0f, s);
}

// Activation gradient; wq == nullptr: W is quantized per input channel here.
int dgrad_impl(const void* dY, const void* W, const fp4_weight_cache* wq, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
               void* dA, void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (M <= 0 || K <= 0 || N <= 0 || (N % 32) != 0 || (K % 8) != 0) return FP4_ERR_SHAPE;
  if (!dY || (!W && !wq) || !dA) return FP4_ERR_NULL;
  if (!aligned16(dY) || (W && !aligned16(W)) || !aligned16(dA)) return FP4_ERR_ARG;
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_DGRAD, M, K, N, dt)) return FP4_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int bf16 = dt == FP4_BF16;
  Carver c(reinterpret_cast<void*>(align_up((size_t)(uintptr_t)workspace, 256)));
  DgradWs w = carve_dgrad(c, M, K, N);
  int rc = fp4_launch_quantize_rows(dY, bf16, M, N, N, w.qdY, w.gdY, s);   // per token
  if (rc) return rc;
  const uint8_t* qW = w.qW;
  const float* gWk = w.gWk;
  if (wq) {
    qW = wq->qWk;
    gWk = wq->gamma_Wk;
  } else {
    rc = fp4_launch_quantize_rows(W, bf16, K, N, N, w.qW, w.gWk, s);       // per input channel
    if (rc) return rc;
  }
  return fp4_launch_gemm(w.qdY, w.gdY, qW, gWk, M, K, N, nullptr, dA, bf16, K, nullptr, 0, 0, nullptr, 0.0f, 0.0f, s);
}
}  // namespace

extern "C" int fp4_linear_fwd(const void* A, const void* W, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
                              double alpha, void* Y, const fp4_fwd_ctx* saved, void* workspace,
                              size_t workspace_bytes, void* stream) {
  return fwd_impl(A, W, nullptr, dt, M, K, N, alpha, Y, saved, workspace, workspace_bytes, stream);
}

extern "C" int fp4_linear_fwd_mixed(const void* A, const void* W, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
                                    fp4_format act_fmt, fp4_format wgt_fmt, double alpha, void* Y,
                                    const fp4_fwd_ctx* saved, void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  const bool a8 = act_fmt == FP4_FMT_E4M3 && wgt_fmt == FP4_FMT_E2M1;   // W4A8
  const bool w8 = act_fmt == FP4_FMT_E2M1 && wgt_fmt == FP4_FMT_E4M3;   // W8A4
  if (!a8 && !w8) return FP4_ERR_DTYPE;
  if (M <= 0 || K <= 0 || N <= 0 || (K % 128) != 0 || (N % 8) != 0) return FP4_ERR_SHAPE;
  if (!(alpha > 0.5) || !(alpha <= 1.0) || (a8 && alpha != 1.0)) return FP4_ERR_ARG;   // the clamp belongs to 4-bit activations
  if (!A || !W || !Y || !saved || !saved->gamma_W) return FP4_ERR_NULL;
  if (!aligned16(A) || !aligned16(W) || !aligned16(Y)) return FP4_ERR_ARG;
  const bool occ = alpha < 1.0;
  const int64_t k = tail_count(M * K, alpha);
  if (occ) {
    if (saved->scope != FP4_OCC_TENSOR) return FP4_ERR_DTYPE;
    if (!saved->thresholds || !saved->row_ptr || !saved->nnz) return FP4_ERR_NULL;
    if (saved->capacity < 2 * k) return FP4_ERR_CAPACITY;
    if (saved->capacity > 0 && (!saved->col_idx || !saved->val)) return FP4_ERR_NULL;
    if (2 * k > provisioned_entries(M, K)) return FP4_ERR_ARG;
  }
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_FWD_MIXED, M, K, N, dt)) return FP4_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int bf16 = dt == FP4_BF16;
  Carver c(reinterpret_cast<void*>(align_up((size_t)(uintptr_t)workspace, 256)));
  FwdWs w = carve_fwd_mixed(c, M, K, N, dt);
  int rc;
  if (w8) rc = fp8_launch_quantize_cols(W, bf16, K, N, N, w.qWt, saved->gamma_W, w.amax, s);
  else rc = fp4_launch_quantize_cols(W, bf16, K, N, N, nullptr, 0, w.qWt, saved->gamma_W, w.amax, s);
  if (rc) return rc;
  const float* addend = nullptr;
  if (a8) {
    rc = fp8_launch_quantize_rows(A, bf16, M, K, K, w.qA, w.gA, s);
    if (rc) return rc;
  } else if (occ) {
    const int64_t cap = std::min(saved->capacity, provisioned_entries(M, K));
    rc = fp4_launch_thresholds(A, bf16, M, K, K, k, saved->thresholds, w.occ.select, w.occ.total, s);
    if (!rc) rc = fp4_launch_occ_count(A, bf16, M, K, K, saved->thresholds, w.occ.row_cnt, s);
    if (!rc) rc = fp4_launch_scan_rows(w.occ.row_cnt, M, saved->row_ptr, saved->nnz, s);
    if (rc) return rc;
    rc = fp4_launch_occ_rows(A, bf16, M, K, K, saved->thresholds, w.qA, w.gA, nullptr, saved->col_idx, saved->val,
                             w.occ.tmp_col, w.occ.tmp_val, saved->row_ptr, cap, nullptr, s);
    if (rc == 1) {
      rc = fp4_launch_order_rows(saved->row_ptr, M, K, cap, w.occ.tmp_col, w.occ.tmp_val, saved->col_idx, saved->val, s);
      if (rc == 1)
        rc = fp4_launch_csr_gather(w.occ.tmp_col, w.occ.tmp_val, M, cap, saved->row_ptr, saved->col_idx, saved->val, s);
    }
    if (rc) return rc;
    float* R = bf16 ? w.R : reinterpret_cast<float*>(Y);
    rc = fp4_launch_spmm(saved->row_ptr, saved->col_idx, saved->val, cap, M, K, W, bf16, N, R, w.sp_scratch,
                         fp4_spmm_long_list_cap(provisioned_entries(M, K)), s);
    if (rc) return rc;
    addend = R;
  } else {
    rc = fp4_launch_quantize_rows(A, bf16, M, K, K, w.qA, w.gA, s);
    if (rc) return rc;
  }
  if (!occ && (saved->thresholds || saved->row_ptr || saved->nnz)) {
    hipLaunchKernelGGL(init_no_occ_kernel, dim3((unsigned)((M + 1 + 255) / 256)), dim3(256), 0, s, saved->thresholds,
                       saved->row_ptr, M, saved->nnz);
    if (hipGetLastError() != hipSuccess) return FP4_ERR_HIP;
  }
  return fp4_launch_gemm_mixed(w.qA, w.gA, w.qWt, saved->gamma_W, a8 ? 1 : 0, M, N, K, addend, Y, bf16, N, s);
}

extern "C" int fp4_linear_fwd_cached(const void* A, const void* W, const fp4_weight_cache* wq, fp4_dtype dt,
                                     int64_t M, int64_t K, int64_t N, double alpha, void* Y,
                                     const fp4_fwd_ctx* saved, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  if (!wq) return FP4_ERR_NULL;
  if (!cache_ok(wq)) return wq->qWt && wq->gamma_W && wq->qWk && wq->gamma_Wk ? FP4_ERR_ARG : FP4_ERR_NULL;
  return fwd_impl(A, W, wq, dt, M, K, N, alpha, Y, saved, workspace, workspace_bytes, stream);
}

extern "C" int fp4_prepare_weights(const void* W, fp4_dtype dt, int64_t K, int64_t N, const fp4_weight_cache* wq,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (K <= 0 || N <= 0 || (K % 32) != 0 || (N % 32) != 0) return FP4_ERR_SHAPE;
  if (!W || !wq) return FP4_ERR_NULL;
  if (!cache_ok(wq)) return wq->qWt && wq->gamma_W && wq->qWk && wq->gamma_Wk ? FP4_ERR_ARG : FP4_ERR_NULL;
  if (!aligned16(W)) return FP4_ERR_ARG;
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_PREPARE, 0, K, N, dt)) return FP4_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int bf16 = dt == FP4_BF16;
  uint32_t* amax = reinterpret_cast<uint32_t*>(align_up((size_t)(uintptr_t)workspace, 256));
  int rc = fp4_launch_quantize_cols(W, bf16, K, N, N, nullptr, 0, wq->qWt, wq->gamma_W, amax, s);   // forward's operand
  if (rc) return rc;
  return fp4_launch_quantize_rows(W, bf16, K, N, N, wq->qWk, wq->gamma_Wk, s);                   // dgrad's operand
}

extern "C" int fp4_linear_fwd_granularity(const void* A, const void* W, fp4_dtype dt, int64_t M, int64_t K, int64_t N,
                                          int act_tensorwise, int wgt_tensorwise, double alpha, void* Y,
                                          const fp4_fwd_ctx* saved, void* workspace, size_t workspace_bytes, void* stream) {
  return fwd_impl(A, W, nullptr, dt, M, K, N, alpha, Y, saved, workspace, workspace_bytes, stream, act_tensorwise != 0,
                  wgt_tensorwise != 0);
}

extern "C" int fp4_linear_bwd_dgrad(const void* dY, const void* W, fp4_dtype dt, int64_t M, int64_t K,
                                    int64_t N, void* dA, void* workspace, size_t workspace_bytes,
                                    void* stream) {
  if (!W) return FP4_ERR_NULL;
  return dgrad_impl(dY, W, nullptr, dt, M, K, N, dA, workspace, workspace_bytes, stream);
}

extern "C" int fp4_linear_bwd_dgrad_cached(const void* dY, const fp4_weight_cache* wq, fp4_dtype dt, int64_t M,
                                           int64_t K, int64_t N, void* dA, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  if (!wq) return FP4_ERR_NULL;
  if (!cache_ok(wq)) return wq->qWt && wq->gamma_W && wq->qWk && wq->gamma_Wk ? FP4_ERR_ARG : FP4_ERR_NULL;
  return dgrad_impl(dY, nullptr, wq, dt, M, K, N, dA, workspace, workspace_bytes, stream);
}

extern "C" int fp4_linear_bwd_wgrad(const void* A, const void* dY, const void* W, fp4_dtype dt, int64_t M,
                                    int64_t K, int64_t N, const fp4_fwd_ctx* saved, float dge_k,
                                    float dge_cap, float* dW, void* workspace, size_t workspace_bytes,
                                    void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (M <= 0 || K <= 0 || N <= 0 || (M % 32) != 0 || (K % 8) != 0 || (N % 8) != 0) return FP4_ERR_SHAPE;
  if (!A || !dY || !W || !dW || !saved || !saved->gamma_W) return FP4_ERR_NULL;
  if (dge_k > 0.0f && !(dge_cap > 0.0f)) return FP4_ERR_ARG;
  if (!aligned16(A) || !aligned16(dY) || !aligned16(W) || !aligned16(dW)) return FP4_ERR_ARG;
  // The residual is in play when the forward pass saved one (capacity > 0 with its arrays).
  const bool occ = saved->capacity > 0 && saved->row_ptr && saved->col_idx && saved->val && saved->nnz &&
                   saved->thresholds;
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_WGRAD, M, K, N, dt)) return FP4_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const int bf16 = dt == FP4_BF16;
  Carver c(reinterpret_cast<void*>(align_up((size_t)(uintptr_t)workspace, 256)));
  WgradWs w = carve_wgrad(c, M, K, N);
  if (saved->scope != FP4_OCC_TENSOR && saved->scope != FP4_OCC_TOKEN) return FP4_ERR_DTYPE;
  const int token = occ && saved->scope == FP4_OCC_TOKEN;   // thresholds: one pair per token
  // as the forward pass: entries beyond what the workspaces provide for cannot exist
  const int64_t cap = occ ? std::min(saved->capacity, provisioned_entries(M, K)) : 0;
  int rc = FP4_OK;
  if (occ)
    rc = fp4_launch_csr_transpose(saved->row_ptr, saved->col_idx, saved->val, saved->nnz, M, K, cap,
                                  w.t_ptr, w.t_idx, w.t_val, w.u_idx, w.u_val, w.t_scratch, s);
  // A_c per input channel (codes [K x M/2]); dY per output channel (codes [N x M/2])
  if (!rc) rc = fp4_launch_quantize_cols(A, bf16, M, K, K, occ ? saved->thresholds : nullptr, token, w.qAt, w.gAk, w.amax, s);
  if (!rc) rc = fp4_launch_quantize_cols(dY, bf16, M, N, N, nullptr, 0, w.qdYt, w.gdYn, w.amax, s);
  if (rc) return rc;
  const float* addend = nullptr;
  if (occ) {
    rc = fp4_launch_spmm(w.t_ptr, w.t_idx, w.t_val, cap, K, M, dY, bf16, N, dW, w.sp_scratch,
                         fp4_spmm_long_list_cap(provisioned_entries(M, K)), s);
    if (rc) return rc;
    addend = dW;
  }
  return fp4_launch_gemm(w.qAt, w.gAk, w.qdYt, w.gdYn, K, N, M, addend, dW, 0, N, W, bf16, N, saved->gamma_W,
                         dge_k, dge_cap, s);
}

// Both gradients of a layer in one call: dY is read once for its row-wise codes (activation gradient)
// and its column maxima (weight gradient) together; everything else as the two separate entry points.
extern "C" int fp4_linear_bwd(const void* dY, const void* A, const void* W, const fp4_weight_cache* wq, fp4_dtype dt,
                              int64_t M, int64_t K, int64_t N, const fp4_fwd_ctx* saved, float dge_k, float dge_cap,
                              void* dA, float* dW, void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (M <= 0 || K <= 0 || N <= 0 || (M % 32) != 0 || (N % 32) != 0 || (K % 8) != 0) return FP4_ERR_SHAPE;
  if (!dY || !A || !W || !dA || !dW || !saved || !saved->gamma_W) return FP4_ERR_NULL;
  if (wq && !cache_ok(wq)) return wq->qWt && wq->gamma_W && wq->qWk && wq->gamma_Wk ? FP4_ERR_ARG : FP4_ERR_NULL;
  if (dge_k > 0.0f && !(dge_cap > 0.0f)) return FP4_ERR_ARG;
  if (!aligned16(dY) || !aligned16(A) || !aligned16(W) || !aligned16(dA) || !aligned16(dW)) return FP4_ERR_ARG;
  if (saved->scope != FP4_OCC_TENSOR && saved->scope != FP4_OCC_TOKEN) return FP4_ERR_DTYPE;
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_BWD, M, K, N, dt)) return FP4_ERR_WORKSPACE;
  const bool occ = saved->capacity > 0 && saved->row_ptr && saved->col_idx && saved->val && saved->nnz && saved->thresholds;
  const int token = occ && saved->scope == FP4_OCC_TOKEN;
  hipStream_t s = (hipStream_t)stream;
  const int bf16 = dt == FP4_BF16;
  Carver c(reinterpret_cast<void*>(align_up((size_t)(uintptr_t)workspace, 256)));
  DgradWs d = carve_dgrad(c, M, K, N);
  WgradWs w = carve_wgrad(c, M, K, N);
  uint16_t* part = c.take<uint16_t>((size_t)fp4_dual_axis_part_elems(M, N));
  // dY: per token (codes for the activation gradient) and, in the same read, per-block column maxima
  int rc = fp4_launch_quantize_rows_colmax(dY, bf16, M, N, N, d.qdY, d.gdY, part, s);
  const bool dual = rc == 0;
  if (rc == 1) rc = fp4_launch_quantize_rows(dY, bf16, M, N, N, d.qdY, d.gdY, s);
  if (rc) return rc;
  // activation gradient
  const uint8_t* qW = d.qW;
  const float* gWk = d.gWk;
  if (wq) { qW = wq->qWk; gWk = wq->gamma_Wk; }
  else {
    rc = fp4_launch_quantize_rows(W, bf16, K, N, N, d.qW, d.gWk, s);
    if (rc) return rc;
  }
  rc = fp4_launch_gemm(d.qdY, d.gdY, qW, gWk, M, K, N, nullptr, dA, bf16, K, nullptr, 0, 0, nullptr, 0.0f, 0.0f, s);
  if (rc) return rc;
  // weight gradient
  const int64_t cap = occ ? std::min(saved->capacity, provisioned_entries(M, K)) : 0;
  if (occ) {
    rc = fp4_launch_csr_transpose(saved->row_ptr, saved->col_idx, saved->val, saved->nnz, M, K, cap, w.t_ptr, w.t_idx,
                                  w.t_val, w.u_idx, w.u_val, w.t_scratch, s);
    if (rc) return rc;
  }
  rc = fp4_launch_quantize_cols(A, bf16, M, K, K, occ ? saved->thresholds : nullptr, token, w.qAt, w.gAk, w.amax, s);
  if (rc) return rc;
  if (dual) rc = fp4_launch_quantize_cols_known_max(dY, M, N, N, part, w.qdYt, w.gdYn, s);
  else rc = fp4_launch_quantize_cols(dY, bf16, M, N, N, nullptr, 0, w.qdYt, w.gdYn, w.amax, s);
  if (rc) return rc;
  const float* addend = nullptr;
  if (occ) {
    rc = fp4_launch_spmm(w.t_ptr, w.t_idx, w.t_val, cap, K, M, dY, bf16, N, dW, w.sp_scratch,
                         fp4_spmm_long_list_cap(provisioned_entries(M, K)), s);
    if (rc) return rc;
    addend = dW;
  }
  return fp4_launch_gemm(w.qAt, w.gAk, w.qdYt, w.gdYn, K, N, M, addend, dW, 0, N, W, bf16, N, saved->gamma_W, dge_k,
                         dge_cap, s);
}

extern "C" int fp4_residual_spmm(const int64_t* row_ptr, const int32_t* col_idx, const float* val,
                                 int64_t P, int64_t Q, const void* D, fp4_dtype dt, int64_t N, float* R,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (!dtype_ok(dt)) return FP4_ERR_DTYPE;
  if (P < 0 || Q < 0 || N < 0 || (N % 8) != 0) return FP4_ERR_SHAPE;
  if (P == 0 || N == 0) return FP4_OK;
  if (!row_ptr || !D || !R) return FP4_ERR_NULL;
  if (!aligned16(D) || !aligned16(R)) return FP4_ERR_ARG;
  if (!workspace || workspace_bytes < fp4_workspace_bytes(FP4_OP_SPMM, P, Q, N, dt)) return FP4_ERR_WORKSPACE;
  int32_t* scratch = reinterpret_cast<int32_t*>(align_up((size_t)(uintptr_t)workspace, 256));
  // no entry limit besides row_ptr itself; the long-row list is sized by P
  return fp4_launch_spmm(row_ptr, col_idx, val, INT64_MAX, P, Q, D, dt == FP4_BF16, N, R, scratch, P + 2,
                         (hipStream_t)stream);
}
