// Outlier clamping and compensation (Sec. 3.2): exact per-tensor quantile thresholds by
// radix selection, canonical CSR of the clamped-away residual, its transpose for the weight
// gradient, and the sparse x dense high-precision product.
#include "fp4_common.h"

#include <algorithm>

namespace {

struct BF16 {};
struct F32 {};

constexpr int SEL_BINS = 2048;  // 11-bit digits

// Selection state kept in the workspace between passes.
struct SelState {
  unsigned long long rank[2];  // remaining 0-based rank of the lo / hi order statistic
  uint32_t prefix[2];          // key bits fixed so far (right-aligned)
  uint32_t pad[2];
};

template <class DT>
FP4_D uint32_t load_key(const void* x, int64_t off) {
  if constexpr (__is_same(DT, BF16)) {
    uint32_t h = reinterpret_cast<const uint16_t*>(x)[off];
    return f32_order_key(h << 16) >> 16;  // 16-bit key
  } else {
    return f32_order_key(reinterpret_cast<const uint32_t*>(x)[off]);
  }
}

__global__ void sel_init_kernel(SelState* st, unsigned long long* hist, unsigned long long k,
                                unsigned long long n, unsigned long long* total) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < 2 * SEL_BINS) hist[i] = 0;
  if (i == 0) {
    st->rank[0] = k;
    st->rank[1] = n - 1 - k;
    st->prefix[0] = st->prefix[1] = 0;
    if (total) *total = 0;
  }
}

// One digit pass: histogram of key digit (key >> shift) & (2^bits - 1) over the elements whose
// higher bits equal the prefix found so far (first pass: all elements, one shared histogram).
template <class DT>
__global__ __launch_bounds__(256) void sel_hist_kernel(const void* x, int64_t rows, int64_t cols,
                                                       int64_t ld, int shift, int bits, int first,
                                                       const SelState* st, unsigned long long* hist) {
  __shared__ uint32_t h[2][SEL_BINS];
  for (int i = threadIdx.x; i < 2 * SEL_BINS; i += 256) (&h[0][0])[i] = 0;
  __syncthreads();
  const uint32_t mask = (1u << bits) - 1u;
  const uint32_t p0 = st->prefix[0], p1 = st->prefix[1];
  const int hs = shift + bits;
  const int64_t n = rows * cols;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / cols, c = i - r * cols;
    const uint32_t key = load_key<DT>(x, r * ld + c);
    const uint32_t d = (key >> shift) & mask;
    if (first) {
      atomicAdd(&h[0][d], 1u);
    } else {
      const uint32_t hi_bits = hs >= 32 ? 0u : (key >> hs);
      if (hi_bits == p0) atomicAdd(&h[0][d], 1u);
      if (hi_bits == p1) atomicAdd(&h[1][d], 1u);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * SEL_BINS; i += 256) {
    uint32_t v = (&h[0][0])[i];
    if (v) atomicAdd(&hist[i], (unsigned long long)v);
  }
}

// Pick, for each of the two targets, the bin that holds its rank; extend the prefix, reduce
// the rank, clear the histograms.  After the last pass the prefix is the full key: decode it.
__global__ __launch_bounds__(256) void sel_pick_kernel(SelState* st, unsigned long long* hist, int bits,
                                                       int first, int last, int key_bits,
                                                       float* thresholds) {
  __shared__ unsigned long long part[256];
  const int nb = 1 << bits;
  const int per = (nb + 255) / 256;
  for (int s = 0; s < 2; ++s) {
    const unsigned long long* hsrc = hist + (first ? 0 : s * SEL_BINS);
    unsigned long long sum = 0;
    for (int j = 0; j < per; ++j) {
      int b = threadIdx.x * per + j;
      if (b < nb) sum += hsrc[b];
    }
    part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      unsigned long long r = st->rank[s], cum = 0;
      int t = 0;
      while (t < 255 && cum + part[t] <= r) { cum += part[t]; ++t; }
      int b = t * per;
      const int bend = min(nb, b + per);
      while (b < bend - 1 && cum + hsrc[b] <= r) { cum += hsrc[b]; ++b; }
      st->rank[s] = r - cum;
      st->prefix[s] = (st->prefix[s] << bits) | (uint32_t)b;
      if (last) {
        uint32_t key = st->prefix[s];
        if (key_bits == 16) {
          // 16-bit keys are the top half of the fp32 key of a bf16 value; undo the map on
          // 16 bits so the low half of the fp32 pattern stays zero
          const uint32_t h = (key & 0x8000u) ? (key & 0x7fffu) : (~key & 0xffffu);
          thresholds[s] = u2f(h << 16);
        } else {
          thresholds[s] = u2f(f32_from_order_key(key));
        }
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < 2 * SEL_BINS; i += 256) hist[i] = 0;
}

// ---- CSR finalisation ---------------------------------------------------------------------
// ptr[0] = 0, ptr[i+1] = sum cnt[0..i]; optional copy of the total.  One workgroup.
__global__ __launch_bounds__(1024) void scan_counts_kernel(const int32_t* cnt, int64_t n, int64_t* ptr,
                                                           int64_t* total_out) {
  __shared__ long long s[1024];
  __shared__ long long carry;
  if (threadIdx.x == 0) { carry = 0; ptr[0] = 0; }
  __syncthreads();
  for (int64_t base = 0; base < n; base += 1024) {
    const int64_t i = base + threadIdx.x;
    long long v = i < n ? cnt[i] : 0;
    s[threadIdx.x] = v;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      long long add = threadIdx.x >= o ? s[threadIdx.x - o] : 0;
      __syncthreads();
      s[threadIdx.x] += add;
      __syncthreads();
    }
    if (i < n) ptr[i + 1] = carry + s[threadIdx.x];
    __syncthreads();
    if (threadIdx.x == 1023) carry += s[1023];
    __syncthreads();
  }
  if (threadIdx.x == 0 && total_out) *total_out = carry;
}

// One wave per row: move the row's temporary entries to their canonical place, ascending
// column order (rank of a column among the row's columns; columns are distinct).
__global__ __launch_bounds__(256) void csr_gather_kernel(const int32_t* tmp_col, const float* tmp_val,
                                                         const int64_t* row_start, const int32_t* row_cnt,
                                                         const int64_t* row_ptr, int64_t rows, int64_t capacity,
                                                         int32_t* col_idx, float* val) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int L = row_cnt[row];
  const int64_t src = row_start[row], dst = row_ptr[row];
  if (src + L > capacity || dst + L > capacity) return;  // truncated output, nnz tells
  for (int i = lane; i < L; i += 64) {
    const int32_t c = tmp_col[src + i];
    int rank = 0;
    for (int j = 0; j < L; ++j) rank += tmp_col[src + j] < c ? 1 : 0;
    col_idx[dst + rank] = c;
    val[dst + rank] = tmp_val[src + i];
  }
}

// ---- CSR transpose (P x Q -> Q x P) -----------------------------------------------------------
__global__ void fill_i32_kernel(int32_t* p, int64_t n, int32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ void csr_count_cols_kernel(const int32_t* col_idx, const int64_t* nnz, int64_t capacity,
                                      int32_t* cnt) {
  const int64_t n = min((int64_t)*nnz, capacity);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    atomicAdd(&cnt[col_idx[i]], 1);
}

__global__ __launch_bounds__(256) void csr_transpose_fill_kernel(const int64_t* row_ptr, const int32_t* col_idx,
                                                                 const float* val, int64_t rows, int64_t capacity,
                                                                 const int64_t* t_ptr, int32_t* cursor,
                                                                 int32_t* t_idx, float* t_val) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int64_t b = row_ptr[row], e = min(row_ptr[row + 1], capacity);
  for (int64_t i = b + lane; i < e; i += 64) {
    const int32_t c = col_idx[i];
    const int64_t pos = t_ptr[c] + atomicAdd(&cursor[c], 1);
    t_idx[pos] = (int32_t)row;
    t_val[pos] = val[i];
  }
}

// Order each transposed row by index so the product below sums in a fixed order.  One
// workgroup per row; rows up to SORT_MAX entries are sorted in LDS (bitonic), longer rows
// are left in arrival order.
constexpr int SORT_MAX = 16384;
__global__ __launch_bounds__(256) void csr_sort_rows_kernel(const int64_t* ptr, int64_t rows, int32_t* idx,
                                                            float* val) {
  __shared__ unsigned long long s_kv[SORT_MAX];
  const int64_t row = blockIdx.x;
  const int64_t b = ptr[row];
  const int L = (int)(ptr[row + 1] - b);
  if (L < 2 || L > SORT_MAX) return;
  int n = 1;
  while (n < L) n <<= 1;
  for (int i = threadIdx.x; i < n; i += 256)
    s_kv[i] = i < L ? (((unsigned long long)(uint32_t)idx[b + i] << 32) | f2u(val[b + i])) : ~0ull;
  __syncthreads();
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = threadIdx.x; i < n; i += 256) {
        const int p = i ^ j;
        if (p > i) {
          const bool up = (i & k) == 0;
          unsigned long long a = s_kv[i], c = s_kv[p];
          if ((a > c) == up) { s_kv[i] = c; s_kv[p] = a; }
        }
      }
      __syncthreads();
    }
  }
  for (int i = threadIdx.x; i < L; i += 256) {
    idx[b + i] = (int32_t)(s_kv[i] >> 32);
    val[b + i] = u2f((uint32_t)s_kv[i]);
  }
}

// ---- sparse x dense: R[p, :] = sum_e val[e] * D[col[e], :] ------------------------------------
template <class DT>
FP4_D void load8d(const void* base, int64_t off, int valid, float (&v)[8]) {
  if (valid >= 8) {
    if constexpr (__is_same(DT, BF16)) {
      u32x4 r = *reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(base) + off);
      v[0] = u2f(r.x << 16); v[1] = u2f(r.x & 0xffff0000u);
      v[2] = u2f(r.y << 16); v[3] = u2f(r.y & 0xffff0000u);
      v[4] = u2f(r.z << 16); v[5] = u2f(r.z & 0xffff0000u);
      v[6] = u2f(r.w << 16); v[7] = u2f(r.w & 0xffff0000u);
    } else {
      const f32x4* p = reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(base) + off);
      f32x4 a = p[0], b = p[1];
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
      v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float f = 0.0f;
      if (e < valid) {
        if constexpr (__is_same(DT, BF16))
          f = bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(base)[off + e]);
        else
          f = reinterpret_cast<const float*>(base)[off + e];
      }
      v[e] = f;
    }
  }
}

template <class DT>
__global__ __launch_bounds__(256) void spmm_rows_kernel(const int64_t* row_ptr, const int32_t* col_idx,
                                                        const float* val, int64_t capacity, const void* D,
                                                        int64_t N, float* R) {
  const int64_t row = blockIdx.x;
  const int64_t col = ((int64_t)blockIdx.y * 256 + threadIdx.x) * 8;
  if (col >= N) return;
  const int valid = (int)min((int64_t)8, N - col);
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
  const int64_t b = row_ptr[row], en = min(row_ptr[row + 1], capacity);
  for (int64_t i = b; i < en; ++i) {
    const int32_t c = col_idx[i];
    const float s = val[i];
    float d[8];
    load8d<DT>(D, (int64_t)c * N + col, valid, d);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = fmaf(s, d[e], acc[e]);
  }
  float* o = R + row * N + col;
  if (valid >= 8 && (N % 4) == 0) {
    f32x4 a = {acc[0], acc[1], acc[2], acc[3]}, c4 = {acc[4], acc[5], acc[6], acc[7]};
    reinterpret_cast<f32x4*>(o)[0] = a;
    reinterpret_cast<f32x4*>(o)[1] = c4;
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (e < valid) o[e] = acc[e];
  }
}

}  // namespace

// ---- internal launchers -----------------------------------------------------------------------
size_t fp4_select_scratch_bytes() {
  return align_up(sizeof(SelState), 256) + align_up(2 * SEL_BINS * sizeof(unsigned long long), 256);
}

// Thresholds lo = v[k], hi = v[n-1-k] of the ascending-sorted tensor into thresholds[0..1].
// Also zeroes *total (the residual entry counter) when given.
int fp4_launch_thresholds(const void* x, int bf16, int64_t rows, int64_t cols, int64_t ld, int64_t k,
                          float* thresholds, void* scratch, unsigned long long* total, hipStream_t s) {
  SelState* st = reinterpret_cast<SelState*>(scratch);
  unsigned long long* hist =
      reinterpret_cast<unsigned long long*>(reinterpret_cast<uint8_t*>(scratch) + align_up(sizeof(SelState), 256));
  const int64_t n = rows * cols;
  hipLaunchKernelGGL(sel_init_kernel, dim3(2 * SEL_BINS / 256), dim3(256), 0, s, st, hist,
                     (unsigned long long)k, (unsigned long long)n, total);
  const int key_bits = bf16 ? 16 : 32;
  int digits[3];
  int nd;
  if (bf16) { digits[0] = 11; digits[1] = 5; nd = 2; }
  else { digits[0] = 11; digits[1] = 11; digits[2] = 10; nd = 3; }
  int shift = key_bits;
  const unsigned grid = (unsigned)std::min<int64_t>((n + 256 * 16 - 1) / (256 * 16), 2048);
  for (int p = 0; p < nd; ++p) {
    shift -= digits[p];
    if (bf16)
      hipLaunchKernelGGL((sel_hist_kernel<BF16>), dim3(grid), dim3(256), 0, s, x, rows, cols, ld, shift,
                         digits[p], p == 0, st, hist);
    else
      hipLaunchKernelGGL((sel_hist_kernel<F32>), dim3(grid), dim3(256), 0, s, x, rows, cols, ld, shift,
                         digits[p], p == 0, st, hist);
    hipLaunchKernelGGL(sel_pick_kernel, dim3(1), dim3(256), 0, s, st, hist, digits[p], p == 0, p == nd - 1,
                       key_bits, thresholds);
  }
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

int fp4_launch_csr_finalize(const int32_t* tmp_col, const float* tmp_val, const int64_t* row_start,
                            const int32_t* row_cnt, int64_t rows, int64_t capacity, int64_t* row_ptr,
                            int32_t* col_idx, float* val, int64_t* nnz, hipStream_t s) {
  hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(1024), 0, s, row_cnt, rows, row_ptr, nnz);
  hipLaunchKernelGGL(csr_gather_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, tmp_col, tmp_val,
                     row_start, row_cnt, row_ptr, rows, capacity, col_idx, val);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

// scratch: cnt[Q] + cursor[Q] int32
int fp4_launch_csr_transpose(const int64_t* row_ptr, const int32_t* col_idx, const float* val,
                             const int64_t* nnz, int64_t P, int64_t Q, int64_t capacity, int64_t* t_ptr,
                             int32_t* t_idx, float* t_val, int32_t* scratch, hipStream_t s) {
  int32_t* cnt = scratch;
  int32_t* cursor = scratch + Q;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((2 * Q + 255) / 256)), dim3(256), 0, s, scratch, 2 * Q, 0);
  const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((capacity + 255) / 256, 4096));
  hipLaunchKernelGGL(csr_count_cols_kernel, dim3(grid), dim3(256), 0, s, col_idx, nnz, capacity, cnt);
  hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(1024), 0, s, cnt, Q, t_ptr, (int64_t*)nullptr);
  hipLaunchKernelGGL(csr_transpose_fill_kernel, dim3((unsigned)((P + 3) / 4)), dim3(256), 0, s, row_ptr,
                     col_idx, val, P, capacity, t_ptr, cursor, t_idx, t_val);
  hipLaunchKernelGGL(csr_sort_rows_kernel, dim3((unsigned)Q), dim3(256), 0, s,
                     t_ptr, Q, t_idx, t_val);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

int fp4_launch_spmm(const int64_t* row_ptr, const int32_t* col_idx, const float* val, int64_t capacity,
                    int64_t P, const void* D, int bf16, int64_t N, float* R, hipStream_t s) {
  if (P == 0 || N == 0) return FP4_OK;
  dim3 grid((unsigned)P, (unsigned)((N + 2047) / 2048));
  if (bf16)
    hipLaunchKernelGGL((spmm_rows_kernel<BF16>), grid, dim3(256), 0, s, row_ptr, col_idx, val, capacity, D, N, R);
  else
    hipLaunchKernelGGL((spmm_rows_kernel<F32>), grid, dim3(256), 0, s, row_ptr, col_idx, val, capacity, D, N, R);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

extern "C" int fp4_residual_spmm(const int64_t* row_ptr, const int32_t* col_idx, const float* val,
                                 int64_t P, int64_t Q, const void* D, fp4_dtype dt, int64_t N, float* R,
                                 void* stream) {
  if (dt != FP4_F32 && dt != FP4_BF16) return FP4_ERR_DTYPE;
  if (P < 0 || Q < 0 || N < 0 || (N % 8) != 0) return FP4_ERR_SHAPE;
  if (P == 0 || N == 0) return FP4_OK;
  if (!row_ptr || !D || !R) return FP4_ERR_NULL;
  if (!aligned16(D) || !aligned16(R)) return FP4_ERR_ARG;
  return fp4_launch_spmm(row_ptr, col_idx, val, INT64_MAX, P, D, dt == FP4_BF16, N, R, (hipStream_t)stream);
}
