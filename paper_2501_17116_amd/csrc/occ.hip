// Outlier clamping and compensation (Sec. 3.2): exact per-tensor quantile thresholds by
// radix selection, and the ordering of the clamped-away residual of long rows into canonical
// CSR.  (The clamp itself is fused into the quantization pass; the transpose for the weight
// gradient and the sparse x dense product live with the sparse kernels.)
#include "fp4_common.h"

#include <algorithm>

namespace {

struct BF16 {};
struct F32 {};

typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr int SEL_BINS = 2048;  // 11-bit digits
constexpr int SEL_THREADS = 1024;   // per workgroup: the 64 KiB of LDS tables allow two workgroups per CU,
                                    // so their size decides how many loads a CU has in flight

// Selection state kept in the workspace between passes.
struct SelState {
  unsigned long long rank[2];  // remaining 0-based rank of the lo / hi order statistic
  uint32_t prefix[2];          // key bits fixed so far (right-aligned)
  uint32_t pad[2];
};

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
// The workgroup histogram is replicated (by lane) to thin out same-address LDS atomics: real
// tensors put most of their mass in a few dozen exponent bins.
template <class DT>
FP4_D uint32_t key_of(uint32_t raw) {   // raw: bf16 bits (low 16) or fp32 bits
  if constexpr (__is_same(DT, BF16)) return f32_order_key(raw << 16) >> 16;
  else return f32_order_key(raw);
}

template <class DT>
__global__ __launch_bounds__(SEL_THREADS) void sel_hist_kernel(const void* x, int64_t rows, int64_t cols,
                                                       int64_t ld, int shift, int bits, int first,
                                                       const SelState* st, unsigned long long* hist) {
  __shared__ uint32_t h[8 * SEL_BINS];   // first pass: 8 replicas; later: 4 replicas x 2 targets
  for (int i = threadIdx.x; i < 8 * SEL_BINS; i += SEL_THREADS) h[i] = 0;
  __syncthreads();
  const uint32_t mask = (1u << bits) - 1u;
  const uint32_t p0 = st->prefix[0], p1 = st->prefix[1];
  const int hs = shift + bits;
  const int lane = threadIdx.x & 63;
  uint32_t* const hrep = first ? &h[(lane & 7) * SEL_BINS] : &h[(lane & 3) * 2 * SEL_BINS];
  auto visit = [&](uint32_t raw) {
    const uint32_t key = key_of<DT>(raw);
    const uint32_t d = (key >> shift) & mask;
    if (first) {
      atomicAdd(&hrep[d], 1u);
    } else {
      const uint32_t hi_bits = hs >= 32 ? 0u : (key >> hs);
      if (hi_bits == p0) atomicAdd(&hrep[d], 1u);
      if (hi_bits == p1) atomicAdd(&hrep[SEL_BINS + d], 1u);
    }
  };
  constexpr int EPV = __is_same(DT, BF16) ? 8 : 4;   // elements per 16-byte load
  const bool flat = (ld == cols) && (cols % EPV) == 0;
  if (flat) {
    const int64_t nvec = rows * cols / EPV;
    const u32x4* xv = reinterpret_cast<const u32x4*>(x);
    auto visit_vec = [&](const u32x4& r) {
      if constexpr (__is_same(DT, BF16)) {
        visit(r.x & 0xffffu); visit(r.x >> 16); visit(r.y & 0xffffu); visit(r.y >> 16);
        visit(r.z & 0xffffu); visit(r.z >> 16); visit(r.w & 0xffffu); visit(r.w >> 16);
      } else {
        visit(r.x); visit(r.y); visit(r.z); visit(r.w);
      }
    };
    // four loads in flight per lane: with the LDS tables limiting a CU to two workgroups, one
    // load at a time leaves the memory pipe mostly idle
    const int64_t stride = (int64_t)gridDim.x * SEL_THREADS;
    int64_t i = (int64_t)blockIdx.x * SEL_THREADS + threadIdx.x;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
      const u32x4 r0 = xv[i], r1 = xv[i + stride], r2 = xv[i + 2 * stride], r3 = xv[i + 3 * stride];
      visit_vec(r0); visit_vec(r1); visit_vec(r2); visit_vec(r3);
    }
    for (; i < nvec; i += stride) visit_vec(xv[i]);
  } else {
    const int64_t n = rows * cols;
    for (int64_t i = (int64_t)blockIdx.x * SEL_THREADS + threadIdx.x; i < n; i += (int64_t)gridDim.x * SEL_THREADS) {
      const int64_t r = i / cols, c = i - r * cols;
      if constexpr (__is_same(DT, BF16)) visit(reinterpret_cast<const uint16_t*>(x)[r * ld + c]);
      else visit(reinterpret_cast<const uint32_t*>(x)[r * ld + c]);
    }
  }
  __syncthreads();
  if (first) {
    for (int i = threadIdx.x; i < SEL_BINS; i += SEL_THREADS) {
      uint32_t v = 0;
#pragma unroll
      for (int r = 0; r < 8; ++r) v += h[r * SEL_BINS + i];
      if (v) atomicAdd(&hist[i], (unsigned long long)v);
    }
  } else {
    for (int i = threadIdx.x; i < 2 * SEL_BINS; i += SEL_THREADS) {
      uint32_t v = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) v += h[r * 2 * SEL_BINS + i];
      if (v) atomicAdd(&hist[i], (unsigned long long)v);
    }
  }
}

// Pick, for each of the two targets, the bin that holds its rank; extend the prefix, reduce
// the rank, clear the histograms.  After the last pass the prefix is the full key: decode it.
__global__ __launch_bounds__(256) void sel_pick_kernel(SelState* st, unsigned long long* hist, int bits,
                                                       int first, int last, int key_bits,
                                                       float* thresholds) {
  constexpr int PER = SEL_BINS / 256;   // bins a thread owns when all SEL_BINS are in use
  __shared__ unsigned long long s_w[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nb = 1 << bits;
  const int per = (nb + 255) / 256;
  // both targets' bins and ranks are requested before either scan starts
  unsigned long long vv[2][PER], rr[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const unsigned long long* hsrc = hist + (first ? 0 : s * SEL_BINS);
    rr[s] = st->rank[s];
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const int b = tid * per + j;
      vv[s][j] = (j < per && b < nb) ? hsrc[b] : 0;
    }
  }
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    unsigned long long (&v)[PER] = vv[s];
    unsigned long long sum = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) sum += v[j];
    // inclusive prefix of the threads' sums: the thread whose range [excl, incl) holds the rank
    // owns the bin (the last thread, should the rank lie beyond the total)
    unsigned long long incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned long long up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += s_w[w];
    const unsigned long long r = rr[s];
    const unsigned long long excl = incl - sum;
    if ((excl <= r && r < incl) || (tid == 255 && r >= incl)) {
      unsigned long long cum = excl;
      int j = 0;
      const int jend = min(per, nb - tid * per);   // bins of this thread that exist (may be <= 0)
#pragma unroll
      for (int q = 0; q < PER - 1; ++q)
        if (j == q && q < jend - 1 && cum + v[q] <= r) { cum += v[q]; ++j; }
      const int b = min(tid * per + j, nb - 1);
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
  for (int i = tid; i < 2 * SEL_BINS; i += 256) hist[i] = 0;
}

// ---- CSR finalisation ---------------------------------------------------------------------
// ptr[0] = 0, ptr[i+1] = sum cnt[0..i]; optional copy of the total.  One workgroup; a thread
// takes 16 consecutive counts, so one block scan covers 16384 of them.
__global__ __launch_bounds__(1024) void scan_counts_kernel(const int32_t* cnt, int64_t n, int64_t* ptr,
                                                           int64_t* total_out) {
  __shared__ long long s_w[16];
  __shared__ long long carry;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) { carry = 0; ptr[0] = 0; }
  __syncthreads();
  for (int64_t base = 0; base < n; base += 16 * 1024) {
    const int64_t i0 = base + (int64_t)threadIdx.x * 16;
    int32_t c[16];
    if (i0 + 16 <= n) {   // 64 aligned bytes: four loads in flight instead of sixteen guarded ones in a row
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const i32x4 t = reinterpret_cast<const i32x4*>(cnt + i0)[q];
        c[4 * q] = t.x; c[4 * q + 1] = t.y; c[4 * q + 2] = t.z; c[4 * q + 3] = t.w;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j) c[j] = i0 + j < n ? cnt[i0 + j] : 0;
    }
    long long v[16];
    long long sum = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      sum += c[j];
      v[j] = sum;   // inclusive inside the thread
    }
    long long incl = sum;   // inclusive over the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const long long up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    long long before = carry + incl - sum;
    for (int w = 0; w < wave; ++w) before += s_w[w];
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (i0 + j < n) ptr[i0 + j + 1] = before + v[j];
    __syncthreads();
    if (threadIdx.x == 1023) carry = before + sum;
    __syncthreads();
  }
  if (threadIdx.x == 0 && total_out) *total_out = carry;
}

// One wave per row: move the row's temporary entries to their canonical place (same segment
// of the final arrays), ascending column order (rank of a column among the row's columns; columns are distinct).
__global__ __launch_bounds__(256) void csr_gather_kernel(const int32_t* tmp_col, const float* tmp_val,
                                                         const int64_t* row_ptr, int64_t rows, int64_t capacity,
                                                         int32_t* col_idx, float* val) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int64_t src = row_ptr[row];
  const int64_t en = row_ptr[row + 1];
  if (en > capacity) return;  // truncated output, nnz tells
  const int L = (int)(en - src);
  for (int i = lane; i < L; i += 64) {
    const int32_t c = tmp_col[src + i];
    int rank = 0;
    for (int j = 0; j < L; ++j) rank += tmp_col[src + j] < c ? 1 : 0;
    col_idx[src + rank] = c;
    val[src + rank] = tmp_val[src + i];
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
  const unsigned grid =
      (unsigned)std::max<int64_t>(1, std::min<int64_t>((n + SEL_THREADS * 64 - 1) / (SEL_THREADS * 64), 512));
  for (int p = 0; p < nd; ++p) {
    shift -= digits[p];
    if (bf16)
      hipLaunchKernelGGL((sel_hist_kernel<BF16>), dim3(grid), dim3(SEL_THREADS), 0, s, x, rows, cols, ld, shift,
                         digits[p], p == 0, st, hist);
    else
      hipLaunchKernelGGL((sel_hist_kernel<F32>), dim3(grid), dim3(SEL_THREADS), 0, s, x, rows, cols, ld, shift,
                         digits[p], p == 0, st, hist);
    hipLaunchKernelGGL(sel_pick_kernel, dim3(1), dim3(256), 0, s, st, hist, digits[p], p == 0, p == nd - 1,
                       key_bits, thresholds);
  }
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

int fp4_launch_scan_rows(const int32_t* row_cnt, int64_t rows, int64_t* row_ptr, int64_t* nnz, hipStream_t s) {
  hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(1024), 0, s, row_cnt, rows, row_ptr, nnz);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}

int fp4_launch_csr_gather(const int32_t* tmp_col, const float* tmp_val, int64_t rows, int64_t capacity,
                          const int64_t* row_ptr, int32_t* col_idx, float* val, hipStream_t s) {
  hipLaunchKernelGGL(csr_gather_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, tmp_col, tmp_val,
                     row_ptr, rows, capacity, col_idx, val);
  FP4_CHECK_LAUNCH();
  return FP4_OK;
}
